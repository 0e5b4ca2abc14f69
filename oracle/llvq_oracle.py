"""ctypes access to the LLVQ oracle (oracle/llvq_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests, the smoke check and the
cpu_baseline leg of the benchmark may import this module.  The GPU library and
its Python binding never do.

The C file is the oracle; this module only marshals numpy arrays into it and
reduces the matrix product to a library routine (numpy's fp64 matmul over the
oracle-decoded dense matrix) so that the C triple loop has something other
than itself to be compared with.
"""
import atexit
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "llvq_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

M_MAX_DEFAULT = 13


def build(force=False):
    """Compile the oracle with gcc (plain C, no GPU code)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_loaded = {}      # m_max -> path of the library image initialised for it


def _image_for(m_max):
    """The C oracle keeps its tables in globals, one ball cut per loaded image: every distinct m_max gets a
    private copy of the shared object, so that oracles for different cuts can be alive at the same time."""
    import shutil
    import tempfile
    path = build()
    if m_max not in _loaded:
        if _loaded:
            fd, private = tempfile.mkstemp(prefix="liboracle_m%d_" % m_max, suffix=".so")
            os.close(fd)
            shutil.copyfile(path, private)
            atexit.register(lambda f=private: os.path.exists(f) and os.remove(f))
            path = private
        _loaded[m_max] = path
    return _loaded[m_max]


class Oracle:
    def __init__(self, m_max=M_MAX_DEFAULT):
        lib = ctypes.CDLL(_image_for(m_max))
        u64, i32 = ctypes.c_uint64, ctypes.c_int
        p = ctypes.c_void_p
        lib.oracle_init.argtypes = [i32]; lib.oracle_init.restype = i32
        lib.oracle_num_points.restype = u64
        lib.oracle_num_classes.restype = i32
        lib.oracle_shell_size.argtypes = [i32]; lib.oracle_shell_size.restype = u64
        lib.oracle_golay_word.argtypes = [i32]; lib.oracle_golay_word.restype = ctypes.c_uint32
        lib.oracle_golay_sorted.argtypes = [i32]; lib.oracle_golay_sorted.restype = ctypes.c_uint32
        lib.oracle_class_info.argtypes = [i32] + [p] * 12
        lib.oracle_decode.argtypes = [u64, p]; lib.oracle_decode.restype = i32
        lib.oracle_encode.argtypes = [p, p]; lib.oracle_encode.restype = i32
        lib.oracle_is_member.argtypes = [p]; lib.oracle_is_member.restype = i32
        lib.oracle_decode_batch.argtypes = [p, u64, p]; lib.oracle_decode_batch.restype = u64
        lib.oracle_decode_range.argtypes = [u64, u64, p]; lib.oracle_decode_range.restype = u64
        lib.oracle_encode_batch.argtypes = [p, u64, p]; lib.oracle_encode_batch.restype = u64
        lib.oracle_dequant_batch.argtypes = [p, p, u64, p]; lib.oracle_dequant_batch.restype = u64
        lib.oracle_matmul.argtypes = [p, p, i32, i32, p, i32, p]; lib.oracle_matmul.restype = None
        lib.oracle_nearest_batch.argtypes = [p, u64, i32, p, p]; lib.oracle_nearest_batch.restype = None
        self.lib = lib
        self.m_max = m_max
        n = lib.oracle_init(m_max)
        if n <= 0:
            raise ValueError("oracle_init failed for m_max=%r" % (m_max,))
        self.num_classes = n
        self.num_points = int(lib.oracle_num_points())

    # -- tables -------------------------------------------------------------------------
    def shell_size(self, m):
        return int(self.lib.oracle_shell_size(m))

    def golay_words(self):
        return np.array([self.lib.oracle_golay_word(u) for u in range(4096)], dtype=np.uint32)

    def golay_sorted(self):
        return np.array([self.lib.oracle_golay_sorted(u) for u in range(4096)], dtype=np.uint32)

    def class_info(self, j):
        i32, u64 = ctypes.c_int, ctypes.c_uint64
        m, odd, w, nv, B = i32(), i32(), i32(), i32(), i32()
        A, P1, P0, size, off = u64(), u64(), u64(), u64(), u64()
        vals = (i32 * 8)(); cnts = (i32 * 8)()
        r = ctypes.byref
        self.lib.oracle_class_info(j, r(m), r(odd), r(w), r(nv), vals, cnts, r(A), r(B), r(P1), r(P0), r(size), r(off))
        return dict(m=m.value, odd=odd.value, w=w.value, B=B.value, A=A.value, P1=P1.value, P0=P0.value,
                    size=size.value, offset=off.value,
                    leader={vals[i]: cnts[i] for i in range(nv.value)})

    def classes(self):
        return [self.class_info(j) for j in range(self.num_classes)]

    # -- codec --------------------------------------------------------------------------
    def decode(self, idx):
        """idx: array of uint64 indices -> (int8 [n,24], number of out-of-range indices)."""
        idx = np.ascontiguousarray(idx, dtype=np.uint64)
        out = np.empty((idx.size, 24), dtype=np.int8)
        bad = self.lib.oracle_decode_batch(idx.ctypes.data, idx.size, out.ctypes.data)
        return out, int(bad)

    def decode_range(self, first, n):
        out = np.empty((n, 24), dtype=np.int8)
        bad = self.lib.oracle_decode_range(int(first), int(n), out.ctypes.data)
        return out, int(bad)

    def encode(self, pts):
        pts = np.ascontiguousarray(pts, dtype=np.int8)
        idx = np.empty(pts.shape[0], dtype=np.uint64)
        bad = self.lib.oracle_encode_batch(pts.ctypes.data, pts.shape[0], idx.ctypes.data)
        return idx, int(bad)

    def is_member(self, x):
        x = np.ascontiguousarray(x, dtype=np.int32)
        return bool(self.lib.oracle_is_member(x.ctypes.data))

    # -- nearest point of the ball cut ---------------------------------------------------
    def nearest(self, w, metric="angular"):
        """w: [n, 24] floats -> (int8 [n, 24] nearest points, float64 [n] scores).
        angular: score <w, x>/||x||; euclidean: score <w, x> - ||x||^2 / 2."""
        w = np.ascontiguousarray(w, dtype=np.float64).reshape(-1, 24)
        out = np.empty((w.shape[0], 24), dtype=np.int8)
        score = np.empty(w.shape[0], dtype=np.float64)
        self.lib.oracle_nearest_batch(w.ctypes.data, w.shape[0], {"angular": 0, "euclidean": 1}[metric],
                                      out.ctypes.data, score.ctypes.data)
        return out, score

    # -- shape-gain and matrix product --------------------------------------------------
    def dequant(self, idx, gain_f16):
        """w = g * x/||x|| in fp64; gain_f16 is a float16 array."""
        idx = np.ascontiguousarray(idx, dtype=np.uint64).ravel()
        g = np.ascontiguousarray(gain_f16, dtype=np.float16).ravel().view(np.uint16)
        out = np.empty((idx.size, 24), dtype=np.float64)
        self.lib.oracle_dequant_batch(idx.ctypes.data, g.ctypes.data, idx.size, out.ctypes.data)
        return out

    def matmul(self, x, idx, gain_f16):
        """y[M,N] = x[M,24*KB] @ W_hat[N,24*KB]^T in fp64, plain loops in C.  idx, gain: [N,KB]."""
        idx = np.ascontiguousarray(idx, dtype=np.uint64)
        N, KB = idx.shape
        g = np.ascontiguousarray(gain_f16, dtype=np.float16).view(np.uint16)
        x64 = np.ascontiguousarray(np.asarray(x).astype(np.float64)).reshape(-1, 24 * KB)
        y = np.empty((x64.shape[0], N), dtype=np.float64)
        self.lib.oracle_matmul(idx.ctypes.data, g.ctypes.data, N, KB, x64.ctypes.data, x64.shape[0], y.ctypes.data)
        return y

    def matmul_dense(self, x, idx, gain_f16):
        """Same product through a library routine: dense W_hat from `dequant`, then numpy's fp64 matmul."""
        idx = np.ascontiguousarray(idx, dtype=np.uint64)
        N, KB = idx.shape
        W = self.dequant(idx, gain_f16).reshape(N, KB * 24)
        x64 = np.asarray(x).astype(np.float64).reshape(-1, 24 * KB)
        return x64 @ W.T
