"""ctypes binding with the same names as the C ABI (include/llvq.h).  Argument marshalling only."""
import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
_LIB = os.path.join(_HERE, "libllvq.so")

LLVQ_IDX_U48, LLVQ_IDX_U64, LLVQ_IDX_U24 = 0, 1, 2
LLVQ_F16, LLVQ_BF16, LLVQ_F32 = 0, 1, 2
LLVQ_ANGULAR, LLVQ_EUCLIDEAN = 0, 1

HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-std=c++17", "-fPIC", "-shared"]
HIPCC_LIBS = ["-L/opt/rocm/lib", "-lrocblas"]


class LLVQError(RuntimeError):
    pass


def lib_path():
    return _LIB


def build_library():
    """Compile the HIP kernels and the host table builder for gfx950 into libllvq.so (in-tree)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = [os.path.join(_CSRC, "llvq_kernels.hip"), os.path.join(_CSRC, "llvq_tables.cpp")]
    subprocess.check_call([hipcc] + HIPCC_FLAGS + ["-o", _LIB] + srcs + HIPCC_LIBS)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        raise LLVQError("libllvq.so is not built (run __graft_entry__.build()); there is no CPU fallback")
    lib = ctypes.CDLL(_LIB)
    vp, i32, u64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_size_t
    lib.llvq_create.argtypes = [ctypes.POINTER(vp), i32, i32]; lib.llvq_create.restype = i32
    lib.llvq_destroy.argtypes = [vp]; lib.llvq_destroy.restype = None
    lib.llvq_strerror.argtypes = [i32]; lib.llvq_strerror.restype = ctypes.c_char_p
    lib.llvq_last_hip_error.argtypes = [vp]; lib.llvq_last_hip_error.restype = ctypes.c_char_p
    lib.llvq_num_points.argtypes = [vp]; lib.llvq_num_points.restype = u64
    lib.llvq_num_classes.argtypes = [vp]; lib.llvq_num_classes.restype = i32
    lib.llvq_decode_i8.argtypes = [vp, vp, i32, sz, vp, vp]; lib.llvq_decode_i8.restype = i32
    lib.llvq_decode.argtypes = [vp, vp, i32, vp, sz, vp, i32, vp]; lib.llvq_decode.restype = i32
    lib.llvq_matmul.argtypes = [vp, vp, i32, i32, vp, i32, vp, i32, i32, vp, vp]; lib.llvq_matmul.restype = i32
    lib.llvq_matmul_multi.argtypes = [vp, vp, i32, i32, i32, vp, i32, vp, vp, i32, vp, vp]; lib.llvq_matmul_multi.restype = i32
    lib.llvq_matmul_ws.argtypes = [vp, vp, i32, i32, vp, i32, vp, i32, i32, vp, vp, sz, vp]; lib.llvq_matmul_ws.restype = i32
    lib.llvq_shell_offset.argtypes = [vp, i32]; lib.llvq_shell_offset.restype = u64
    lib.llvq_decode_i8_coded.argtypes = [vp, vp, i32, i32, u64, sz, vp, vp]; lib.llvq_decode_i8_coded.restype = i32
    lib.llvq_decode_coded.argtypes = [vp, vp, i32, i32, u64, vp, vp, sz, vp, i32, vp]; lib.llvq_decode_coded.restype = i32
    lib.llvq_matmul_coded.argtypes = [vp, vp, i32, i32, vp, i32, i32, u64, vp, vp, i32, i32, vp, vp]; lib.llvq_matmul_coded.restype = i32
    lib.llvq_encode.argtypes = [vp, vp, sz, vp, i32, vp]; lib.llvq_encode.restype = i32
    lib.llvq_repack.argtypes = [vp, vp, i32, vp, sz, vp, vp]; lib.llvq_repack.restype = i32
    lib.llvq_quantize.argtypes = [vp, vp, sz, i32, vp, vp, i32, vp, vp]; lib.llvq_quantize.restype = i32
    lib.llvq_gptq_workspace_bytes.argtypes = [i32]; lib.llvq_gptq_workspace_bytes.restype = sz
    lib.llvq_gptq_quantize.argtypes = [vp, vp, i32, i32, sz, vp, vp, i32, vp, vp, sz, vp]; lib.llvq_gptq_quantize.restype = i32
    lib.llvq_gptq_quantize_levels.argtypes = [vp, vp, i32, i32, sz, vp, vp, i32, vp, vp, i32, vp, sz, vp]; lib.llvq_gptq_quantize_levels.restype = i32
    lib.llvq_gptq_group_scales_workspace_bytes.argtypes = [i32, i32]; lib.llvq_gptq_group_scales_workspace_bytes.restype = sz
    lib.llvq_gptq_group_scales.argtypes = [vp, vp, vp, i32, i32, sz, vp, ctypes.c_float, vp, vp, vp, sz, vp]; lib.llvq_gptq_group_scales.restype = i32
    lib.llvq_validate.argtypes = [vp, vp, i32, sz, ctypes.POINTER(u64), vp]; lib.llvq_validate.restype = i32
    lib.llvq_validate_static.argtypes = [vp, vp, i32, sz, vp, vp]; lib.llvq_validate_static.restype = i32
    _lib = lib
    return lib


def _stream_handle(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


class LLVQ:
    """A context for Lambda_24(m_max) on one device.  Tensors are torch CUDA (ROCm) tensors owned by the caller."""

    def __init__(self, m_max=13, device=0):
        self._lib = _load()
        h = ctypes.c_void_p()
        rc = self._lib.llvq_create(ctypes.byref(h), m_max, device)
        if rc != 0:
            raise LLVQError("llvq_create: %s" % self._lib.llvq_strerror(rc).decode())
        self._h = h
        self.m_max = m_max
        self.device = device

    def close(self):
        if getattr(self, "_h", None):
            self._lib.llvq_destroy(self._h)
            self._h = None

    __del__ = close

    def _check(self, rc, what):
        if rc != 0:
            raise LLVQError("%s: %s (%s)" % (what, self._lib.llvq_strerror(rc).decode(),
                                             self._lib.llvq_last_hip_error(self._h).decode()))

    @property
    def num_points(self):
        return int(self._lib.llvq_num_points(self._h))

    @property
    def num_classes(self):
        return int(self._lib.llvq_num_classes(self._h))

    def llvq_shell_offset(self, m):
        return int(self._lib.llvq_shell_offset(self._h, m))

    @staticmethod
    def _idx_fmt(idx, fmt=None):
        import torch
        if fmt == LLVQ_IDX_U24:
            if idx.dtype != torch.uint8:
                raise LLVQError("24-bit words are passed as a uint8 tensor, 3 bytes per word")
            return LLVQ_IDX_U24, idx.numel() // 3
        if idx.dtype == torch.uint8:
            return LLVQ_IDX_U48, idx.numel() // 6
        if idx.dtype in (torch.int64, torch.uint64):
            return LLVQ_IDX_U64, idx.numel()
        raise LLVQError("indices must be uint8 (6 bytes per index) or int64/uint64")

    def llvq_decode_i8(self, idx, out=None, n_blocks=None, stream=None):
        import torch
        fmt, n = self._idx_fmt(idx)
        n = n if n_blocks is None else n_blocks
        if out is None:
            out = torch.empty((n, 24), dtype=torch.int8, device=idx.device)
        self._check(self._lib.llvq_decode_i8(self._h, idx.data_ptr(), fmt, n, out.data_ptr(), _stream_handle(stream)),
                    "llvq_decode_i8")
        return out

    def llvq_decode(self, idx, gain, out_dtype=None, out=None, stream=None):
        import torch
        fmt, n = self._idx_fmt(idx)
        out_dtype = out_dtype or torch.float16
        code = {torch.float16: LLVQ_F16, torch.bfloat16: LLVQ_BF16, torch.float32: LLVQ_F32}[out_dtype]
        if gain.dtype != torch.float16 or gain.numel() != n:
            raise LLVQError("gain must be float16 with one entry per block")
        if out is None:
            out = torch.empty((n, 24), dtype=out_dtype, device=idx.device)
        self._check(self._lib.llvq_decode(self._h, idx.data_ptr(), fmt, gain.data_ptr(), n, out.data_ptr(), code,
                                          _stream_handle(stream)), "llvq_decode")
        return out

    def llvq_matmul(self, x, idx, gain, N, KB, out=None, stream=None, workspace=None):
        import torch
        fmt, n = self._idx_fmt(idx)
        if n != N * KB or gain.numel() != N * KB or gain.dtype != torch.float16:
            raise LLVQError("idx and gain must hold N*KB blocks; gain float16")
        code = {torch.float16: LLVQ_F16, torch.bfloat16: LLVQ_BF16}[x.dtype]
        x2 = x.reshape(-1, 24 * KB)
        M = x2.shape[0]
        if out is None:
            out = torch.empty((M, N), dtype=torch.float32, device=x.device)
        if workspace is not None:
            self._check(self._lib.llvq_matmul_ws(self._h, x2.data_ptr(), code, M, idx.data_ptr(), fmt, gain.data_ptr(), N, KB,
                                                 out.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                                 _stream_handle(stream)), "llvq_matmul_ws")
            return out
        self._check(self._lib.llvq_matmul(self._h, x2.data_ptr(), code, M, idx.data_ptr(), fmt, gain.data_ptr(), N, KB,
                                          out.data_ptr(), _stream_handle(stream)), "llvq_matmul")
        return out

    def llvq_matmul_multi(self, x, idxs, gains, Ns, KB, outs=None, stream=None):
        """y_i = W_i x for up to four matrices that share x: lists of index tensors, gain tensors and row counts."""
        import torch
        n_items = len(idxs)
        if not (len(gains) == len(Ns) == n_items) or (outs is not None and len(outs) != n_items):
            raise LLVQError("idxs, gains, Ns and outs must have the same length")
        code = {torch.float16: LLVQ_F16, torch.bfloat16: LLVQ_BF16}[x.dtype]
        x2 = x.reshape(-1, 24 * KB)
        M = x2.shape[0]
        fmt = None
        for idx, gain, N in zip(idxs, gains, Ns):
            f, n = self._idx_fmt(idx)
            if fmt is not None and f != fmt:
                raise LLVQError("all matrices must use the same index format")
            fmt = f
            if n != N * KB or gain.numel() != N * KB or gain.dtype != torch.float16:
                raise LLVQError("idx and gain must hold N*KB blocks; gain float16")
        if outs is None:
            outs = [torch.empty((M, N), dtype=torch.float32, device=x.device) for N in Ns]
        P = ctypes.c_void_p * max(n_items, 1)
        a_idx = P(*[t.data_ptr() for t in idxs])
        a_gain = P(*[t.data_ptr() for t in gains])
        a_y = P(*[t.data_ptr() for t in outs])
        a_n = (ctypes.c_int * max(n_items, 1))(*[int(N) for N in Ns])
        self._check(self._lib.llvq_matmul_multi(self._h, x2.data_ptr(), code, M, n_items, a_idx, fmt if fmt is not None else 0,
                                                a_gain, a_n, KB, a_y, _stream_handle(stream)), "llvq_matmul_multi")
        return outs

    # ---- coded words: shape index in the low shape_bits (+ base_index), gain code above them ------------------
    def llvq_decode_i8_coded(self, idx, shape_bits, base_index=0, fmt=None, out=None, stream=None):
        import torch
        fmt, n = self._idx_fmt(idx, fmt)
        if out is None:
            out = torch.empty((n, 24), dtype=torch.int8, device=idx.device)
        self._check(self._lib.llvq_decode_i8_coded(self._h, idx.data_ptr(), fmt, shape_bits, base_index, n, out.data_ptr(),
                                                   _stream_handle(stream)), "llvq_decode_i8_coded")
        return out

    @staticmethod
    def _gain_args(gain_lut, gain, n):
        import torch
        for t, what in ((gain_lut, "gain_lut"), (gain, "gain")):
            if t is not None and t.dtype != torch.float16:
                raise LLVQError("%s must be float16" % what)
        if gain is not None and gain.numel() != n:
            raise LLVQError("gain must hold one entry per block")
        return (gain_lut.data_ptr() if gain_lut is not None else None, gain.data_ptr() if gain is not None else None)

    def llvq_decode_coded(self, idx, shape_bits, base_index=0, gain_lut=None, gain=None, fmt=None, out_dtype=None, out=None,
                          stream=None):
        import torch
        fmt, n = self._idx_fmt(idx, fmt)
        out_dtype = out_dtype or torch.float16
        code = {torch.float16: LLVQ_F16, torch.bfloat16: LLVQ_BF16, torch.float32: LLVQ_F32}[out_dtype]
        p_lut, p_gain = self._gain_args(gain_lut, gain, n)
        if gain_lut is not None and gain_lut.numel() != 1 << ((24 if fmt == LLVQ_IDX_U24 else 48) - shape_bits):
            raise LLVQError("gain_lut must hold 2^(word bits - shape_bits) entries")
        if out is None:
            out = torch.empty((n, 24), dtype=out_dtype, device=idx.device)
        self._check(self._lib.llvq_decode_coded(self._h, idx.data_ptr(), fmt, shape_bits, base_index, p_lut, p_gain, n,
                                                out.data_ptr(), code, _stream_handle(stream)), "llvq_decode_coded")
        return out

    def llvq_matmul_coded(self, x, idx, N, KB, shape_bits, base_index=0, gain_lut=None, gain=None, fmt=None, out=None,
                          stream=None):
        import torch
        fmt, n = self._idx_fmt(idx, fmt)
        if n != N * KB:
            raise LLVQError("idx must hold N*KB words")
        p_lut, p_gain = self._gain_args(gain_lut, gain, n)
        if gain_lut is not None and gain_lut.numel() != 1 << ((24 if fmt == LLVQ_IDX_U24 else 48) - shape_bits):
            raise LLVQError("gain_lut must hold 2^(word bits - shape_bits) entries")
        code = {torch.float16: LLVQ_F16, torch.bfloat16: LLVQ_BF16}[x.dtype]
        x2 = x.reshape(-1, 24 * KB)
        M = x2.shape[0]
        if out is None:
            out = torch.empty((M, N), dtype=torch.float32, device=x.device)
        self._check(self._lib.llvq_matmul_coded(self._h, x2.data_ptr(), code, M, idx.data_ptr(), fmt, shape_bits, base_index,
                                                p_lut, p_gain, N, KB, out.data_ptr(), _stream_handle(stream)),
                    "llvq_matmul_coded")
        return out

    def llvq_encode(self, pts, fmt=LLVQ_IDX_U48, out=None, stream=None):
        """pts: int8 [n, 24] -> indices, uint8 [n, 6] (LLVQ_IDX_U48) or int64 [n] (LLVQ_IDX_U64); all ones = not a point"""
        import torch
        if pts.dtype != torch.int8 or pts.numel() % 24:
            raise LLVQError("points must be int8 with 24 coordinates each")
        n = pts.numel() // 24
        if out is None:
            out = (torch.empty((n, 6), dtype=torch.uint8, device=pts.device) if fmt == LLVQ_IDX_U48
                   else torch.empty(n, dtype=torch.int64, device=pts.device))
        self._check(self._lib.llvq_encode(self._h, pts.data_ptr(), n, out.data_ptr(), fmt, _stream_handle(stream)), "llvq_encode")
        return out

    def llvq_repack(self, idx, gain, out=None, stream=None):
        """idx (uint8 6 bytes per block, or int64) + gain float16 -> int64 [n]: index | gain bits << 48"""
        import torch
        fmt, n = self._idx_fmt(idx)
        if gain.dtype != torch.float16 or gain.numel() != n:
            raise LLVQError("gain must hold one float16 per block")
        if out is None:
            out = torch.empty(n, dtype=torch.int64, device=idx.device)
        self._check(self._lib.llvq_repack(self._h, idx.data_ptr(), fmt, gain.data_ptr(), n, out.data_ptr(), _stream_handle(stream)),
                    "llvq_repack")
        return out

    def llvq_quantize(self, w, metric=LLVQ_ANGULAR, fmt=LLVQ_IDX_U48, want_idx=True, stream=None):
        """w: float32 [n, 24] -> (points int8 [n, 24], indices or None, scores float32 [n])"""
        import torch
        if w.dtype != torch.float32 or w.numel() % 24:
            raise LLVQError("blocks must be float32 with 24 coordinates each")
        n = w.numel() // 24
        pts = torch.empty((n, 24), dtype=torch.int8, device=w.device)
        score = torch.empty(n, dtype=torch.float32, device=w.device)
        idx = None
        if want_idx:
            idx = (torch.empty((n, 6), dtype=torch.uint8, device=w.device) if fmt == LLVQ_IDX_U48
                   else torch.empty(n, dtype=torch.int64, device=w.device))
        self._check(self._lib.llvq_quantize(self._h, w.data_ptr(), n, metric, pts.data_ptr(),
                                            idx.data_ptr() if idx is not None else None, fmt, score.data_ptr(),
                                            _stream_handle(stream)), "llvq_quantize")
        return pts, idx, score

    def llvq_gptq_quantize(self, W, U, fmt=LLVQ_IDX_U48, gain_levels=None, stream=None):
        """W: float32 [N, 24*KB], overwritten with the quantised layer; U: float32 [K, K] upper factor of H^-1.
        Returns (indices [N, KB(, 6)], gains float16 [N, KB])."""
        import torch
        N, K = W.shape
        if W.dtype != torch.float32 or U.dtype != torch.float32 or K % 24 or tuple(U.shape) != (K, K) or not W.is_contiguous() or not U.is_contiguous():
            raise LLVQError("W must be contiguous float32 [N, 24*KB] and U float32 [K, K]")
        KB = K // 24
        idx = (torch.empty((N, KB, 6), dtype=torch.uint8, device=W.device) if fmt == LLVQ_IDX_U48
               else torch.empty((N, KB), dtype=torch.int64, device=W.device))
        gain = torch.empty((N, KB), dtype=torch.float16, device=W.device)
        ws = torch.empty(int(self._lib.llvq_gptq_workspace_bytes(N)), dtype=torch.uint8, device=W.device)
        if gain_levels is not None:
            if gain_levels.dtype != torch.float16 or not gain_levels.is_contiguous():
                raise LLVQError("gain_levels must be a contiguous float16 tensor (ascending levels)")
            self._check(self._lib.llvq_gptq_quantize_levels(self._h, W.data_ptr(), N, KB, K, U.data_ptr(), idx.data_ptr(), fmt,
                                                            gain.data_ptr(), gain_levels.data_ptr(), gain_levels.numel(), ws.data_ptr(),
                                                            ws.numel(), _stream_handle(stream)), "llvq_gptq_quantize_levels")
        else:
            self._check(self._lib.llvq_gptq_quantize(self._h, W.data_ptr(), N, KB, K, U.data_ptr(), idx.data_ptr(), fmt,
                                                     gain.data_ptr(), ws.data_ptr(), ws.numel(), _stream_handle(stream)),
                        "llvq_gptq_quantize")
        return idx, gain

    def llvq_gptq_group_scales(self, Wq, W0, H, gain, lam=0.0, stream=None):
        """closed-form group scales in place on Wq and gain; returns the scales s [N, KB] (float32)"""
        import torch
        N, K = Wq.shape
        if (Wq.dtype != torch.float32 or W0.dtype != torch.float32 or H.dtype != torch.float32 or gain.dtype != torch.float16 or K % 24
                or tuple(W0.shape) != (N, K) or tuple(H.shape) != (K, K) or tuple(gain.shape) != (N, K // 24)
                or not (Wq.is_contiguous() and W0.is_contiguous() and H.is_contiguous() and gain.is_contiguous())):
            raise LLVQError("Wq, W0 contiguous float32 [N, 24*KB], H float32 [K, K], gain float16 [N, KB]")
        KB = K // 24
        s = torch.empty((N, KB), dtype=torch.float32, device=Wq.device)
        ws = torch.empty(int(self._lib.llvq_gptq_group_scales_workspace_bytes(N, KB)), dtype=torch.uint8, device=Wq.device)
        self._check(self._lib.llvq_gptq_group_scales(self._h, Wq.data_ptr(), W0.data_ptr(), N, KB, K, H.data_ptr(), float(lam),
                                                     gain.data_ptr(), s.data_ptr(), ws.data_ptr(), ws.numel(), _stream_handle(stream)),
                    "llvq_gptq_group_scales")
        return s

    def llvq_validate(self, idx, stream=None):
        fmt, n = self._idx_fmt(idx)
        bad = ctypes.c_uint64()
        self._check(self._lib.llvq_validate(self._h, idx.data_ptr(), fmt, n, ctypes.byref(bad), _stream_handle(stream)),
                    "llvq_validate")
        return int(bad.value)

    def llvq_validate_static(self, idx, out=None, stream=None):
        """Count of out-of-range indices into a one-element int64 device tensor; no synchronisation, no allocation
        inside the library (`out` is allocated here when the caller passes none)."""
        import torch
        fmt, n = self._idx_fmt(idx)
        if out is None:
            out = torch.empty(1, dtype=torch.int64, device=idx.device)
        self._check(self._lib.llvq_validate_static(self._h, idx.data_ptr(), fmt, n, out.data_ptr(), _stream_handle(stream)),
                    "llvq_validate_static")
        return out
