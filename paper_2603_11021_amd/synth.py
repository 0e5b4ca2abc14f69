"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds none of the method's arithmetic: it only draws indices uniformly below a given code size, log-normal
gains and normal activations, with the shapes of the workloads (Llama-3 8B / 70B linear layers, blocks of 24
along the input channels, K zero-padded to a multiple of 24), and packs indices into 6 little-endian bytes.
"""
import numpy as np

N_POINTS_M13 = 280974212784720      # |Lambda_24(13)|, paper Table 1
N_SHELL2 = 196560                   # minimal vectors, paper Table 1
BASE_SEED = 20260311

LLAMA3_8B = {"q": (4096, 4096), "k": (1024, 4096), "v": (1024, 4096), "o": (4096, 4096),
             "gate": (14336, 4096), "up": (14336, 4096), "down": (4096, 14336)}
LLAMA3_70B = {"q": (8192, 8192), "k": (1024, 8192), "v": (1024, 8192), "o": (8192, 8192),
              "gate": (28672, 8192), "up": (28672, 8192), "down": (8192, 28672)}


def blocks_per_row(K):
    return (K + 23) // 24


def rng_for(config, ordinal=0):
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * config + ordinal))


def indices(rng, shape, n_points=N_POINTS_M13):
    return rng.integers(0, n_points, size=shape, dtype=np.uint64)


def gains(rng, shape):
    return np.exp(0.5 * rng.standard_normal(size=shape)).astype(np.float16)


def activations(rng, M, K, dtype=np.float16):
    """M x K_pad activations ~N(0,1), columns K..K_pad-1 zero; float32 values already rounded to `dtype`
    (np.float16, or the string "bf16" for bfloat16 round-to-nearest-even)."""
    KB = blocks_per_row(K)
    x = np.zeros((M, 24 * KB), dtype=np.float32)
    x[:, :K] = rng.standard_normal(size=(M, K)).astype(np.float32)
    if dtype == "bf16":
        u = x.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32)
    return x.astype(np.float16).astype(np.float32)


def pack_u48(idx):
    """uint64 indices -> uint8 array of 6 little-endian bytes per index (same leading shape, last dim * 6)."""
    idx = np.ascontiguousarray(idx, dtype=np.uint64)
    b = idx.reshape(-1, 1).view(np.uint8).reshape(-1, 8)[:, :6]
    return np.ascontiguousarray(b).reshape(idx.shape + (6,))


def pack_u24(words):
    """uint64 words below 2^24 -> uint8 array of 3 little-endian bytes per word."""
    words = np.ascontiguousarray(words, dtype=np.uint64)
    b = words.reshape(-1, 1).view(np.uint8).reshape(-1, 8)[:, :3]
    return np.ascontiguousarray(b).reshape(words.shape + (3,))


def chi_gain_levels(bits, dim=24, scale=1.0):
    """2^bits reconstruction levels for the norm of a `dim`-dimensional standard normal block: the medians of
    2^bits equiprobable cells of the chi distribution (paper App. I, gain code matched to chi_24), as float16.
    Input generator only: the levels are passed to both the library and the oracle as data."""
    from scipy.stats import chi
    n = 1 << bits
    return (scale * chi.ppf((np.arange(n) + 0.5) / n, dim) / np.sqrt(dim)).astype(np.float16)


def layer(config, ordinal, N, K, M=1, n_points=N_POINTS_M13, x_dtype=np.float16):
    """One synthetic quantised linear layer: (idx uint64 [N,KB], gain float16 [N,KB], x float32 [M,24*KB])."""
    rng = rng_for(config, ordinal)
    KB = blocks_per_row(K)
    return indices(rng, (N, KB), n_points), gains(rng, (N, KB)), activations(rng, M, K, x_dtype)
