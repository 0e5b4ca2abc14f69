"""GPU parity tests of the coded-word entry points (gain bits inside the word, single-shell 24-bit words):
the HIP path through the C ABI against the oracle fed with the unpacked (index, gain) pairs."""
import numpy as np
import pytest

from paper_2603_11021_amd import synth, LLVQ_IDX_U24

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_11021_amd import LLVQ
    return LLVQ(13, 0)


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _rel(y, ref):
    return np.abs(np.asarray(y, dtype=np.float64) - ref).max() / np.abs(ref).max()


def test_shell_offsets_are_table1(gpu, oracle13):
    # paper Table 1: N(2) = 196,560, N(3) = 16,969,680, N(4) = 415,003,680, N(13)
    assert [gpu.llvq_shell_offset(m) for m in (2, 3, 4, 5)] == [0, 196560, 16969680, 415003680]
    assert gpu.llvq_shell_offset(14) == synth.N_POINTS_M13
    sizes = [int(oracle13.shell_size(m)) for m in range(2, 14)]
    assert [gpu.llvq_shell_offset(m) for m in range(2, 15)] == [sum(sizes[:i]) for i in range(13)]


@pytest.mark.parametrize("gain_bits", [1, 2, 4])
def test_gain_bits_inside_the_word(gpu, oracle13, gain_bits):
    """48-bit word = gain code above a (48 - gain_bits)-bit shape index over the largest ball cut that fits"""
    import torch
    shape_bits = 48 - gain_bits
    n_shape = min(synth.N_POINTS_M13, 1 << shape_bits)
    N, KB = 123, 47
    rng = synth.rng_for(8, gain_bits)
    shape = synth.indices(rng, (N, KB), n_shape)
    code = rng.integers(0, 1 << gain_bits, size=(N, KB), dtype=np.uint64)
    shape[0, :2] = (0, n_shape - 1)
    code[0, :2] = ((1 << gain_bits) - 1, 0)
    words = (code << np.uint64(shape_bits)) | shape
    lut = synth.chi_gain_levels(gain_bits, scale=0.02)
    gain = lut[code.astype(np.int64)]                                         # what the oracle is given
    d48 = _dev(synth.pack_u48(words).reshape(-1))
    d64 = _dev(words.view(np.int64).reshape(-1))
    d_lut = _dev(lut)
    # shape-gain reconstruction
    want = oracle13.dequant(shape.reshape(-1), gain.reshape(-1))
    for d in (d48, d64):
        got = gpu.llvq_decode_coded(d, shape_bits, gain_lut=d_lut, out_dtype=torch.float32).cpu().numpy().astype(np.float64)
        assert (np.abs(got - want) <= 3 * 2.0 ** -24 * np.abs(want) + 1e-30).all()
    # integer coordinates: the gain bits are ignored
    wi, bad = oracle13.decode(shape.reshape(-1))
    assert bad == 0
    assert np.array_equal(gpu.llvq_decode_i8_coded(d48, shape_bits).cpu().numpy(), wi)
    # fused product, lane-per-block kernel (M <= 2) and matrix-core kernel
    for M in (1, 2, 19):
        x = synth.activations(rng, M, 24 * KB)
        ref = oracle13.matmul(x, shape, gain)
        for d in (d48, d64):
            y = gpu.llvq_matmul_coded(_dev(x).half(), d, N, KB, shape_bits, gain_lut=d_lut).cpu().numpy()
            assert _rel(y, ref) <= (1e-5 if M <= 2 else TOL)
    # same words, gains from a per-block array instead of the table: upper bits ignored
    x = synth.activations(rng, 1, 24 * KB)
    g2 = synth.gains(rng, (N, KB))
    y = gpu.llvq_matmul_coded(_dev(x).half(), d48, N, KB, shape_bits, gain=_dev(g2.reshape(-1))).cpu().numpy()
    assert _rel(y, oracle13.matmul(x, shape, g2)) <= 1e-5


def test_single_shell_24bit_words(gpu, oracle13):
    """shell 3 alone: 16,773,120 points < 2^24, one 3-byte word per block of 24 weights (1 bit per weight)"""
    import torch
    base = gpu.llvq_shell_offset(3)
    n3 = gpu.llvq_shell_offset(4) - base
    assert n3 == 16773120
    N, KB = 70, 171
    rng = synth.rng_for(8, 24)
    words = synth.indices(rng, (N, KB), n3)
    words[0, :3] = (0, n3 - 1, 12345)
    gain = synth.gains(rng, (N, KB))
    idx = words + np.uint64(base)
    d24 = _dev(synth.pack_u24(words).reshape(-1))
    wi, bad = oracle13.decode(idx.reshape(-1))
    assert bad == 0 and ((wi.astype(np.int64) ** 2).sum(axis=1) == 48).all()
    got = gpu.llvq_decode_i8_coded(d24, 24, base, fmt=LLVQ_IDX_U24).cpu().numpy()
    assert np.array_equal(got, wi)
    want = oracle13.dequant(idx.reshape(-1), gain.reshape(-1))
    got = gpu.llvq_decode_coded(d24, 24, base, gain=_dev(gain.reshape(-1)), fmt=LLVQ_IDX_U24, out_dtype=torch.float32)
    got = got.cpu().numpy().astype(np.float64)
    assert (np.abs(got - want) <= 3 * 2.0 ** -24 * np.abs(want) + 1e-30).all()
    for M in (1, 2, 8):
        x = synth.activations(rng, M, 24 * KB)
        y = gpu.llvq_matmul_coded(_dev(x).half(), d24, N, KB, 24, base, gain=_dev(gain.reshape(-1)), fmt=LLVQ_IDX_U24).cpu().numpy()
        assert _rel(y, oracle13.matmul(x, idx, gain)) <= (1e-5 if M <= 2 else TOL)
    # no gain bits at all: a gain table with one level (constant-norm code, 3 bytes per block: the paper's App. C setting)
    one = np.array([0.0123], dtype=np.float16)
    x = synth.activations(rng, 1, 24 * KB)
    y = gpu.llvq_matmul_coded(_dev(x).half(), d24, N, KB, 24, base, gain_lut=_dev(one), fmt=LLVQ_IDX_U24).cpu().numpy()
    assert _rel(y, oracle13.matmul(x, idx, np.full(idx.shape, one[0], dtype=np.float16))) <= 1e-5
    # 23 shape bits + 1 gain bit inside the 24-bit word, over the first 2^23 points of the shell
    shape = synth.indices(rng, (N, KB), 1 << 23)
    code = rng.integers(0, 2, size=(N, KB), dtype=np.uint64)
    lut = synth.chi_gain_levels(1)
    w2 = (code << np.uint64(23)) | shape
    x = synth.activations(rng, 1, 24 * KB)
    y = gpu.llvq_matmul_coded(_dev(x).half(), _dev(synth.pack_u24(w2).reshape(-1)), N, KB, 23, base, gain_lut=_dev(lut),
                              fmt=LLVQ_IDX_U24).cpu().numpy()
    assert _rel(y, oracle13.matmul(x, shape + np.uint64(base), lut[code.astype(np.int64)])) <= 1e-5


def test_single_shell_words_past_the_end():
    """with a context for Lambda_24(3) the 4,096 words >= n(3) of a 24-bit single-shell code give the zero block"""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_11021_amd import LLVQ
    from oracle.llvq_oracle import Oracle
    o = Oracle(3)
    g = LLVQ(3, 0)
    base = g.llvq_shell_offset(3)
    words = np.array([0, 16773119, 16773120, (1 << 24) - 1, 777], dtype=np.uint64)
    want, bad = o.decode(words + np.uint64(base))
    assert bad == 2 and not want[2].any() and not want[3].any()
    got = g.llvq_decode_i8_coded(_dev(synth.pack_u24(words).reshape(-1)), 24, base, fmt=LLVQ_IDX_U24).cpu().numpy()
    assert np.array_equal(got, want)
    g.close()


def test_coded_argument_checks(gpu):
    import torch
    from paper_2603_11021_amd import LLVQError
    d = torch.zeros(6 * 8, dtype=torch.uint8, device="cuda:0")
    lut = torch.ones(1 << 13, dtype=torch.float16, device="cuda:0")
    x = torch.zeros(24 * 8, dtype=torch.float16, device="cuda:0")
    with pytest.raises(LLVQError):
        gpu.llvq_decode_i8_coded(d, 0)                        # no shape bits
    with pytest.raises(LLVQError):
        gpu.llvq_decode_i8_coded(d, 49)                       # more than the word holds
    with pytest.raises(LLVQError):
        gpu.llvq_matmul_coded(x, d, 1, 8, 35, gain_lut=lut)   # a 13-bit gain table is refused
    with pytest.raises(LLVQError):
        gpu.llvq_matmul_coded(x, d, 1, 8, 47)                 # neither a gain table nor per-block gains
    # empty input is a no-op
    e = torch.empty(0, dtype=torch.uint8, device="cuda:0")
    assert gpu.llvq_decode_i8_coded(e, 47).shape == (0, 24)


@pytest.mark.parametrize("src_fmt", ["u48", "u64"])
def test_packed_words_carry_index_and_gain(gpu, oracle13, src_fmt):
    """llvq_repack writes index | gain bits << 48; the coded calls with 64-bit words, 48 shape bits, no gain table and
    no gain array read both from the word: bit-exact packing, decode and products against the oracle"""
    import torch
    N, K, M = 300, 24 * 57 - 3, 2
    idx, gain, x = synth.layer(6, 6100, N, K, M)
    KB = idx.shape[1]
    flat = idx.reshape(-1)
    d_idx = _dev(synth.pack_u48(flat).reshape(-1)) if src_fmt == "u48" else _dev(flat.astype(np.int64))
    d_gain = _dev(gain.reshape(-1))
    packed = gpu.llvq_repack(d_idx, d_gain)
    want = flat | (gain.reshape(-1).view(np.uint16).astype(np.uint64) << np.uint64(48))
    assert np.array_equal(packed.cpu().numpy().view(np.uint64), want)
    # integer coordinates ignore the gain bits
    pts = gpu.llvq_decode_i8_coded(packed, 48).cpu().numpy()
    ref_pts, _ = oracle13.decode(flat)
    assert np.array_equal(pts, ref_pts)
    for dt, rel in ((torch.float16, 2.0 ** -11), (torch.float32, 0.0)):
        w = gpu.llvq_decode_coded(packed, 48, out_dtype=dt).float().cpu().numpy().astype(np.float64)
        ref = oracle13.dequant(flat, gain.reshape(-1))
        assert (np.abs(w - ref) <= (rel + 3 * 2.0 ** -24) * np.abs(ref) + 1e-30).all()
    ref = oracle13.matmul(x, idx, gain)
    for m_rows in (1, M):                                    # vector-ALU kernel, and the same with two rows
        y = gpu.llvq_matmul_coded(_dev(x[:m_rows]).half(), packed, N, KB, 48).cpu().numpy()
        assert _rel(y, ref[:m_rows]) <= TOL
    x16 = synth.activations(synth.rng_for(6, 6101), 16, K)
    y = gpu.llvq_matmul_coded(_dev(x16).half(), packed, N, KB, 48).cpu().numpy()      # matrix-core kernel
    assert _rel(y, oracle13.matmul(x16, idx, gain)) <= TOL
    x300 = synth.activations(synth.rng_for(6, 6102), 100, K, "bf16")
    y = gpu.llvq_matmul_coded(_dev(x300).to(torch.bfloat16), packed, N, KB, 48).cpu().numpy()   # strip kernel
    assert _rel(y, oracle13.matmul(x300, idx, gain)) <= TOL


def test_coded_formats_on_a_long_launch(gpu, oracle13):
    """the three word formats on a layer long enough for the long-launch kernels (all tables in LDS, batches of 64
    blocks taken from a counter): 24-bit single-shell words, packed 64-bit words, 47 + 1 bits in 48-bit words;
    products on sampled rows and decoded blocks on sampled positions against the oracle"""
    import torch
    N, KB = 9000, 171                                  # 1,539,000 blocks: 94 wave-batches per compute unit
    K = 24 * KB
    rng = synth.rng_for(8, 99)
    rows = np.sort(np.random.default_rng(5).choice(N, 1500, replace=False))
    pos = np.sort(np.random.default_rng(6).choice(N * KB, 30000, replace=False))
    x = synth.activations(rng, 1, K)
    d_x = _dev(x).half()
    gain = synth.gains(rng, (N, KB))
    d_gain = _dev(gain.reshape(-1))
    # 24-bit words over shell 3
    base = gpu.llvq_shell_offset(3)
    n3 = gpu.llvq_shell_offset(4) - base
    words = synth.indices(rng, (N, KB), n3)
    d24 = _dev(synth.pack_u24(words).reshape(-1))
    y = gpu.llvq_matmul_coded(d_x, d24, N, KB, 24, base, gain=d_gain, fmt=LLVQ_IDX_U24).cpu().numpy()
    assert _rel(y[:, rows], oracle13.matmul(x, words[rows] + np.uint64(base), gain[rows])) <= 1e-5
    pts = gpu.llvq_decode_i8_coded(d24, 24, base, fmt=LLVQ_IDX_U24)
    want, _ = oracle13.decode(words.reshape(-1)[pos] + np.uint64(base))
    assert np.array_equal(pts[torch.from_numpy(pos).to("cuda:0")].cpu().numpy(), want)
    # packed 64-bit words: index + fp16 gain
    idx = synth.indices(rng, (N, KB))
    packed = gpu.llvq_repack(_dev(synth.pack_u48(idx).reshape(-1)), d_gain)
    y = gpu.llvq_matmul_coded(d_x, packed, N, KB, 48).cpu().numpy()
    assert _rel(y[:, rows], oracle13.matmul(x, idx[rows], gain[rows])) <= 1e-5
    w = gpu.llvq_decode_coded(packed, 48, out_dtype=torch.float32)
    ref = oracle13.dequant(idx.reshape(-1)[pos], gain.reshape(-1)[pos])
    got = w[torch.from_numpy(pos).to("cuda:0")].cpu().numpy().astype(np.float64)
    assert (np.abs(got - ref) <= 3 * 2.0 ** -24 * np.abs(ref) + 1e-30).all()
    # 47 shape bits + 1 gain bit in a 48-bit word
    shape = synth.indices(rng, (N, KB), 1 << 47)
    code = rng.integers(0, 2, size=(N, KB), dtype=np.uint64)
    lut = synth.chi_gain_levels(1, scale=0.02)
    d48 = _dev(synth.pack_u48((code << np.uint64(47)) | shape).reshape(-1))
    y = gpu.llvq_matmul_coded(d_x, d48, N, KB, 47, gain_lut=_dev(lut)).cpu().numpy()
    assert _rel(y[:, rows], oracle13.matmul(x, shape[rows], lut[code[rows].astype(np.int64)])) <= 1e-5
    # the same three formats through the prefill kernel for M >= 384 (panels of 128 rows x 512 tokens; the gain table
    # adds a load to the part of the decode that leaves reads in flight across steps)
    rows = rows[:200]
    x400 = synth.activations(rng, 400, K)
    d_x400 = _dev(x400).half()
    y = gpu.llvq_matmul_coded(d_x400, d24, N, KB, 24, base, gain=d_gain, fmt=LLVQ_IDX_U24).cpu().numpy()
    assert _rel(y[:, rows], oracle13.matmul(x400, words[rows] + np.uint64(base), gain[rows])) <= TOL
    y = gpu.llvq_matmul_coded(d_x400, packed, N, KB, 48).cpu().numpy()
    assert _rel(y[:, rows], oracle13.matmul(x400, idx[rows], gain[rows])) <= TOL
    y = gpu.llvq_matmul_coded(d_x400, d48, N, KB, 47, gain_lut=_dev(lut)).cpu().numpy()
    assert _rel(y[:, rows], oracle13.matmul(x400, shape[rows], lut[code[rows].astype(np.int64)])) <= TOL


def test_repack_empty_and_invalid(gpu):
    import torch
    from paper_2603_11021_amd import LLVQError
    out = gpu.llvq_repack(torch.empty(0, dtype=torch.uint8, device="cuda:0"), torch.empty(0, dtype=torch.float16, device="cuda:0"))
    assert out.numel() == 0
    with pytest.raises(LLVQError):                            # no gain anywhere with 48-bit words: nothing to read it from
        gpu.llvq_matmul_coded(torch.zeros(1, 24, dtype=torch.float16, device="cuda:0"),
                              torch.zeros(6, dtype=torch.uint8, device="cuda:0"), 1, 1, 48)
