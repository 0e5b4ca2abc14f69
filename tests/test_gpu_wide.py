"""Contexts for the larger unions of shells (m_max up to 19, paper Table 1 row m = 19; 55-bit indices): the decoder of
these contexts against Oracle(19), bit-exact for coordinates, within the matmul bar for the fused product."""
import numpy as np
import pytest

from paper_2603_11021_amd import synth, LLVQ_IDX_U64

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def gpu19():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2603_11021_amd import LLVQ
    return LLVQ(19, 0)


@pytest.fixture(scope="module")
def oracle19():
    from oracle.llvq_oracle import Oracle
    return Oracle(19)


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def test_wide_context_reports_table_1(gpu19, oracle19):
    assert gpu19.num_points == 23546209100646960 == oracle19.num_points
    assert gpu19.num_classes == 1457
    assert gpu19.llvq_shell_offset(14) == 280974212784720
    assert gpu19.llvq_shell_offset(2) == 0 and gpu19.llvq_shell_offset(20) == gpu19.num_points


def test_wide_decode_is_bit_exact_on_every_class_and_random_indices(gpu19, oracle19):
    rng = synth.rng_for(19, 0)
    idx = []
    for c in oracle19.classes():
        off, size = int(c["offset"]), int(c["size"])
        idx += [off, off + size - 1] + [off + int(v) for v in rng.integers(0, size, size=30, dtype=np.uint64)]
    idx = np.concatenate([np.array(idx, dtype=np.uint64), rng.integers(0, oracle19.num_points, size=400000, dtype=np.uint64)])
    got = gpu19.llvq_decode_i8(_dev(idx.view(np.int64))).cpu().numpy()
    want, bad = oracle19.decode(idx)
    assert bad == 0 and np.array_equal(got, want)
    # 48-bit storage addresses the first 2^48 points of the same code
    low = rng.integers(0, 1 << 48, size=50000, dtype=np.uint64)
    got = gpu19.llvq_decode_i8(_dev(synth.pack_u48(low).reshape(-1))).cpu().numpy()
    assert np.array_equal(got, oracle19.decode(low)[0])


def test_wide_out_of_range_and_validate(gpu19, oracle19):
    import torch
    N = oracle19.num_points
    idx = np.array([0, N - 1, N, N + 5, (1 << 56) - 1, 12345], dtype=np.uint64)
    got = gpu19.llvq_decode_i8(_dev(idx.view(np.int64))).cpu().numpy()
    want, _ = oracle19.decode(idx[[0, 1, 5]])
    assert np.array_equal(got[[0, 1, 5]], want) and not got[2:5].any()
    assert gpu19.llvq_validate(_dev(idx.view(np.int64))) == 3
    out = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    gpu19.llvq_validate_static(_dev(idx.view(np.int64)), out=out)
    assert int(out.cpu()[0]) == 3
    # the upper 8 bits of a 64-bit word are ignored
    tagged = idx.copy()
    tagged[5] |= np.uint64(0xAB) << np.uint64(56)
    assert np.array_equal(gpu19.llvq_decode_i8(_dev(tagged.view(np.int64))).cpu().numpy()[5], want[2])


@pytest.mark.parametrize("dt", ["float16", "bfloat16", "float32"])
def test_wide_shape_gain_decode(gpu19, oracle19, dt):
    import torch
    rng = synth.rng_for(19, 1)
    idx = rng.integers(0, oracle19.num_points, size=30011, dtype=np.uint64)
    gain = synth.gains(rng, idx.shape)
    tdt = getattr(torch, dt)
    got = gpu19.llvq_decode(_dev(idx.view(np.int64)), _dev(gain), out_dtype=tdt).float().cpu().numpy().astype(np.float64)
    want = oracle19.dequant(idx, gain)
    tol = {"float16": 2 ** -10, "bfloat16": 2 ** -8, "float32": 2 ** -22}[dt]
    assert np.abs(got - want).max() <= tol * np.abs(want).max()
    assert (np.abs(got - want) <= tol * np.abs(want) + 1e-7).all()


@pytest.mark.parametrize("N,K,M,xd", [(300, 24 * 31, 1, "f16"), (64, 1000, 3, "bf16"), (1024, 4096, 1, "f16"), (37, 24 * 5, 16, "f16")])
def test_wide_matmul(gpu19, oracle19, N, K, M, xd):
    import torch
    rng = synth.rng_for(19, 10 + N)
    KB = synth.blocks_per_row(K)
    idx = rng.integers(0, oracle19.num_points, size=(N, KB), dtype=np.uint64)
    gain = synth.gains(rng, (N, KB))
    x = synth.activations(rng, M, K, "bf16" if xd == "bf16" else np.float16)
    d_x = _dev(x).to(torch.bfloat16 if xd == "bf16" else torch.float16)
    y = gpu19.llvq_matmul(d_x, _dev(idx.view(np.int64).reshape(-1)), _dev(gain.reshape(-1)), N, KB).cpu().numpy().astype(np.float64)
    ref = oracle19.matmul(x, idx, gain)
    err = np.abs(y - ref).max() / np.abs(ref).max()
    assert err <= TOL, err
    assert err <= 1e-5                      # fp32 accumulation of exact products


def test_wide_context_refuses_what_it_does_not_implement(gpu19):
    import torch
    from paper_2603_11021_amd import LLVQError
    pts = torch.zeros((4, 24), dtype=torch.int8, device="cuda:0")
    with pytest.raises(LLVQError, match="not implemented"):
        gpu19.llvq_encode(pts)
    x = torch.zeros((17, 24), dtype=torch.float16, device="cuda:0")
    idx = torch.zeros(2, dtype=torch.int64, device="cuda:0")
    g = torch.ones(2, dtype=torch.float16, device="cuda:0")
    with pytest.raises(LLVQError, match="not implemented"):
        gpu19.llvq_matmul(x, idx, g, 2, 1)
