"""Adapter gradient with O_A kept in bf16 (falqon_db_bf16) against the oracle's db_wide."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_24061_amd as fq
from gpu_common import np_of, relf, sample_indices

pytestmark = pytest.mark.gpu

TOL = 1e-3      # the bar for products; fp32 accumulation of exact bf16 products lands near 1e-6


def _inputs(T, m, r, seed):
    g = torch.Generator().manual_seed(seed)
    dy = torch.randn(T, m, generator=g)
    dy[:, : max(1, m // 97)] *= 30.0                                   # a few large columns, like gradient outliers
    o_a = (torch.randn(T, r, generator=g) * 2.5).to(torch.bfloat16)
    dyq, s_dy, _ = oracle.quantize(dy.numpy(), oracle.E5M2)
    return dyq, np.float32(s_dy), o_a


def _run(dyq, s_dy, o_a, m, r, buf=None, lr=0.0):
    T = dyq.shape[0]
    ws = torch.empty(fq.workspace_bytes(T, 16, m, r), dtype=torch.uint8, device="cuda")
    d_b = torch.full((m, r), float("nan"), device="cuda")
    fq.db_bf16(torch.from_numpy(dyq).cuda(), torch.tensor([s_dy], device="cuda"), o_a.cuda(), d_b,
               buf, lr, ws)
    torch.cuda.synchronize()
    return d_b


# tokens: below one tile, ragged tail, several round trips of four tiles, many splits; features and
# ranks: single and several tiles with ragged edges
SHAPES = [(1, 16, 16), (100, 48, 16), (128, 128, 64), (777, 272, 32), (2100, 400, 80), (4096, 1040, 64),
          (5000, 144, 256), (9001, 2064, 48)]


@pytest.mark.parametrize("T,m,r", SHAPES)
def test_matches_oracle(T, m, r):
    dyq, s_dy, o_a = _inputs(T, m, r, seed=T + m + r)
    d_b = _run(dyq, s_dy, o_a, m, r)
    want = oracle.db_wide(dyq, s_dy, o_a.float().numpy())
    got = np_of(d_b)
    assert np.isfinite(got).all()
    assert relf(got, want) < TOL
    assert relf(got, want) < 1e-5                                      # what the arithmetic actually allows
    # element by element: every entry within a few fp32 roundings of the largest partial sum
    scale = np.abs(want).max()
    assert np.abs(got - want).max() <= 1e-5 * scale


def test_exact_integer_case_is_bit_exact():
    """Small integers and s_dy a power of two: every product and partial sum is an integer below
    2^24, so fp32 accumulation in any order gives the exact result."""
    T, m, r = 1000, 160, 48
    g = np.random.default_rng(3)
    dy_int = g.integers(-4, 5, size=(T, m)).astype(np.float32)
    oa_int = g.integers(-8, 9, size=(T, r)).astype(np.float32)
    dyq = oracle.fp8_encode(dy_int * 2.0, oracle.E5M2)                   # s_dy = 2
    d_b = _run(dyq, np.float32(2.0), torch.from_numpy(oa_int).to(torch.bfloat16), m, r)
    want = dy_int.astype(np.float64).T @ oa_int.astype(np.float64)
    assert np.array_equal(np_of(d_b).astype(np.float64), want)
    assert np.array_equal(oracle.db_wide(dyq, np.float32(2.0), oa_int), want)


def test_subnormal_and_extreme_gradient_codes_widen_exactly():
    """Every finite E5M2 code, subnormals and the largest value included, times 1 and times -2."""
    codes = np.array([c for c in range(256) if (c & 0x7F) < 0x7C], np.uint8)
    T = 16
    m = 256
    dyq = np.zeros((T, m), np.uint8)
    dyq[0, : codes.size] = codes                                          # one token carries each code once
    o_a = torch.zeros(T, 16)
    o_a[0, 0], o_a[0, 1] = 1.0, -2.0
    d_b = _run(dyq, np.float32(1.0), o_a.to(torch.bfloat16), m, 16)
    vals = oracle.fp8_decode(codes, oracle.E5M2)
    got = np_of(d_b).astype(np.float64)
    assert np.array_equal(got[: codes.size, 0], vals)
    assert np.array_equal(got[: codes.size, 1], -2.0 * vals)
    assert not got[:, 2:].any() and not got[codes.size:].any()


def test_buffer_step_and_repeatability():
    T, m, r = 1500, 272, 64
    dyq, s_dy, o_a = _inputs(T, m, r, seed=11)
    lr = 2e-4
    buf0 = torch.randn(m, r, generator=torch.Generator().manual_seed(5)) * 1e-3
    buf = buf0.clone().cuda()
    d_b = _run(dyq, s_dy, o_a, m, r, buf=buf, lr=lr)
    d_b_again = _run(dyq, s_dy, o_a, m, r)
    assert torch.equal(d_b, d_b_again)                                    # fixed summation order
    want_buf = oracle.delta_accumulate(buf0.numpy(), np_of(d_b).astype(np.float64), np.float32(lr))
    assert np.array_equal(np_of(buf), want_buf)


def test_full_size_config2_sampled_rows():
    T, m, r = 4096, 4096, 64
    dyq, s_dy, o_a = _inputs(T, m, r, seed=2)
    d_b = _run(dyq, s_dy, o_a, m, r)
    rows = sample_indices(m, 96, seed=4)
    want = oracle.db_wide(dyq, s_dy, o_a.float().numpy(), rows)
    assert relf(np_of(d_b)[rows], want) < 1e-5


def test_closer_to_the_ideal_gradient_than_the_e4m3_variant():
    """Same dy~, same saved O_A: dropping the cast of O_A to E4M3 removes that rounding error."""
    T, n, m, r = 2048, 512, 512, 64
    import workloads
    d = workloads.make_inputs(T=T, n=n, m=m, r=r, seed=21)
    from gpu_common import layer_on_gpu, oracle_weights
    wcat, s_w = oracle_weights(d["w"], d["a"])
    layer = layer_on_gpu(T, n, m, r, 8, wcat, s_w)
    layer.forward(d["x"].cuda())
    layer.backward(d["dy"].cuda(), accumulate=False)
    narrow = np_of(layer.d_b).astype(np.float64)
    wide = torch.empty(m, r, device="cuda")
    fq.db_bf16(layer.dyq, layer.s_dy, layer.o_a, wide, None, 0.0, layer.ws)
    torch.cuda.synchronize()
    ideal = oracle.fp8_decode(np_of(layer.dyq), oracle.E5M2).T @ np_of(layer.o_a).astype(np.float64) / float(layer.s_dy.item())
    assert relf(np_of(wide), ideal) < 1e-5
    assert relf(np_of(wide), ideal) < 0.01 * relf(narrow, ideal)


def test_argument_errors():
    dyq = torch.zeros(64, 64, dtype=torch.uint8, device="cuda")
    s = torch.ones(1, device="cuda")
    o_a = torch.zeros(64, 16, dtype=torch.bfloat16, device="cuda")
    d_b = torch.zeros(64, 16, device="cuda")
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(fq.FalqonError):
        fq.db_bf16(dyq, s, o_a, d_b, None, 0.0, small)
    with pytest.raises(fq.FalqonError):
        fq.db_bf16(torch.zeros(64, 40, dtype=torch.uint8, device="cuda"), s, o_a, torch.zeros(40, 16, device="cuda"),
                   None, 0.0, torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))          # m % 16 != 0
