"""GPU parity of falqon_quantize against the CPU oracle: FP8 codes, scale and amax bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_24061_amd as fq
from gpu_common import np_of

pytestmark = pytest.mark.gpu


def _run(x: torch.Tensor, fmt, scale_in=None):
    xg = x.cuda()
    q = torch.full(xg.shape, 0xAA, dtype=torch.uint8, device="cuda")
    s = torch.zeros(1, device="cuda")
    amax = torch.zeros(1, device="cuda")
    ws = torch.empty(8192, dtype=torch.uint8, device="cuda")
    s_in = None if scale_in is None else torch.tensor([scale_in], dtype=torch.float32, device="cuda")
    fq.quantize(xg, fmt, q, s, ws, scale_in=s_in, amax_out=amax)
    torch.cuda.synchronize()
    return np_of(q), np.float32(s.item()), np.float32(amax.item())


def _check(x: torch.Tensor, fmt, scale_in=None):
    q, s, amax = _run(x, fmt, scale_in)
    xf = x.float().numpy()
    q_ref, s_ref, amax_ref = oracle.quantize(xf, fmt, scale_in=scale_in)
    assert s.tobytes() == s_ref.tobytes(), (s, s_ref)
    assert amax.tobytes() == amax_ref.tobytes(), (amax, amax_ref)
    bad = np.flatnonzero(q.ravel() != q_ref.ravel())
    assert bad.size == 0, (bad[:5], q.ravel()[bad[:5]], q_ref.ravel()[bad[:5]], xf.ravel()[bad[:5]])


@pytest.mark.parametrize("fmt", [fq.E4M3, fq.E5M2])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("shape", [(1, 16), (37, 48), (256, 512), (1000, 4096), (3, 65536 + 16)])
def test_quantize_matches_oracle(fmt, dtype, shape):
    g = torch.Generator().manual_seed(hash((fmt, shape)) % 1000)
    x = (torch.randn(*shape, generator=g) * torch.exp(torch.randn(shape[0], 1, generator=g) * 2)).to(dtype)
    _check(x, fmt)


@pytest.mark.parametrize("fmt", [fq.E4M3, fq.E5M2])
def test_quantize_outlier_dominated_scale_and_subnormal_codes(fmt):
    g = torch.Generator().manual_seed(3)
    x = torch.randn(512, 1024, generator=g)
    x[:, 7] *= 20.0
    x[100, 7] = 3000.0            # amax far above the bulk: most codes fall into the subnormal range
    _check(x.to(torch.bfloat16), fmt)
    _check(x, fmt)


def test_quantize_with_supplied_scale_saturates_like_the_oracle():
    g = torch.Generator().manual_seed(4)
    a = torch.randn(64, 512, generator=g) / 64
    _check(a, fq.E4M3, scale_in=np.float32(21000.0))      # many entries beyond 448 / s: must clip, not NaN
    q, _, _ = _run(a, fq.E4M3, np.float32(21000.0))
    assert np.all((q & 0x7F) != 0x7F)
    assert np.any((q & 0x7F) == 0x7E)


@pytest.mark.parametrize("fmt", [fq.E4M3, fq.E5M2])
def test_quantize_all_zero_and_empty(fmt):
    _check(torch.zeros(8, 32), fmt)
    q = torch.empty(0, 32, dtype=torch.uint8, device="cuda")
    s = torch.zeros(1, device="cuda")
    ws = torch.empty(8192, dtype=torch.uint8, device="cuda")
    fq.quantize(torch.empty(0, 32, device="cuda"), fmt, q, s, ws)
    torch.cuda.synchronize()
    assert np.float32(s.item()) == np.float32(oracle.fp8_max(fmt)) / np.float32(1e-12)


def test_quantize_every_bf16_bit_pattern():
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    x = bits.view(torch.bfloat16)
    x = x[torch.isfinite(x.float())]
    x = x[: (x.numel() // 16) * 16].contiguous()
    for fmt in (fq.E4M3, fq.E5M2):
        # unit scale: the cast alone
        q, s, _ = _run(x.reshape(1, -1), fmt, np.float32(1.0))
        ref = oracle.fp8_encode(x.float().numpy(), fmt)
        assert np.array_equal(q.ravel(), ref)
        q, s, _ = _run(x.reshape(1, -1), fmt, np.float32(0.37))
        ref = oracle.fp8_encode(x.float().numpy() * np.float32(0.37), fmt)
        assert np.array_equal(q.ravel(), ref)


@pytest.mark.parametrize("fmt", [fq.E4M3, fq.E5M2])
def test_cast_every_finite_fp32_bit_pattern(fmt):
    """All 2^32 fp32 inputs through the C ABI with unit scale, in 32 slices of 2^27."""
    chunk = 1 << 27
    ws = torch.empty(8192, dtype=torch.uint8, device="cuda")
    s = torch.zeros(1, device="cuda")
    one = torch.ones(1, device="cuda")
    q = torch.empty(chunk, dtype=torch.uint8, device="cuda")
    base = torch.arange(chunk, dtype=torch.int32, device="cuda")
    for c in range(32):
        bits = base + torch.tensor((c * chunk) - (1 << 31), dtype=torch.int64).to(torch.int32).cuda()
        x = bits.view(torch.float32)
        fq.quantize(x, fmt, q, s, ws, scale_in=one)
        got = q.cpu().numpy()
        xf = x.cpu().numpy()
        ref = oracle.fp8_encode(xf, fmt)
        fin = np.isfinite(xf)
        bad = np.flatnonzero((got != ref) & fin)
        assert bad.size == 0, (c, xf[bad[:4]], got[bad[:4]], ref[bad[:4]])
        print(f"slice {c} ok", flush=True)


def test_quantize_more_than_2_to_31_elements():
    """Index arithmetic beyond 32 bits: a tensor of 2^31 + 2^16 elements whose largest magnitude is
    its very last element.  The scale must see it, and codes are compared where 32-bit offsets would
    wrap: at the start, across the 2^31 boundary and at the end."""
    cols = 4096
    rows = (1 << 31) // cols + 16
    g = torch.Generator().manual_seed(31)
    block = torch.randn(4096, cols, generator=g).to(torch.bfloat16)
    x = block.repeat(rows // 4096 + 1, 1)[:rows].contiguous()
    x[-1, -1] = 1000.0
    x[(1 << 31) // cols, 5] = -700.0
    xg = x.cuda()
    q = torch.empty(rows, cols, dtype=torch.uint8, device="cuda")
    s = torch.zeros(1, device="cuda")
    amax = torch.zeros(1, device="cuda")
    ws = torch.empty(8192, dtype=torch.uint8, device="cuda")
    fq.quantize(xg, fq.E4M3, q, s, ws, amax_out=amax)
    torch.cuda.synchronize()
    assert amax.item() == 1000.0
    _, s_ref, _ = oracle.quantize(np.full((1, 16), 1000.0, np.float32), oracle.E4M3)
    assert np.float32(s.item()).tobytes() == s_ref.tobytes()
    boundary = (1 << 31) // cols
    for lo, hi in ((0, 256), (boundary - 128, boundary + 128), (rows - 256, rows)):
        ref, _, _ = oracle.quantize(x[lo:hi].float().numpy(), oracle.E4M3, scale_in=s_ref)
        assert np.array_equal(np_of(q[lo:hi]), ref), (lo, hi)


@pytest.mark.parametrize("fmt", [fq.E4M3, fq.E5M2])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("rows,cols,pad_x,pad_q", [(37, 48, 16, 32), (300, 1024, 48, 0), (129, 272, 0, 16),
                                                   (2050, 4096, 32, 64)])
def test_quantize_row_strided_input_and_output(fmt, dtype, rows, cols, pad_x, pad_q):
    """Row strides larger than the row length (ld_x > cols, ld_q > cols): the padding elements of x,
    which here hold values far above the tensor's own maximum, must not enter the scale, and the
    padding bytes of q must stay as they were."""
    g = torch.Generator().manual_seed(rows + cols)
    big = torch.full((rows, cols + pad_x), 1.0e6).to(dtype)
    big[:, :cols] = (torch.randn(rows, cols, generator=g) * torch.exp(torch.randn(rows, 1, generator=g))).to(dtype)
    xg = big.cuda()[:, :cols]
    qbig = torch.full((rows, cols + pad_q), 0xAA, dtype=torch.uint8, device="cuda")
    q = qbig[:, :cols]
    s = torch.zeros(1, device="cuda")
    amax = torch.zeros(1, device="cuda")
    ws = torch.empty(8192, dtype=torch.uint8, device="cuda")
    fq.quantize(xg, fmt, q, s, ws, amax_out=amax)
    torch.cuda.synchronize()
    q_ref, s_ref, amax_ref = oracle.quantize(big[:, :cols].float().numpy(), fmt)
    assert np.float32(s.item()).tobytes() == s_ref.tobytes()
    assert np.float32(amax.item()).tobytes() == amax_ref.tobytes()
    got = np_of(qbig)
    assert np.array_equal(got[:, :cols], q_ref)
    assert np.all(got[:, cols:] == 0xAA)
