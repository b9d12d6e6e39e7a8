"""The building block falqon_fp8_gemm: the plain FP8 product against the oracle, and the product
launches of the melded calls (adapter share as a side job) against those calls."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_24061_amd as fq
import workloads
from gpu_common import layer_on_gpu, np_of, oracle_weights, relf

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,N,K", [(70, 48, 80), (300, 272, 400), (2100, 1040, 528)])
@pytest.mark.parametrize("kn", [False, True])
def test_plain_product_matches_the_oracle(M, N, K, kn):
    """C = A . op(B) / (s_a s_b) on random codes.  The oracle's merged-forward product is that
    definition for [N,K] operands; for [K,N] the oracle's input-gradient product is."""
    g = np.random.default_rng(M + N + K + kn)
    fmt_a = fq.E5M2 if kn else fq.E4M3
    a = oracle.fp8_encode(g.normal(size=(M, K)).astype(np.float32) * 3, fmt_a)
    b = oracle.fp8_encode(g.normal(size=((K, N) if kn else (N, K))).astype(np.float32) * 3, oracle.E4M3)
    s_a, s_b = np.float32(1.7), np.float32(0.3)
    c = torch.empty(M, N, dtype=torch.float32, device="cuda")
    fq.fp8_gemm(torch.from_numpy(a).cuda(), fmt_a, torch.from_numpy(b).cuda(), kn,
                torch.tensor([s_a], device="cuda"), torch.tensor([s_b], device="cuda"), c)
    torch.cuda.synchronize()
    if kn:
        ref = oracle.dx(a, b, s_a, s_b, K)                    # rows [0, K) of a [K, N] "weight": dX = A . B
    else:
        ref = oracle.melded_fwd(a, b, s_b, s_a, N, 0)         # all N rows are backbone rows: Y = A . B^T
    assert relf(np_of(c), ref) < 1e-3


@pytest.mark.parametrize("T,n,m,r", [(2400, 3328, 3584, 64), (2400, 3344, 3568, 32)])
def test_product_launch_with_side_job_is_the_one_the_melded_calls_issue(T, n, m, r):
    d = workloads.make_inputs(T, n, m, r, seed=4400 + m, outliers=True)
    wcat, s_w = oracle_weights(d["w"], d["a"])
    layer = layer_on_gpu(T, n, m, r, 8, wcat, s_w, torch.bfloat16)
    layer.forward(d["x"].cuda())
    layer.backward(d["dy"].cuda(), accumulate=False)
    torch.cuda.synchronize()
    ws = torch.empty_like(layer.ws)
    y = torch.empty_like(layer.y)
    fq.fp8_gemm(layer.xq, fq.E4M3, layer.wq[:m], False, layer.s_x, layer.s_w, y, side=layer.wq[m:], side_ws=ws)
    codes = torch.from_numpy(oracle.quantize(np_of(layer.o_a), oracle.E4M3,
                                             scale_in=np.float32(448.0) / max(np.float32(layer.amax_oa.item()), np.float32(1e-12)))[0]).cuda()
    dx = torch.empty_like(layer.dx)
    fq.fp8_gemm(layer.dyq, fq.E5M2, layer.wq[:m], True, layer.s_dy, layer.s_w, dx, side=codes, side_ws=ws)
    torch.cuda.synchronize()
    assert torch.equal(y, layer.y) and torch.equal(dx, layer.dx)
    with pytest.raises(fq.FalqonError):                        # a small product has no such launch
        fq.fp8_gemm(layer.xq[:64], fq.E4M3, layer.wq[:m], False, layer.s_x, layer.s_w, y[:64], side=layer.wq[m:], side_ws=ws)
