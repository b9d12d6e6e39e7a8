"""The register-only matrix-core loop (a measurement aid) computes what its header says."""
import pytest
import torch

import paper_2510_24061_amd as fq

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("code_a,code_b,val", [(0x38, 0x38, 1.0), (0x40, 0xB8, -2.0), (0x00, 0x38, 0.0)])
def test_probe_sums_constant_operands(code_a, code_b, val):
    # every operand element is the same value, so each accumulator element is iters * 64 * a * b
    # and a lane's 16 blocks x 16 elements sum to 256 times that (exact in fp32 at these sizes)
    wgs, iters = 3, 5
    a = torch.full((8192,), code_a, dtype=torch.uint8, device="cuda")
    b = torch.full((8192,), code_b, dtype=torch.uint8, device="cuda")
    sink = torch.full((wgs * 256,), float("nan"), device="cuda")
    fq.mfma_probe(a, b, wgs, iters, sink)
    torch.cuda.synchronize()
    assert torch.equal(sink.cpu(), torch.full((wgs * 256,), 256.0 * iters * 64 * val))


def test_probe_rejects_bad_arguments():
    a = torch.zeros(8192, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(256, device="cuda")
    with pytest.raises(ValueError):
        fq.mfma_probe(a[:4096], a, 1, 1, sink)
    with pytest.raises(ValueError):
        fq.mfma_probe(a, a, 2, 1, sink)
    with pytest.raises(fq.FalqonError):
        fq.mfma_probe(a, a, 1, 0, sink)
