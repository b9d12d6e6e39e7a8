"""The proxy update that takes no workspace (static device scratch inside the library) against the
ordinary entry point: bit-identical indices, weight bytes and buffer, on two calls in a row, the
second on a smaller layer (the scratch keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import paper_2510_24061_amd as fq
import workloads
from gpu_common import np_of, oracle_weights

pytestmark = pytest.mark.gpu


def _case(n, m, r, k, seed, clear):
    d = workloads.make_inputs(4, n, m, r, seed=seed, outliers=False)
    wcat, _ = oracle_weights(d["w"], d["a"])
    buf = workloads.make_delta_buffer(m, r, seed=seed + 1, scale=5e-3, ties=True)
    out = []
    for static in (False, True):
        wq = torch.from_numpy(wcat).cuda()
        delta = buf.clone().cuda()
        idx = torch.full((k,), -1, dtype=torch.int32, device="cuda")
        if static:
            fq.proxy_update_static(delta, wq, m, r, k, idx, clear_selected=clear)
        else:
            ws = torch.empty(fq.workspace_bytes(16, n, m, r), dtype=torch.uint8, device="cuda")
            fq.proxy_update(delta, wq, m, r, k, idx, ws, clear_selected=clear)
        torch.cuda.synchronize()
        out.append((np_of(idx).copy(), np_of(wq).copy(), np_of(delta).copy()))
    (i0, w0, b0), (i1, w1, b1) = out
    assert np.array_equal(i0, i1), (n, m, r, k)
    assert np.array_equal(w0, w1)
    assert b0.tobytes() == b1.tobytes()
    assert np.any(w0[:m] != wcat[:m])
    return i0


def test_static_scratch_update_equals_the_workspace_update_twice_in_a_row():
    print("static update: 4096 x 4096, k = 32", flush=True)
    _case(4096, 4096, 64, 32, seed=801, clear=True)
    print("static update: 208 x 384, k = 5 (smaller, same scratch)", flush=True)
    _case(384, 208, 16, 5, seed=802, clear=True)
    print("static update: 1040 x 1024, k = 64, buffer rows kept", flush=True)
    _case(1024, 1040, 64, 64, seed=803, clear=False)
