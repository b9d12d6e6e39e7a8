"""The library on a non-default stream and under HIP graph capture.

Every call only enqueues kernels on the caller's stream (no allocation, no synchronisation, no
memset), so a whole training step can be captured into a graph.  A replay must reproduce the eager
step byte for byte; the graph is replayed several times with eager work and synchronisations in
between, and every replay is checked."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_24061_amd as fq
import workloads
from gpu_common import layer_on_gpu, np_of, oracle_weights

pytestmark = pytest.mark.gpu


def _state(layer):
    return [np_of(t).copy() for t in (layer.wq, layer.y, layer.o_a, layer.amax_oa, layer.dx, layer.d_b,
                                      layer.delta_buf, layer.idx, layer.xq, layer.dyq, layer.s_x, layer.s_dy)]


def _fresh(T, n, m, r, k, wcat, s_w):
    layer = layer_on_gpu(T, n, m, r, k, wcat, s_w)
    layer.delta_buf.zero_()
    return layer


@pytest.mark.parametrize("shape", [(256, 512, 512, 16, 8), (2304, 1024, 3600, 64, 16)])
def test_step_on_side_stream_matches_default_stream(shape):
    T, n, m, r, k = shape
    d = workloads.make_inputs(T, n, m, r, seed=77 + T, outliers=True)
    wcat, s_w = oracle_weights(d["w"], d["a"])
    x, dy = d["x"].cuda(), d["dy"].cuda()
    ref = _fresh(T, n, m, r, k, wcat, s_w)
    ref.forward(x); ref.backward(dy); ref.update()
    torch.cuda.synchronize()
    want = _state(ref)
    side = torch.cuda.Stream()
    layer = _fresh(T, n, m, r, k, wcat, s_w)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        layer.forward(x); layer.backward(dy); layer.update()
    side.synchronize()
    for a, b in zip(_state(layer), want):
        assert a.tobytes() == b.tobytes()


@pytest.mark.parametrize("shape", [(256, 512, 512, 16, 8), (2304, 1024, 3600, 64, 16)])
def test_captured_step_replays_like_the_eager_step(shape):
    T, n, m, r, k = shape
    d = workloads.make_inputs(T, n, m, r, seed=78 + T, outliers=True)
    wcat, s_w = oracle_weights(d["w"], d["a"])
    x, dy = d["x"].cuda(), d["dy"].cuda()
    wq0 = torch.from_numpy(wcat).cuda()

    # eager: three consecutive steps, state recorded after each
    eager = _fresh(T, n, m, r, k, wcat, s_w)
    want = []
    for _ in range(3):
        eager.forward(x); eager.backward(dy); eager.update()
        torch.cuda.synchronize()
        want.append(_state(eager))

    layer = _fresh(T, n, m, r, k, wcat, s_w)
    # warm up on a side stream (loads the code objects, sets kernel attributes), then restore the state
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        layer.forward(x); layer.backward(dy); layer.update()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    layer.wq.copy_(wq0); layer.delta_buf.zero_()
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer.forward(x); layer.backward(dy); layer.update()
    layer.wq.copy_(wq0); layer.delta_buf.zero_()                     # capture does not run the step
    scratch = torch.empty(1 << 20, device="cuda")
    for i in range(3):
        graph.replay()
        torch.cuda.synchronize()
        got = _state(layer)
        for a, b in zip(got, want[i]):
            assert a.tobytes() == b.tobytes(), f"replay {i}"
        scratch.normal_()                                             # eager work between replays
        (scratch * 2).sum().item()
