"""Helpers shared by the GPU parity tests (no arithmetic of the method)."""
import numpy as np
import torch

import oracle
import paper_2510_24061_amd as fq


def relf(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def np_of(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.float().numpy()
    return t.numpy()


def oracle_weights(w: torch.Tensor, a: torch.Tensor):
    """Initialization steps without the SVD, on the CPU oracle: codes of [W ; A] and s_w."""
    wq, s_w, _ = oracle.quantize(w.numpy(), oracle.E4M3)
    aq, _, _ = oracle.quantize(a.numpy(), oracle.E4M3, scale_in=s_w)
    return np.concatenate([wq, aq]), s_w


def layer_on_gpu(T, n, m, r, k, wcat: np.ndarray, s_w, out_dtype=torch.bfloat16) -> fq.MeldedLinear:
    """A GPU layer whose weight state is the oracle's (so both sides start from the same bytes)."""
    layer = fq.MeldedLinear(T, n, m, r, k, out_dtype=out_dtype)
    layer.wq.copy_(torch.from_numpy(wcat))
    layer.s_w.fill_(float(s_w))
    return layer


def sample_indices(total: int, count: int, seed: int) -> np.ndarray:
    g = np.random.default_rng(seed)
    if total <= count:
        return np.arange(total, dtype=np.int64)
    # always include the first and last index (tile corners), the rest at random
    rest = g.choice(np.arange(1, total - 1), size=count - 2, replace=False)
    return np.sort(np.concatenate([[0, total - 1], rest])).astype(np.int64)
