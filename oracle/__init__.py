"""CPU oracle for the melded FP8-LoRA layer: numpy front end of falqon_oracle.c.

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg; never by the GPU package.  All arithmetic lives in
the C file; this module only marshals numpy arrays into it and composes its
functions in the order the paper's algorithms give.
"""
import ctypes
import os

import numpy as np

from . import build as _build

E4M3 = 0
E5M2 = 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        c = ctypes
        p = c.c_void_p
        L.orc_fp8_max.restype = c.c_double
        L.orc_fp8_max.argtypes = [c.c_int]
        L.orc_fp8_decode.restype = c.c_double
        L.orc_fp8_decode.argtypes = [c.c_uint8, c.c_int]
        L.orc_fp8_encode.restype = c.c_uint8
        L.orc_fp8_encode.argtypes = [c.c_float, c.c_int]
        L.orc_round_bf16.restype = c.c_float
        L.orc_round_bf16.argtypes = [c.c_double]
        L.orc_round_bf16_array.argtypes = [p, c.c_int64, p]
        L.orc_fp8_encode_array.argtypes = [p, c.c_int64, c.c_int, p]
        L.orc_fp8_decode_array.argtypes = [p, c.c_int64, c.c_int, p]
        L.orc_quantize.argtypes = [p, c.c_int64, c.c_int, p, p, p, p]
        L.orc_melded_fwd.argtypes = [p, p, c.c_float, c.c_float, c.c_int64, c.c_int64, c.c_int64, c.c_int64,
                                     p, c.c_int64, p, c.c_int64, p]
        L.orc_dx.argtypes = [p, p, c.c_float, c.c_float, c.c_int64, c.c_int64, c.c_int64,
                             p, c.c_int64, p, c.c_int64, p]
        L.orc_db.argtypes = [p, c.c_float, p, c.c_float, c.c_int64, c.c_int64, c.c_int64,
                             p, c.c_int64, p, p, p]
        L.orc_db_wide.argtypes = [p, c.c_float, p, c.c_int64, c.c_int64, c.c_int64, p, c.c_int64, p]
        L.orc_delta_accumulate.argtypes = [p, p, c.c_int64, c.c_float]
        L.orc_adamw_delta.argtypes = [p, p, p, p, c.c_int64, c.c_int64, c.c_double, c.c_double, c.c_double,
                                      c.c_double, c.c_double]
        L.orc_sum_squares.restype = c.c_double
        L.orc_sum_squares.argtypes = [p, c.c_int64]
        L.orc_clip_coef.restype = c.c_double
        L.orc_clip_coef.argtypes = [c.c_double, c.c_double]
        L.orc_row_scores.argtypes = [p, c.c_int64, c.c_int64, p]
        L.orc_topk_rows.argtypes = [p, c.c_int64, c.c_int64, p]
        L.orc_proxy_update.argtypes = [p, p, c.c_int64, c.c_int64, c.c_int64, c.c_int64, p, c.c_int]
        L.orc_init_residual.argtypes = [p, p, c.c_float, c.c_int64, p]
        L.orc_adapter_inner_grad.argtypes = [p, c.c_float, p, c.c_float, c.c_int64, c.c_int64, c.c_int64, p]
        L.orc_da.argtypes = [p, c.c_float, p, c.c_int64, c.c_int64, c.c_int64, p, c.c_int64, p]
        L.orc_num_threads.restype = c.c_int
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _sel(sel):
    if sel is None:
        return None, 0
    s = _c(sel, np.int64)
    return s, s.size


def num_threads() -> int:
    return int(lib().orc_num_threads())


def fp8_max(fmt: int) -> float:
    return float(lib().orc_fp8_max(fmt))


def fp8_encode(values, fmt: int) -> np.ndarray:
    v = _c(values, np.float32)
    out = np.empty(v.shape, np.uint8)
    lib().orc_fp8_encode_array(_ptr(v), v.size, fmt, _ptr(out))
    return out


def fp8_decode(codes, fmt: int) -> np.ndarray:
    c = _c(codes, np.uint8)
    out = np.empty(c.shape, np.float64)
    lib().orc_fp8_decode_array(_ptr(c), c.size, fmt, _ptr(out))
    return out


def round_bf16(values) -> np.ndarray:
    v = _c(values, np.float64)
    out = np.empty(v.shape, np.float32)
    lib().orc_round_bf16_array(_ptr(v), v.size, _ptr(out))
    return out


def quantize(x, fmt: int, scale_in=None):
    """Q_fp8 of the whole tensor.  Returns (codes, scale, amax)."""
    xf = _c(x, np.float32)
    q = np.empty(xf.shape, np.uint8)
    s_out = np.zeros(1, np.float32)
    a_out = np.zeros(1, np.float32)
    s_in = None if scale_in is None else np.array([scale_in], np.float32)
    lib().orc_quantize(_ptr(xf), xf.size, fmt, _ptr(s_in), _ptr(q), _ptr(s_out), _ptr(a_out))
    return q, np.float32(s_out[0]), np.float32(a_out[0])


def melded_fwd(xq, wq, s_w, s_x, m: int, r: int, rows=None, cols=None) -> np.ndarray:
    """fp64 merged output [rows, cols] (all tokens / all m+r columns when None)."""
    xq = _c(xq, np.uint8)
    wq = _c(wq, np.uint8)
    T, n = xq.shape
    assert wq.shape == (m + r, n)
    rs, nr = _sel(rows)
    cs, nc = _sel(cols)
    out = np.empty((nr if rs is not None else T, nc if cs is not None else m + r), np.float64)
    lib().orc_melded_fwd(_ptr(xq), _ptr(wq), float(s_w), float(s_x), T, n, m, r,
                         _ptr(rs), nr, _ptr(cs), nc, _ptr(out))
    return out


def dx(dyq, wq, s_dy, s_w, m: int, rows=None, cols=None) -> np.ndarray:
    dyq = _c(dyq, np.uint8)
    wq = _c(wq, np.uint8)
    T = dyq.shape[0]
    n = wq.shape[1]
    assert dyq.shape[1] == m and wq.shape[0] >= m
    rs, nr = _sel(rows)
    cs, nc = _sel(cols)
    out = np.empty((nr if rs is not None else T, nc if cs is not None else n), np.float64)
    lib().orc_dx(_ptr(dyq), _ptr(wq), float(s_dy), float(s_w), T, n, m,
                 _ptr(rs), nr, _ptr(cs), nc, _ptr(out))
    return out


def db(dyq, s_dy, o_a, amax_oa, rows=None):
    """Returns (dB fp64 [rows, r], E4M3 codes of O_A [T, r], s_oa)."""
    dyq = _c(dyq, np.uint8)
    oa = _c(o_a, np.float32)
    T, m = dyq.shape
    r = oa.shape[1]
    assert oa.shape[0] == T
    rs, nr = _sel(rows)
    out = np.empty((nr if rs is not None else m, r), np.float64)
    oaq = np.empty((T, r), np.uint8)
    s_oa = np.zeros(1, np.float32)
    lib().orc_db(_ptr(dyq), float(s_dy), _ptr(oa), float(amax_oa), T, m, r,
                 _ptr(rs), nr, _ptr(out), _ptr(oaq), _ptr(s_oa))
    return out, oaq, np.float32(s_oa[0])


def db_wide(dyq, s_dy, o_a, rows=None) -> np.ndarray:
    """dB fp64 [rows, r] with O_A taken as given (16-bit values), not cast to E4M3."""
    dyq = _c(dyq, np.uint8)
    oa = _c(o_a, np.float32)
    T, m = dyq.shape
    r = oa.shape[1]
    assert oa.shape[0] == T
    rs, nr = _sel(rows)
    out = np.empty((nr if rs is not None else m, r), np.float64)
    lib().orc_db_wide(_ptr(dyq), float(s_dy), _ptr(oa), T, m, r, _ptr(rs), nr, _ptr(out))
    return out


def delta_accumulate(buf, d_b, lr) -> np.ndarray:
    b = np.array(buf, np.float32, copy=True)
    g = _c(d_b, np.float64)
    assert b.shape == g.shape
    lib().orc_delta_accumulate(_ptr(b), _ptr(g), b.size, float(lr))
    return b


def adamw_delta(d_b, exp_avg, exp_avg_sq, buf, step, lr=2e-4, beta1=0.9, beta2=0.999, eps=1e-8, clip_coef=1.0):
    """One optimizer step into the proxy buffer; returns new (exp_avg, exp_avg_sq, buf), all fp32."""
    g = _c(d_b, np.float32)
    m = np.array(exp_avg, np.float32, copy=True)
    v = np.array(exp_avg_sq, np.float32, copy=True)
    b = np.array(buf, np.float32, copy=True)
    assert g.shape == m.shape == v.shape == b.shape
    lib().orc_adamw_delta(_ptr(g), _ptr(m), _ptr(v), _ptr(b), g.size, int(step), float(lr), float(beta1),
                          float(beta2), float(eps), float(clip_coef))
    return m, v, b


def sum_squares(g) -> float:
    a = _c(g, np.float32)
    return float(lib().orc_sum_squares(_ptr(a), a.size))


def clip_coef(sum_sq: float, max_norm: float = 0.3) -> float:
    return float(lib().orc_clip_coef(float(sum_sq), float(max_norm)))


def row_scores(buf) -> np.ndarray:
    b = _c(buf, np.float32)
    m, r = b.shape
    out = np.empty(m, np.float64)
    lib().orc_row_scores(_ptr(b), m, r, _ptr(out))
    return out


def topk_rows(score, k: int) -> np.ndarray:
    s = _c(score, np.float64)
    idx = np.empty(k, np.int32)
    lib().orc_topk_rows(_ptr(s), s.size, k, _ptr(idx))
    return idx


def proxy_update(buf, wq, m: int, r: int, k: int, clear_selected: bool = True):
    """Returns (idx int32[k], new concatenated weight, new buffer); inputs are not modified."""
    b = np.array(buf, np.float32, copy=True)
    w = np.array(wq, np.uint8, copy=True)
    n = w.shape[1]
    assert w.shape[0] == m + r and b.shape == (m, r)
    idx = np.empty(k, np.int32)
    lib().orc_proxy_update(_ptr(b), _ptr(w), n, m, r, k, _ptr(idx), 1 if clear_selected else 0)
    return idx, w, b


def init_residual(w, wq, s_w) -> np.ndarray:
    """E = DQ(W~) - W in fp32 (initialization algorithm, residual step, with the sign of the reformulation equation)."""
    wf = _c(w, np.float32)
    q = _c(wq, np.uint8)
    assert wf.shape == q.shape
    e = np.empty(wf.shape, np.float32)
    lib().orc_init_residual(_ptr(wf), _ptr(q), float(s_w), wf.size, _ptr(e))
    return e


def adapter_inner_grad(dyq, s_dy, btq, s_b) -> np.ndarray:
    """G = bf16( dy~ . B~ / (s_dy s_b) ): the gradient at the adapter's inner activation A x (LoRA backward
    equation, first product of dL/dA = B^T dL/dO x^T).  btq is B^T as E4M3 codes [r, m]; returns fp32 [T, r]."""
    dyq = _c(dyq, np.uint8)
    btq = _c(btq, np.uint8)
    T, m = dyq.shape
    r = btq.shape[0]
    assert btq.shape == (r, m)
    g = np.empty((T, r), np.float32)
    lib().orc_adapter_inner_grad(_ptr(dyq), float(s_dy), _ptr(btq), float(s_b), T, m, r, _ptr(g))
    return g


def da(xq, s_x, g, rows=None) -> np.ndarray:
    """(dL/dA)^T = x~^T . G / s_x, fp64 [rows of n, r] (LoRA backward equation, second product)."""
    xq = _c(xq, np.uint8)
    gg = _c(g, np.float32)
    T, n = xq.shape
    r = gg.shape[1]
    assert gg.shape[0] == T
    rs, nr = _sel(rows)
    out = np.empty((nr if rs is not None else n, r), np.float64)
    lib().orc_da(_ptr(xq), float(s_x), _ptr(gg), T, n, r, _ptr(rs), nr, _ptr(out))
    return out


def svd_factors(e, r: int):
    """Both factors of the rank-r truncated SVD of E by the library's full SVD in fp64 (initialization
    algorithm, decomposition step): B = U_r sqrt(S_r) [m, r], A = sqrt(S_r) V_r^T [r, n], and all singular values."""
    u, sv, vt = np.linalg.svd(np.asarray(e, np.float64), full_matrices=False)
    root = np.sqrt(sv[:r])
    return u[:, :r] * root[None, :], root[:, None] * vt[:r], sv


def svd_right_factor(e, r: int):
    """Rank-r truncated SVD of E (initialization algorithm, decomposition step) by the library's full SVD in fp64:
    E ~ B A with B = U_r sqrt(S_r), A = sqrt(S_r) V_r^T.  Returns (A fp64 [r, n], S fp64 [min(m, n)])."""
    u, sv, vt = np.linalg.svd(np.asarray(e, np.float64), full_matrices=False)
    return np.sqrt(sv[:r])[:, None] * vt[:r], sv


def init_adapter(w, r: int):
    """Lines 3-6 of the initialization algorithm: W~, s_w <- Q(W); E; A^ <- SVD(E, r); A~ <- cast(A^ s_w).
    Returns dict(wq, s_w, e, a_hat, a_q, sv)."""
    wq, s_w, _ = quantize(w, E4M3)
    e = init_residual(w, wq, s_w)
    a_hat, sv = svd_right_factor(e, r)
    a_q, _, _ = quantize(a_hat.astype(np.float32), E4M3, scale_in=s_w)
    return dict(wq=wq, s_w=s_w, e=e, a_hat=a_hat, a_q=a_q, sv=sv)


# --------------------------------------------------------------------------------------
# Whole calls, composed as the paper's algorithms order them.
# --------------------------------------------------------------------------------------

def layer_fwd(x, wq, s_w, m: int, r: int, rows=None, cols=None):
    """Forward loop body: quantize x (E4M3), merged product, split.

    Returns dict(xq, s_x, merged) with merged = fp64 [rows, cols] of the merged output;
    with rows=cols=None also y (fp64 [T,m]), o_a (bf16-rounded, fp32 [T,r]) and amax_oa.
    """
    xq, s_x, _ = quantize(x, E4M3)
    merged = melded_fwd(xq, wq, s_w, s_x, m, r, rows, cols)
    out = dict(xq=xq, s_x=s_x, merged=merged)
    if rows is None and cols is None:
        out["y"] = merged[:, :m]
        o_a = round_bf16(merged[:, m:])
        out["o_a"] = o_a
        out["amax_oa"] = np.float32(np.max(np.abs(o_a))) if o_a.size else np.float32(0)
    return out


def layer_bwd(dy, wq, s_w, o_a, amax_oa, m: int, r: int, delta_buf=None, lr=0.0,
              dx_rows=None, dx_cols=None):
    """Backward loop body: quantize dY (E5M2), input gradient, adapter gradient, buffer step."""
    dyq, s_dy, _ = quantize(dy, E5M2)
    g_x = dx(dyq, wq, s_dy, s_w, m, dx_rows, dx_cols)
    g_b, oaq, s_oa = db(dyq, s_dy, o_a, amax_oa)
    out = dict(dyq=dyq, s_dy=s_dy, dx=g_x, db=g_b, oaq=oaq, s_oa=s_oa)
    if delta_buf is not None:
        out["delta_buf"] = delta_accumulate(delta_buf, g_b, lr)
    return out
