"""ctypes binding of libfalqon.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their device
pointers and the current HIP stream through the C ABI (include/falqon.h) and returns.
Nothing is computed here, and there is no fallback: if the library is missing or a call
fails, an exception is raised.
"""
import ctypes
import os
from typing import Optional

import torch

E4M3, E5M2 = 0, 1
BF16, F32 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfalqon.so")
_lib = None


class FalqonError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: falqon status {status} ({status_string(status)})")


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """Load libfalqon.so (built in-tree by paper_2510_24061_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2510_24061_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        c = ctypes
        vp, i64, f32p = c.c_void_p, c.c_int64, c.c_void_p
        L.falqon_status_string.restype = c.c_char_p
        L.falqon_status_string.argtypes = [c.c_int]
        L.falqon_workspace_bytes.restype = c.c_size_t
        L.falqon_workspace_bytes.argtypes = [i64, i64, i64, i64]
        L.falqon_quantize.restype = c.c_int
        L.falqon_quantize.argtypes = [vp, c.c_int, i64, i64, i64, c.c_int, f32p, vp, i64, f32p, f32p,
                                      vp, c.c_size_t, vp]
        L.falqon_melded_fwd.restype = c.c_int
        L.falqon_melded_fwd.argtypes = [vp, vp, f32p, i64, i64, i64, i64, vp, f32p, vp, c.c_int, vp, f32p,
                                        vp, c.c_size_t, vp]
        L.falqon_melded_bwd.restype = c.c_int
        L.falqon_melded_bwd.argtypes = [vp, vp, f32p, vp, f32p, i64, i64, i64, i64, vp, f32p, vp, c.c_int,
                                        f32p, f32p, c.c_float, vp, vp, c.c_size_t, vp]
        L.falqon_row_score_bytes.restype = c.c_size_t
        L.falqon_row_score_bytes.argtypes = [i64]
        L.falqon_proxy_update.restype = c.c_int
        L.falqon_proxy_update.argtypes = [f32p, vp, i64, i64, i64, i64, vp, c.c_int, vp, vp, c.c_size_t, vp]
        L.falqon_proxy_update_static.restype = c.c_int
        L.falqon_proxy_update_static.argtypes = [f32p, vp, i64, i64, i64, i64, vp, c.c_int, vp]
        L.falqon_db_bf16.restype = c.c_int
        L.falqon_db_bf16.argtypes = [vp, f32p, vp, i64, i64, i64, vp, vp, c.c_float, vp, c.c_size_t, vp]
        L.falqon_fp8_gemm.restype = c.c_int
        L.falqon_fp8_gemm.argtypes = [vp, c.c_int, vp, c.c_int, i64, i64, i64, f32p, f32p, vp, c.c_int,
                                      vp, i64, vp, c.c_size_t, vp]
        L.falqon_grad_sqnorm.restype = c.c_int
        L.falqon_grad_sqnorm.argtypes = [f32p, i64, vp, vp, c.c_size_t, vp]
        L.falqon_adamw_delta.restype = c.c_int
        L.falqon_adamw_delta.argtypes = [f32p, f32p, f32p, f32p, i64, i64, i64, c.c_double, c.c_double, c.c_double,
                                         c.c_double, vp, c.c_double, vp]
        L.falqon_init_residual.restype = c.c_int
        L.falqon_init_residual.argtypes = [f32p, vp, f32p, i64, i64, f32p, vp]
        L.falqon_svd_workspace_bytes.restype = c.c_size_t
        L.falqon_svd_workspace_bytes.argtypes = [i64, i64, i64]
        L.falqon_svd_right_factor.restype = c.c_int
        L.falqon_svd_right_factor.argtypes = [f32p, i64, i64, i64, f32p, c.c_int, f32p, f32p, f32p, vp, c.c_size_t, vp]
        L.falqon_da.restype = c.c_int
        L.falqon_da.argtypes = [vp, f32p, vp, f32p, vp, f32p, i64, i64, i64, i64, vp, f32p, f32p, vp, c.c_size_t, vp]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().falqon_status_string(int(status)).decode()


def workspace_bytes(T: int, n: int, m: int, r: int) -> int:
    return int(lib().falqon_workspace_bytes(T, n, m, r))


def _p(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _check(status: int, where: str):
    if status != 0:
        raise FalqonError(status, where)


def _dev(*tensors):
    for t in tensors:
        if t is not None and not (t.is_cuda and t.is_contiguous()):
            raise ValueError("tensors must be contiguous GPU tensors")


def quantize(x: torch.Tensor, fmt: int, q: torch.Tensor, scale_out: torch.Tensor,
             ws: torch.Tensor, scale_in: Optional[torch.Tensor] = None,
             amax_out: Optional[torch.Tensor] = None) -> None:
    """falqon_quantize on a 2-D (or flat) tensor.  x and q may be row-strided views (unit stride along a
    row, any row stride that is a multiple of 16 elements): their row strides are passed as ld_x and ld_q."""
    _dev(scale_out, ws, scale_in, amax_out)
    if x.dim() == 2 and q.dim() == 2:
        rows, cols = x.shape
        if not (x.is_cuda and q.is_cuda) or q.shape != x.shape or (cols > 1 and (x.stride(1) != 1 or q.stride(1) != 1)):
            raise ValueError("x and q must be GPU tensors of one shape with unit stride along rows")
        ld_x = x.stride(0) if rows > 1 else cols
        ld_q = q.stride(0) if rows > 1 else cols
    else:
        _dev(x, q)
        rows, cols = 1, x.numel()
        ld_x = ld_q = cols
    st = lib().falqon_quantize(_p(x), _dtype_code(x), rows, cols, ld_x, fmt, _p(scale_in), _p(q), ld_q,
                               _p(scale_out), _p(amax_out), _p(ws), ws.numel() * ws.element_size(), _stream())
    _check(st, "falqon_quantize")


def melded_fwd(x, wq, s_w, m: int, r: int, xq, s_x, y, o_a, amax_oa, ws) -> None:
    """x = None: xq and s_x are inputs (already quantized by another layer's call or by quantize())."""
    _dev(x, wq, s_w, xq, s_x, y, o_a, amax_oa, ws)
    T, n = xq.shape
    st = lib().falqon_melded_fwd(_p(x) if x is not None else None, _p(wq), _p(s_w), T, n, m, r, _p(xq), _p(s_x), _p(y), _dtype_code(y),
                                 _p(o_a), _p(amax_oa), _p(ws), ws.numel() * ws.element_size(), _stream())
    _check(st, "falqon_melded_fwd")


def row_score_bytes(m: int) -> int:
    return int(lib().falqon_row_score_bytes(m))


def melded_bwd(dy, wq, s_w, o_a, amax_oa, n: int, r: int, dyq, s_dy, dx, d_b, delta_buf, lr: float, ws,
               row_scores=None) -> None:
    """dx = None: the input-gradient product is skipped.  delta_buf = None: no buffer step.
    row_scores (uint8/float64 tensor of row_score_bytes(m) bytes): left for a proxy_update that follows."""
    _dev(dy, wq, s_w, o_a, amax_oa, dyq, s_dy, dx, d_b, delta_buf, ws, row_scores)
    T, m = dy.shape
    st = lib().falqon_melded_bwd(_p(dy), _p(wq), _p(s_w), _p(o_a), _p(amax_oa), T, n, m, r, _p(dyq), _p(s_dy),
                                 _p(dx), _dtype_code(dx) if dx is not None else BF16, _p(d_b), _p(delta_buf), float(lr),
                                 _p(row_scores),
                                 _p(ws), ws.numel() * ws.element_size(), _stream())
    _check(st, "falqon_melded_bwd")


def proxy_update(delta_buf, wq, m: int, r: int, k: int, idx_out, ws, clear_selected: bool = True,
                 row_scores=None) -> None:
    """row_scores: the array melded_bwd filled for this very buffer content (else the scores are formed here)."""
    _dev(delta_buf, wq, idx_out, ws, row_scores)
    n = wq.shape[1]
    st = lib().falqon_proxy_update(_p(delta_buf), _p(wq), n, m, r, k, _p(idx_out), 1 if clear_selected else 0,
                                   _p(row_scores), _p(ws), ws.numel() * ws.element_size(), _stream())
    _check(st, "falqon_proxy_update")


def proxy_update_static(delta_buf, wq, m: int, r: int, k: int, idx_out, clear_selected: bool = True) -> None:
    """falqon_proxy_update on the library's static device scratch: no workspace, nothing allocated."""
    _dev(delta_buf, wq, idx_out)
    n = wq.shape[1]
    st = lib().falqon_proxy_update_static(_p(delta_buf), _p(wq), n, m, r, k, _p(idx_out), 1 if clear_selected else 0,
                                          _stream())
    _check(st, "falqon_proxy_update_static")


def fp8_gemm(a, a_fmt: int, b, b_is_kn: bool, s_a, s_b, c, side=None, side_ws=None) -> None:
    """C = A . op(B) / (s_a s_b): a [M,K] FP8; b E4M3 [N,K] or, with b_is_kn, [K,N].
    With `side` (adapter rows [r,K], or O_A codes [M,r] when b_is_kn) and a workspace it is the product
    launch of the melded forward / backward call, the adapter's product (or its partial sums) included."""
    _dev(a, b, s_a, s_b, c, side, side_ws)
    M, K = a.shape
    N = b.shape[1] if b_is_kn else b.shape[0]
    r = 0 if side is None else (side.shape[1] if b_is_kn else side.shape[0])
    st = lib().falqon_fp8_gemm(_p(a), a_fmt, _p(b), 1 if b_is_kn else 0, M, N, K, _p(s_a), _p(s_b), _p(c),
                               _dtype_code(c), _p(side), r, _p(side_ws),
                               0 if side_ws is None else side_ws.numel() * side_ws.element_size(), _stream())
    _check(st, "falqon_fp8_gemm")


def db_bf16(dyq, s_dy, o_a, d_b, delta_buf, lr: float, ws) -> None:
    """d_b = dyq^T o_a / s_dy with O_A kept in bf16 (variant of the adapter gradient); optional buffer step."""
    _dev(dyq, s_dy, o_a, d_b, ws)
    if delta_buf is not None:
        _dev(delta_buf)
    T, m = dyq.shape
    r = o_a.shape[1]
    st = lib().falqon_db_bf16(_p(dyq), _p(s_dy), _p(o_a), T, m, r, _p(d_b),
                              _p(delta_buf) if delta_buf is not None else None, float(lr), _p(ws),
                              ws.numel() * ws.element_size(), _stream())
    _check(st, "falqon_db_bf16")


def grad_sqnorm(g, sum_sq, ws) -> None:
    """*sum_sq (device fp64 scalar) += sum of squares of g (fp32)."""
    _dev(g, sum_sq, ws)
    st = lib().falqon_grad_sqnorm(_p(g), g.numel(), _p(sum_sq), _p(ws), ws.numel() * ws.element_size(), _stream())
    _check(st, "falqon_grad_sqnorm")


def adamw_delta(d_b, exp_avg, exp_avg_sq, delta_buf, step: int, lr: float = 2e-4, beta1: float = 0.9,
                beta2: float = 0.999, eps: float = 1e-8, sum_sq=None, max_norm: float = 0.3) -> None:
    """AdamW step on the (clipped) adapter gradient, written into the proxy buffer."""
    _dev(d_b, exp_avg, exp_avg_sq, delta_buf)
    if sum_sq is not None:
        _dev(sum_sq)
    m, r = d_b.shape
    st = lib().falqon_adamw_delta(_p(d_b), _p(exp_avg), _p(exp_avg_sq), _p(delta_buf), m, r, int(step), lr, beta1,
                                  beta2, eps, _p(sum_sq) if sum_sq is not None else None, max_norm, _stream())
    _check(st, "falqon_adamw_delta")


def init_residual(w, wq, s_w, e) -> None:
    """e = DQ(wq) - w (fp32 [m, n])."""
    _dev(w, wq, s_w, e)
    m, n = w.shape
    st = lib().falqon_init_residual(_p(w), _p(wq), _p(s_w), m, n, _p(e), _stream())
    _check(st, "falqon_init_residual")


def svd_workspace_bytes(m: int, n: int, r: int) -> int:
    return int(lib().falqon_svd_workspace_bytes(m, n, r))


def da(dyq, s_dy, btq, s_b, xq, s_x, g, amax_g, d_at, ws) -> None:
    """Gradient of the adapter factor A: g = bf16(dyq btq^T / (s_dy s_b)), d_at = xq^T g / s_x (fp32 [n, r]).
    ws: workspace_bytes(T, m, n, r) bytes (n and m exchanged)."""
    _dev(dyq, s_dy, btq, s_b, xq, s_x, g, amax_g, d_at, ws)
    T, m = dyq.shape
    n = xq.shape[1]
    r = btq.shape[0]
    st = lib().falqon_da(_p(dyq), _p(s_dy), _p(btq), _p(s_b), _p(xq), _p(s_x), T, n, m, r, _p(g), _p(amax_g), _p(d_at),
                         _p(ws), ws.numel() * ws.element_size(), _stream())
    _check(st, "falqon_da")


def svd_right_factor(e, r: int, omega, iters: int, a_out, sigma_out, ws, bt_out=None) -> None:
    """a_out = sqrt(S_r) V_r^T of e (fp32 [m, n]); omega is a Gaussian fp32 [r + 8, n] start matrix.
    bt_out (fp32 [r, m], optional): the left factor transposed, (U_r sqrt(S_r))^T."""
    _dev(e, omega, a_out, sigma_out, ws, bt_out)
    m, n = e.shape
    st = lib().falqon_svd_right_factor(_p(e), m, n, r, _p(omega), iters, _p(a_out), _p(sigma_out), _p(bt_out), _p(ws),
                                       ws.numel() * ws.element_size(), _stream())
    _check(st, "falqon_svd_right_factor")


class MeldedLinear:
    """Buffers of one melded layer plus the four calls, for tests and the benchmark.

    State kept between steps: wq = [W~ ; A~] (E4M3, [(m+r), n]), s_w, delta_buf (fp32 [m, r]).
    Everything else is per-step output or scratch.  All memory is allocated once here.
    """

    def __init__(self, T: int, n: int, m: int, r: int, k: int, out_dtype=torch.bfloat16, device="cuda",
                 share_transients_with: Optional["MeldedLinear"] = None):
        """share_transients_with: another layer of the same shape whose per-step buffers (x~, y, dy~,
        dx, workspace) this one aliases; for stacks whose layers run one after the other."""
        self.T, self.n, self.m, self.r, self.k = T, n, m, r, k
        dev = torch.device(device)
        u8, f32 = torch.uint8, torch.float32
        self.wq = torch.zeros(m + r, n, dtype=u8, device=dev)
        self.s_w = torch.zeros(1, dtype=f32, device=dev)
        self.delta_buf = torch.zeros(m, r, dtype=f32, device=dev)
        self.o_a = torch.empty(T, r, dtype=torch.bfloat16, device=dev)
        self.amax_oa = torch.zeros(1, dtype=f32, device=dev)
        self.d_b = torch.empty(m, r, dtype=f32, device=dev)
        self.idx = torch.zeros(k, dtype=torch.int32, device=dev)
        self.row_scores = torch.empty(row_score_bytes(m) // 8, dtype=torch.float64, device=dev)
        self._scores_fresh = False      # row_scores describe delta_buf as it is now
        o = share_transients_with
        if o is not None:
            if (o.T, o.n, o.m, o.r) != (T, n, m, r) or o.y.dtype != out_dtype:
                raise ValueError("transient buffers can only be shared between layers of one shape")
            self.xq, self.s_x, self.y, self.dyq, self.s_dy, self.dx, self.ws = o.xq, o.s_x, o.y, o.dyq, o.s_dy, o.dx, o.ws
            return
        self.xq = torch.empty(T, n, dtype=u8, device=dev)
        self.s_x = torch.zeros(1, dtype=f32, device=dev)
        self.y = torch.empty(T, m, dtype=out_dtype, device=dev)
        self.dyq = torch.empty(T, m, dtype=u8, device=dev)
        self.s_dy = torch.zeros(1, dtype=f32, device=dev)
        self.dx = torch.empty(T, n, dtype=out_dtype, device=dev)
        nbytes = workspace_bytes(T, n, m, r)
        if nbytes == 0:
            raise ValueError("invalid layer shape")
        self.ws = torch.empty(nbytes, dtype=u8, device=dev)

    def init_weights(self, w: torch.Tensor, a: torch.Tensor) -> None:
        """Initialization steps that need no SVD: W~, s_w <- Q(W); A~ <- cast(A * s_w); buffer <- 0."""
        s_tmp = torch.zeros(1, dtype=torch.float32, device=self.wq.device)
        quantize(w.contiguous(), E4M3, self.wq[: self.m], self.s_w, self.ws)
        quantize(a.contiguous(), E4M3, self.wq[self.m:], s_tmp, self.ws, scale_in=self.s_w)
        self.delta_buf.zero_()

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        melded_fwd(x, self.wq, self.s_w, self.m, self.r, self.xq, self.s_x, self.y, self.o_a, self.amax_oa, self.ws)
        return self.y

    def backward(self, dy: torch.Tensor, lr: float = 2e-4, accumulate: bool = True) -> torch.Tensor:
        """With the buffer step the call also leaves the buffer's row scores for the update that follows."""
        melded_bwd(dy, self.wq, self.s_w, self.o_a, self.amax_oa, self.n, self.r, self.dyq, self.s_dy, self.dx,
                   self.d_b, self.delta_buf if accumulate else None, lr, self.ws,
                   row_scores=self.row_scores if accumulate else None)
        self._scores_fresh = accumulate
        return self.dx

    def adamw_step(self, step: int, sum_sq: Optional[torch.Tensor] = None, lr: float = 2e-4, beta1: float = 0.9,
                   beta2: float = 0.999, eps: float = 1e-8, max_norm: float = 0.3) -> None:
        """DeltaBuffer <- AdamW(d_b) (after backward(accumulate=False)); moments are allocated on first use."""
        if not hasattr(self, "exp_avg"):
            self.exp_avg = torch.zeros_like(self.d_b)
            self.exp_avg_sq = torch.zeros_like(self.d_b)
        adamw_delta(self.d_b, self.exp_avg, self.exp_avg_sq, self.delta_buf, step, lr, beta1, beta2, eps, sum_sq,
                    max_norm)
        self._scores_fresh = False

    def update(self, clear_selected: bool = True, reuse_scores: bool = False) -> torch.Tensor:
        """reuse_scores: take the row scores the last backward() left instead of forming them again.  Only
        the caller knows whether delta_buf was written in between (this class sees its own calls only), so
        it has to ask for it; it is honoured only directly after a backward() with the buffer step."""
        scores = self.row_scores if (reuse_scores and self._scores_fresh) else None
        proxy_update(self.delta_buf, self.wq, self.m, self.r, self.k, self.idx, self.ws, clear_selected,
                     row_scores=scores)
        self._scores_fresh = False
        return self.idx
