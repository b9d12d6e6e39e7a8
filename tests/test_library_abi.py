"""Host-side checks of libfalqon.so that need no GPU: the library loads, exports every symbol
that include/falqon.h declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2510_24061_amd as fq
    if not os.path.exists(fq.lib_path()):
        from paper_2510_24061_amd import build
        build.build()
    return fq.lib()


def test_exports_every_declared_symbol(L):
    header = open(os.path.join(ROOT, "include", "falqon.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(falqon_[a-z_]+)\s*\(", header))
    assert {"falqon_quantize", "falqon_melded_fwd", "falqon_melded_bwd", "falqon_proxy_update",
            "falqon_workspace_bytes", "falqon_status_string"} <= names
    for name in names:
        assert hasattr(L, name), name


def test_status_strings(L):
    import paper_2510_24061_amd as fq
    assert fq.status_string(0) == "ok"
    assert len({fq.status_string(i) for i in range(8)}) == 8


def test_workspace_bytes(L):
    import paper_2510_24061_amd as fq
    assert fq.workspace_bytes(4096, 4096, 4096, 64) >= 4096 + 8 * 4096
    assert fq.workspace_bytes(4096, 4096, 4096, 64) < 64 << 20
    assert fq.workspace_bytes(0, 4096, 4096, 64) == 0
    assert fq.workspace_bytes(16, 4100, 4096, 64) == 0          # n not a multiple of 16
    assert fq.workspace_bytes(16, 4096, 4096, 272) == 0         # r > 256


def _vp(v):
    return ctypes.c_void_p(v)


def test_argument_validation_happens_before_any_launch(L):
    """Fake, never-dereferenced device addresses: every call must return an error status
    without launching (this machine may have no GPU at all)."""
    ok = 0x10000            # 16-byte aligned fake address
    odd = 0x10004
    ws_bytes = L.falqon_workspace_bytes(64, 64, 64, 16)
    q = L.falqon_quantize
    assert q(None, 0, 4, 16, 16, 0, None, _vp(ok), 16, _vp(ok), None, _vp(ok), 4096, None) == 1      # NULL x
    assert q(_vp(ok), 7, 4, 16, 16, 0, None, _vp(ok), 16, _vp(ok), None, _vp(ok), 4096, None) == 4   # dtype
    assert q(_vp(ok), 0, 4, 16, 16, 2, None, _vp(ok), 16, _vp(ok), None, _vp(ok), 4096, None) == 4   # fmt
    assert q(_vp(ok), 0, 4, 24, 24, 0, None, _vp(ok), 24, _vp(ok), None, _vp(ok), 4096, None) == 2   # cols % 16
    assert q(_vp(ok), 0, 4, 32, 16, 0, None, _vp(ok), 32, _vp(ok), None, _vp(ok), 4096, None) == 2   # ld < cols
    assert q(_vp(odd), 0, 4, 16, 16, 0, None, _vp(ok), 16, _vp(ok), None, _vp(ok), 4096, None) == 3  # align
    assert q(_vp(ok), 0, 4, 16, 16, 0, None, _vp(ok), 16, _vp(ok), None, None, 0, None) == 5         # no ws
    assert q(_vp(ok), 0, 4, 16, 16, 0, None, _vp(ok), 16, _vp(ok), None, _vp(ok), 100, None) == 5    # small ws

    f = L.falqon_melded_fwd
    args = dict(x=ok, wq=ok, s_w=ok, T=64, n=64, m=64, r=16, xq=ok, s_x=ok, y=ok, yt=0, o_a=ok, amax=ok,
                ws=ok, wsb=ws_bytes)

    def fwd(**kw):
        a = dict(args, **kw)
        return f(_vp(a["x"]), _vp(a["wq"]), _vp(a["s_w"]), a["T"], a["n"], a["m"], a["r"], _vp(a["xq"]),
                 _vp(a["s_x"]), _vp(a["y"]), a["yt"], _vp(a["o_a"]), _vp(a["amax"]), _vp(a["ws"]), a["wsb"], None)

    assert fwd(xq=None) == 1 and fwd(wq=None) == 1 and fwd(amax=None) == 1       # x alone may be NULL
    assert fwd(x=None, xq=None) == 1 and fwd(x=odd) == 3
    assert fwd(T=0) == 2 and fwd(n=72) == 2 and fwd(m=0) == 2 and fwd(r=8) == 2 and fwd(r=512) == 2
    assert fwd(y=odd) == 3 and fwd(yt=5) == 4
    assert fwd(ws=None) == 5 and fwd(wsb=ws_bytes - 1) == 5

    b = L.falqon_melded_bwd

    def bwd(**kw):
        a = dict(dy=ok, wq=ok, s_w=ok, o_a=ok, amax=ok, T=64, n=64, m=64, r=16, dyq=ok, s_dy=ok, dx=ok, dxt=0,
                 d_b=ok, buf=ok, sc=None, ws=ok, wsb=ws_bytes)
        a.update(kw)
        return b(_vp(a["dy"]), _vp(a["wq"]), _vp(a["s_w"]), _vp(a["o_a"]), _vp(a["amax"]), a["T"], a["n"], a["m"],
                 a["r"], _vp(a["dyq"]), _vp(a["s_dy"]), _vp(a["dx"]), a["dxt"], _vp(a["d_b"]), _vp(a["buf"]),
                 ctypes.c_float(1e-3), _vp(a["sc"]), _vp(a["ws"]), a["wsb"], None)

    assert bwd(dy=None) == 1 and bwd(d_b=None) == 1 and bwd(o_a=None) == 1
    assert bwd(sc=ok, buf=None) == 1                                           # scores are those of the stepped buffer
    assert bwd(sc=odd) == 3
    assert bwd(m=24) == 2 and bwd(T=-1) == 2
    assert bwd(dx=odd) == 3 and bwd(buf=odd) == 3 and bwd(dxt=9) == 4
    assert bwd(wsb=0) == 5

    p = L.falqon_proxy_update

    def upd(**kw):
        a = dict(buf=ok, wq=ok, n=64, m=64, r=16, k=4, idx=ok, sc=None, ws=ok, wsb=ws_bytes)
        a.update(kw)
        return p(_vp(a["buf"]), _vp(a["wq"]), a["n"], a["m"], a["r"], a["k"], _vp(a["idx"]), 1, _vp(a["sc"]),
                 _vp(a["ws"]), a["wsb"], None)

    assert upd(buf=None) == 1 and upd(idx=None) == 1 and upd(sc=odd) == 3
    assert L.falqon_row_score_bytes(4096) == 8 * (4096 + 64) and L.falqon_row_score_bytes(100) == 8 * 102
    assert L.falqon_row_score_bytes(0) == 0 and L.falqon_row_score_bytes(70000) == 0
    assert upd(k=0) == 2 and upd(k=65) == 2 and upd(m=131072, k=1) == 2
    assert upd(wq=odd) == 3
    assert upd(ws=None) == 5 and upd(wsb=16) == 5


def test_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2510_24061_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "import oracle" not in text and "from oracle" not in text, fn
                assert "falqon_oracle" not in text and "orc_" not in text, fn


def test_optimizer_argument_validation(L):
    import paper_2510_24061_amd as fq
    fq.lib()
    ok, odd = 0x10000, 0x10004
    n = L.falqon_grad_sqnorm
    assert n(None, 64, _vp(ok), _vp(ok), 4096, None) == 1
    assert n(_vp(ok), 64, None, _vp(ok), 4096, None) == 1
    assert n(_vp(ok), 0, _vp(ok), _vp(ok), 4096, None) == 2 and n(_vp(ok), 66, _vp(ok), _vp(ok), 4096, None) == 2
    assert n(_vp(odd), 64, _vp(ok), _vp(ok), 4096, None) == 3 and n(_vp(ok), 64, _vp(odd), _vp(ok), 4096, None) == 3
    assert n(_vp(ok), 64, _vp(ok), None, 4096, None) == 5 and n(_vp(ok), 64, _vp(ok), _vp(ok), 100, None) == 5

    a = L.falqon_adamw_delta

    def adam(d_b=ok, m1=ok, m2=ok, buf=ok, m=64, r=16, step=1, lr=2e-4, b1=0.9, b2=0.999, eps=1e-8, ss=None,
             mx=0.3):
        return a(_vp(d_b), _vp(m1), _vp(m2), _vp(buf), m, r, step, lr, b1, b2, eps, _vp(ss), mx, None)

    assert adam(d_b=None) == 1 and adam(m1=None) == 1 and adam(m2=None) == 1 and adam(buf=None) == 1
    assert adam(m=0) == 2 and adam(r=8) == 2 and adam(r=512) == 2 and adam(step=0) == 2
    assert adam(b1=1.0) == 2 and adam(b2=-0.1) == 2 and adam(eps=0.0) == 2 and adam(ss=ok, mx=0.0) == 2
    assert adam(buf=odd) == 3 and adam(ss=odd) == 3


def test_initialization_argument_validation(L):
    ok, odd = 0x10000, 0x10004
    res = L.falqon_init_residual
    assert res(None, _vp(ok), _vp(ok), 64, 64, _vp(ok), None) == 1 and res(_vp(ok), _vp(ok), _vp(ok), 64, 64, None, None) == 1
    assert res(_vp(ok), _vp(ok), _vp(ok), 0, 64, _vp(ok), None) == 2 and res(_vp(ok), _vp(ok), _vp(ok), 64, 66, _vp(ok), None) == 2
    assert res(_vp(odd), _vp(ok), _vp(ok), 64, 64, _vp(ok), None) == 3
    assert L.falqon_svd_workspace_bytes(4096, 4096, 64) > 72 * 4096 * 8
    assert L.falqon_svd_workspace_bytes(4096, 4096, 128) == 0 and L.falqon_svd_workspace_bytes(4096, 4096, 20) == 0
    assert L.falqon_svd_workspace_bytes(16, 4096, 16) == 0            # fewer rows than vectors
    svd = L.falqon_svd_right_factor
    wsb = L.falqon_svd_workspace_bytes(256, 256, 16)

    def f(e=ok, m=256, n=256, r=16, om=ok, it=2, a=ok, sg=ok, bt=None, ws=ok, wb=wsb):
        return svd(_vp(e), m, n, r, _vp(om), it, _vp(a), _vp(sg), _vp(bt), _vp(ws), wb, None)

    assert f(e=None) == 1 and f(om=None) == 1 and f(a=None) == 1 and f(sg=None) == 1
    assert f(r=12) == 2 and f(r=128) == 2 and f(m=254) == 2 and f(it=-1) == 2 and f(it=100) == 2
    assert f(a=odd) == 3 and f(bt=odd) == 3 and f(ws=None) == 5 and f(wb=wsb - 1) == 5


def test_db_bf16_argument_validation(L):
    f = L.falqon_db_bf16
    ok, odd = 0x10000, 0x10004
    big = L.falqon_workspace_bytes(64, 16, 64, 16)
    import ctypes as c
    lr = c.c_float(0.0)
    assert f(None, _vp(ok), _vp(ok), 64, 64, 16, _vp(ok), None, lr, _vp(ok), big, None) == 1
    assert f(_vp(ok), _vp(ok), _vp(ok), 64, 64, 16, None, None, lr, _vp(ok), big, None) == 1
    assert f(_vp(ok), _vp(ok), _vp(ok), 0, 64, 16, _vp(ok), None, lr, _vp(ok), big, None) == 2
    assert f(_vp(ok), _vp(ok), _vp(ok), 64, 40, 16, _vp(ok), None, lr, _vp(ok), big, None) == 2
    assert f(_vp(ok), _vp(ok), _vp(ok), 64, 64, 272, _vp(ok), None, lr, _vp(ok), big, None) == 2
    assert f(_vp(odd), _vp(ok), _vp(ok), 64, 64, 16, _vp(ok), None, lr, _vp(ok), big, None) == 3
    assert f(_vp(ok), _vp(ok), _vp(ok), 64, 64, 16, _vp(ok), _vp(odd), lr, _vp(ok), big, None) == 3
    assert f(_vp(ok), _vp(ok), _vp(ok), 64, 64, 16, _vp(ok), None, lr, None, big, None) == 5
    assert f(_vp(ok), _vp(ok), _vp(ok), 64, 64, 16, _vp(ok), None, lr, _vp(ok), big - 1, None) == 5


def test_static_scratch_update_rejects_sizes_beyond_its_limit(L):
    import paper_2510_24061_amd as fq
    ok = _vp(0x10000)
    f = L.falqon_proxy_update_static
    assert f(ok, ok, 256, 16400, 16, 4, ok, 1, None) == 7          # m beyond 16384
    assert f(ok, ok, 256, 16384, 256, 300, ok, 1, None) == 7       # k * r beyond 65536
    assert f(ok, ok, 256, 4096, 64, 0, ok, 1, None) == 2           # an ordinary shape error comes first
    assert f(None, ok, 256, 4096, 64, 4, ok, 1, None) == 1
    assert f(ok, _vp(0x10004), 256, 4096, 64, 4, ok, 1, None) == 3
    assert fq.status_string(7).startswith("size beyond")


def test_fp8_gemm_argument_validation(L):
    f = L.falqon_fp8_gemm
    ok, odd = _vp(0x10000), _vp(0x10004)
    big = L.falqon_workspace_bytes(2400, 3328, 3584, 64)

    def g(a=ok, af=0, b=ok, kn=0, M=2400, N=3584, K=3328, sa=ok, sb=ok, c=ok, ct=0, side=None, r=0, ws=None, wsb=0):
        return f(a, af, b, kn, M, N, K, sa, sb, c, ct, side, r, ws, wsb, None)

    assert g(a=None) == 1 and g(c=None) == 1 and g(sa=None) == 1
    assert g(af=3) == 4 and g(ct=2) == 4
    assert g(N=24) == 2 and g(K=8) == 2 and g(M=0) == 2
    assert g(b=odd) == 3
    # with the adapter's share as a side job: the shapes of a melded call, and a workspace
    assert g(side=ok, r=64, ws=None, wsb=big) == 5
    assert g(side=ok, r=64, ws=ok, wsb=big - 1) == 5
    assert g(side=ok, r=20, ws=ok, wsb=big) == 2                       # r not a multiple of 16
    assert g(side=ok, r=256, ws=ok, wsb=1 << 40) == 2                   # a rank beyond what 14 tile columns can share out
    assert g(side=ok, r=64, ws=ok, wsb=big, M=64) == 2                  # a small product does not use this launch
    assert g(side=odd, r=64, ws=ok, wsb=big) == 3
    assert g(side=ok, r=64, ws=ok, wsb=big, kn=1, af=0) == 4            # input-gradient orientation takes E5M2
    assert g(side=ok, r=64, ws=ok, wsb=big, kn=0, af=1) == 4


def test_da_argument_validation(L):
    f = L.falqon_da
    ok, odd = _vp(0x10000), _vp(0x10004)
    big = L.falqon_workspace_bytes(64, 128, 64, 16)              # (T, m, n, r): n and m exchanged

    def g(dyq=ok, btq=ok, xq=ok, T=64, n=64, m=128, r=16, gg=ok, am=ok, dat=ok, ws=ok, wb=big):
        return f(dyq, ok, btq, ok, xq, ok, T, n, m, r, gg, am, dat, ws, wb, None)

    assert g(dyq=None) == 1 and g(btq=None) == 1 and g(xq=None) == 1 and g(gg=None) == 1 and g(dat=None) == 1
    assert g(r=8) == 2 and g(n=72) == 2 and g(T=0) == 2
    assert g(xq=odd) == 3 and g(dat=odd) == 3
    assert g(ws=None) == 5 and g(wb=big - 1) == 5
