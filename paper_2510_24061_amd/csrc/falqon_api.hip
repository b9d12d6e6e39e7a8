// C ABI of libfalqon: argument validation on the host, then kernel launches on the caller's
// stream.  Nothing here allocates, synchronises or keeps state.
#include <cmath>

#include "falqon_internal.h"
#include "row_scores.h"

namespace falqon {

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

WsLayout ws_layout(int64_t T, int64_t n, int64_t m, int64_t r)
{
    WsLayout w;
    size_t off = 0;
    // partial counts: the larger of what the two ways of forming each adapter product need
    const OaTailPlan po = plan_oa_tail(T, n, m, r);
    const DbTailPlan pd = plan_db_tail(T, n, m, r);
    int oa_parts = oa_splits(T, r), db_parts = db_splits(T, m);
    if (po.use && po.splits > oa_parts) oa_parts = po.splits;
    if (pd.use && pd.groups > db_parts) db_parts = pd.groups;
    w.amax_partials = off; off = align_up(off + sizeof(float) * kMaxAmaxBlocks, 256);
    w.scores = off;        off = align_up(off + sizeof(double) * static_cast<size_t>(m + (m + 63) / 64), 256);
    w.delta_sel = off;     off = align_up(off + sizeof(float) * static_cast<size_t>(m) * static_cast<size_t>(r), 256);
    w.db_partials = off;   off = align_up(off + sizeof(float) * static_cast<size_t>(db_parts) *
                                                    static_cast<size_t>(m) * static_cast<size_t>(r), 256);
    w.oa_partials = off;   off = align_up(off + sizeof(float) * static_cast<size_t>(oa_parts) *
                                                    static_cast<size_t>(T) * static_cast<size_t>(r), 256);
    w.oa_codes = off;      off = align_up(off + static_cast<size_t>(T) * static_cast<size_t>(r), 256);
    w.total = off;
    return w;
}

int oa_splits(int64_t T, int64_t r)
{
    // the O_A product runs on 128x128 tiles; split K until about one workgroup per CU
    const int64_t tiles = ((T + 127) / 128) * ((r + 127) / 128);
    int s = 1;
    while (s < 8 && tiles * s * 2 <= 256) s *= 2;               // a power of two, at most 8
    return s;
}

static bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

static bool bad_layer_shape(int64_t T, int64_t n, int64_t m, int64_t r)
{
    return T < 1 || n < 16 || m < 16 || r < 16 || (n % 16) || (m % 16) || (r % 16) || r > 256 ||
           T > (int64_t(1) << 24) || n > (int64_t(1) << 20) || m > (int64_t(1) << 20);
}

}  // namespace falqon

using namespace falqon;

extern "C" {

const char* falqon_status_string(falqon_status s)
{
    switch (s) {
        case FALQON_OK: return "ok";
        case FALQON_ERR_NULL: return "null pointer";
        case FALQON_ERR_SHAPE: return "bad shape";
        case FALQON_ERR_ALIGN: return "pointer not 16-byte aligned";
        case FALQON_ERR_ENUM: return "unknown format or dtype";
        case FALQON_ERR_WORKSPACE: return "workspace missing or too small";
        case FALQON_ERR_HIP: return "HIP launch failed";
        case FALQON_ERR_LIMIT: return "size beyond the limit of the library's static scratch";
    }
    return "unknown status";
}

size_t falqon_workspace_bytes(int64_t T, int64_t n, int64_t m, int64_t r)
{
    if (bad_layer_shape(T, n, m, r)) return 0;
    return ws_layout(T, n, m, r).total;
}

size_t falqon_row_score_bytes(int64_t m)
{
    if (m < 1 || m > 65536) return 0;
    return sizeof(double) * static_cast<size_t>(m + score_blocks(m));
}

falqon_status falqon_quantize(const void* x, falqon_dtype xt, int64_t rows, int64_t cols, int64_t ld_x,
                              falqon_fmt fmt, const float* scale_in,
                              uint8_t* q, int64_t ld_q, float* scale_out, float* amax_out,
                              void* ws, size_t ws_bytes, void* stream)
{
    if (xt != FALQON_BF16 && xt != FALQON_F32) return FALQON_ERR_ENUM;
    if (fmt != FALQON_E4M3 && fmt != FALQON_E5M2) return FALQON_ERR_ENUM;
    if (rows < 0 || cols < 0 || (cols % 16) || ld_x < cols || ld_q < cols || (ld_x % 16) || (ld_q % 16))
        return FALQON_ERR_SHAPE;
    if (rows > (int64_t(1) << 40) / (cols > 0 ? cols : 1)) return FALQON_ERR_SHAPE;
    const bool empty = rows == 0 || cols == 0;
    if (!scale_out || (!empty && (!x || !q))) return FALQON_ERR_NULL;
    if (!empty && (misaligned(x) || misaligned(q))) return FALQON_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(scale_out) & 3u) || (amax_out && (reinterpret_cast<uintptr_t>(amax_out) & 3u)) ||
        (scale_in && (reinterpret_cast<uintptr_t>(scale_in) & 3u)))
        return FALQON_ERR_ALIGN;
    if (!ws || ws_bytes < sizeof(float) * kMaxAmaxBlocks) return FALQON_ERR_WORKSPACE;
    if (misaligned(ws)) return FALQON_ERR_ALIGN;
    hipError_t e = launch_quantize(x, xt, empty ? 0 : rows, cols > 0 ? cols : 16, ld_x, fmt, scale_in, q, ld_q,
                                   scale_out, amax_out, static_cast<float*>(ws), nullptr,
                                   static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

falqon_status falqon_melded_fwd(const void* x, const uint8_t* wq, const float* s_w,
                                int64_t T, int64_t n, int64_t m, int64_t r,
                                uint8_t* xq, float* s_x, void* y, falqon_dtype yt,
                                void* o_a, float* amax_oa,
                                void* ws, size_t ws_bytes, void* stream)
{
    if (yt != FALQON_BF16 && yt != FALQON_F32) return FALQON_ERR_ENUM;
    if (bad_layer_shape(T, n, m, r)) return FALQON_ERR_SHAPE;
    if (!wq || !s_w || !xq || !s_x || !y || !o_a || !amax_oa) return FALQON_ERR_NULL;     // x may be NULL
    if ((x && misaligned(x)) || misaligned(wq) || misaligned(xq) || misaligned(y) || misaligned(o_a))
        return FALQON_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(s_w) & 3u) || (reinterpret_cast<uintptr_t>(s_x) & 3u) ||
        (reinterpret_cast<uintptr_t>(amax_oa) & 3u))
        return FALQON_ERR_ALIGN;
    const WsLayout L = ws_layout(T, n, m, r);
    if (!ws || ws_bytes < L.total) return FALQON_ERR_WORKSPACE;
    if (misaligned(ws)) return FALQON_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* w8 = static_cast<uint8_t*>(ws);

    // x~, s_x <- Q_E4M3(x); the cast pass also resets the running maximum of O_A.  Without x the
    // caller's x~ and s_x are used as they are (several layers reading one input quantize it once).
    hipError_t e = x ? launch_quantize(x, FALQON_BF16, T, n, n, FALQON_E4M3, nullptr, xq, n, s_x, nullptr,
                                       reinterpret_cast<float*>(w8 + L.amax_partials),
                                       reinterpret_cast<uint32_t*>(amax_oa), st)
                     : launch_zero_word(reinterpret_cast<uint32_t*>(amax_oa), st);
    if (e != hipSuccess) return FALQON_ERR_HIP;

    // O_merged <- x~ W~'^T / (s_w s_x), split into y and O_A.  When the r adapter columns fit
    // into the last, partly empty tile column of the backbone product they ride along in the one
    // GEMM, whose epilogue splits them off; otherwise they would add a whole, almost empty tile
    // column (a second round over the CUs) and are formed from the same x~ by a split-K launch of
    // the same kernel on the adapter rows instead.
    const int64_t tile = gemm_tile_n(T, m + r);
    const bool merged = (m + r + tile - 1) / tile == (m + tile - 1) / tile;
    GemmArgs g;
    g.a = xq; g.lda = n; g.a_fmt = 0;
    g.b = wq; g.ldb = n; g.b_is_kn = 0;
    g.M = T; g.N = merged ? m + r : m; g.K = n;
    g.sa = s_x; g.sb = s_w;
    g.c0 = y; g.ldc0 = m; g.c0_is_f32 = (yt == FALQON_F32); g.n_split = m;
    g.c1 = o_a; g.ldc1 = r; g.amax1 = reinterpret_cast<uint32_t*>(amax_oa);
    if (merged) {
        e = launch_gemm(g, st);
        return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
    }
    // O_A <- x~ A~^T / (s_w s_x).  On the large tiles the backbone workgroups form it: inside their
    // own K-steps, finished, where a tile row has enough tile columns to share it out; else as a
    // side job ahead of the tile that leaves fp32 partials over K slices, which one more pass adds
    // in order, rounds to bf16 and takes the maximum of.
    float* part = reinterpret_cast<float*>(w8 + L.oa_partials);
    const OaTailPlan po = plan_oa_tail(T, n, m, r);
    if (po.use) {
        TailArgs t;
        t.side = wq + m * n; t.r = r; t.partial = part; t.splits = po.splits; t.steps_per_split = po.steps_per_split;
        t.row_parts = po.row_parts;
        e = launch_gemm_fwd_tail(g, t, st);
        if (e != hipSuccess) return FALQON_ERR_HIP;
        if (po.splits > 0)                                       // (no partials: the launch wrote O_A and its maximum)
            e = launch_sum_partials_bf16(part, po.splits, T * r, static_cast<uint16_t*>(o_a),
                                         reinterpret_cast<uint32_t*>(amax_oa), st);
        return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
    }
    // Otherwise: the same GEMM kernel on the adapter rows, K split over workgroups.  Nothing orders
    // the two products, so when the backbone product runs on the large tiles both go out as one launch.
    const int splits = oa_splits(T, r);
    int64_t kps = (n + splits - 1) / splits;
    kps = (kps + 127) / 128 * 128;
    GemmArgs h;
    h.a = xq; h.lda = n; h.a_fmt = 0;
    h.b = wq + m * n; h.ldb = n; h.b_is_kn = 0;
    h.M = T; h.N = r; h.K = n;
    h.sa = s_x; h.sb = s_w;
    h.c0 = part; h.ldc0 = r; h.c0_is_f32 = 1; h.n_split = r;
    h.c1 = nullptr; h.ldc1 = 0; h.amax1 = nullptr;
    h.splits = splits; h.k_per_split = kps;
    if (gemm_fwd_pair_supported(g, h)) {
        e = launch_gemm_fwd_pair(g, h, st);
    } else {
        e = launch_gemm(g, st);
        if (e == hipSuccess) e = launch_gemm(h, st);
    }
    if (e != hipSuccess) return FALQON_ERR_HIP;
    e = launch_sum_partials_bf16(part, splits, T * r, static_cast<uint16_t*>(o_a),
                                 reinterpret_cast<uint32_t*>(amax_oa), st);
    return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

falqon_status falqon_melded_bwd(const void* dy, const uint8_t* wq, const float* s_w,
                                const void* o_a, const float* amax_oa,
                                int64_t T, int64_t n, int64_t m, int64_t r,
                                uint8_t* dyq, float* s_dy, void* dx, falqon_dtype dxt,
                                float* d_b, float* delta_buf, float lr, double* row_scores,
                                void* ws, size_t ws_bytes, void* stream)
{
    if (dxt != FALQON_BF16 && dxt != FALQON_F32) return FALQON_ERR_ENUM;
    if (row_scores && !delta_buf) return FALQON_ERR_NULL;
    if (row_scores && (reinterpret_cast<uintptr_t>(row_scores) & 7u)) return FALQON_ERR_ALIGN;
    if (bad_layer_shape(T, n, m, r)) return FALQON_ERR_SHAPE;
    if (!dy || !wq || !s_w || !o_a || !amax_oa || !dyq || !s_dy || !d_b) return FALQON_ERR_NULL;   // dx may be NULL
    if (misaligned(dy) || misaligned(wq) || misaligned(o_a) || misaligned(dyq) || (dx && misaligned(dx)) ||
        misaligned(d_b) || (delta_buf && misaligned(delta_buf)))
        return FALQON_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(s_w) & 3u) || (reinterpret_cast<uintptr_t>(s_dy) & 3u) ||
        (reinterpret_cast<uintptr_t>(amax_oa) & 3u))
        return FALQON_ERR_ALIGN;
    const WsLayout L = ws_layout(T, n, m, r);
    if (!ws || ws_bytes < L.total) return FALQON_ERR_WORKSPACE;
    if (misaligned(ws)) return FALQON_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* w8 = static_cast<uint8_t*>(ws);

    // dy~, s_dy <- Q_E5M2(dy).  When the adapter gradient is formed by side jobs of the dX tiles, the
    // cast pass also casts the saved O_A to E4M3 (its maximum is known from the forward pass).
    const DbTailPlan pd = dx ? plan_db_tail(T, n, m, r) : DbTailPlan{false, 0};
    SideCast sc{static_cast<const uint16_t*>(o_a), amax_oa, w8 + L.oa_codes, T * r};
    hipError_t e = launch_quantize(dy, FALQON_BF16, T, m, m, FALQON_E5M2, nullptr, dyq, m, s_dy, nullptr,
                                   reinterpret_cast<float*>(w8 + L.amax_partials), nullptr, st, pd.use ? &sc : nullptr);
    if (e != hipSuccess) return FALQON_ERR_HIP;

    // dX <- dy~ W~ / (s_dy s_w): the backbone rows of the concatenated weight, read as [K = m, N = n]
    GemmArgs g;
    g.a = dyq; g.lda = m; g.a_fmt = 1;
    g.b = wq; g.ldb = n; g.b_is_kn = 1;
    g.M = T; g.N = n; g.K = m;
    g.sa = s_dy; g.sb = s_w;
    g.c0 = dx; g.ldc0 = n; g.c0_is_f32 = (dxt == FALQON_F32); g.n_split = n;
    g.c1 = nullptr; g.ldc1 = 0; g.amax1 = nullptr;
    // dB <- dy~^T O_A~ / (s_dy s_oa);  DeltaBuffer += -lr dB.  Its partial pass reads only dy~ and
    // O_A, so nothing orders it against the dX product: on the large tiles both go out as one launch.
    const DbArgs d = make_db_args(dyq, o_a, amax_oa, T, m, r, reinterpret_cast<float*>(w8 + L.db_partials),
                                  pd.use ? pd.groups : db_splits(T, m));
    if (pd.use) {
        TailArgs t;
        t.side = w8 + L.oa_codes; t.r = r; t.partial = d.partial; t.splits = 0; t.steps_per_split = 0; t.row_parts = 1;
        e = launch_gemm_dx_tail(g, t, st);
    } else if (!dx) {
        e = launch_db_partial(d, st);                      // the layer's input needs no gradient
    } else if (gemm_dx_db_pair_supported(g)) {
        e = launch_gemm_dx_db_pair(g, d, st);
    } else {
        e = launch_gemm(g, st);
        if (e == hipSuccess) e = launch_db_partial(d, st);
    }
    if (e != hipSuccess) return FALQON_ERR_HIP;
    e = launch_db_reduce(d, s_dy, d_b, delta_buf, lr, st, row_scores);
    return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

falqon_status falqon_db_bf16(const uint8_t* dyq, const float* s_dy, const void* o_a,
                             int64_t T, int64_t m, int64_t r, float* d_b, float* delta_buf, float lr,
                             void* ws, size_t ws_bytes, void* stream)
{
    if (bad_layer_shape(T, 16, m, r)) return FALQON_ERR_SHAPE;
    if (!dyq || !s_dy || !o_a || !d_b) return FALQON_ERR_NULL;
    if (misaligned(dyq) || misaligned(o_a) || misaligned(d_b) || (delta_buf && misaligned(delta_buf)) ||
        (reinterpret_cast<uintptr_t>(s_dy) & 3u))
        return FALQON_ERR_ALIGN;
    const WsLayout L = ws_layout(T, 16, m, r);
    if (!ws || ws_bytes < L.total) return FALQON_ERR_WORKSPACE;
    if (misaligned(ws)) return FALQON_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const DbArgs d = make_db_args(dyq, o_a, nullptr, T, m, r,
                                  reinterpret_cast<float*>(static_cast<uint8_t*>(ws) + L.db_partials), db_splits(T, m));
    hipError_t e = launch_db_wide_partial(d, st);
    if (e == hipSuccess) e = launch_db_reduce(d, s_dy, d_b, delta_buf, lr, st);
    return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

falqon_status falqon_da(const uint8_t* dyq, const float* s_dy, const uint8_t* btq, const float* s_b,
                        const uint8_t* xq, const float* s_x, int64_t T, int64_t n, int64_t m, int64_t r,
                        void* g, float* amax_g, float* d_at, void* ws, size_t ws_bytes, void* stream)
{
    if (bad_layer_shape(T, n, m, r)) return FALQON_ERR_SHAPE;
    if (!dyq || !s_dy || !btq || !s_b || !xq || !s_x || !g || !amax_g || !d_at) return FALQON_ERR_NULL;
    if (misaligned(dyq) || misaligned(btq) || misaligned(xq) || misaligned(g) || misaligned(d_at) ||
        (reinterpret_cast<uintptr_t>(s_dy) & 3u) || (reinterpret_cast<uintptr_t>(s_b) & 3u) ||
        (reinterpret_cast<uintptr_t>(s_x) & 3u) || (reinterpret_cast<uintptr_t>(amax_g) & 3u))
        return FALQON_ERR_ALIGN;
    // the second product has the layer's input width in the place of its output width
    const WsLayout L = ws_layout(T, m, n, r);
    if (!ws || ws_bytes < L.total) return FALQON_ERR_WORKSPACE;
    if (misaligned(ws)) return FALQON_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* w8 = static_cast<uint8_t*>(ws);

    // G <- dy~ B~ / (s_dy s_b): a product with only r output columns, so K is split over workgroups;
    // fp32 partials, then the pass that adds them in order, rounds to bf16 and takes the maximum
    hipError_t e = launch_zero_word(reinterpret_cast<uint32_t*>(amax_g), st);
    if (e != hipSuccess) return FALQON_ERR_HIP;
    const int splits = oa_splits(T, r);
    int64_t kps = (m + splits - 1) / splits;
    kps = (kps + 127) / 128 * 128;
    float* part = reinterpret_cast<float*>(w8 + L.oa_partials);
    GemmArgs h;
    h.a = dyq; h.lda = m; h.a_fmt = 1;
    h.b = btq; h.ldb = m; h.b_is_kn = 0;
    h.M = T; h.N = r; h.K = m;
    h.sa = s_dy; h.sb = s_b;
    h.c0 = part; h.ldc0 = r; h.c0_is_f32 = 1; h.n_split = r;
    h.c1 = nullptr; h.ldc1 = 0; h.amax1 = nullptr;
    h.splits = splits; h.k_per_split = kps;
    e = launch_gemm(h, st);
    if (e != hipSuccess) return FALQON_ERR_HIP;
    e = launch_sum_partials_bf16(part, splits, T * r, static_cast<uint16_t*>(g), reinterpret_cast<uint32_t*>(amax_g), st);
    if (e != hipSuccess) return FALQON_ERR_HIP;
    // dA^T <- x~^T G / s_x on the bf16 matrix cores (E4M3 is exact in bf16), token splits, ordered sum
    const DbArgs d = make_db_args(xq, g, nullptr, T, n, r, reinterpret_cast<float*>(w8 + L.db_partials), db_splits(T, n));
    e = launch_db_wide_partial(d, st, false);
    if (e == hipSuccess) e = launch_db_reduce(d, s_x, d_at, nullptr, 0.0f, st);
    return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

falqon_status falqon_proxy_update(float* delta_buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                                  int32_t* idx_out, int clear_selected, const double* row_scores,
                                  void* ws, size_t ws_bytes, void* stream)
{
    if (bad_layer_shape(1, n, m, r) || m > 65536 || k < 1 || k > m) return FALQON_ERR_SHAPE;
    if (!delta_buf || !wq || !idx_out) return FALQON_ERR_NULL;
    if (misaligned(delta_buf) || misaligned(wq) || (reinterpret_cast<uintptr_t>(idx_out) & 3u) ||
        (reinterpret_cast<uintptr_t>(row_scores) & 7u))
        return FALQON_ERR_ALIGN;
    const WsLayout L = ws_layout(1, n, m, r);
    if (!ws || ws_bytes < L.db_partials) return FALQON_ERR_WORKSPACE;
    if (misaligned(ws)) return FALQON_ERR_ALIGN;
    uint8_t* w8 = static_cast<uint8_t*>(ws);
    hipError_t e = launch_proxy_update(delta_buf, wq, n, m, r, k, idx_out, clear_selected,
                                       reinterpret_cast<double*>(w8 + L.scores), row_scores,
                                       reinterpret_cast<float*>(w8 + L.delta_sel), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

falqon_status falqon_proxy_update_static(float* delta_buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                                         int32_t* idx_out, int clear_selected, void* stream)
{
    if (bad_layer_shape(1, n, m, r) || m > 65536 || k < 1 || k > m) return FALQON_ERR_SHAPE;
    if (m > kStaticMaxRows || k * r > kStaticMaxSelected) return FALQON_ERR_LIMIT;
    if (!delta_buf || !wq || !idx_out) return FALQON_ERR_NULL;
    if (misaligned(delta_buf) || misaligned(wq) || (reinterpret_cast<uintptr_t>(idx_out) & 3u))
        return FALQON_ERR_ALIGN;
    hipError_t e = launch_proxy_update_static(delta_buf, wq, n, m, r, k, idx_out, clear_selected,
                                              static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

falqon_status falqon_fp8_gemm(const uint8_t* a, falqon_fmt a_fmt, const uint8_t* b, int b_is_kn,
                              int64_t M, int64_t N, int64_t K, const float* s_a, const float* s_b,
                              void* c, falqon_dtype ct,
                              const uint8_t* side, int64_t r, void* side_ws, size_t side_ws_bytes, void* stream)
{
    if (a_fmt != FALQON_E4M3 && a_fmt != FALQON_E5M2) return FALQON_ERR_ENUM;
    if (ct != FALQON_BF16 && ct != FALQON_F32) return FALQON_ERR_ENUM;
    if (M < 1 || N < 16 || K < 16 || (N % 16) || (K % 16) || M > (int64_t(1) << 24) || N > (int64_t(1) << 20) ||
        K > (int64_t(1) << 20))
        return FALQON_ERR_SHAPE;
    if (!a || !b || !s_a || !s_b || !c) return FALQON_ERR_NULL;
    if (misaligned(a) || misaligned(b) || misaligned(c)) return FALQON_ERR_ALIGN;
    GemmArgs g;
    g.a = a; g.lda = K; g.a_fmt = a_fmt == FALQON_E5M2 ? 1 : 0;
    g.b = b; g.ldb = b_is_kn ? N : K; g.b_is_kn = b_is_kn ? 1 : 0;
    g.M = M; g.N = N; g.K = K;
    g.sa = s_a; g.sb = s_b;
    g.c0 = c; g.ldc0 = N; g.c0_is_f32 = (ct == FALQON_F32); g.n_split = N;
    g.c1 = nullptr; g.ldc1 = 0; g.amax1 = nullptr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (!side) {
        hipError_t e = launch_gemm(g, st);
        return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
    }
    // The product launch of a melded call: the same product with the adapter's share as a side job.
    // The layer's (n, m) are (K, N) in the forward orientation and (N, K) in the input-gradient one.
    const int64_t n = b_is_kn ? N : K, m = b_is_kn ? K : N;
    if (bad_layer_shape(M, n, m, r)) return FALQON_ERR_SHAPE;
    if ((b_is_kn != 0) != (a_fmt == FALQON_E5M2)) return FALQON_ERR_ENUM;
    if (misaligned(side)) return FALQON_ERR_ALIGN;
    const WsLayout L = ws_layout(M, n, m, r);
    if (!side_ws || side_ws_bytes < L.total) return FALQON_ERR_WORKSPACE;
    if (misaligned(side_ws)) return FALQON_ERR_ALIGN;
    uint8_t* w8 = static_cast<uint8_t*>(side_ws);
    TailArgs t;
    t.side = side; t.r = r; t.splits = 0; t.steps_per_split = 0; t.row_parts = 1;
    hipError_t e;
    if (!b_is_kn) {
        const OaTailPlan po = plan_oa_tail(M, n, m, r);
        const int64_t tile = gemm_tile_n(M, m + r);
        if (!po.use || (m + r + tile - 1) / tile == (m + tile - 1) / tile) return FALQON_ERR_SHAPE;
        t.partial = reinterpret_cast<float*>(w8 + L.oa_partials); t.splits = po.splits; t.steps_per_split = po.steps_per_split;
        t.row_parts = po.row_parts;
        if (po.splits == 0) {                                    // O_A (bf16) instead of partials
            g.c1 = w8 + L.oa_partials; g.ldc1 = r;
        }
        e = launch_gemm_fwd_tail(g, t, st);
    } else {
        const DbTailPlan pd = plan_db_tail(M, n, m, r);
        if (!pd.use) return FALQON_ERR_SHAPE;
        t.partial = reinterpret_cast<float*>(w8 + L.db_partials);
        e = launch_gemm_dx_tail(g, t, st);
    }
    return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

falqon_status falqon_grad_sqnorm(const float* g, int64_t count, double* sum_sq,
                                 void* ws, size_t ws_bytes, void* stream)
{
    if (count < 4 || (count % 4) || count > (int64_t(1) << 40)) return FALQON_ERR_SHAPE;
    if (!g || !sum_sq) return FALQON_ERR_NULL;
    if (misaligned(g) || (reinterpret_cast<uintptr_t>(sum_sq) & 7u)) return FALQON_ERR_ALIGN;
    if (!ws || ws_bytes < 4096) return FALQON_ERR_WORKSPACE;
    if (misaligned(ws)) return FALQON_ERR_ALIGN;
    hipError_t e = launch_grad_sqnorm(g, count, sum_sq, static_cast<double*>(ws), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

falqon_status falqon_adamw_delta(const float* d_b, float* exp_avg, float* exp_avg_sq, float* delta_buf,
                                 int64_t m, int64_t r, int64_t step, double lr, double beta1, double beta2,
                                 double eps, const double* sum_sq, double max_norm, void* stream)
{
    if (m < 16 || r < 16 || (m % 16) || (r % 16) || r > 256 || m > (int64_t(1) << 20)) return FALQON_ERR_SHAPE;
    if (step < 1 || !(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0) || !(eps > 0.0))
        return FALQON_ERR_SHAPE;
    if (sum_sq && !(max_norm > 0.0)) return FALQON_ERR_SHAPE;
    if (!d_b || !exp_avg || !exp_avg_sq || !delta_buf) return FALQON_ERR_NULL;
    if (misaligned(d_b) || misaligned(exp_avg) || misaligned(exp_avg_sq) || misaligned(delta_buf) ||
        (reinterpret_cast<uintptr_t>(sum_sq) & 7u))
        return FALQON_ERR_ALIGN;
    // 1 - beta and the bias corrections in double on the host, handed over as fp32 factors
    AdamFactors f;
    f.beta1 = static_cast<float>(beta1); f.one_minus_beta1 = static_cast<float>(1.0 - beta1);
    f.beta2 = static_cast<float>(beta2); f.one_minus_beta2 = static_cast<float>(1.0 - beta2);
    f.eps = static_cast<float>(eps);
    f.step_size = static_cast<float>(lr / (1.0 - pow(beta1, static_cast<double>(step))));
    f.inv_sqrt_bias2 = static_cast<float>(1.0 / sqrt(1.0 - pow(beta2, static_cast<double>(step))));
    f.max_norm = max_norm;
    hipError_t e = launch_adamw_delta(d_b, exp_avg, exp_avg_sq, delta_buf, m * r, f, sum_sq,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

static bool bad_svd_shape(int64_t m, int64_t n, int64_t r)
{
    return m < 16 || n < 16 || (m % 4) || (n % 4) || r < 16 || r > 120 || (r % 8) || r + 8 > m || r + 8 > n ||
           m > (int64_t(1) << 20) || n > (int64_t(1) << 20);
}

falqon_status falqon_init_residual(const float* w, const uint8_t* wq, const float* s_w, int64_t m, int64_t n,
                                   float* e, void* stream)
{
    if (m < 1 || n < 4 || (n % 4) || m > (int64_t(1) << 20) || n > (int64_t(1) << 20)) return FALQON_ERR_SHAPE;
    if (!w || !wq || !s_w || !e) return FALQON_ERR_NULL;
    if (misaligned(w) || misaligned(wq) || misaligned(e) || (reinterpret_cast<uintptr_t>(s_w) & 3u))
        return FALQON_ERR_ALIGN;
    hipError_t err = launch_init_residual(w, wq, s_w, m * n, e, static_cast<hipStream_t>(stream));
    return err == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

size_t falqon_svd_workspace_bytes(int64_t m, int64_t n, int64_t r)
{
    if (bad_svd_shape(m, n, r)) return 0;
    return svd_layout(m, n, r).total;
}

falqon_status falqon_svd_right_factor(const float* e, int64_t m, int64_t n, int64_t r, const float* omega,
                                      int iters, float* a_out, float* sigma_out, float* bt_out,
                                      void* ws, size_t ws_bytes, void* stream)
{
    if (bad_svd_shape(m, n, r) || iters < 0 || iters > 64) return FALQON_ERR_SHAPE;
    if (!e || !omega || !a_out || !sigma_out) return FALQON_ERR_NULL;
    if (misaligned(e) || misaligned(omega) || misaligned(a_out) || (reinterpret_cast<uintptr_t>(sigma_out) & 3u) ||
        (bt_out && misaligned(bt_out)))
        return FALQON_ERR_ALIGN;
    if (!ws || ws_bytes < svd_layout(m, n, r).total) return FALQON_ERR_WORKSPACE;
    if (misaligned(ws)) return FALQON_ERR_ALIGN;
    hipError_t err = launch_svd_right_factor(e, m, n, r, omega, iters, a_out, sigma_out, bt_out, static_cast<uint8_t*>(ws),
                                             static_cast<hipStream_t>(stream));
    return err == hipSuccess ? FALQON_OK : FALQON_ERR_HIP;
}

}  // extern "C"
