// Internal declarations shared by the translation units of libfalqon (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "falqon.h"

namespace falqon {

// ---- workspace -------------------------------------------------------------------------
// One layout serves all four calls; the regions never overlap so a forward, a backward
// and an update of the same layer may share one workspace when run in stream order.
constexpr int kMaxAmaxBlocks = 1024;   // per-block partial maxima written by the amax pass
constexpr int kDbSplitMax = 32;        // upper bound on the token splits of the dB contraction

struct WsLayout {
    size_t amax_partials;   // float[kMaxAmaxBlocks]
    size_t scores;          // double[m + ceil(m / 64)]: row scores of the proxy buffer and their block maxima
    size_t delta_sel;       // float[m][r]: buffer rows picked by the proxy update, in rank order
    size_t db_partials;     // float[splits][m][r]
    size_t oa_partials;     // float[splits][T][r]
    size_t oa_codes;        // uint8[T][r]: the saved O_A cast to E4M3 for the adapter gradient
    size_t total;
};
WsLayout ws_layout(int64_t T, int64_t n, int64_t m, int64_t r);
int db_splits(int64_t T, int64_t m);

// ---- quantizer (quantize.hip) ------------------------------------------------------------
// Two launches: per-block partial maxima, then scale + cast.  `zero_word` (nullable) is a
// device word the cast pass clears, used to reset the running maximum of O_A.
// `side` (nullable): a small dense bf16 tensor of `count` elements (a multiple of 16) with a known
// maximum that the cast pass casts to E4M3 along the way, q = cast(x * (448 / max(*amax, 1e-12f))).
struct SideCast { const uint16_t* x; const float* amax; uint8_t* q; int64_t count; };
hipError_t launch_quantize(const void* x, falqon_dtype xt, int64_t rows, int64_t cols, int64_t ld_x,
                           falqon_fmt fmt, const float* scale_in, uint8_t* q, int64_t ld_q,
                           float* scale_out, float* amax_out, float* partials, uint32_t* zero_word,
                           hipStream_t stream, const SideCast* side = nullptr);
// Clears one device word with a kernel (a memset node is not safe inside a captured graph here).
hipError_t launch_zero_word(uint32_t* w, hipStream_t stream);

// ---- FP8 GEMMs (gemm.hip) ----------------------------------------------------------------
// C[M,N] = A[M,K] . op(B) * 1 / (sa * sb), fp32 accumulation on the FP8 matrix cores.
//   b_is_kn = 0: B is [N,K] (K contiguous)  - forward, against the concatenated weight
//   b_is_kn = 1: B is [K,N] (N contiguous)  - input gradient, against the backbone rows
// Columns [0, n_split) go to c0 (ldc0), columns [n_split, N) go to c1 as bf16 (ldc1) and
// their running absolute maximum (after bf16 rounding) is folded into *amax1.
struct GemmArgs {
    const uint8_t* a; int64_t lda; int a_fmt;      // a_fmt: 0 = E4M3, 1 = E5M2
    const uint8_t* b; int64_t ldb; int b_is_kn;    // B is always E4M3
    int64_t M, N, K;
    const float* sa; const float* sb;              // device scalars
    void* c0; int64_t ldc0; int c0_is_f32; int64_t n_split;
    void* c1; int64_t ldc1; uint32_t* amax1;
    int splits = 1; int64_t k_per_split = int64_t(1) << 40;   // split K: c0 becomes [splits][M][ldc0] partials
};
hipError_t launch_gemm(const GemmArgs& g, hipStream_t stream);
int64_t gemm_tile_n(int64_t M, int64_t N);   // width of the output tiles launch_gemm picks for an M x N product
// g (large product, 256x256 tiles) and h (a split-K product on 128x128 tiles) in one launch; both
// [N,K], E4M3.  Results are those of launch_gemm(g) and launch_gemm(h).
bool gemm_fwd_pair_supported(const GemmArgs& g, const GemmArgs& h);
hipError_t launch_gemm_fwd_pair(const GemmArgs& g, const GemmArgs& h, hipStream_t stream);

// What every 256x256 backbone tile does for the adapter besides its own tile (gemm.hip).
//   forward launch:        side = adapter rows A~ [r][K] (row stride g.ldb).
//                          splits > 0: partial[splits][M][r], rescaled; tile columns in sets of
//                          row_parts: set s < splits covers K-steps [s * steps_per_split,
//                          +steps_per_split), each member a part of the token rows.
//                          splits = 0 (row_parts = 0, steps_per_split = rank blocks per wave, 1, 2 or 4):
//                          no partials; the launch writes O_A as bf16 to g.c1 (row stride g.ldc1) and
//                          raises g.amax1 (if not null) to its maximum
//   input-gradient launch: side = O_A codes [T][r] (E4M3, cast by the dy quantizer's cast pass);
//                          partial[groups][m][r], raw sums; splits / steps_per_split unused
struct TailArgs {
    const uint8_t* side; int64_t r; float* partial; int splits; int steps_per_split; int row_parts;
};
struct OaTailPlan { bool use; int splits; int steps_per_split; int row_parts; };
struct DbTailPlan { bool use; int groups; };
OaTailPlan plan_oa_tail(int64_t T, int64_t n, int64_t m, int64_t r);     // forward of a [T,n] x [m+r,n] layer
DbTailPlan plan_db_tail(int64_t T, int64_t n, int64_t m, int64_t r);     // backward of the same layer
hipError_t launch_gemm_fwd_tail(const GemmArgs& g, const TailArgs& t, hipStream_t stream);
hipError_t launch_gemm_dx_tail(const GemmArgs& g, const TailArgs& t, hipStream_t stream);

// ---- O_A from split-K partials (partials.hip) ---------------------------------------------------
// out[count] (bf16) = sum over splits of partial[split][count]; folds max|out| into *amax.
hipError_t launch_sum_partials_bf16(const float* partial, int splits, int64_t count, uint16_t* out, uint32_t* amax,
                                    hipStream_t stream);
int oa_splits(int64_t T, int64_t r);

// ---- adapter gradient (db.hip, db_tile.h) ------------------------------------------------------
// Two passes: fp32 partials per token split, then their ordered sum with the rescale and the
// optional proxy-buffer step.
struct DbArgs {
    const uint8_t* dyq; const uint16_t* o_a; const float* amax_oa;
    int64_t T, m, r, tokens_per_split;
    float* partial;                                                    // [splits][m][r]
    int i_tiles, splits, p_tiles;                                      // grid of the partial pass
};
DbArgs make_db_args(const uint8_t* dyq, const void* o_a, const float* amax_oa, int64_t T, int64_t m, int64_t r,
                    float* partials, int splits);
hipError_t launch_db_partial(const DbArgs& d, hipStream_t stream);
// score (nullable, used only with delta_buf): row scores of the buffer after the step, in the layout
// of row_scores.h (m scores, then one maximum per block of 64 rows).
hipError_t launch_db_reduce(const DbArgs& d, const float* s_dy, float* d_b, float* delta_buf, float lr,
                            hipStream_t stream, double* score = nullptr);
// Variant with O_A kept in bf16 (db_wide.hip): d.amax_oa is not read and may be null, also in the reduce.
// left_e5m2 = false: the codes in d.dyq are E4M3 (the second product of the gradient of A, with x~ on the left).
hipError_t launch_db_wide_partial(const DbArgs& d, hipStream_t stream, bool left_e5m2 = true);
// Input-gradient GEMM g ([K,N] right operand, E5M2 left operand, 256x256 tiles) and the partial pass
// of the adapter gradient in one launch: both read only dy~ (and O_A, the weight).
bool gemm_dx_db_pair_supported(const GemmArgs& g);
hipError_t launch_gemm_dx_db_pair(const GemmArgs& g, const DbArgs& d, hipStream_t stream);

// ---- proxy update (proxy.hip) ----------------------------------------------------------------
// scores: scratch for m + ceil(m / 64) doubles (row_scores.h), written by the score pass; scores_in
// (nullable): such an array already filled by the kernel that wrote the buffer, the score pass is
// skipped.  delta_sel: scratch for k * r floats.
hipError_t launch_proxy_update(float* delta_buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                               int32_t* idx_out, int clear_selected, double* scores, const double* scores_in,
                               float* delta_sel, hipStream_t stream);

// The same update on the library's own static device scratch (no workspace, no allocation).
constexpr int64_t kStaticMaxRows = 16384;          // m
constexpr int64_t kStaticMaxSelected = 65536;      // k * r
hipError_t launch_proxy_update_static(float* delta_buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                                      int32_t* idx_out, int clear_selected, hipStream_t stream);

// ---- initialization (init.hip) -----------------------------------------------------------------
hipError_t launch_init_residual(const float* w, const uint8_t* wq, const float* s_w, int64_t count, float* e,
                                hipStream_t stream);
struct SvdLayout { size_t z, y, h, p, lambda, order, part, total; };   // offsets into the workspace, l = r + 8 vectors
SvdLayout svd_layout(int64_t m, int64_t n, int64_t r);
// bt_out (nullable): the left factor, transposed: B^ = U_r sqrt(S_r) as fp32 [r, m]
hipError_t launch_svd_right_factor(const float* e, int64_t m, int64_t n, int64_t r, const float* omega, int iters,
                                   float* a_out, float* sigma_out, float* bt_out, uint8_t* ws, hipStream_t stream);

// ---- optimizer step into the proxy buffer (optimizer.hip) ------------------------------------
// partials: at least 256 doubles of scratch
hipError_t launch_grad_sqnorm(const float* g, int64_t count, double* sum_sq, double* partials, hipStream_t stream);
struct AdamFactors {
    float beta1, one_minus_beta1, beta2, one_minus_beta2, eps;
    float step_size;         // lr / (1 - beta1^t)
    float inv_sqrt_bias2;    // 1 / sqrt(1 - beta2^t)
    double max_norm;
};
hipError_t launch_adamw_delta(const float* d_b, float* exp_avg, float* exp_avg_sq, float* delta_buf, int64_t count,
                              const AdamFactors& f, const double* sum_sq, hipStream_t stream);

}  // namespace falqon
