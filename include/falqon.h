/*
 * falqon.h - C ABI of the MI355X (gfx950) melded FP8-LoRA linear layer.
 *
 * The layer is the hot path of FALQON (arXiv 2510.24061): an FP8 linear layer whose
 * LoRA adapter is melded into the FP8-quantized backbone weight.  Four operations:
 *
 *   falqon_quantize      per-tensor FP8 quantizer Q_fp8
 *   falqon_melded_fwd    quantize x, one FP8 product against the concatenated weight
 *                        [W~ ; A~], split into the layer output and O_A = A x
 *   falqon_melded_bwd    quantize dY, input gradient dX = dY~ W~, adapter gradient
 *                        dB = dY~^T O_A, optional proxy-buffer step
 *   falqon_proxy_update  row scores of the proxy buffer, top-k rows, requantize-and-
 *                        write of those rows of W~
 * and, between the last two, the optimizer step that fills the proxy buffer
 * (falqon_grad_sqnorm, falqon_adamw_delta) in place of the plain SGD step that
 * falqon_melded_bwd can apply itself.
 *
 * Conventions (all calls)
 *   - Orientation is row-major with tokens first: X[T,n], W~'[(m+r),n], Y[T,m],
 *     O_A[T,r], dY[T,m], dX[T,n], dB[m,r], DeltaBuffer[m,r].  (The paper writes
 *     activations as n x d columns, O = W x; T is its d.)
 *   - Every pointer is a DEVICE pointer unless it is called "host".  Scales and amax
 *     values are device scalars, so no call synchronises with the host.
 *   - Arguments marked "in/out" are outputs of the call's own first step when its source
 *     tensor is given and inputs when that source is NULL: xq and s_x of falqon_melded_fwd
 *     (written by the call's quantizer when x is given; read as they are when x is NULL).
 *   - The caller owns every buffer.  The library allocates nothing and keeps no state
 *     between calls.  `ws` is caller-provided scratch of at least
 *     falqon_workspace_bytes() bytes; its contents are undefined after a call.
 *   - Calls validate their arguments on the host first; on error nothing is launched.
 *     Otherwise they enqueue kernels on `stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and return without waiting.
 *   - Tensors are dense.  Pointers must be 16-byte aligned.  n, m and r must be
 *     multiples of 16, r <= 256, T >= 1.
 *   - FP8 codes are OCP E4M3 (max 448, no infinity) and OCP E5M2 (max 57344): the two
 *     formats the paper fixes through their largest values.  Casts round to nearest,
 *     ties to even, and saturate.  Non-finite inputs never fault; their outputs are
 *     unspecified.
 *   - Re-entrant for distinct buffers and streams.  Two calls that share an output
 *     buffer or a workspace must be ordered by the caller.
 */
#ifndef FALQON_H
#define FALQON_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FALQON_OK = 0,
    FALQON_ERR_NULL = 1,       /* a required pointer is NULL */
    FALQON_ERR_SHAPE = 2,      /* a size is out of range or not a multiple of 16 */
    FALQON_ERR_ALIGN = 3,      /* a pointer is not 16-byte aligned */
    FALQON_ERR_ENUM = 4,       /* unknown format or dtype */
    FALQON_ERR_WORKSPACE = 5,  /* ws is NULL or smaller than falqon_workspace_bytes() */
    FALQON_ERR_HIP = 6,        /* a HIP launch failed */
    FALQON_ERR_LIMIT = 7       /* a size exceeds the fixed scratch of an entry point that takes no workspace */
} falqon_status;

typedef enum { FALQON_E4M3 = 0, FALQON_E5M2 = 1 } falqon_fmt;
typedef enum { FALQON_BF16 = 0, FALQON_F32 = 1 } falqon_dtype;

/* Human-readable name of a status code (host, static storage). */
const char* falqon_status_string(falqon_status s);

/*
 * Scratch bytes any of the calls below needs for a layer of this shape (host function,
 * no device access).  Returns 0 if the shape is invalid.
 */
size_t falqon_workspace_bytes(int64_t T, int64_t n, int64_t m, int64_t r);

/*
 * Per-tensor quantizer (quantization equation of "Low-precision floating-point
 * quantization"; with scale_in it is the A-integration equation, which casts the
 * adapter A with the backbone's scale).
 *
 *   amax = max |x|
 *   s    = fmt_max / max(amax, 1e-12f)      (one fp32 division; the scale multiplies up
 *                                            to the format's range and divides on rescale)
 *   q    = cast_fmt( fl32(x * s) )          (one fp32 multiply, then the cast)
 *
 *   x          in   [rows, cols] of dtype xt, row stride ld_x elements
 *   q          out  [rows, cols] FP8 codes, row stride ld_q bytes
 *   scale_in   in   nullable.  NULL: derive s from amax.  Else use *scale_in as s.
 *   scale_out  out  the scale used
 *   amax_out   out  nullable; max |x|
 * cols, ld_x and ld_q must be multiples of 16.  rows*cols = 0 is allowed (s = fmt_max/1e-12).
 */
falqon_status falqon_quantize(const void* x, falqon_dtype xt, int64_t rows, int64_t cols, int64_t ld_x,
                              falqon_fmt fmt, const float* scale_in,
                              uint8_t* q, int64_t ld_q, float* scale_out, float* amax_out,
                              void* ws, size_t ws_bytes, void* stream);

/*
 * Melded forward (forward loop of the gradient-computation algorithm; merged-output
 * equation):
 *
 *   xq, s_x   = Q_E4M3(x)
 *   O_merged  = xq . wq^T / (s_w * s_x)             [T, m+r], fp32 accumulation
 *   y         = O_merged[:, :m]
 *   o_a       = bf16( O_merged[:, m:] )             saved for the backward pass
 *   amax_oa   = max |o_a|
 *
 *   x        in   bf16 [T, n]; NULL: the first line is skipped and xq, s_x are inputs (layers that
 *                 read the same activation, such as the q, k and v projections, quantize it once)
 *   wq       in   E4M3 [(m+r), n]: m backbone rows, then the r adapter rows cast with s_w
 *   s_w      in   device scalar, the backbone's scale
 *   xq, s_x  in/out  E4M3 [T, n] and its scale: the operands the product is formed from.  Out when
 *                 x is given, in when x is NULL
 *   y        out  [T, m] of dtype yt
 *   o_a      out  bf16 [T, r]
 *   amax_oa  out  device scalar
 */
falqon_status falqon_melded_fwd(const void* x, const uint8_t* wq, const float* s_w,
                                int64_t T, int64_t n, int64_t m, int64_t r,
                                uint8_t* xq, float* s_x, void* y, falqon_dtype yt,
                                void* o_a, float* amax_oa,
                                void* ws, size_t ws_bytes, void* stream);

/*
 * Melded backward (first two lines of the backward-and-update loop, plus the input
 * gradient that an FP8 linear layer owes its predecessor; gradients are E5M2):
 *
 *   dyq, s_dy = Q_E5M2(dy)
 *   dx        = dyq . wq[:m] / (s_dy * s_w)          only the backbone rows take part
 *   s_oa      = 448 / max(amax_oa, 1e-12f);  oaq = cast_E4M3( fl32(o_a * s_oa) )
 *   d_b       = dyq^T . oaq / (s_dy * s_oa)          modified LoRA-backward equation
 *   delta_buf += -lr * d_b                           if delta_buf != NULL (plain SGD as
 *                                                    the optimizer that fills the buffer)
 *   row_scores_i = sum_p |delta_buf[i,p]|            if row_scores != NULL: the first line of
 *                                                    falqon_proxy_update, on the buffer this step leaves
 *
 *   dy         in   bf16 [T, m]
 *   o_a, amax_oa in bf16 [T, r] and device scalar, as falqon_melded_fwd produced them
 *   dyq, s_dy  out  E5M2 [T, m] and its scale
 *   dx         out  [T, n] of dtype dxt; NULL: the input-gradient product is skipped (a layer whose
 *                   input needs no gradient, such as the first projections behind a frozen embedding)
 *   d_b        out  fp32 [m, r]
 *   delta_buf  i/o  nullable fp32 [m, r]
 *   row_scores out  nullable (needs delta_buf); falqon_row_score_bytes(m) bytes, 8-byte aligned.  The
 *                   kernel that writes the buffer has its rows at hand, so it can leave their scores
 *                   for a falqon_proxy_update that follows with the buffer unchanged (one launch less).
 *                   The array's content beyond "valid input of falqon_proxy_update" is internal.
 */
falqon_status falqon_melded_bwd(const void* dy, const uint8_t* wq, const float* s_w,
                                const void* o_a, const float* amax_oa,
                                int64_t T, int64_t n, int64_t m, int64_t r,
                                uint8_t* dyq, float* s_dy, void* dx, falqon_dtype dxt,
                                float* d_b, float* delta_buf, float lr, double* row_scores,
                                void* ws, size_t ws_bytes, void* stream);

/* Bytes of a row-score array for m buffer rows (host function); 0 if m is out of range. */
size_t falqon_row_score_bytes(int64_t m);

/*
 * Row-wise proxy update (update equation; last two lines of the backward-and-update loop):
 *
 *   score_i = sum_p |delta_buf[i,p]|                 fp64, p ascending
 *   idx     = the k rows of largest score, larger first, ties by smaller row index
 *   for i in idx, all j:
 *       acc = value(wq[i,j]);  for p ascending: acc += delta_buf[i,p] * value(wq[m+p,j])   (fp64)
 *       wq[i,j] = cast_E4M3( (float)acc )
 *   if clear_selected: delta_buf[i,:] = +0 for i in idx
 *
 * The adapter is the one stored in rows [m, m+r) of wq, so both terms carry the scale
 * s_w, which cancels and stays fixed.  Rows outside idx and the adapter rows are not
 * written.  1 <= k <= m, m <= 65536.
 *
 *   delta_buf  i/o  fp32 [m, r]
 *   wq         i/o  E4M3 [(m+r), n]
 *   idx_out    out  int32 [k], device
 *   row_scores in   nullable: the array falqon_melded_bwd filled for this very buffer content; the
 *                   scores are then not formed again.  The caller vouches that the buffer has not
 *                   changed since (another backward step, an optimizer step or an update makes the
 *                   array stale); NULL is always correct.
 */
falqon_status falqon_proxy_update(float* delta_buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                                  int32_t* idx_out, int clear_selected, const double* row_scores,
                                  void* ws, size_t ws_bytes, void* stream);

/*
 * falqon_proxy_update for callers that cannot allocate device memory and so have no workspace to
 * pass: code under HIP graph capture, tight loops, harnesses that forbid hipMalloc.  Same
 * arguments (the scores are always formed here), same kernels and bit-identical results; the
 * scratch (row scores with their block maxima, and the staged rows of the selection) lives in a
 * static device array of the library, 386 KiB per GPU, held until the process ends.  The call
 * allocates and frees nothing.
 *
 * Limits: m <= 16384 and k * r <= 65536, else FALQON_ERR_LIMIT and nothing is launched.
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two
 * streams, two threads) race; order them.  The first call on a device looks up the array's
 * address (once per device, kept for the life of the process, guarded by a mutex); make that call
 * outside a graph capture.  Nothing in the array needs clearing between calls: each call writes
 * every score and every staged row it later reads.
 */
falqon_status falqon_proxy_update_static(float* delta_buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                                         int32_t* idx_out, int clear_selected, void* stream);

/*
 * Building block: one FP8 product with rescale, C = A . op(B) / (s_a * s_b), fp32 accumulation.
 * This is the FP8 matmul-and-rescale equation on its own; falqon_melded_fwd and
 * falqon_melded_bwd run the same kernel.  It is exported so that a benchmark can time the
 * product in isolation and can assemble a conventional separate-path FP8 LoRA layer (the
 * comparison the paper draws in its preliminary analysis) from the same kernels.
 *
 *   a      in   FP8 [M, K], K contiguous, format a_fmt
 *   b      in   E4M3; b_is_kn = 0: [N, K] (K contiguous); b_is_kn = 1: [K, N] (N contiguous)
 *   s_a, s_b  in  device scalars
 *   c      out  [M, N] of dtype ct
 * K and N must be multiples of 16.
 *
 * With side != NULL it is the product launch of a melded call, exactly as that call issues it
 * (one launch; what the call adds is the quantizer before it and, where the adapter's product
 * leaves the launch as partial sums, the ordered sum after it): the workgroups of the product
 * also form the adapter's small product, into side_ws.
 *   b_is_kn = 0 (melded forward; a = x~ E4M3 [T, n], b = backbone rows [m, n]):
 *       side = adapter rows A~ [r, n] E4M3; x~ A~^T, finished (bf16) where every tile row has
 *       enough tile columns to share it out (m > 768 and 16 ceil(m / 256) >= r), else fp32 partials over
 *       slices of K
 *   b_is_kn = 1 (melded backward; a = dy~ E5M2 [T, m], b = backbone rows [m, n]):
 *       side = O_A cast to E4M3 [T, r]; partials of dy~^T O_A~ over groups of tokens
 *   side_ws  scratch of at least falqon_workspace_bytes(T, n, m, r) bytes
 * Only for shapes at which the melded calls use this launch (large products, the adapter columns
 * not inside the backbone's last tile column, r <= 64 unless the forward product is finished in
 * the launch); FALQON_ERR_SHAPE otherwise.  What side_ws holds afterwards is internal; the entry
 * exists so that this launch can be timed on its own.
 */
falqon_status falqon_fp8_gemm(const uint8_t* a, falqon_fmt a_fmt, const uint8_t* b, int b_is_kn,
                              int64_t M, int64_t N, int64_t K, const float* s_a, const float* s_b,
                              void* c, falqon_dtype ct,
                              const uint8_t* side, int64_t r, void* side_ws, size_t side_ws_bytes, void* stream);

/*
 * Variant of the adapter gradient in falqon_melded_bwd (modified LoRA-backward equation, first line
 * of the backward-and-update loop) that keeps the saved O_A at its 16-bit precision; the paper does
 * not fix the precision of this small product's operands:
 *   d_b[i,p] = ( sum_t value_E5M2(dyq[t,i]) * o_a[t,p] ) / s_dy          (fp32 accumulation)
 *   delta_buf != NULL:  delta_buf += -lr * d_b
 * E5M2 values are exact in bf16, so nothing is rounded before the accumulation.  dyq and s_dy are
 * the ones falqon_melded_bwd returned; a caller that wants this gradient calls falqon_melded_bwd
 * with delta_buf = NULL and then this function, which overwrites d_b and takes the buffer step.
 *
 *   dyq        in   E5M2 [T, m]
 *   s_dy       in   device scalar
 *   o_a        in   bf16 [T, r]
 *   d_b        out  fp32 [m, r]
 *   delta_buf  i/o  fp32 [m, r], nullable
 *   ws         at least falqon_workspace_bytes(T, 16, m, r)
 * Shapes as for falqon_melded_bwd.
 */
falqon_status falqon_db_bf16(const uint8_t* dyq, const float* s_dy, const void* o_a,
                             int64_t T, int64_t m, int64_t r, float* d_b, float* delta_buf, float lr,
                             void* ws, size_t ws_bytes, void* stream);

/*
 * Variant in which the adapter factor A is trained too (the paper's appendix "Ablation on matrix A
 * update", which reports what forming this gradient costs): the gradient of A from the LoRA
 * backward equation, dL/dA = B^T dL/dO x^T, as two products on the FP8 operands the melded calls
 * leave behind:
 *
 *   g     = bf16( dyq . btq^T / (s_dy * s_b) )     [T, r]  gradient at the inner activation A x
 *   d_at  = xq^T . g / s_x                          [n, r]  = (dL/dA)^T, fp32 accumulation
 *
 * g is kept at 16-bit precision like the saved O_A (the paper does not fix the precision of these
 * small products); FP8 values are exact in bf16, so the second product runs on the bf16 matrix
 * cores with nothing rounded before the accumulation.  B is implicit in the melded weight; a
 * caller that wants this variant keeps B^T from the initialization (falqon_svd_right_factor's
 * bt_out) cast to E4M3 with falqon_quantize.  Applying a change of A to the melded weight is not
 * part of the method as published and not of this library.
 *
 *   dyq, s_dy  in   E5M2 [T, m] and scale, as falqon_melded_bwd returned them
 *   btq, s_b   in   B^T as E4M3 codes [r, m] and its scale
 *   xq, s_x    in   E4M3 [T, n] and scale, as falqon_melded_fwd returned them
 *   g          out  bf16 [T, r];  amax_g  out  device scalar, max |g|
 *   d_at       out  fp32 [n, r]
 *   ws         at least falqon_workspace_bytes(T, m, n, r) bytes (n and m exchanged)
 */
falqon_status falqon_da(const uint8_t* dyq, const float* s_dy, const uint8_t* btq, const float* s_b,
                        const uint8_t* xq, const float* s_x, int64_t T, int64_t n, int64_t m, int64_t r,
                        void* g, float* amax_g, float* d_at, void* ws, size_t ws_bytes, void* stream);

/*
 * Optimizer step into the proxy buffer: "DeltaBuffer <- Optimizer(dL/dB, lr)", the second line of
 * the loop of the paper's backward-and-update algorithm, with the optimizer its experiments name
 * (AdamW with a maximum gradient norm of 0.3; "Detailed experimental settings").  Two calls:
 *
 * falqon_grad_sqnorm adds the sum of squares of one gradient tensor to a device accumulator, in
 * fp64 and in a fixed order (bitwise reproducible).  Called once per layer on a zeroed
 * accumulator it yields the squared global gradient norm that clipping needs.
 *
 *   g        in      fp32 [count], count a multiple of 4
 *   sum_sq   in/out  device double, incremented
 *   ws       scratch of at least 4096 bytes
 *
 * falqon_adamw_delta performs, element by element in fp32,
 *   g = c * dB,  c = min(1, max_norm / (sqrt(*sum_sq) + 1e-6))   (c = 1 when sum_sq is NULL)
 *   exp_avg    = beta1 * exp_avg    + (1 - beta1) * g
 *   exp_avg_sq = beta2 * exp_avg_sq + (1 - beta2) * g * g
 *   delta_buf += -(lr / (1 - beta1^step)) * exp_avg / (sqrt(exp_avg_sq) / sqrt(1 - beta2^step) + eps)
 * B itself is never stored (the buffer holds only its change), so there is no decoupled weight
 * decay term.  Use it with falqon_melded_bwd called with delta_buf = NULL.
 *
 *   d_b         in      fp32 [m, r]
 *   exp_avg, exp_avg_sq  in/out  fp32 [m, r], zero before the first step
 *   delta_buf   in/out  fp32 [m, r]
 *   lr, beta1, beta2, eps, max_norm  host doubles; 1 - beta and the bias corrections are formed in
 *               double on the host and handed to the kernel as fp32 factors
 *   step        1-based count of optimizer steps taken, this one included
 *   sum_sq      in      device double (squared global gradient norm) or NULL for no clipping
 * Errors: FALQON_ERR_SHAPE also for step < 1, betas outside [0, 1), eps <= 0 or max_norm <= 0.
 */
falqon_status falqon_grad_sqnorm(const float* g, int64_t count, double* sum_sq,
                                 void* ws, size_t ws_bytes, void* stream);
falqon_status falqon_adamw_delta(const float* d_b, float* exp_avg, float* exp_avg_sq, float* delta_buf,
                                 int64_t m, int64_t r, int64_t step, double lr, double beta1, double beta2,
                                 double eps, const double* sum_sq, double max_norm, void* stream);

/*
 * Initialization (the paper's initialization algorithm; once per layer, off the hot path):
 *
 *   W~, s_w <- Q(W)                   falqon_quantize
 *   E = DQ(W~) - W                    falqon_init_residual   (the sign the reformulation
 *                                     equation fixes: DQ(W~) = W + E, E ~ B^ A^)
 *   B^, A^ <- SVD(E, r)               falqon_svd_right_factor: A^ = sqrt(S_r) V_r^T; B^ is
 *                                     never needed (it is implicit in W~)
 *   A~ <- cast(A^ * s_w)              falqon_quantize with scale_in = s_w into rows [m, m+r)
 *
 * falqon_init_residual: e[i,j] = fl32( fl32(value(wq[i,j]) / s_w) - w[i,j] ), fp32 [m, n].
 *
 * falqon_svd_right_factor: randomized subspace iteration with l = r + 8 vectors started from the
 * caller's Gaussian matrix omega (fp32 [l, n]) and `iters` rounds of multiplication by E^T E, then a
 * Rayleigh-Ritz step (l x l symmetric eigenproblem in fp64).  a_out (fp32 [r, n]) has orthogonal
 * rows with squared norms sigma_out[i] (the Ritz values, approximations from below of the r
 * largest singular values, in descending order); the sign of each row is arbitrary.  The row space
 * converges to that of the exact truncated SVD at the rate (sigma_{l+1} / sigma_r)^(2 iters + 1).
 * bt_out (nullable, fp32 [r, m]): the other factor, transposed, B^ = U_r sqrt(S_r) with the same
 * signs, so that bt_out^T a_out approximates the rank-r part of E (only the A-update variant,
 * falqon_da, needs it).
 * 16 <= r <= 120, r a multiple of 8; m, n multiples of 4; ws of falqon_svd_workspace_bytes(m, n, r).
 */
falqon_status falqon_init_residual(const float* w, const uint8_t* wq, const float* s_w, int64_t m, int64_t n,
                                   float* e, void* stream);
size_t falqon_svd_workspace_bytes(int64_t m, int64_t n, int64_t r);
falqon_status falqon_svd_right_factor(const float* e, int64_t m, int64_t n, int64_t r, const float* omega,
                                      int iters, float* a_out, float* sigma_out, float* bt_out,
                                      void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FALQON_H */
