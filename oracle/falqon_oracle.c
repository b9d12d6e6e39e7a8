/*
 * CPU oracle for the melded FP8-LoRA linear layer (FALQON, arXiv 2510.24061).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * layer computes; the GPU library shares no code with it and must never call it.
 * Only the tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Every floating-point result is formed in fp64 unless the paper's method fixes
 * fp32 (the scale, the scaled value handed to the FP8 cast, the proxy buffer).
 * OpenMP only distributes independent output rows over cores; it never changes
 * the order in which any single output is accumulated.
 *
 * Orientation: row-major, tokens first.  The paper writes activations as
 * x in R^{n x d} and O = W x (Background, "Low-rank adaptation"); here
 * X[T,n] holds the same data transposed (T = the paper's d), so O = X W^T.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC (never -ffast-math).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* FP8 formats (Background, "Low-precision floating-point quantization":      */
/* max(E4M3) = 448 and max(E5M2) = 57344 identify the OCP 8-bit formats).     */
/*   fmt 0: E4M3 - 4 exponent bits, bias 7, 3 mantissa bits, no infinity,     */
/*          S.1111.111 is NaN, largest finite 1.75 * 2^8 = 448.               */
/*   fmt 1: E5M2 - 5 exponent bits, bias 15, 2 mantissa bits, IEEE-like       */
/*          (exponent field 31 = Inf/NaN), largest finite 1.75 * 2^15.        */
/* ------------------------------------------------------------------------- */
typedef struct { int mbits; int bias; int emax_field; double maxv; } fmt_desc;

static fmt_desc fmt_of(int fmt)
{
    fmt_desc d;
    if (fmt == 0) { d.mbits = 3; d.bias = 7;  d.emax_field = 15; d.maxv = 448.0; }
    else          { d.mbits = 2; d.bias = 15; d.emax_field = 30; d.maxv = 57344.0; }
    return d;
}

double orc_fp8_max(int fmt) { return fmt_of(fmt).maxv; }

/* Exact value of an FP8 code.  NaN codes decode to NaN, E5M2 Inf to Inf. */
double orc_fp8_decode(uint8_t code, int fmt)
{
    fmt_desc d = fmt_of(fmt);
    int sign = code >> 7;
    int efield = (code & 0x7F) >> d.mbits;
    int mant = code & ((1 << d.mbits) - 1);
    double v;
    if (fmt == 0 && (code & 0x7F) == 0x7F) v = NAN;
    else if (fmt == 1 && efield == 31) v = mant ? NAN : INFINITY;
    else if (efield == 0) v = ldexp((double)mant, 1 - d.bias - d.mbits);           /* subnormal */
    else v = ldexp((double)((1 << d.mbits) + mant), efield - d.bias - d.mbits);    /* normal */
    return sign ? -v : v;
}

/*
 * Round-to-nearest cast of an fp32 value to FP8 (the rounding bracket of the
 * paper's quantization equation).  Ties go to the even mantissa; magnitudes
 * above the format's largest finite value saturate to it; subnormals are kept;
 * the sign of zero is kept.  NaN maps to the format's NaN.
 */
uint8_t orc_fp8_encode(float v, int fmt)
{
    fmt_desc d = fmt_of(fmt);
    uint8_t sign = signbit(v) ? 0x80 : 0x00;
    double a = fabs((double)v);
    if (isnan(v)) return (uint8_t)(sign | (fmt == 0 ? 0x7F : 0x7E));
    uint8_t maxcode = (uint8_t)((d.emax_field << d.mbits) | (fmt == 0 ? 0x6 : 0x3));
    if (a >= d.maxv) return (uint8_t)(sign | maxcode);
    if (a == 0.0) return sign;
    int e;                      /* a = f * 2^e with f in [0.5, 1)  =>  floor(log2 a) = e - 1 */
    (void)frexp(a, &e);
    int ex = e - 1;
    int emin = 1 - d.bias;      /* exponent of the smallest normal; subnormals share its spacing */
    if (ex < emin) ex = emin;
    /* spacing of representable values in this binade is 2^(ex - mbits) */
    double q = ldexp(a, d.mbits - ex);          /* exact: power-of-two scaling */
    double rq = nearbyint(q);                   /* default rounding mode: nearest, ties to even */
    /* rq in [0, 2^(mbits+1)]; code arithmetic carries into the exponent field on its own:
       normal:    field = ex + bias, mantissa = rq - 2^mbits
       subnormal: field = 0,         mantissa = rq  (rq = 2^mbits is the smallest normal) */
    int code = ((ex + d.bias - 1) << d.mbits) + (int)rq;
    return (uint8_t)(sign | (uint8_t)code);
}

void orc_fp8_encode_array(const float* v, int64_t count, int fmt, uint8_t* out)
{
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) out[i] = orc_fp8_encode(v[i], fmt);
}

void orc_fp8_decode_array(const uint8_t* c, int64_t count, int fmt, double* out)
{
    for (int64_t i = 0; i < count; ++i) out[i] = orc_fp8_decode(c[i], fmt);
}

/* Round an fp64 value to the nearest bfloat16 (ties to even), returned as fp32. */
float orc_round_bf16(double v)
{
    if (isnan(v) || isinf(v) || v == 0.0) return (float)v;
    int e;
    (void)frexp(fabs(v), &e);
    int ex = e - 1;
    if (ex < -126) ex = -126;                   /* bf16 shares fp32's exponent range */
    double q = ldexp(v, 7 - ex);                /* 8 significant bits */
    double r = ldexp(nearbyint(q), ex - 7);
    return (float)r;                            /* exact: at most 8 significant bits */
}

void orc_round_bf16_array(const double* v, int64_t count, float* out)
{
    for (int64_t i = 0; i < count; ++i) out[i] = orc_round_bf16(v[i]);
}

/* ------------------------------------------------------------------------- */
/* Per-tensor quantizer Q_fp8 (quantization equation of the Background        */
/* section; with a supplied scale it is the A-integration equation, where A   */
/* is cast with the backbone's scale).                                        */
/* The printed scale max|X|/max(FP8) cannot be meant literally (it would map  */
/* the largest entry to amax^2/448 while the rescale divides by the scale);   */
/* the scale multiplies up to the format's range: s = max(FP8)/max|X|.        */
/*   amax  = max |x|            (exact)                                       */
/*   s     = fmt_max / max(amax, 1e-12f)     one fp32 division                */
/*   code  = encode( fl32(x * s) )           one fp32 multiply, then the cast */
/* ------------------------------------------------------------------------- */
void orc_quantize(const float* x, int64_t count, int fmt, const float* scale_in,
                  uint8_t* q, float* scale_out, float* amax_out)
{
    float amax = 0.0f;
    for (int64_t i = 0; i < count; ++i) {
        float a = fabsf(x[i]);
        if (a > amax) amax = a;
    }
    float s;
    if (scale_in) s = *scale_in;
    else {
        float den = amax > 1e-12f ? amax : 1e-12f;
        s = (float)orc_fp8_max(fmt) / den;
    }
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        volatile float scaled = x[i] * s;       /* volatile: force the fp32 rounding of the product */
        q[i] = orc_fp8_encode(scaled, fmt);
    }
    if (scale_out) *scale_out = s;
    if (amax_out) *amax_out = amax;
}

/* ------------------------------------------------------------------------- */
/* Melded forward (merged-output equation; forward loop of the gradient-      */
/* computation algorithm):                                                    */
/*   O_merged[t,c] = ( sum_j dec(xq[t,j]) * dec(wq[c,j]) ) / (s_w * s_x)      */
/* for c in [0, m+r); columns [0,m) are the layer output, [m,m+r) are O_A.    */
/* wq is the concatenated weight [(m+r), n]: m backbone rows, then r rows of  */
/* the adapter A cast with the backbone's scale.                              */
/* row_sel / col_sel (nullable) restrict the computed outputs to chosen       */
/* tokens / merged columns: out is [n_rows, n_cols] over the selected sets.   */
/* ------------------------------------------------------------------------- */
void orc_melded_fwd(const uint8_t* xq, const uint8_t* wq, float s_w, float s_x,
                    int64_t T, int64_t n, int64_t m, int64_t r,
                    const int64_t* row_sel, int64_t n_rows,
                    const int64_t* col_sel, int64_t n_cols,
                    double* out)
{
    double lut[256];
    for (int c = 0; c < 256; ++c) lut[c] = orc_fp8_decode((uint8_t)c, 0);
    if (!row_sel) n_rows = T;
    if (!col_sel) n_cols = m + r;
    double denom = (double)s_w * (double)s_x;
    #pragma omp parallel for schedule(dynamic, 1)
    for (int64_t a = 0; a < n_rows; ++a) {
        int64_t t = row_sel ? row_sel[a] : a;
        const uint8_t* xr = xq + t * n;
        for (int64_t b = 0; b < n_cols; ++b) {
            int64_t c = col_sel ? col_sel[b] : b;
            const uint8_t* wr = wq + c * n;
            double acc = 0.0;
            for (int64_t j = 0; j < n; ++j) acc += lut[xr[j]] * lut[wr[j]];
            out[a * n_cols + b] = acc / denom;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Input gradient (FP8 matmul-and-rescale equation applied to the backward    */
/* pass; gradients are E5M2, weights E4M3 - "Detailed experimental settings").*/
/* Only the m backbone rows of the concatenated weight take part: nothing     */
/* downstream consumes O_A, so no gradient flows through the adapter rows.    */
/*   dX[t,j] = ( sum_{i<m} dec5(dyq[t,i]) * dec4(wq[i,j]) ) / (s_dy * s_w)    */
/* ------------------------------------------------------------------------- */
void orc_dx(const uint8_t* dyq, const uint8_t* wq, float s_dy, float s_w,
            int64_t T, int64_t n, int64_t m,
            const int64_t* row_sel, int64_t n_rows,
            const int64_t* col_sel, int64_t n_cols,
            double* out)
{
    double lut4[256], lut5[256];
    for (int c = 0; c < 256; ++c) { lut4[c] = orc_fp8_decode((uint8_t)c, 0); lut5[c] = orc_fp8_decode((uint8_t)c, 1); }
    if (!row_sel) n_rows = T;
    if (!col_sel) n_cols = n;
    double denom = (double)s_dy * (double)s_w;
    /* Tokens are independent.  Within a token the loop runs i outermost so the weight is
       read along its rows; each output still adds its terms in ascending i. */
    #pragma omp parallel for schedule(dynamic, 1)
    for (int64_t a = 0; a < n_rows; ++a) {
        int64_t t = row_sel ? row_sel[a] : a;
        const uint8_t* gr = dyq + t * m;
        double* acc = out + a * n_cols;
        for (int64_t b = 0; b < n_cols; ++b) acc[b] = 0.0;
        for (int64_t i = 0; i < m; ++i) {
            double g = lut5[gr[i]];
            const uint8_t* wr = wq + i * n;
            for (int64_t b = 0; b < n_cols; ++b) {
                int64_t j = col_sel ? col_sel[b] : b;
                acc[b] += g * lut4[wr[j]];
            }
        }
        for (int64_t b = 0; b < n_cols; ++b) acc[b] = acc[b] / denom;
    }
}

/* ------------------------------------------------------------------------- */
/* Adapter gradient in its reformulated shape dL/dB = dL/dO (A x)^T           */
/* (modified LoRA-backward equation; first line of the backward loop).        */
/* The saved O_A (bf16 values, given here as fp32) is cast to E4M3 with its   */
/* own per-tensor scale s_oa = 448 / max(amax_oa, 1e-12f):                    */
/*   oaq[t,p] = encode( fl32(o_a[t,p] * s_oa) )                               */
/*   dB[i,p]  = ( sum_t dec5(dyq[t,i]) * dec4(oaq[t,p]) ) / (s_dy * s_oa)     */
/* row_sel (nullable) restricts the computed rows i of dB.                    */
/* ------------------------------------------------------------------------- */
void orc_db(const uint8_t* dyq, float s_dy, const float* o_a, float amax_oa,
            int64_t T, int64_t m, int64_t r,
            const int64_t* row_sel, int64_t n_rows,
            double* out, uint8_t* oaq_out /* nullable [T,r] */, float* s_oa_out /* nullable */)
{
    double lut4[256], lut5[256];
    for (int c = 0; c < 256; ++c) { lut4[c] = orc_fp8_decode((uint8_t)c, 0); lut5[c] = orc_fp8_decode((uint8_t)c, 1); }
    float den = amax_oa > 1e-12f ? amax_oa : 1e-12f;
    float s_oa = 448.0f / den;
    uint8_t* oaq = (uint8_t*)malloc((size_t)(T * r));
    for (int64_t e = 0; e < T * r; ++e) {
        volatile float scaled = o_a[e] * s_oa;
        oaq[e] = orc_fp8_encode(scaled, 0);
    }
    if (!row_sel) n_rows = m;
    double denom = (double)s_dy * (double)s_oa;
    /* Rows of dB are independent.  For one row the loop runs t outermost so O_A is read
       along its rows; each output still adds its terms in ascending t. */
    #pragma omp parallel for schedule(dynamic, 8)
    for (int64_t a = 0; a < n_rows; ++a) {
        int64_t i = row_sel ? row_sel[a] : a;
        double* acc = out + a * r;
        for (int64_t p = 0; p < r; ++p) acc[p] = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double g = lut5[dyq[t * m + i]];
            const uint8_t* orow = oaq + t * r;
            for (int64_t p = 0; p < r; ++p) acc[p] += g * lut4[orow[p]];
        }
        for (int64_t p = 0; p < r; ++p) acc[p] = acc[p] / denom;
    }
    if (oaq_out) memcpy(oaq_out, oaq, (size_t)(T * r));
    if (s_oa_out) *s_oa_out = s_oa;
    free(oaq);
}

/* ------------------------------------------------------------------------- */
/* The same adapter gradient with the saved O_A kept at its 16-bit precision  */
/* (the paper does not say in which precision the operands of this small      */
/* product are held; E5M2 values are exactly representable in bf16, so only   */
/* the cast of O_A to E4M3 is dropped):                                       */
/*   dB[i,p] = ( sum_t dec5(dyq[t,i]) * o_a[t,p] ) / s_dy                     */
/* ------------------------------------------------------------------------- */
void orc_db_wide(const uint8_t* dyq, float s_dy, const float* o_a,
                 int64_t T, int64_t m, int64_t r,
                 const int64_t* row_sel, int64_t n_rows, double* out)
{
    double lut5[256];
    for (int c = 0; c < 256; ++c) lut5[c] = orc_fp8_decode((uint8_t)c, 1);
    if (!row_sel) n_rows = m;
    #pragma omp parallel for schedule(dynamic, 8)
    for (int64_t a = 0; a < n_rows; ++a) {
        int64_t i = row_sel ? row_sel[a] : a;
        double* acc = out + a * r;
        for (int64_t p = 0; p < r; ++p) acc[p] = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double g = lut5[dyq[t * m + i]];
            const float* orow = o_a + t * r;
            for (int64_t p = 0; p < r; ++p) acc[p] += g * (double)orow[p];
        }
        for (int64_t p = 0; p < r; ++p) acc[p] = acc[p] / (double)s_dy;
    }
}

/* ------------------------------------------------------------------------- */
/* Proxy buffer accumulation: stand-in for "DeltaBuffer <- Optimizer(dB, lr)" */
/* of the backward-and-update algorithm, as plain SGD on the change of B:     */
/*   buf[i,p] = fl32( buf[i,p] + fl32( -lr * fl32(dB[i,p]) ) )                */
/* The buffer accumulates across steps (it "stores only changes of B").       */
/* ------------------------------------------------------------------------- */
void orc_delta_accumulate(float* buf, const double* d_b, int64_t count, float lr)
{
    for (int64_t e = 0; e < count; ++e) {
        float g = (float)d_b[e];
        volatile float step = -lr * g;
        volatile float sum = buf[e] + step;
        buf[e] = sum;
    }
}

/* ------------------------------------------------------------------------- */
/* Optimizer step into the proxy buffer: "DeltaBuffer <- Optimizer(dB, lr)"   */
/* of the backward-and-update algorithm with the optimizer the experiments    */
/* name (AdamW, maximum gradient norm 0.3; "Detailed experimental settings"). */
/* B itself is never stored, only its change, so the decoupled weight decay   */
/* has nothing to act on and is taken as zero (the default of the recipe the  */
/* paper follows); the step is then Adam with bias correction:                */
/*   g   = c * dB                       c = clip coefficient (below)          */
/*   m   = b1*m + (1-b1)*g              v = b2*v + (1-b2)*g*g                 */
/*   dlt = -(lr / (1-b1^t)) * m / ( sqrt(v)/sqrt(1-b2^t) + eps )              */
/*   buf = buf + dlt                                                          */
/* Each element is formed in fp64 from the fp32 state and rounded to fp32     */
/* when stored (moments and buffer are fp32 arrays).                          */
/* ------------------------------------------------------------------------- */
void orc_adamw_delta(const float* d_b, float* exp_avg, float* exp_avg_sq, float* buf, int64_t count,
                     int64_t step, double lr, double beta1, double beta2, double eps, double clip_coef)
{
    double bias1 = 1.0 - pow(beta1, (double)step);
    double bias2 = 1.0 - pow(beta2, (double)step);
    for (int64_t e = 0; e < count; ++e) {
        double g = clip_coef * (double)d_b[e];
        double m = beta1 * (double)exp_avg[e] + (1.0 - beta1) * g;
        double v = beta2 * (double)exp_avg_sq[e] + (1.0 - beta2) * g * g;
        double denom = sqrt(v) / sqrt(bias2) + eps;
        double dlt = -(lr / bias1) * m / denom;
        exp_avg[e] = (float)m;
        exp_avg_sq[e] = (float)v;
        buf[e] = (float)((double)buf[e] + dlt);
    }
}

/* Sum of squares of a gradient tensor in fp64, elements in index order: one   */
/* term of the global gradient norm.                                           */
double orc_sum_squares(const float* g, int64_t count)
{
    double s = 0.0;
    for (int64_t e = 0; e < count; ++e) s += (double)g[e] * (double)g[e];
    return s;
}

/* Clip coefficient of gradient-norm clipping over all adapter gradients:      */
/* total = sqrt(sum of squares of every gradient), c = min(1, max/(total+1e-6)) */
double orc_clip_coef(double sum_squares, double max_norm)
{
    double c = max_norm / (sqrt(sum_squares) + 1e-6);
    return c < 1.0 ? c : 1.0;
}

/* ------------------------------------------------------------------------- */
/* Row-wise proxy update (update equation; last two lines of the backward-    */
/* and-update algorithm):                                                     */
/*   score_i = sum_p |buf[i,p]|            fp64, p ascending                  */
/*   idx     = the k rows of largest score; larger score first, equal scores  */
/*             by smaller row index (plain full sort)                         */
/*   for i in idx, every column j:                                            */
/*       acc = dec(wq[i,j]);  for p ascending: acc += buf[i,p]*dec(wq[m+p,j]) */
/*       wq[i,j] = encode( (float)acc )                                       */
/* The adapter used is the one stored in rows [m, m+r) of the concatenated    */
/* weight; both terms then carry the backbone's scale, which cancels, so the  */
/* sum is formed directly on code values and the scale stays fixed.           */
/* With clear_selected the folded rows of the buffer are reset to +0.         */
/* ------------------------------------------------------------------------- */
typedef struct { double score; int64_t row; } score_row;

static int cmp_score_row(const void* pa, const void* pb)
{
    const score_row* a = (const score_row*)pa;
    const score_row* b = (const score_row*)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    if (a->row < b->row) return -1;
    if (a->row > b->row) return 1;
    return 0;
}

void orc_row_scores(const float* buf, int64_t m, int64_t r, double* score)
{
    for (int64_t i = 0; i < m; ++i) {
        double s = 0.0;
        for (int64_t p = 0; p < r; ++p) s += fabs((double)buf[i * r + p]);
        score[i] = s;
    }
}

void orc_topk_rows(const double* score, int64_t m, int64_t k, int32_t* idx)
{
    score_row* all = (score_row*)malloc(sizeof(score_row) * (size_t)m);
    for (int64_t i = 0; i < m; ++i) { all[i].score = score[i]; all[i].row = i; }
    qsort(all, (size_t)m, sizeof(score_row), cmp_score_row);
    for (int64_t a = 0; a < k; ++a) idx[a] = (int32_t)all[a].row;
    free(all);
}

void orc_proxy_update(float* buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                      int32_t* idx, int clear_selected)
{
    double lut4[256];
    for (int c = 0; c < 256; ++c) lut4[c] = orc_fp8_decode((uint8_t)c, 0);
    double* score = (double*)malloc(sizeof(double) * (size_t)m);
    orc_row_scores(buf, m, r, score);
    orc_topk_rows(score, m, k, idx);
    free(score);
    const uint8_t* aq = wq + m * n;             /* adapter rows of the concatenated weight */
    for (int64_t a = 0; a < k; ++a) {
        int64_t i = idx[a];
        for (int64_t j = 0; j < n; ++j) {
            double acc = lut4[wq[i * n + j]];
            for (int64_t p = 0; p < r; ++p) acc += (double)buf[i * r + p] * lut4[aq[p * n + j]];
            wq[i * n + j] = orc_fp8_encode((float)acc, 0);
        }
    }
    if (clear_selected)
        for (int64_t a = 0; a < k; ++a)
            for (int64_t p = 0; p < r; ++p) buf[(int64_t)idx[a] * r + p] = 0.0f;
}

/* ------------------------------------------------------------------------- */
/* Initialization, residual step (initialization algorithm; the               */
/* reformulation equation fixes the sign): the quantization error the adapter */
/* is read out of,                                                            */
/*   E[i,j] = fl32( fl32( dec(wq[i,j]) / s_w ) - w[i,j] )  =  DQ(W~) - W      */
/* so that DQ(W~) = W + E and the rank-r part of E plays the role of B A.     */
/* ------------------------------------------------------------------------- */
void orc_init_residual(const float* w, const uint8_t* wq, float s_w, int64_t count, float* e)
{
    for (int64_t i = 0; i < count; ++i) {
        volatile float dq = (float)orc_fp8_decode(wq[i], 0) / s_w;
        volatile float d = dq - w[i];
        e[i] = d;
    }
}

/* ------------------------------------------------------------------------- */
/* Variant in which the adapter factor A is trained too (appendix "Ablation   */
/* on matrix A update").  LoRA backward equation:                             */
/*   dL/dA = B^T dL/dO x^T                                                    */
/* In the layer's orientation (tokens first) that is two products:            */
/*   G[t,p]     = sum_i dY[t,i] B[i,p]          (the gradient at A x)         */
/*   dA^T[j,p]  = sum_t x[t,j] G[t,p]                                         */
/* with the FP8 operands the layer already has: dy~ (E5M2, scale s_dy),       */
/* x~ (E4M3, scale s_x), and B^T cast to E4M3 with a scale s_b of its own,    */
/* stored as bt[p][i].  G is kept at 16-bit precision, like the saved O_A     */
/* (the paper does not fix the precision of these small products):            */
/*   G[t,p]    = bf16( ( sum_i dec5(dyq[t,i]) dec4(btq[p,i]) ) / (s_dy s_b) ) */
/*   dAt[j,p]  = ( sum_t dec4(xq[t,j]) G[t,p] ) / s_x                         */
/* ------------------------------------------------------------------------- */
void orc_adapter_inner_grad(const uint8_t* dyq, float s_dy, const uint8_t* btq, float s_b,
                            int64_t T, int64_t m, int64_t r, float* g_out)
{
    double lut5[256], lut4[256];
    for (int c = 0; c < 256; ++c) { lut5[c] = orc_fp8_decode((uint8_t)c, 1); lut4[c] = orc_fp8_decode((uint8_t)c, 0); }
    const double denom = (double)s_dy * (double)s_b;
    #pragma omp parallel for schedule(dynamic, 8)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t p = 0; p < r; ++p) {
            double acc = 0.0;
            for (int64_t i = 0; i < m; ++i) acc += lut5[dyq[t * m + i]] * lut4[btq[p * m + i]];
            g_out[t * r + p] = orc_round_bf16(acc / denom);
        }
    }
}

void orc_da(const uint8_t* xq, float s_x, const float* g, int64_t T, int64_t n, int64_t r,
            const int64_t* row_sel, int64_t n_rows, double* out)
{
    double lut4[256];
    for (int c = 0; c < 256; ++c) lut4[c] = orc_fp8_decode((uint8_t)c, 0);
    if (!row_sel) n_rows = n;
    #pragma omp parallel for schedule(dynamic, 8)
    for (int64_t a = 0; a < n_rows; ++a) {
        int64_t j = row_sel ? row_sel[a] : a;
        double* acc = out + a * r;
        for (int64_t p = 0; p < r; ++p) acc[p] = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double xv = lut4[xq[t * n + j]];
            const float* grow = g + t * r;
            for (int64_t p = 0; p < r; ++p) acc[p] += xv * (double)grow[p];
        }
        for (int64_t p = 0; p < r; ++p) acc[p] = acc[p] / (double)s_x;
    }
}

int orc_num_threads(void)
{
    int nthreads = 1;
    #pragma omp parallel
    {
        #pragma omp master
        {
#ifdef _OPENMP
            extern int omp_get_num_threads(void);
            nthreads = omp_get_num_threads();
#endif
        }
    }
    return nthreads;
}
