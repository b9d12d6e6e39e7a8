// Initialization (the paper's initialization algorithm): the quantization residual
//   E = DQ(W~) - W            (its residual step, with the sign the reformulation equation fixes)
// and the right factor of its rank-r truncated SVD,  A^ = sqrt(S_r) V_r^T  (its decomposition step),
// which the caller then casts with the backbone's scale (its last step, falqon_quantize with scale_in).
//
// This runs once per layer, before training; it is off the hot path.  The SVD is a randomized
// subspace iteration (the paper only says "SVD"; a truncated factor is all it needs):
//   Z0 = orth(Omega)                         l = r + 8 rows of length n, Omega Gaussian (caller's);
//                                            orth = Cholesky QR applied twice
//   repeat q times:  Y = orth(Z E^T);  Z = orth(Y E)
//   Y = Z E^T;  H = Y Y^T (l x l, fp64);  H = P diag(lambda) P^T  (cyclic Jacobi, fp64)
//   A^[i,:] = lambda_i^(1/4) * sum_c P[c,i] Z[c,:]      for the r largest lambda_i = sigma_i^2
// Products with E accumulate in fp32 (matrix cores, slices of the contraction added in order);
// everything l x l (Gram matrices, Cholesky factors, the eigenproblem) is fp64.
#include "falqon_internal.h"

namespace falqon {
namespace {

constexpr int kThreads = 256;

__global__ void __launch_bounds__(kThreads)
init_residual_kernel(const float* __restrict__ w, const uint8_t* __restrict__ wq, const float* __restrict__ s_w,
                     int64_t count, float* __restrict__ e)
{
    const float s = *s_w;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads * 4;
    for (int64_t i = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4; i < count; i += stride) {
        const float4 wv = *reinterpret_cast<const float4*>(w + i);
        const uint32_t c = *reinterpret_cast<const uint32_t*>(wq + i);
        float4 o;
        // IEEE division and subtraction, unfused, as the definition has them
        o.x = __fsub_rn(__fdiv_rn(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(c), 0), s), wv.x);
        o.y = __fsub_rn(__fdiv_rn(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(c), 1), s), wv.y);
        o.z = __fsub_rn(__fdiv_rn(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(c), 2), s), wv.z);
        o.w = __fsub_rn(__fdiv_rn(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(c), 3), s), wv.w);
        *reinterpret_cast<float4*>(e + i) = o;
    }
}

__global__ void __launch_bounds__(kThreads)
copy_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t count)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < count; i += stride) dst[i] = src[i];
}

constexpr int kMaxL = 128;                 // vectors in the subspace (r + 8 <= 128)
constexpr int kMaxSlices = 16;             // slices of the contracted dimension in the two products

typedef float v16f __attribute__((ext_vector_type(16)));

// The two products with E run on the fp32 matrix cores (v_mfma_f32_32x32x2_f32), operands loaded
// straight from memory into the instruction's layout: lane t supplies row (t % 32) of its
// operand and depth index (t / 32).  A contraction does not care in which order its terms are
// taken as long as both operands agree, so depth index h of four consecutive instructions stands
// for four consecutive memory elements 4 h .. 4 h + 3 of an eight-element step: one 16-byte load
// per lane and operand where the operand is contiguous along the contracted dimension.
// The accumulator of (first, second) operand holds, in lane t, column (t % 32) = the second
// operand's row, and in register v the first operand's row 8 (v / 4) + 4 (t / 32) + v % 4.
// One wave owns 32 rows (or columns) of E and all l <= 32 NBV vectors over one slice of the
// contracted dimension; the slices' results are added in order by sum_slices_kernel.

// part[s][c][i] = sum over columns j of slice s of Z[c][j] E[i][j]
template <int NBV>
__global__ void __launch_bounds__(kThreads)
apply_e_kernel(const float* __restrict__ e, int64_t m, int64_t n, const float* __restrict__ z, int l,
               float* __restrict__ part, int64_t per_slice)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, h = lane >> 5;
    const int64_t i0 = (static_cast<int64_t>(blockIdx.x) * (kThreads / 64) + wave) * 32;
    if (i0 >= m) return;                                             // (no barrier in this kernel)
    const int64_t j_begin = static_cast<int64_t>(blockIdx.y) * per_slice;
    const int64_t j_end = j_begin + per_slice < n ? j_begin + per_slice : n;
    const int64_t row = i0 + (lane & 31);
    const float* const erow = e + (row < m ? row : m - 1) * n;
    v16f acc[NBV];
#pragma unroll
    for (int b = 0; b < NBV; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.0f;
    const float4 zero = make_float4(0.0f, 0.0f, 0.0f, 0.0f);

    for (int64_t j0 = j_begin; j0 < j_end; j0 += 8) {
        const int64_t jj = j0 + 4 * h;                               // n and per_slice are multiples of 4 and 8
        const bool in = jj < j_end;
        const float4 ev = (in && row < m) ? *reinterpret_cast<const float4*>(erow + jj) : zero;
#pragma unroll
        for (int b = 0; b < NBV; ++b) {
            const int c = b * 32 + (lane & 31);
            const float4 zv = (in && c < l) ? *reinterpret_cast<const float4*>(z + static_cast<int64_t>(c) * n + jj) : zero;
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(zv.x, ev.x, acc[b], 0, 0, 0);
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(zv.y, ev.y, acc[b], 0, 0, 0);
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(zv.z, ev.z, acc[b], 0, 0, 0);
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(zv.w, ev.w, acc[b], 0, 0, 0);
        }
    }
    if (row >= m) return;
    float* const out = part + static_cast<int64_t>(blockIdx.y) * l * m;
#pragma unroll
    for (int b = 0; b < NBV; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int c = b * 32 + 8 * (v / 4) + 4 * h + v % 4;
            if (c < l) out[static_cast<int64_t>(c) * m + row] = acc[b][v];
        }
}

// part[s][c][j] = sum over rows i of slice s of Y[c][i] E[i][j]
template <int NBV>
__global__ void __launch_bounds__(kThreads)
apply_et_kernel(const float* __restrict__ e, int64_t m, int64_t n, const float* __restrict__ y, int l,
                float* __restrict__ part, int64_t per_slice)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, h = lane >> 5;
    const int64_t j0 = (static_cast<int64_t>(blockIdx.x) * (kThreads / 64) + wave) * 32;
    if (j0 >= n) return;                                             // (no barrier in this kernel)
    const int64_t i_begin = static_cast<int64_t>(blockIdx.y) * per_slice;
    const int64_t i_end = i_begin + per_slice < m ? i_begin + per_slice : m;
    const int64_t col = j0 + (lane & 31);
    const float* const ecol = e + (col < n ? col : n - 1);
    v16f acc[NBV];
#pragma unroll
    for (int b = 0; b < NBV; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.0f;
    const float4 zero = make_float4(0.0f, 0.0f, 0.0f, 0.0f);

    for (int64_t i0 = i_begin; i0 < i_end; i0 += 8) {
        const int64_t ii = i0 + 4 * h;                               // m and per_slice are multiples of 4 and 8
        const bool in = ii < i_end;
        float ev[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) ev[t] = (in && col < n) ? ecol[(ii + t) * n] : 0.0f;
#pragma unroll
        for (int b = 0; b < NBV; ++b) {
            const int c = b * 32 + (lane & 31);
            const float4 yv = (in && c < l) ? *reinterpret_cast<const float4*>(y + static_cast<int64_t>(c) * m + ii) : zero;
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(yv.x, ev[0], acc[b], 0, 0, 0);
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(yv.y, ev[1], acc[b], 0, 0, 0);
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(yv.z, ev[2], acc[b], 0, 0, 0);
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(yv.w, ev[3], acc[b], 0, 0, 0);
        }
    }
    if (col >= n) return;
    float* const out = part + static_cast<int64_t>(blockIdx.y) * l * n;
#pragma unroll
    for (int b = 0; b < NBV; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int c = b * 32 + 8 * (v / 4) + 4 * h + v % 4;
            if (c < l) out[static_cast<int64_t>(c) * n + col] = acc[b][v];
        }
}

// out[i] = part[0][i] + part[1][i] + ... in that order
__global__ void __launch_bounds__(kThreads)
sum_slices_kernel(const float* __restrict__ part, int slices, int64_t count, float* __restrict__ out)
{
    const int64_t i = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4;
    if (i >= count) return;                                          // count is a multiple of 4
    float4 s = *reinterpret_cast<const float4*>(part + i);
    for (int k = 1; k < slices; ++k) {
        const float4 v = *reinterpret_cast<const float4*>(part + static_cast<int64_t>(k) * count + i);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    *reinterpret_cast<float4*>(out + i) = s;
}

// Orthonormalisation of the l rows of V[l][len] by Cholesky QR, applied twice: G = V V^T (fp64,
// gram_kernel), G = L L^T, V <- L^-1 V by forward substitution.  Everything of size len runs over
// the whole chip; only the l x l factorisation is one workgroup.  The second application brings the
// rows to orthonormal at the precision they are stored in whenever cond(V) < 1e8, which a product
// with E of a set of orthonormal vectors is far from reaching.  A row whose pivot is not positive
// (a vector in the span of the earlier ones) is set to zero.
//
// Right-looking factorisation in LDS.  Output: the strict lower triangle of L, and on the diagonal
// the reciprocal of the pivot (0 for a dropped row).
__global__ void __launch_bounds__(kThreads)
cholesky_kernel(const double* __restrict__ g, int l, double* __restrict__ lfac)
{
    extern __shared__ double s_l[];                                   // [l][l]
    for (int q = threadIdx.x; q < l * l; q += kThreads) s_l[q] = g[q];
    __syncthreads();
    const double tiny = 1e-28 * fmax(s_l[0], 1e-300);
    for (int c = 0; c < l; ++c) {
        const double d = s_l[c * l + c];
        const bool dead = !(d > tiny);
        const double rinv = dead ? 0.0 : 1.0 / sqrt(d);
        __syncthreads();                                              // everyone has read the pivot
        for (int k = c + threadIdx.x; k < l; k += kThreads)
            s_l[k * l + c] = (k == c) ? rinv : s_l[k * l + c] * rinv;
        __syncthreads();
        const int rem = l - 1 - c;                                    // trailing block, lower half only
        for (int q = threadIdx.x; q < rem * rem; q += kThreads) {
            const int k = c + 1 + q / rem, j = c + 1 + q % rem;
            if (j <= k) s_l[k * l + j] -= s_l[k * l + c] * s_l[j * l + c];
        }
        __syncthreads();
    }
    for (int q = threadIdx.x; q < l * l; q += kThreads) lfac[q] = (q % l <= q / l) ? s_l[q] : 0.0;
}

// V <- L^-1 V in place: one lane per column of V, rows solved in order; the column lives in LDS.
__global__ void __launch_bounds__(64)
solve_lower_kernel(float* __restrict__ v, int l, int64_t len, const double* __restrict__ lfac)
{
    __shared__ float s_q[kMaxL][64];
    const int tj = threadIdx.x;
    const int64_t j = static_cast<int64_t>(blockIdx.x) * 64 + tj;
    if (j >= len) return;                                             // no barrier below: a lane only touches its own column
    for (int c = 0; c < l; ++c) s_q[c][tj] = v[static_cast<int64_t>(c) * len + j];
    for (int c = 0; c < l; ++c) {
        const double* row = lfac + static_cast<int64_t>(c) * l;
        double acc = static_cast<double>(s_q[c][tj]);
        for (int p = 0; p < c; ++p) acc -= row[p] * static_cast<double>(s_q[p][tj]);
        const float q = static_cast<float>(acc * row[c]);
        s_q[c][tj] = q;
        v[static_cast<int64_t>(c) * len + j] = q;
    }
}

// H[a][b] = sum_i Y[a][i] Y[b][i] in fp64; grid (l, l)
__global__ void __launch_bounds__(kThreads)
gram_kernel(const float* __restrict__ y, int l, int64_t m, double* __restrict__ h)
{
    __shared__ double s_red[kThreads / 64];
    const float* ya = y + static_cast<int64_t>(blockIdx.x) * m;
    const float* yb = y + static_cast<int64_t>(blockIdx.y) * m;
    double d = 0.0;
    for (int64_t i = threadIdx.x; i < m; i += kThreads) d += static_cast<double>(ya[i]) * static_cast<double>(yb[i]);
    for (int off = 32; off > 0; off >>= 1) d += __shfl_xor(d, off, 64);
    if ((threadIdx.x & 63) == 0) s_red[threadIdx.x >> 6] = d;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int w = 0; w < kThreads / 64; ++w) t += s_red[w];
        h[static_cast<int64_t>(blockIdx.x) * l + blockIdx.y] = t;
    }
}

// Symmetric eigen-decomposition of H (l x l, l even, fp64) by two-sided Jacobi with the round-robin
// ordering: each round rotates l/2 disjoint index pairs at once.  One workgroup; H lives in LDS,
// the eigenvectors P (columns) beside it where both fit (P_IN_LDS, l <= 96: a round then touches no
// memory), in global memory otherwise.  Stops after the first sweep without a rotation, or after
// `sweeps`.  On exit lambda[i] = H[i][i] and order[k] is the
// index of the k-th largest eigenvalue.
// 1024 threads: a round is three short LDS-bound phases between barriers, the more lanes the shorter
constexpr int kJacobiThreads = 1024;

template <bool P_IN_LDS>
__global__ void __launch_bounds__(kJacobiThreads)
jacobi_eig_kernel(const double* __restrict__ h_in, int l, double* __restrict__ p, double* __restrict__ lambda,
                  int* __restrict__ order, int sweeps)
{
    extern __shared__ double s_h[];                                   // [l][l], (P [l][l],) then c[l/2], s[l/2], pairs
    double* const s_p = P_IN_LDS ? s_h + l * l : p;                   // the eigenvectors while they are rotated
    double* const s_c = s_h + (P_IN_LDS ? 2 : 1) * l * l;
    double* const s_s = s_c + l / 2;
    int* const s_pp = reinterpret_cast<int*>(s_s + l / 2);            // pairs of this round: p[k], q[k]
    int* const s_rot = s_pp + l;                                      // rotations taken in this sweep
    for (int q = threadIdx.x; q < l * l; q += kJacobiThreads) {
        s_h[q] = h_in[q];
        s_p[q] = (q / l == q % l) ? 1.0 : 0.0;
    }
    __syncthreads();
    const int half = l / 2;
    // round-robin ordering: position 0 keeps index 0, positions 1 .. l-1 rotate by one per round
    auto at = [&](int pos, int round) { return pos == 0 ? 0 : (pos - 1 + (l - 1) - round % (l - 1)) % (l - 1) + 1; };
    for (int sweep = 0; sweep < sweeps; ++sweep) {
        if (threadIdx.x == 0) *s_rot = 0;
        __syncthreads();
        for (int round = 0; round < l - 1; ++round) {
            // pairs (positions k and l-1-k) and their rotations from the current 2x2 blocks
            for (int k = threadIdx.x; k < half; k += kJacobiThreads) {
                int a = at(k, round), b = at(l - 1 - k, round);
                if (a > b) { const int t = a; a = b; b = t; }
                s_pp[2 * k] = a; s_pp[2 * k + 1] = b;
                const double haa = s_h[a * l + a], hbb = s_h[b * l + b], hab = s_h[a * l + b];
                double c = 1.0, s = 0.0;
                // an off-diagonal entry below the rounding level of its two diagonal ones is left alone
                if (fabs(hab) > 1e-300 && fabs(hab) > 1e-16 * sqrt(fabs(haa * hbb))) {
                    atomicAdd(s_rot, 1);
                    const double tau = (hbb - haa) / (2.0 * hab);
                    const double t = (tau >= 0.0 ? 1.0 : -1.0) / (fabs(tau) + sqrt(1.0 + tau * tau));
                    c = 1.0 / sqrt(1.0 + t * t);
                    s = t * c;
                }
                s_c[k] = c; s_s[k] = s;
            }
            __syncthreads();
            // columns: H <- H J, P <- P J   (pairs are disjoint, so all of them at once)
            for (int q = threadIdx.x; q < half * l; q += kJacobiThreads) {
                const int k = q / l, i = q - k * l;
                const int a = s_pp[2 * k], b = s_pp[2 * k + 1];
                const double c = s_c[k], s = s_s[k];
                const double ha = s_h[i * l + a], hb = s_h[i * l + b];
                s_h[i * l + a] = c * ha - s * hb;
                s_h[i * l + b] = s * ha + c * hb;
                const double pa = s_p[i * l + a], pb = s_p[i * l + b];
                s_p[i * l + a] = c * pa - s * pb;
                s_p[i * l + b] = s * pa + c * pb;
            }
            __syncthreads();
            // rows: H <- J^T H
            for (int q = threadIdx.x; q < half * l; q += kJacobiThreads) {
                const int k = q / l, j = q - k * l;
                const int a = s_pp[2 * k], b = s_pp[2 * k + 1];
                const double c = s_c[k], s = s_s[k];
                const double ha = s_h[a * l + j], hb = s_h[b * l + j];
                s_h[a * l + j] = c * ha - s * hb;
                s_h[b * l + j] = s * ha + c * hb;
            }
            __syncthreads();
        }
        if (*s_rot == 0) break;                                       // converged (same value in every lane)
        __syncthreads();
    }
    if (P_IN_LDS)
        for (int q = threadIdx.x; q < l * l; q += kJacobiThreads) p[q] = s_p[q];
    for (int i = threadIdx.x; i < l; i += kJacobiThreads) lambda[i] = s_h[i * l + i];
    __syncthreads();
    // rank by eigenvalue, larger first, equal values by smaller index
    for (int i = threadIdx.x; i < l; i += kJacobiThreads) {
        const double li = s_h[i * l + i];
        int rank = 0;
        for (int j = 0; j < l; ++j) {
            const double lj = s_h[j * l + j];
            rank += (lj > li || (lj == li && j < i)) ? 1 : 0;
        }
        order[rank] = i;
    }
}

// A^[k][j] = lambda_k^(1/4) * sum_c P[c][order[k]] Z[c][j];  sigma[k] = sqrt(lambda_k)
__global__ void __launch_bounds__(kThreads)
rotate_kernel(const float* __restrict__ z, int l, int64_t n, const double* __restrict__ p,
              const double* __restrict__ lambda, const int* __restrict__ order, int r,
              float* __restrict__ a_out, float* __restrict__ sigma_out, int inverse_scale)
{
    const int k = blockIdx.y;
    const int col = order[k];
    const double lam = lambda[col] > 0.0 ? lambda[col] : 0.0;
    // right factor: z holds unit vectors, row k becomes sqrt(sigma_k) v_k.  Left factor (inverse_scale):
    // z holds E v (length sigma_k u_k after the rotation), row k becomes sqrt(sigma_k) u_k.
    const double root = sqrt(sqrt(lam));
    const double scale = inverse_scale ? (root > 0.0 ? 1.0 / root : 0.0) : root;
    const int64_t j = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (j < n) {
        double acc = 0.0;
        for (int c = 0; c < l; ++c) acc += p[c * l + col] * static_cast<double>(z[static_cast<int64_t>(c) * n + j]);
        a_out[static_cast<int64_t>(k) * n + j] = static_cast<float>(scale * acc);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && sigma_out) sigma_out[k] = static_cast<float>(sqrt(lam));
}

}  // namespace

hipError_t launch_init_residual(const float* w, const uint8_t* wq, const float* s_w, int64_t count, float* e,
                                hipStream_t stream)
{
    int64_t blocks = (count / 4 + kThreads - 1) / kThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > 8192) blocks = 8192;
    init_residual_kernel<<<static_cast<unsigned>(blocks), kThreads, 0, stream>>>(w, wq, s_w, count, e);
    return hipGetLastError();
}

SvdLayout svd_layout(int64_t m, int64_t n, int64_t r)
{
    const size_t l = static_cast<size_t>(r) + 8;
    auto up = [](size_t v) { return (v + 255) / 256 * 256; };
    SvdLayout L;
    size_t off = 0;
    L.z = off;      off = up(off + sizeof(float) * l * static_cast<size_t>(n));
    L.y = off;      off = up(off + sizeof(float) * l * static_cast<size_t>(m));
    L.h = off;      off = up(off + sizeof(double) * l * l);
    L.p = off;      off = up(off + sizeof(double) * l * l);
    L.lambda = off; off = up(off + sizeof(double) * l);
    L.order = off;  off = up(off + sizeof(int) * l);
    L.part = off;   off = up(off + sizeof(float) * kMaxSlices * l * static_cast<size_t>(m > n ? m : n));
    L.total = off;
    return L;
}

// rows of v[l][len] <- orthonormal (Cholesky QR twice); h and lfac are l x l fp64 scratch
static hipError_t orthonormalize_rows(float* v, int l, int64_t len, double* h, double* lfac, hipStream_t stream)
{
    const size_t lds = sizeof(double) * static_cast<size_t>(l) * l;
    hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void*>(&cholesky_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (err != hipSuccess) return err;
    for (int pass = 0; pass < 2; ++pass) {
        gram_kernel<<<dim3(l, l), kThreads, 0, stream>>>(v, l, len, h);
        cholesky_kernel<<<1, kThreads, lds, stream>>>(h, l, lfac);
        solve_lower_kernel<<<static_cast<unsigned>((len + 63) / 64), 64, 0, stream>>>(v, l, len, lfac);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
    }
    return hipSuccess;
}

hipError_t launch_svd_right_factor(const float* e, int64_t m, int64_t n, int64_t r, const float* omega, int iters,
                                   float* a_out, float* sigma_out, float* bt_out, uint8_t* ws, hipStream_t stream)
{
    const int l = static_cast<int>(r) + 8;
    const SvdLayout L = svd_layout(m, n, r);
    float* z = reinterpret_cast<float*>(ws + L.z);
    float* y = reinterpret_cast<float*>(ws + L.y);
    double* h = reinterpret_cast<double*>(ws + L.h);
    double* p = reinterpret_cast<double*>(ws + L.p);
    double* lambda = reinterpret_cast<double*>(ws + L.lambda);
    int* order = reinterpret_cast<int*>(ws + L.order);
    float* part = reinterpret_cast<float*>(ws + L.part);
    // Y[l][m] = Z E^T (transposed == false) or Z[l][n] = Y E: slices of the contracted dimension so that about
    // 2048 waves stream E, then the ordered sum of the slices
    auto product = [&](bool transposed, const float* vec, float* out) -> hipError_t {
        const int64_t rows = transposed ? n : m, depth = transposed ? m : n;
        const int64_t blocks = (rows + 31) / 32;
        int64_t slices = 2048 / blocks;
        if (slices < 1) slices = 1;
        if (slices > kMaxSlices) slices = kMaxSlices;
        int64_t per = ((depth + slices - 1) / slices + 7) / 8 * 8;
        slices = (depth + per - 1) / per;
        const dim3 grid(static_cast<unsigned>((blocks + kThreads / 64 - 1) / (kThreads / 64)), static_cast<unsigned>(slices));
        float* dst = slices > 1 ? part : out;
        const int nbv = (l + 31) / 32;
#define FQ_PRODUCT(NBV)                                                                                   \
        if (transposed) apply_et_kernel<NBV><<<grid, kThreads, 0, stream>>>(e, m, n, vec, l, dst, per);   \
        else apply_e_kernel<NBV><<<grid, kThreads, 0, stream>>>(e, m, n, vec, l, dst, per)
        if (nbv == 1) { FQ_PRODUCT(1); } else if (nbv == 2) { FQ_PRODUCT(2); } else if (nbv == 3) { FQ_PRODUCT(3); } else { FQ_PRODUCT(4); }
#undef FQ_PRODUCT
        hipError_t pe = hipGetLastError();
        if (pe != hipSuccess || slices == 1) return pe;
        const int64_t count = static_cast<int64_t>(l) * rows;          // a multiple of 4 (m and n are)
        sum_slices_kernel<<<static_cast<unsigned>((count / 4 + kThreads - 1) / kThreads), kThreads, 0, stream>>>(
            part, static_cast<int>(slices), count, out);
        return hipGetLastError();
    };
    hipError_t err;
#define FQ_CHECK_LAUNCH() do { err = hipGetLastError(); if (err != hipSuccess) return err; } while (0)
    copy_kernel<<<1024, kThreads, 0, stream>>>(omega, z, static_cast<int64_t>(l) * n);
    FQ_CHECK_LAUNCH();
    err = orthonormalize_rows(z, l, n, h, p, stream);
    if (err != hipSuccess) return err;
    for (int it = 0; it < iters; ++it) {
        err = product(false, z, y);
        if (err != hipSuccess) return err;
        err = orthonormalize_rows(y, l, m, h, p, stream);
        if (err != hipSuccess) return err;
        err = product(true, y, z);
        if (err != hipSuccess) return err;
        err = orthonormalize_rows(z, l, n, h, p, stream);
        if (err != hipSuccess) return err;
    }
    err = product(false, z, y);
    if (err != hipSuccess) return err;
    gram_kernel<<<dim3(l, l), kThreads, 0, stream>>>(y, l, m, h);
    FQ_CHECK_LAUNCH();
    // H, and the eigenvectors too while both fit the LDS (l <= 96; rotated in memory otherwise)
    const size_t mat = sizeof(double) * static_cast<size_t>(l) * l;
    const size_t rest = sizeof(double) * static_cast<size_t>(l) + sizeof(int) * (static_cast<size_t>(l) + 4);
    const bool p_in_lds = 2 * mat + rest <= 160 * 1024;
    const size_t lds = (p_in_lds ? 2 : 1) * mat + rest;
    const void* jacobi = p_in_lds ? reinterpret_cast<const void*>(&jacobi_eig_kernel<true>)
                                  : reinterpret_cast<const void*>(&jacobi_eig_kernel<false>);
    err = hipFuncSetAttribute(jacobi, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
    if (err != hipSuccess) return err;
    if (p_in_lds) jacobi_eig_kernel<true><<<1, kJacobiThreads, lds, stream>>>(h, l, p, lambda, order, 14);
    else jacobi_eig_kernel<false><<<1, kJacobiThreads, lds, stream>>>(h, l, p, lambda, order, 14);
    FQ_CHECK_LAUNCH();
    rotate_kernel<<<dim3(static_cast<unsigned>((n + kThreads - 1) / kThreads), static_cast<unsigned>(r)), kThreads, 0,
                    stream>>>(z, l, n, p, lambda, order, static_cast<int>(r), a_out, sigma_out, 0);
    FQ_CHECK_LAUNCH();
    if (bt_out) {
        // y still holds E z^T: its rotation by the same eigenvectors is sigma_k u_k, the left singular vectors
        rotate_kernel<<<dim3(static_cast<unsigned>((m + kThreads - 1) / kThreads), static_cast<unsigned>(r)), kThreads, 0,
                        stream>>>(y, l, m, p, lambda, order, static_cast<int>(r), bt_out, nullptr, 1);
        FQ_CHECK_LAUNCH();
    }
#undef FQ_CHECK_LAUNCH
    return hipSuccess;
}

}  // namespace falqon
