// Adapter gradient in its reformulated shape, dL/dB = dL/dO (A x)^T (modified
// LoRA-backward equation; first line of the backward-and-update loop):
//
//   dB[i,p] = ( sum_t value5(dyq[t,i]) * value4(oaq[t,p]) ) / (s_dy * s_oa)
//
// dyq is the E5M2 gradient that the input-gradient GEMM already uses; oaq is the saved
// O_A = A x (bf16) cast to E4M3 inside this kernel's load stage with
// s_oa = 448 / max(amax_oa, 1e-12f), so no separate small-matrix quantize pass exists.
//
// The contraction runs over tokens, the strided dimension of both operands.  Both tiles are
// therefore kept as [token][feature] in LDS and read with ds_read_b64_tr_b8, which returns
// eight consecutive tokens of one feature per lane: the matrix-core operand layout.
// The kernel is bound by the single read of dyq, so tokens are split over many workgroups;
// each split writes an fp32 partial and a second pass adds the partials in a fixed order
// (bitwise reproducible, no floating-point atomics) and applies the proxy-buffer step.
#include "db_tile.h"
#include "row_scores.h"

namespace falqon {
namespace {

using namespace dbt;

__device__ __attribute__((aligned(16))) uint8_t g_zero16[16];

__global__ void __launch_bounds__(kThreads)
db_partial_kernel(const DbArgs d)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t s_tiles[];
    db_partial_tile(d, blockIdx.x, blockIdx.y, blockIdx.z, s_tiles, g_zero16);
}

// buf + fl32(-lr * g): product and sum are rounded separately, as the step is defined.  The
// rounding intrinsics do not stop the compiler from fusing the pair, the pragma does.
__device__ __forceinline__ float buffer_step(float buf, float lr, float g)
{
#pragma clang fp contract(off)
    const float step = -lr * g;
    return buf + step;
}

// dB = (sum of partials, split ascending) / (s_dy * s_oa);  delta_buf += -lr * dB.
// A workgroup owns 64 rows of dB.  With `score` set (only together with delta_buf) it keeps the new
// buffer rows in LDS and leaves their L1 norms and the block's largest norm for the proxy update.
__global__ void __launch_bounds__(kThreads)
db_reduce_kernel(const float* __restrict__ partial, int splits, int64_t m, int r,
                 const float* __restrict__ s_dy, const float* __restrict__ amax_oa,
                 float* __restrict__ d_b, float* delta_buf, float lr, double* __restrict__ score)
{
    extern __shared__ float s_rows[];                                              // 64 x (r + 4) floats when score is set
    const float s_oa_scale = amax_oa ? 448.0f / fmaxf(*amax_oa, 1e-12f) : 1.0f;    // no amax: O_A was not cast
    const float inv = 1.0f / ((*s_dy) * s_oa_scale);
    const int64_t count = m * r;
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kScoreRows;
    const int64_t e0 = row0 * r;
    int64_t e_end = e0 + static_cast<int64_t>(kScoreRows) * r;
    if (e_end > count) e_end = count;
    const int r4 = r / 4, pitch = r + 4;
    constexpr int B = 8, U = 4;                                    // splits per batch, float4 positions per thread and pass
    for (int64_t base = e0 + threadIdx.x * 4; base < e_end; base += static_cast<int64_t>(U) * kThreads * 4) {
        float4 s[U];
        for (int sp0 = 0; sp0 < splits; sp0 += B) {
            float4 v[U][B];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t e = base + static_cast<int64_t>(u) * kThreads * 4;
                const int64_t ee = e < e_end ? e : e0;                   // beyond the block: a valid address, value unused
#pragma unroll
                for (int b = 0; b < B; ++b) {
                    const int sp = sp0 + b < splits ? sp0 + b : splits - 1;
                    v[u][b] = *reinterpret_cast<const float4*>(partial + sp * count + ee);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int b = 0; b < B; ++b) {
                    if (sp0 + b == 0) s[u] = v[u][b];
                    else if (sp0 + b < splits) { s[u].x += v[u][b].x; s[u].y += v[u][b].y; s[u].z += v[u][b].z; s[u].w += v[u][b].w; }
                }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t e = base + static_cast<int64_t>(u) * kThreads * 4;
            if (e >= e_end) continue;
            float4 g = s[u];
            g.x *= inv; g.y *= inv; g.z *= inv; g.w *= inv;
            *reinterpret_cast<float4*>(d_b + e) = g;
            if (delta_buf) {
                float4 d = *reinterpret_cast<const float4*>(delta_buf + e);
                d.x = buffer_step(d.x, lr, g.x);
                d.y = buffer_step(d.y, lr, g.y);
                d.z = buffer_step(d.z, lr, g.z);
                d.w = buffer_step(d.w, lr, g.w);
                *reinterpret_cast<float4*>(delta_buf + e) = d;
                if (score) {
                    const int64_t q4 = (e - e0) / 4;
                    *reinterpret_cast<float4*>(s_rows + (q4 / r4) * pitch + (q4 % r4) * 4) = d;
                }
            }
        }
    }
    if (score) {
        __syncthreads();
        score_rows_from_lds(s_rows, r, row0, m, score);
    }
}

}  // namespace

int db_splits(int64_t T, int64_t m)
{
    const int64_t i_tiles = (m + BI - 1) / BI;
    int64_t splits = (384 + i_tiles - 1) / i_tiles;          // aim at one to two workgroups per CU
    const int64_t max_by_tokens = (T + BT - 1) / BT;
    if (splits > max_by_tokens) splits = max_by_tokens;
    if (splits > kDbSplitMax) splits = kDbSplitMax;
    int p2 = 1;                                              // round down to a power of two
    while (p2 * 2 <= splits) p2 *= 2;
    return p2;
}

DbArgs make_db_args(const uint8_t* dyq, const void* o_a, const float* amax_oa, int64_t T, int64_t m, int64_t r,
                    float* partials, int splits)
{
    DbArgs d;
    d.dyq = dyq; d.o_a = static_cast<const uint16_t*>(o_a); d.amax_oa = amax_oa;
    d.T = T; d.m = m; d.r = r;
    // tokens per split: a multiple of the step so that every split starts on a tile boundary
    int64_t tps = (T + splits - 1) / splits;
    d.tokens_per_split = (tps + BT - 1) / BT * BT;
    d.partial = partials;
    d.i_tiles = static_cast<int>((m + BI - 1) / BI); d.splits = splits; d.p_tiles = static_cast<int>((r + BP - 1) / BP);
    return d;
}

hipError_t launch_db_partial(const DbArgs& d, hipStream_t stream)
{
    const dim3 grid(static_cast<unsigned>(d.i_tiles), static_cast<unsigned>(d.splits), static_cast<unsigned>(d.p_tiles));
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&db_partial_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kDbLdsBytes));
    if (e != hipSuccess) return e;
    db_partial_kernel<<<grid, kThreads, kDbLdsBytes, stream>>>(d);
    return hipGetLastError();
}

hipError_t launch_db_reduce(const DbArgs& d, const float* s_dy, float* d_b, float* delta_buf, float lr,
                            hipStream_t stream, double* score)
{
    if (d.splits < 1) return hipErrorInvalidValue;
    if (!delta_buf) score = nullptr;                              // the scores are those of the buffer the step leaves
    const size_t lds = score ? sizeof(float) * kScoreRows * (static_cast<size_t>(d.r) + 4) : 0;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&db_reduce_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e != hipSuccess) return e;
    }
    db_reduce_kernel<<<static_cast<unsigned>(score_blocks(d.m)), kThreads, lds, stream>>>(
        d.partial, d.splits, d.m, static_cast<int>(d.r), s_dy, d.amax_oa, d_b, delta_buf, lr, score);
    return hipGetLastError();
}

}  // namespace falqon
