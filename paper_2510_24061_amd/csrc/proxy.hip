// Row-wise proxy update (update equation; last two lines of the backward-and-update loop):
//   k = topk( sum_j |dB_ij| ; k ),   W~[k] = W~[k] + DeltaBuffer[k] A
//
// Three small launches, all latency bound (the update touches k of m rows):
//   1. row scores: L1 norm of every buffer row, fp64, columns ascending
//   2. selection: the rank of a row is the number of rows that beat it (larger score, or
//      equal score and smaller index); rows of rank < k write their index to idx[rank].
//      Counting is exact and order free, so the result is deterministic and already
//      sorted; no sort, no atomics, no host round trip.
//   3. requantize: one workgroup per selected row forms value(W~[i,:]) + buffer[i,:] . value(A~)
//      in fp64 (rank ascending), rounds to fp32, casts to E4M3 and writes the row back;
//      then clears the buffer row.
// The adapter A~ is read from rows [m, m+r) of the concatenated weight, in the same scaled
// domain as W~, so the backbone's scale never enters.
#include "falqon_internal.h"

namespace falqon {
namespace {

constexpr int kThreads = 256;

__global__ void __launch_bounds__(kThreads)
row_score_kernel(const float* __restrict__ buf, int64_t m, int64_t r, double* __restrict__ score)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (i >= m) return;
    const float4* row = reinterpret_cast<const float4*>(buf + i * r);
    double s = 0.0;
    for (int64_t p4 = 0; p4 < r / 4; ++p4) {
        const float4 v = row[p4];
        s += fabs(static_cast<double>(v.x));
        s += fabs(static_cast<double>(v.y));
        s += fabs(static_cast<double>(v.z));
        s += fabs(static_cast<double>(v.w));
    }
    score[i] = s;
}

// One wave per group of kRows rows; lanes stride over all rows j and count those that beat
// each of the wave's rows; a wave reduction gives the ranks.
constexpr int kRows = 4;

__global__ void __launch_bounds__(kThreads)
topk_rank_kernel(const double* __restrict__ score, int64_t m, int64_t k, int32_t* __restrict__ idx)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave_global = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) >> 6;
    const int64_t n_waves = (static_cast<int64_t>(gridDim.x) * kThreads) >> 6;
    for (int64_t base = wave_global * kRows; base < m; base += n_waves * kRows) {
        double si[kRows];
        int cnt[kRows];
#pragma unroll
        for (int q = 0; q < kRows; ++q) {
            const int64_t i = base + q;
            si[q] = i < m ? score[i] : 0.0;
            cnt[q] = 0;
        }
        for (int64_t j = lane; j < m; j += 64) {
            const double sj = score[j];
#pragma unroll
            for (int q = 0; q < kRows; ++q) {
                const int64_t i = base + q;
                cnt[q] += (sj > si[q] || (sj == si[q] && j < i)) ? 1 : 0;
            }
        }
#pragma unroll
        for (int q = 0; q < kRows; ++q) {
            int c = cnt[q];
            for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
            const int64_t i = base + q;
            if (lane == 0 && i < m && c < k) idx[c] = static_cast<int32_t>(i);
        }
    }
}

__device__ __forceinline__ void decode4_e4m3(uint32_t w, double (&d)[4])
{
    d[0] = static_cast<double>(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(w), 0));
    d[1] = static_cast<double>(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(w), 1));
    d[2] = static_cast<double>(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(w), 2));
    d[3] = static_cast<double>(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(w), 3));
}

// grid: k workgroups; workgroup a rewrites row idx[a]
__global__ void __launch_bounds__(kThreads)
row_requantize_kernel(float* buf, uint8_t* wq, int64_t n, int64_t m, int64_t r,
                      const int32_t* __restrict__ idx, int clear_selected)
{
    __shared__ double s_delta[256];                     // r <= 256
    const int64_t i = idx[blockIdx.x];
    if (i < 0 || i >= m) return;                        // cannot happen; keeps every access in range
    for (int p = threadIdx.x; p < r; p += kThreads) s_delta[p] = static_cast<double>(buf[i * r + p]);
    __syncthreads();
    uint32_t* wrow = reinterpret_cast<uint32_t*>(wq + i * n);
    const uint32_t* arows = reinterpret_cast<const uint32_t*>(wq + m * n);
    const int64_t n4 = n / 4;
    for (int64_t c = threadIdx.x; c < n4; c += kThreads) {
        double acc[4];
        decode4_e4m3(wrow[c], acc);
        for (int64_t p = 0; p < r; ++p) {
            double a[4];
            decode4_e4m3(arows[p * n4 + c], a);
            const double d = s_delta[p];
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = fma(d, a[e], acc[e]);     // product is exact in fp64
        }
        float f[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            f[e] = __builtin_amdgcn_fmed3f(static_cast<float>(acc[e]), -448.0f, 448.0f);
        int w = 0;
        w = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], w, false);
        w = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], w, true);
        wrow[c] = static_cast<uint32_t>(w);
    }
    if (clear_selected) {
        __syncthreads();
        for (int p = threadIdx.x; p < r; p += kThreads) buf[i * r + p] = 0.0f;
    }
}

}  // namespace

hipError_t launch_proxy_update(float* delta_buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                               int32_t* idx_out, int clear_selected, double* scores, hipStream_t stream)
{
    row_score_kernel<<<static_cast<unsigned>((m + kThreads - 1) / kThreads), kThreads, 0, stream>>>(delta_buf, m, r,
                                                                                                      scores);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    int64_t groups = (m + kRows - 1) / kRows;                  // one wave per group, 4 waves per workgroup
    int64_t blocks = (groups + 3) / 4;
    if (blocks > 2048) blocks = 2048;
    topk_rank_kernel<<<static_cast<unsigned>(blocks), kThreads, 0, stream>>>(scores, m, k, idx_out);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    row_requantize_kernel<<<static_cast<unsigned>(k), kThreads, 0, stream>>>(delta_buf, wq, n, m, r, idx_out,
                                                                             clear_selected);
    return hipGetLastError();
}

}  // namespace falqon
