// Row-wise proxy update (update equation; last two lines of the backward-and-update loop):
//   k = topk( sum_j |dB_ij| ; k ),   W~[k] = W~[k] + DeltaBuffer[k] A
//
// Three small launches, all latency bound (the update touches k of m rows), so each is shaped
// to have its loads in flight together rather than one after the other:
//   1. row scores: L1 norm of every buffer row, fp64, columns ascending.  A workgroup stages 64
//      rows in LDS with coalesced 16-byte loads; one lane per row then adds them in order.
//   2. selection: the rank of a row is the number of rows that beat it (larger score, or equal
//      score and smaller index); a row of rank c < k writes its index to idx[c].  Counting is
//      exact and order free, so the result is deterministic and already sorted: no sort, no
//      atomics, no host round trip.  The wave that finds a selected row also moves that buffer
//      row to a compact staging array (and clears it in the buffer), which lets the third
//      launch spread one row over several workgroups without a hazard on the buffer.
//   3. requantize: value(W~[i,j]) + sum_p delta[p] * value(A~[p,j]) in fp64 (p ascending),
//      rounded to fp32, cast to E4M3, written back.  A~ is rows [m, m+r) of the concatenated
//      weight, in the same scaled domain as W~, so the backbone's scale never enters.
#include <mutex>

#include "falqon_internal.h"

namespace falqon {
namespace {

constexpr int kThreads = 256;
constexpr int kScoreRows = 64;

// Scratch of the entry point that may not allocate and takes no workspace: row scores for up to
// kStaticMaxRows rows, then the staged buffer rows of the selection (k * r floats).  One copy per GPU,
// held until the process ends; every call on a GPU uses it, so calls that overlap on one GPU race.
constexpr size_t kStaticScoreBytes = sizeof(double) * kStaticMaxRows;
constexpr size_t kStaticBytes = kStaticScoreBytes + sizeof(float) * kStaticMaxSelected;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// grid: ceil(m / 64); dynamic LDS: 64 * (r + 4) floats
__global__ void __launch_bounds__(kThreads)
row_score_kernel(const float* __restrict__ buf, int64_t m, int64_t r, double* __restrict__ score)
{
    extern __shared__ float s_rows[];
    const int pitch = static_cast<int>(r) + 4;                      // +16 B: rows start on different banks
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kScoreRows;
    const int r4 = static_cast<int>(r / 4);
    for (int e = threadIdx.x; e < kScoreRows * r4; e += kThreads) {
        const int row = e / r4, c4 = e - row * r4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row0 + row < m) v = *reinterpret_cast<const float4*>(buf + (row0 + row) * r + c4 * 4);
        *reinterpret_cast<float4*>(s_rows + row * pitch + c4 * 4) = v;
    }
    __syncthreads();
    if (threadIdx.x < kScoreRows && row0 + threadIdx.x < m) {
        const float* row = s_rows + threadIdx.x * pitch;
        double s = 0.0;
        for (int c4 = 0; c4 < r4; ++c4) {
            const float4 v = *reinterpret_cast<const float4*>(row + c4 * 4);
            s += fabs(static_cast<double>(v.x));
            s += fabs(static_cast<double>(v.y));
            s += fabs(static_cast<double>(v.z));
            s += fabs(static_cast<double>(v.w));
        }
        score[row0 + threadIdx.x] = s;
    }
}

// A workgroup ranks 16 rows (4 waves x 4 consecutive rows).  All scores pass through LDS in
// chunks; lanes stride over a chunk and count the rows that beat each of the wave's rows.
// Scores are non-negative doubles, so their bit patterns order them as 64-bit integers.  Row j
// beats row i if key_j > key_i, or key_j == key_i and j < i: for all j below the wave's rows that
// is "key_j >= key_i", for all j above them "key_j > key_i", so the inner loop is one integer
// comparison per pair; only the wave's own four rows need the index compared.
constexpr int kRankRows = 4;
constexpr int kChunk = 4096;                                         // scores per LDS chunk (32 KB)

__global__ void __launch_bounds__(kThreads)
topk_rank_kernel(const double* __restrict__ score, int64_t m, int64_t k, int64_t r, int32_t* __restrict__ idx,
                 float* buf, float* __restrict__ delta_sel, int clear_selected)
{
    __shared__ uint64_t s_key[kChunk];
    const uint64_t* key = reinterpret_cast<const uint64_t*>(score);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t base = (static_cast<int64_t>(blockIdx.x) * 4 + wave) * kRankRows;
    uint64_t ki[kRankRows];
    int cnt[kRankRows];
#pragma unroll
    for (int q = 0; q < kRankRows; ++q) {
        ki[q] = base + q < m ? key[base + q] : 0;
        cnt[q] = 0;
    }
    for (int64_t c0 = 0; c0 < m; c0 += kChunk) {
        const int n_here = static_cast<int>(m - c0 < kChunk ? m - c0 : kChunk);
        __syncthreads();
        {
            uint64_t v[kChunk / kThreads];                           // all loads in flight together
#pragma unroll
            for (int u = 0; u < kChunk / kThreads; ++u) {
                const int e = u * kThreads + threadIdx.x;
                v[u] = e < n_here ? key[c0 + e] : 0;
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < kChunk / kThreads; ++u) s_key[u * kThreads + threadIdx.x] = v[u];
        }
        __syncthreads();
        // rows below the wave's rows: ties count; rows above: they do not
        const int64_t lo_end = base - c0 < 0 ? 0 : (base - c0 > n_here ? n_here : base - c0);
        const int64_t hi_begin = base + kRankRows - c0 < 0 ? 0 : (base + kRankRows - c0 > n_here ? n_here : base + kRankRows - c0);
        // eight keys per lane and step, read together (one LDS latency per step instead of eight);
        // a slot beyond the range reads key 0 of the chunk and is masked out of the count
        for (int e0 = lane; e0 < lo_end; e0 += 64 * 8) {
            uint64_t kj[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) kj[u] = s_key[e0 + 64 * u < lo_end ? e0 + 64 * u : 0];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool in = e0 + 64 * u < lo_end;
#pragma unroll
                for (int q = 0; q < kRankRows; ++q) cnt[q] += (in && kj[u] >= ki[q]) ? 1 : 0;
            }
        }
        for (int e0 = static_cast<int>(hi_begin) + lane; e0 < n_here; e0 += 64 * 8) {
            uint64_t kj[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) kj[u] = s_key[e0 + 64 * u < n_here ? e0 + 64 * u : 0];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool in = e0 + 64 * u < n_here;
#pragma unroll
                for (int q = 0; q < kRankRows; ++q) cnt[q] += (in && kj[u] > ki[q]) ? 1 : 0;
            }
        }
        if (lane < kRankRows && base + lane >= c0 && base + lane < c0 + n_here) {       // the wave's own rows
            const uint64_t kj = s_key[base + lane - c0];
#pragma unroll
            for (int q = 0; q < kRankRows; ++q) cnt[q] += (kj > ki[q] || (kj == ki[q] && lane < q)) ? 1 : 0;
        }
    }
#pragma unroll
    for (int q = 0; q < kRankRows; ++q) {
        int c = cnt[q];
        for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
        const int64_t i = base + q;
        if (i < m && c < k) {                                        // wave-uniform
            if (lane == 0) idx[c] = static_cast<int32_t>(i);
            for (int64_t p = lane; p < r; p += 64) {
                delta_sel[static_cast<int64_t>(c) * r + p] = buf[i * r + p];
                if (clear_selected) buf[i * r + p] = 0.0f;
            }
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

// grid: (k, ceil(n / 1024)); a thread owns four adjacent columns of row idx[blockIdx.x]
__global__ void __launch_bounds__(kThreads)
row_requantize_kernel(uint8_t* wq, int64_t n, int64_t m, int64_t r, const int32_t* __restrict__ idx,
                      const float* __restrict__ delta_sel)
{
    __shared__ double s_delta[256];                                  // r <= 256
    const int64_t i = idx[blockIdx.x];
    if (i < 0 || i >= m) return;                                     // cannot happen; keeps every access in range
    for (int p = threadIdx.x; p < r; p += kThreads)
        s_delta[p] = static_cast<double>(delta_sel[static_cast<int64_t>(blockIdx.x) * r + p]);
    __syncthreads();
    const int64_t n4 = n / 4;
    const int64_t c = static_cast<int64_t>(blockIdx.y) * kThreads + threadIdx.x;
    if (c >= n4) return;
    uint32_t* wrow = reinterpret_cast<uint32_t*>(wq + i * n);
    const uint32_t* arows = reinterpret_cast<const uint32_t*>(wq + m * n);
    double acc[4];
    decode4_e4m3(wrow[c], acc);
    constexpr int U = 16;                                            // r is a multiple of 16
    for (int64_t p0 = 0; p0 < r; p0 += U) {
        uint32_t aw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) aw[u] = arows[(p0 + u) * n4 + c];    // all 16 loads in flight
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            double a[4];
            decode4_e4m3(aw[u], a);
            const double d = s_delta[p0 + u];
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = fma(d, a[e], acc[e]);  // product is exact in fp64
        }
    }
    float f[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) f[e] = __builtin_amdgcn_fmed3f(static_cast<float>(acc[e]), -448.0f, 448.0f);
    int w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(f[0], f[1], w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(f[2], f[3], w, true);
    wrow[c] = static_cast<uint32_t>(w);
}

}  // namespace

// Device address of `scratch` on the current GPU.  In host code the array's name is only a handle:
// the address is looked up once per device and kept; every launch below receives that pointer.
static hipError_t static_scratch(unsigned char** out)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static unsigned char* ptrs[kMaxDevices] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptrs[dev] = static_cast<unsigned char*>(p);
    }
    *out = ptrs[dev];
    return hipSuccess;
}

hipError_t launch_proxy_update_static(float* delta_buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                                      int32_t* idx_out, int clear_selected, hipStream_t stream)
{
    unsigned char* base = nullptr;
    hipError_t e = static_scratch(&base);
    if (e != hipSuccess) return e;
    return launch_proxy_update(delta_buf, wq, n, m, r, k, idx_out, clear_selected, reinterpret_cast<double*>(base),
                               reinterpret_cast<float*>(base + kStaticScoreBytes), stream);
}

hipError_t launch_proxy_update(float* delta_buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                               int32_t* idx_out, int clear_selected, double* scores, float* delta_sel,
                               hipStream_t stream)
{
    const size_t lds = sizeof(float) * kScoreRows * (static_cast<size_t>(r) + 4);
    if (lds > 64 * 1024) {
        hipError_t e0 = hipFuncSetAttribute(reinterpret_cast<const void*>(&row_score_kernel),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        if (e0 != hipSuccess) return e0;
    }
    row_score_kernel<<<static_cast<unsigned>((m + kScoreRows - 1) / kScoreRows), kThreads, lds, stream>>>(
        delta_buf, m, r, scores);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int64_t rows_per_block = 4 * kRankRows;
    topk_rank_kernel<<<static_cast<unsigned>((m + rows_per_block - 1) / rows_per_block), kThreads, 0, stream>>>(
        scores, m, k, r, idx_out, delta_buf, delta_sel, clear_selected);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 grid(static_cast<unsigned>(k), static_cast<unsigned>((n / 4 + kThreads - 1) / kThreads));
    row_requantize_kernel<<<grid, kThreads, 0, stream>>>(wq, n, m, r, idx_out, delta_sel);
    return hipGetLastError();
}

}  // namespace falqon
