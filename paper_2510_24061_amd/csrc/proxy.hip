// Row-wise proxy update (update equation; last two lines of the backward-and-update loop):
//   k = topk( sum_j |dB_ij| ; k ),   W~[k] = W~[k] + DeltaBuffer[k] A
//
// Three small launches, all latency bound (the update touches k of m rows), so each is shaped to
// have its loads in flight together rather than one after the other:
//   1. row scores: L1 norm of every buffer row, fp64, columns ascending, and the largest score of
//      every block of 64 rows (row_scores.h).  Skipped when the kernel that wrote the buffer has
//      already left them (falqon_melded_bwd with its buffer step).
//   2. selection: the rank of a row is the number of rows that beat it (larger score, or equal
//      score and smaller index); a row of rank c < k is selected and its index goes to idx[c].
//      Counting is exact and order free, so the result is deterministic and already sorted: no
//      sort, no atomics, no host round trip.  Only rows that can be selected are ranked: the k-th
//      largest of the block maxima is a lower bound on the k-th largest score (each of those maxima
//      is the score of a different row), so a row below it has at least k rows above it.  The wave
//      that finds a selected row also moves that buffer row to a compact staging array (and clears
//      it in the buffer), which lets the third launch spread one row over several workgroups
//      without a hazard on the buffer.  (Requantizing in the same launch was built and measured
//      slower: the one workgroup that finds a row then walks the whole weight row alone.)
//   3. requantize: value(W~[i,j]) + sum_p delta[p] * value(A~[p,j]) in fp64 (p ascending),
//      rounded to fp32, cast to E4M3, written back.  A~ is rows [m, m+r) of the concatenated
//      weight, in the same scaled domain as W~, so the backbone's scale never enters.
#include <mutex>

#include "falqon_internal.h"
#include "row_scores.h"

namespace falqon {
namespace {

constexpr int kThreads = 256;

// Scratch of the entry point that may not allocate and takes no workspace: row scores for up to
// kStaticMaxRows rows with their block maxima, then the staged buffer rows of the selection (k * r
// floats).  One copy per GPU, held until the process ends; every
// call on a GPU uses it, so calls that overlap on one GPU race.
constexpr size_t kStaticScoreBytes = sizeof(double) * (kStaticMaxRows + kStaticMaxRows / kScoreRows);
constexpr size_t kStaticBytes = kStaticScoreBytes + sizeof(float) * kStaticMaxSelected;
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

// grid: ceil(m / 64); dynamic LDS: 64 * (r + 4) floats
__global__ void __launch_bounds__(kThreads)
row_score_kernel(const float* __restrict__ buf, int64_t m, int r, double* __restrict__ score)
{
    extern __shared__ float s_rows[];
    const int pitch = r + 4;                                         // +16 B: rows start on different banks
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kScoreRows;
    const int r4 = r / 4;
    for (int e = threadIdx.x; e < kScoreRows * r4; e += kThreads) {
        const int row = e / r4, c4 = e - row * r4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row0 + row < m) v = *reinterpret_cast<const float4*>(buf + (row0 + row) * r + c4 * 4);
        *reinterpret_cast<float4*>(s_rows + row * pitch + c4 * 4) = v;
    }
    __syncthreads();
    score_rows_from_lds(s_rows, r, row0, m, score);
}

__device__ __forceinline__ void decode4_e4m3(uint32_t w, double (&d)[4])
{
    d[0] = static_cast<double>(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(w), 0));
    d[1] = static_cast<double>(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(w), 1));
    d[2] = static_cast<double>(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(w), 2));
    d[3] = static_cast<double>(__builtin_amdgcn_cvt_f32_fp8(static_cast<int>(w), 3));
}

// A workgroup owns 16 rows (4 waves x 4 consecutive rows).
// Scores are non-negative doubles, so their bit patterns order them as 64-bit integers.  Row j
// beats row i if key_j > key_i, or key_j == key_i and j < i: for all j below the wave's rows that
// is "key_j >= key_i", for all j above them "key_j > key_i", so the inner loop is one integer
// comparison per pair; only the wave's own four rows need the index compared.
constexpr int kChunk = 4096;                                         // scores that fit the small selection's LDS (32 KB)
static_assert(65536 / kScoreRows <= kChunk, "the block maxima of the largest buffer (m <= 65536) fit the LDS chunk");

// Selection for buffers of up to kChunk rows.  A workgroup ranks 16 rows (4 waves x 4 consecutive
// rows).  All scores sit in LDS; lanes stride over them and count the rows that beat each of the
// wave's rows.  Scores are non-negative doubles, so their bit patterns order them as 64-bit
// integers.  Row j beats row i if key_j > key_i, or key_j == key_i and j < i: for all j below the
// wave's rows that is "key_j >= key_i", for all j above them "key_j > key_i", so the inner loop is
// one integer comparison per pair; only the wave's own four rows need the index compared.
constexpr int kRankRows = 4;

__global__ void __launch_bounds__(kThreads)
topk_rank_kernel(const double* __restrict__ score, int64_t m, int64_t k, int r, int32_t* __restrict__ idx,
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
    const int n_here = static_cast<int>(m);                          // m <= kChunk
    {
        uint64_t v[kChunk / kThreads];                               // all loads in flight together
#pragma unroll
        for (int u = 0; u < kChunk / kThreads; ++u) {
            const int e = u * kThreads + threadIdx.x;
            v[u] = e < n_here ? key[e] : 0;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < kChunk / kThreads; ++u) s_key[u * kThreads + threadIdx.x] = v[u];
    }
    __syncthreads();
    // rows below the wave's rows: ties count; rows above: they do not
    const int64_t lo_end = base > n_here ? n_here : base;
    const int64_t hi_begin = base + kRankRows > n_here ? n_here : base + kRankRows;
    // eight keys per lane and step, read together (one LDS latency per step instead of eight);
    // a slot beyond the range reads key 0 and is masked out of the count
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
    if (lane < kRankRows && base + lane < n_here) {                  // the wave's own rows
        const uint64_t kj = s_key[base + lane];
#pragma unroll
        for (int q = 0; q < kRankRows; ++q) cnt[q] += (kj > ki[q] || (kj == ki[q] && lane < q)) ? 1 : 0;
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

// Selection for larger buffers: rank only rows that can be selected.  The k-th largest of the block
// maxima is a lower bound tau on the k-th largest score (each maximum is the score of a different
// row), so a row below tau has at least k rows above it.  A workgroup owns one block of 64 rows; it
// needs nothing but the block maxima to know whether it can leave, and most do.  One that stays
// lists its rows that reach tau, takes 128 KB of LDS to fetch up to 16384 scores per round trip, and
// counts, all threads together and one listed row at a time, the rows that beat it.
constexpr int kChunkFiltered = 16384;

__global__ void __launch_bounds__(kThreads)
topk_filtered_kernel(const double* __restrict__ score, int64_t m, int64_t k, int r, int32_t* __restrict__ idx,
                     float* buf, float* __restrict__ delta_sel, int clear_selected)
{
    extern __shared__ uint64_t s_key[];                              // kChunkFiltered keys
    __shared__ uint64_t s_tau;
    __shared__ int s_cand[kScoreRows + 4], s_cnt[kScoreRows + 4], s_ncand;
    __shared__ uint64_t s_ckey[kScoreRows + 4];
    const uint64_t* key = reinterpret_cast<const uint64_t*>(score);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * kScoreRows;

    // ---- tau, and whether this block can hold a selected row ----------------------------------------
    const int nb = static_cast<int>(score_blocks(m));
    if (threadIdx.x == 0) { s_tau = 0; s_ncand = 0; }
    if (threadIdx.x < kScoreRows + 4) s_cnt[threadIdx.x] = 0;
    for (int e = threadIdx.x; e < nb; e += kThreads) s_key[e] = key[m + e];
    __syncthreads();
    if (nb >= k) {
        for (int e = threadIdx.x; e < nb; e += kThreads) {
            const uint64_t mine = s_key[e];
            int above = 0;                                           // maxima that beat this one (ties by position)
            for (int j = 0; j < nb; ++j) {
                const uint64_t o = s_key[j];
                above += (o > mine || (o == mine && j < e)) ? 1 : 0;
            }
            if (above == k - 1) s_tau = mine;                        // exactly one position has this count
        }
    }
    __syncthreads();
    const uint64_t tau = s_tau;
    if (s_key[blockIdx.x] < tau) return;                             // workgroup-uniform
    // ---- the block's rows that reach tau, in row order ------------------------------------------------
    if (wave == 0) {
        const int64_t i = row0 + lane;
        const uint64_t mine = i < m ? key[i] : 0;
        const bool in = i < m && mine >= tau;
        const uint64_t mask = __ballot(in);
        if (in) {
            const int pos = __popcll(mask & ((uint64_t(1) << lane) - 1));
            s_cand[pos] = static_cast<int>(i);
            s_ckey[pos] = mine;
        }
        const int total = __popcll(mask);
        if (lane < 4) {                                              // padding so that listed rows can be taken four at a time
            s_cand[total + lane] = -1;
            s_ckey[total + lane] = ~uint64_t(0);
        }
        if (lane == 0) s_ncand = total;
    }
    __syncthreads();                                                 // also: the block maxima in s_key are no longer read
    const int ncand = s_ncand;
    // ---- count, for every listed row, the rows that beat it ---------------------------------------------
    for (int64_t c0 = 0; c0 < m; c0 += kChunkFiltered) {
        const int n_here = static_cast<int>(m - c0 < kChunkFiltered ? m - c0 : kChunkFiltered);
        if (c0 > 0) __syncthreads();
        for (int e0 = threadIdx.x; e0 < n_here; e0 += 32 * kThreads) {   // 32 loads in flight per thread
            uint64_t v[32];
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                const int e = e0 + u * kThreads;
                v[u] = e < n_here ? key[c0 + e] : 0;
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < 32; ++u) {
                const int e = e0 + u * kThreads;
                if (e < n_here) s_key[e] = v[u];
            }
        }
        __syncthreads();
        for (int c = 0; c < ncand; c += 4) {                         // four listed rows per pass over the scores
            int64_t ri[4];
            uint64_t kc[4];
            int cnt[4] = {0, 0, 0, 0};
#pragma unroll
            for (int q = 0; q < 4; ++q) { ri[q] = s_cand[c + q]; kc[q] = s_ckey[c + q]; }
            for (int e = threadIdx.x; e < n_here; e += kThreads) {
                const uint64_t kj = s_key[e];
#pragma unroll
                for (int q = 0; q < 4; ++q) cnt[q] += (kj > kc[q] || (kj == kc[q] && c0 + e < ri[q])) ? 1 : 0;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int v = cnt[q];
                for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
                if (lane == 0 && v) atomicAdd(&s_cnt[c + q], v);     // integer sum in LDS: order immaterial
            }
        }
    }
    __syncthreads();
    // ---- selected rows: index out, buffer row staged and cleared (one wave per row) -------------------
    for (int c = wave; c < ncand; c += 4) {
        const int rank = s_cnt[c];
        if (rank >= k) continue;                                     // wave-uniform
        const int64_t i = s_cand[c];
        if (lane == 0) idx[rank] = static_cast<int32_t>(i);
        for (int64_t p = lane; p < r; p += 64) {
            delta_sel[static_cast<int64_t>(rank) * r + p] = buf[i * r + p];
            if (clear_selected) buf[i * r + p] = 0.0f;
        }
    }
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
                               nullptr, reinterpret_cast<float*>(base + kStaticScoreBytes), stream);
}

hipError_t launch_proxy_update(float* delta_buf, uint8_t* wq, int64_t n, int64_t m, int64_t r, int64_t k,
                               int32_t* idx_out, int clear_selected, double* scores, const double* scores_in,
                               float* delta_sel, hipStream_t stream)
{
    if (!scores_in) {
        const size_t lds = sizeof(float) * kScoreRows * (static_cast<size_t>(r) + 4);
        if (lds > 64 * 1024) {
            hipError_t e0 = hipFuncSetAttribute(reinterpret_cast<const void*>(&row_score_kernel),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
            if (e0 != hipSuccess) return e0;
        }
        row_score_kernel<<<static_cast<unsigned>(score_blocks(m)), kThreads, lds, stream>>>(delta_buf, m, static_cast<int>(r),
                                                                                        scores);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        scores_in = scores;
    }
    if (m > kChunk) {
        constexpr size_t lds_sel = sizeof(uint64_t) * kChunkFiltered;
        hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(&topk_filtered_kernel),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds_sel));
        if (e1 != hipSuccess) return e1;
        topk_filtered_kernel<<<static_cast<unsigned>(score_blocks(m)), kThreads, lds_sel, stream>>>(
            scores_in, m, k, static_cast<int>(r), idx_out, delta_buf, delta_sel, clear_selected);
    } else {
        topk_rank_kernel<<<static_cast<unsigned>((m + 4 * kRankRows - 1) / (4 * kRankRows)), kThreads, 0, stream>>>(
            scores_in, m, k, static_cast<int>(r), idx_out, delta_buf, delta_sel, clear_selected);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 grid(static_cast<unsigned>(k), static_cast<unsigned>((n / 4 + kThreads - 1) / kThreads));
    row_requantize_kernel<<<grid, kThreads, 0, stream>>>(wq, n, m, r, idx_out, delta_sel);
    return hipGetLastError();
}

}  // namespace falqon
