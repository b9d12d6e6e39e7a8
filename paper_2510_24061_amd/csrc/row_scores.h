// Row scores of the proxy buffer (update equation: score_i = sum_p |DeltaBuffer[i,p]|) for a block of
// 64 rows that a workgroup holds in LDS, shared by the update's own score pass and by the kernels
// that write the buffer and can hand the scores on.
//
// Layout of a score array for m rows (doubles): [0, m) the scores; [m, m + ceil(m / 64)) the largest
// score of each block of 64 rows (the selection derives from them a lower bound on the k-th largest
// score and ranks only the rows that reach it).
#pragma once
#include "falqon_internal.h"

namespace falqon {

constexpr int kScoreRows = 64;

__host__ __device__ inline int64_t score_blocks(int64_t m) { return (m + kScoreRows - 1) / kScoreRows; }

// s_rows: kScoreRows rows of r floats at a pitch of r + 4 floats, complete (the caller has
// synchronised).  Lane t of the first wave adds row t in fp64, columns ascending (the order the
// definition gives), writes score[row0 + t]; the block's largest score goes to score[m + block].
// Rows beyond m count as zero.  Must be called by all threads of the workgroup's first wave.
__device__ __forceinline__ void score_rows_from_lds(const float* s_rows, int r, int64_t row0, int64_t m, double* score)
{
    if (threadIdx.x >= kScoreRows) return;
    const int pitch = r + 4;
    double s = 0.0;
    if (row0 + threadIdx.x < m) {
        const float* row = s_rows + threadIdx.x * pitch;
        for (int c4 = 0; c4 < r / 4; ++c4) {
            const float4 v = *reinterpret_cast<const float4*>(row + c4 * 4);
            s += fabs(static_cast<double>(v.x));
            s += fabs(static_cast<double>(v.y));
            s += fabs(static_cast<double>(v.z));
            s += fabs(static_cast<double>(v.w));
        }
        score[row0 + threadIdx.x] = s;
    }
    // non-negative doubles order like their bit patterns
    unsigned long long key = static_cast<unsigned long long>(__double_as_longlong(s));
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long o = __shfl_xor(key, off, 64);
        key = o > key ? o : key;
    }
    if (threadIdx.x == 0) score[m + row0 / kScoreRows] = __longlong_as_double(static_cast<long long>(key));
}

}  // namespace falqon
