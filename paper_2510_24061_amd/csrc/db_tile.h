// Tile body of the adapter-gradient contraction dB = dy~^T O_A~ (modified LoRA-backward equation),
// shared by its own kernel and by the launch that pairs it with the input-gradient GEMM.
#pragma once
#include "falqon_internal.h"

namespace falqon {
namespace dbt {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));

#ifndef FQ_GLOBAL_PTR
#define FQ_GLOBAL_PTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define FQ_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))
#endif

constexpr int BI = 128;    // rows of dB (output features) per workgroup
constexpr int BP = 64;     // columns of dB (rank) per workgroup
constexpr int BT = 128;    // tokens per step
constexpr int kThreads = 256;

// [token][feature] tile with CH 16-byte chunks per token row; chunk c of row t sits at c ^ swz.
template <int CH>
__device__ __forceinline__ int swz_t(int trow) { return trow & (CH - 1); }

// Eight consecutive tokens of one feature per lane; four reads make a 32-token operand.
// Lane s of a 16-lane group supplies the address of token row (s % 16) / 2, feature block
// 8 * (s % 2); lane L then receives feature (L % 16) of the group's 16-feature span.
template <int CH>
__device__ __forceinline__ v8i read_tokens_of_feature(const uint8_t* tile, int feat_base, int kh, int lane)
{
    v8i r;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int trow = kh * 64 + (lane >> 5) * 32 + t * 8 + ((lane & 15) >> 1);
        const int feat = feat_base + ((lane >> 4) & 1) * 16 + (lane & 1) * 8;
        const uint8_t* p = tile + trow * (CH * 16) + ((((feat >> 4) ^ swz_t<CH>(trow)) << 4) | (feat & 15));
        const v2i d = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(p));
        r[2 * t] = d[0];
        r[2 * t + 1] = d[1];
    }
    return r;
}

__device__ __forceinline__ uint32_t cast4_e4m3(float a, float b, float c, float d)
{
    a = __builtin_amdgcn_fmed3f(a, -448.0f, 448.0f);
    b = __builtin_amdgcn_fmed3f(b, -448.0f, 448.0f);
    c = __builtin_amdgcn_fmed3f(c, -448.0f, 448.0f);
    d = __builtin_amdgcn_fmed3f(d, -448.0f, 448.0f);
    int w = 0;
    w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, w, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
    return static_cast<uint32_t>(w);
}

// One tile of the grid (ceil(m / BI), splits, ceil(r / BP)); partial[split][m][r].
// s_tiles: kDbLdsBytes of LDS, 1 KB aligned; zero16: 16 zero bytes in global memory.
// The workgroup's token range is walked in groups of kTiles tiles of BT tokens.  All fetches of a
// group are issued together, so a workgroup pays one memory latency per group, not per tile (the
// matrix-core work per tile is a few hundred cycles; the kernel is all memory latency otherwise).
constexpr int kTiles = 4;
constexpr int kTileBytes = BT * BI + BT * BP;                          // dyq tile + O_A tile (codes)
constexpr size_t kDbLdsBytes = static_cast<size_t>(kTiles) * kTileBytes;

__device__ __forceinline__ void db_partial_tile(const DbArgs& d, const int bi, const int bsplit, const int bp,
                                                uint8_t* const s_tiles, const uint8_t* const zero16)
{
    constexpr int CH_DY = BI / 16, CH_OA = BP / 16;
    const uint8_t* const dyq = d.dyq;
    const uint16_t* const o_a = d.o_a;
    const int64_t T = d.T, m = d.m, r = d.r;
    // s_tiles: [tile]{[token][feature i], [token][rank p]}
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t i0 = static_cast<int64_t>(bi) * BI;
    const int64_t p0 = static_cast<int64_t>(bp) * BP;
    const int64_t t_begin = static_cast<int64_t>(bsplit) * d.tokens_per_split;
    int64_t t_end = t_begin + d.tokens_per_split;
    if (t_end > T) t_end = T;
    const float s_oa_scale = 448.0f / fmaxf(*d.amax_oa, 1e-12f);

    v16f acc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.0f;

    for (int64_t tg = t_begin; tg < t_end; tg += kTiles * BT) {
        __syncthreads();                       // the previous group's operand reads are done
        // dyq tiles: BT rows x BI bytes = 16 KB = 16 wave instructions of 1 KB (8 token rows each).
        // Rows, features and whole tiles out of range are fetched from a block of zeros.
#pragma unroll
        for (int tl = 0; tl < kTiles; ++tl) {
            const int64_t t0 = tg + tl * BT;
#pragma unroll
            for (int it = 0; it < BT * BI / 1024 / 4; ++it) {
                const int q = it * 4 + wave;
                const int trow = q * 8 + (lane >> 3);
                const int c = (lane & 7) ^ swz_t<CH_DY>(trow);
                const int64_t gt = t0 + trow, gi = i0 + c * 16;
                const uint8_t* src = (gt < t_end && gi < m) ? dyq + gt * m + gi : zero16;
                __builtin_amdgcn_global_load_lds(FQ_GLOBAL_PTR(src), FQ_LDS_PTR(s_tiles + tl * kTileBytes + q * 1024), 16, 0, 0);
            }
        }
        // O_A tiles: BT rows x BP bf16 -> E4M3 bytes.  256 threads x 32 values: thread -> (row, half row)
        const int trow = threadIdx.x >> 1, half = threadIdx.x & 1;         // 32 ranks per half
        uint4 w[kTiles][4];
        // rows and ranks out of range read a block of zeros (address select: a load inside a
        // branch would be waited for at the join and serialise the loads)
#pragma unroll
        for (int tl = 0; tl < kTiles; ++tl) {
            const int64_t gt = tg + tl * BT + trow;
#pragma unroll
            for (int v8 = 0; v8 < 4; ++v8) {                               // 8 bf16 per 16-byte load
                const int64_t gp = p0 + half * 32 + v8 * 8;
                const void* src = (gt < t_end && gp < r) ? static_cast<const void*>(o_a + gt * r + gp)
                                                         : static_cast<const void*>(zero16);
                w[tl][v8] = *reinterpret_cast<const uint4*>(src);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int tl = 0; tl < kTiles; ++tl) {
            uint32_t codes[8];
#pragma unroll
            for (int v8 = 0; v8 < 4; ++v8) {
                const uint32_t ww[4] = {w[tl][v8].x, w[tl][v8].y, w[tl][v8].z, w[tl][v8].w};
                float f[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    f[2 * e] = __fmul_rn(__uint_as_float(ww[e] << 16), s_oa_scale);
                    f[2 * e + 1] = __fmul_rn(__uint_as_float(ww[e] & 0xffff0000u), s_oa_scale);
                }
                codes[2 * v8] = cast4_e4m3(f[0], f[1], f[2], f[3]);
                codes[2 * v8 + 1] = cast4_e4m3(f[4], f[5], f[6], f[7]);
            }
            uint8_t* s_oa = s_tiles + tl * kTileBytes + BT * BI;
#pragma unroll
            for (int c = 0; c < 2; ++c) {                                   // two 16-byte chunks
                const int chunk = (half * 2 + c) ^ swz_t<CH_OA>(trow);
                uint4 o;
                o.x = codes[4 * c]; o.y = codes[4 * c + 1]; o.z = codes[4 * c + 2]; o.w = codes[4 * c + 3];
                *reinterpret_cast<uint4*>(s_oa + trow * BP + chunk * 16) = o;
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        // wave w owns features [32 w, 32 w + 32) of the tile and both 32-wide rank blocks
#pragma unroll
        for (int tl = 0; tl < kTiles; ++tl) {
            if (tg + tl * BT >= t_end) break;                               // tiles beyond the range hold zeros
            const uint8_t* s_dy = s_tiles + tl * kTileBytes;
            const uint8_t* s_oa = s_dy + BT * BI;
#pragma unroll
            for (int kh = 0; kh < 2; ++kh) {
                const v8i a = read_tokens_of_feature<CH_DY>(s_dy, wave * 32, kh, lane);
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const v8i bb = read_tokens_of_feature<CH_OA>(s_oa, b * 32, kh, lane);
                    acc[b] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, bb, acc[b], 1 /* E5M2 */, 0 /* E4M3 */,
                                                                              0, 0, 0, 0);
                }
            }
        }
    }

    float* out = d.partial + static_cast<int64_t>(bsplit) * m * r;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int64_t p = p0 + b * 32 + (lane & 31);
        if (p >= r) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t i = i0 + wave * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            if (i < m) out[i * r + p] = acc[b][v];
        }
    }
}

}  // namespace dbt
}  // namespace falqon
