// FP8 GEMMs of the melded layer on the gfx950 matrix cores.
//
//   forward         Y|O_A = X~ . W~'^T / (s_w s_x)     (merged-output equation)
//   input gradient  dX    = dY~ . W~    / (s_dy s_w)   (FP8 matmul-and-rescale equation)
//
// One kernel template serves both.  The left operand is always K-contiguous (tokens x K).
// The right operand is E4M3 and either [N,K] (forward: rows of the concatenated weight) or
// [K,N] (input gradient: the same weight bytes read down its rows, so no transposed copy
// of the weight is ever kept).
//
// Design for CDNA4:
//   - v_mfma_f32_32x32x64_f8f6f4 (the 8-bit path that runs at the full FP8 rate; the older
//     32x32x16 FP8 instruction runs at half of it), fp32 accumulators in registers.
//   - A workgroup owns a BM x BN output tile and walks K in steps of 128 bytes.  Operand
//     tiles go HBM/L2 -> LDS with global_load_lds (16 B per lane, no register staging),
//     double buffered: the loads of step k+1 are in flight while step k is multiplied.
//   - global_load_lds writes lanes to consecutive LDS addresses, so the bank-conflict
//     swizzle is applied on the global side: lane -> (row, physical chunk) is fixed, and
//     the lane fetches the logical chunk that belongs there.
//   - The [K,N] operand is read from LDS with ds_read_b64_tr_b8, which hands each lane
//     eight consecutive K for one N: exactly the matrix-core operand layout.
//   - Out-of-range rows, columns and the K tail are fetched from a 16-byte block of zeros,
//     so ragged shapes need no separate code path.
//   - Workgroup ids are spread round-robin over the 8 XCDs by the hardware; the id -> tile
//     map hands each XCD a compact block of tiles so its L2 sees each operand panel once.
#include "falqon_internal.h"

namespace falqon {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));

#define FQ_GLOBAL_PTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define FQ_LDS_PTR(p) ((void __attribute__((address_space(3)))*)(p))

__device__ __attribute__((aligned(16))) uint8_t g_zero16[16];

constexpr int BK = 128;   // bytes of K per step (two 64-deep MFMAs)

// Swizzle of a K-contiguous tile (128 B = 8 chunks of 16 B per row): the physical chunk of
// logical chunk c in row `row` is c ^ swz_kc(row).  Any 8 or 16 consecutive rows land on
// distinct 16-byte bank groups for a fixed logical chunk.
__device__ __forceinline__ int swz_kc(int row) { return ((row >> 1) ^ ((row & 1) << 2)) & 7; }

// Swizzle of a [K][N] tile with CH chunks of 16 B per K-row.
template <int CH>
__device__ __forceinline__ int swz_kn(int krow) { return CH >= 16 ? ((krow & 7) << 1) : (krow & (CH - 1)); }

__device__ __forceinline__ uint16_t bf16_bits_rne(float v)
{
    uint32_t u = __float_as_uint(v);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

template <int WM, int WN, int MB, int NB, bool B_KN, int A_FMT>
__global__ void __launch_bounds__(64 * WM * WN)
gemm_fp8_kernel(const GemmArgs g, const int tiles_m, const int tiles_n, const int chunk)
{
    constexpr int BM = WM * MB * 32, BN = WN * NB * 32, NW = WM * WN;
    constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK, STAGE = A_BYTES + B_BYTES;
    static_assert((BM / 8) % NW == 0 && (B_BYTES / 1024) % NW == 0, "loads must split evenly over waves");
    __shared__ __attribute__((aligned(1024))) uint8_t lds[2 * STAGE];

    // ---- workgroup -> tile (XCD aware) ----------------------------------------------------
    // Hardware places workgroup b on XCD b % 8.  XCD x takes tiles [x*chunk, (x+1)*chunk) of a
    // raster that walks panels of 4 tile-rows, tile-column by tile-column.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int tile_id = xcd * chunk + slot;
    if (slot >= chunk || tile_id >= tiles_m * tiles_n) return;
    constexpr int PH = 4;
    const int per_panel = PH * tiles_n;
    const int panel = tile_id / per_panel, rem = tile_id - panel * per_panel;
    const int ph = (tiles_m - panel * PH) < PH ? (tiles_m - panel * PH) : PH;
    const int tile_n = rem / ph, tile_m = panel * PH + (rem - tile_n * ph);

    // wave-uniform values live in scalar registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int wm = wave / WN, wn = wave % WN;
    const int64_t m0 = static_cast<int64_t>(tile_m) * BM, n0 = static_cast<int64_t>(tile_n) * BN;
    const int64_t M = g.M, N = g.N, K = g.K;

    // ---- global -> LDS ----------------------------------------------------------------------
    auto issue_stage = [&](int kt, int buf) {
        uint8_t* sA = lds + buf * STAGE;
        uint8_t* sB = sA + A_BYTES;
        const int64_t k0 = static_cast<int64_t>(kt) * BK;
#pragma unroll
        for (int it = 0; it < BM / 8 / NW; ++it) {
            const int i = it * NW + wave;                     // 1 KB = 8 rows per wave instruction
            const int row = i * 8 + (lane >> 3);
            const int c = (lane & 7) ^ swz_kc(row);
            const int64_t gr = m0 + row, gk = k0 + c * 16;
            const uint8_t* src = (gr < M && gk < K) ? g.a + gr * g.lda + gk : g_zero16;
            __builtin_amdgcn_global_load_lds(FQ_GLOBAL_PTR(src), FQ_LDS_PTR(sA + i * 1024), 16, 0, 0);
        }
        if (!B_KN) {
#pragma unroll
            for (int it = 0; it < BN / 8 / NW; ++it) {
                const int i = it * NW + wave;
                const int row = i * 8 + (lane >> 3);
                const int c = (lane & 7) ^ swz_kc(row);
                const int64_t gr = n0 + row, gk = k0 + c * 16;
                const uint8_t* src = (gr < N && gk < K) ? g.b + gr * g.ldb + gk : g_zero16;
                __builtin_amdgcn_global_load_lds(FQ_GLOBAL_PTR(src), FQ_LDS_PTR(sB + i * 1024), 16, 0, 0);
            }
        } else {
            constexpr int CH = BN / 16;                       // chunks per K-row
            constexpr int RPI = 64 / CH;                      // K-rows per wave instruction
#pragma unroll
            for (int it = 0; it < BK / RPI / NW; ++it) {
                const int i = it * NW + wave;
                const int krow = i * RPI + lane / CH;
                const int c = (lane % CH) ^ swz_kn<CH>(krow);
                const int64_t gk = k0 + krow, gn = n0 + c * 16;
                const uint8_t* src = (gk < K && gn < N) ? g.b + gk * g.ldb + gn : g_zero16;
                __builtin_amdgcn_global_load_lds(FQ_GLOBAL_PTR(src), FQ_LDS_PTR(sB + i * 1024), 16, 0, 0);
            }
        }
    };

    // ---- LDS -> matrix-core operands ----------------------------------------------------------
    // 32x32x64: lane l holds row (l % 32) and the 32 K-bytes [32*(l/32), +32) of the 64-deep slice.
    auto read_kc = [&](const uint8_t* tile, int row, int kh) -> v8i {
        const int cb = kh * 4 + (lane >> 5) * 2;
        const int s = swz_kc(row);
        const uint8_t* base = tile + row * BK;
        const v4i lo = *reinterpret_cast<const v4i*>(base + ((cb ^ s) << 4));
        const v4i hi = *reinterpret_cast<const v4i*>(base + (((cb + 1) ^ s) << 4));
        v8i r;
        r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
        r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
        return r;
    };
    // [K][N] tile: ds_read_b64_tr_b8 works on groups of 16 lanes.  Lane s of a group supplies
    // the address of 8 bytes; lane L receives byte (L % 8) of the eight lanes 2q + (L % 16) / 8.
    // Pointing lane s at K-row (s % 16) / 2, column block 8 * (s % 2) therefore returns to
    // lane L eight consecutive K of column (L % 16): four such reads fill a 32-byte operand.
    auto read_kn = [&](const uint8_t* tile, int ncol_base, int kh) -> v8i {
        constexpr int CH = BN / 16;
        v8i r;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int krow = kh * 64 + (lane >> 5) * 32 + t * 8 + ((lane & 15) >> 1);
            const int ncol = ncol_base + ((lane >> 4) & 1) * 16 + (lane & 1) * 8;
            const uint8_t* p = tile + krow * BN + ((((ncol >> 4) ^ swz_kn<CH>(krow)) << 4) | (ncol & 15));
            const v2i d = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                (v2i __attribute__((address_space(3)))*)(p));
            r[2 * t] = d[0];
            r[2 * t + 1] = d[1];
        }
        return r;
    };

    v16f acc[MB][NB];
#pragma unroll
    for (int mi = 0; mi < MB; ++mi)
#pragma unroll
        for (int ni = 0; ni < NB; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;


    const int KT = static_cast<int>((K + BK - 1) / BK);
    issue_stage(0, 0);
    for (int kt = 0; kt < KT; ++kt) {
        __builtin_amdgcn_s_waitcnt(0);          // this wave's LDS-DMA loads of step kt have landed
        __syncthreads();                         // ... everyone's have, and buffer (kt+1)&1 is free
        if (kt + 1 < KT) issue_stage(kt + 1, (kt + 1) & 1);
        const uint8_t* sA = lds + (kt & 1) * STAGE;
        const uint8_t* sB = sA + A_BYTES;
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            v8i af[MB], bf[NB];
#pragma unroll
            for (int mi = 0; mi < MB; ++mi) af[mi] = read_kc(sA, wm * MB * 32 + mi * 32 + (lane & 31), kh);
#pragma unroll
            for (int ni = 0; ni < NB; ++ni) {
                if (!B_KN) bf[ni] = read_kc(sB, wn * NB * 32 + ni * 32 + (lane & 31), kh);
                else bf[ni] = read_kn(sB, wn * NB * 32 + ni * 32, kh);
            }
#pragma unroll
            for (int mi = 0; mi < MB; ++mi)
#pragma unroll
                for (int ni = 0; ni < NB; ++ni)
                    // weight operand first: the accumulator then holds, per lane, one token row
                    // and runs of four consecutive output columns (wide, row-contiguous stores)
                    acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        bf[ni], af[mi], acc[mi][ni], 0 /* E4M3 */, A_FMT, 0, 0, 0, 0);
        }
    }

    // ---- epilogue: rescale, convert, stage through LDS, split, store ----------------------------
    // Accumulator layout of a 32x32 block (weight operand first): lane l holds token row l % 32;
    // register v holds column 8*(v/4) + 4*(l/32) + v%4 of the block.  One pass per 32-row block
    // index mi: every wave parks its 32 x (NB*32) strip in LDS, then the workgroup streams the
    // WM*32 rows out with 16 bytes per lane, row-contiguous.
    const float inv = 1.0f / ((*g.sa) * (*g.sb));
    const bool f32 = g.c0_is_f32 != 0;
    const int es = f32 ? 4 : 2;
    const int pitch = BN * es + 16;                               // +16 B: rows start on different banks
    float oa_max = 0.0f;
    __syncthreads();                                              // all operand reads are done
#pragma unroll
    for (int mi = 0; mi < MB; ++mi) {
        uint8_t* srow = lds + (wm * 32 + (lane & 31)) * pitch;
#pragma unroll
        for (int ni = 0; ni < NB; ++ni) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = wn * NB * 32 + ni * 32 + q * 8 + (lane >> 5) * 4;
                const float v0 = acc[mi][ni][4 * q] * inv, v1 = acc[mi][ni][4 * q + 1] * inv;
                const float v2 = acc[mi][ni][4 * q + 2] * inv, v3 = acc[mi][ni][4 * q + 3] * inv;
                if (f32) {
                    *reinterpret_cast<float4*>(srow + c * 4) = make_float4(v0, v1, v2, v3);
                } else {
                    uint2 pk;
                    pk.x = bf16_bits_rne(v0) | (static_cast<uint32_t>(bf16_bits_rne(v1)) << 16);
                    pk.y = bf16_bits_rne(v2) | (static_cast<uint32_t>(bf16_bits_rne(v3)) << 16);
                    *reinterpret_cast<uint2*>(srow + c * 2) = pk;
                }
            }
        }
        __syncthreads();
        const int segs_per_row = BN * es / 16;
        const int cols_per_seg = 16 / es;
        for (int sidx = threadIdx.x; sidx < WM * 32 * segs_per_row; sidx += 64 * NW) {
            const int srw = sidx / segs_per_row, seg = sidx - srw * segs_per_row;
            const int64_t row = m0 + (srw >> 5) * (MB * 32) + mi * 32 + (srw & 31);
            const int64_t col = n0 + seg * cols_per_seg;
            if (row < M && col < N) {
                const uint4 d = *reinterpret_cast<const uint4*>(lds + srw * pitch + seg * 16);
                if (col < g.n_split) {
                    *reinterpret_cast<uint4*>(static_cast<uint8_t*>(g.c0) + (row * g.ldc0 + col) * es) = d;
                } else {
                    uint16_t* dst = static_cast<uint16_t*>(g.c1) + row * g.ldc1 + (col - g.n_split);
                    const uint32_t w[4] = {d.x, d.y, d.z, d.w};
                    if (f32) {                                     // four fp32 -> four bf16
                        uint2 pk;
                        const uint16_t b0 = bf16_bits_rne(__uint_as_float(w[0])), b1 = bf16_bits_rne(__uint_as_float(w[1]));
                        const uint16_t b2 = bf16_bits_rne(__uint_as_float(w[2])), b3 = bf16_bits_rne(__uint_as_float(w[3]));
                        pk.x = b0 | (static_cast<uint32_t>(b1) << 16);
                        pk.y = b2 | (static_cast<uint32_t>(b3) << 16);
                        *reinterpret_cast<uint2*>(dst) = pk;
                        oa_max = fmaxf(oa_max, fmaxf(fmaxf(fabsf(__uint_as_float(static_cast<uint32_t>(b0) << 16)),
                                                           fabsf(__uint_as_float(static_cast<uint32_t>(b1) << 16))),
                                                     fmaxf(fabsf(__uint_as_float(static_cast<uint32_t>(b2) << 16)),
                                                           fabsf(__uint_as_float(static_cast<uint32_t>(b3) << 16)))));
                    } else {
                        *reinterpret_cast<uint4*>(dst) = d;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            oa_max = fmaxf(oa_max, fmaxf(fabsf(__uint_as_float(w[e] << 16)),
                                                         fabsf(__uint_as_float(w[e] & 0xffff0000u))));
                    }
                }
            }
        }
        __syncthreads();
    }
    if (g.amax1 && n0 + BN > g.n_split) {
        for (int off = 32; off > 0; off >>= 1) oa_max = fmaxf(oa_max, __shfl_xor(oa_max, off, 64));
        // non-negative floats order like their bit patterns
        if (lane == 0 && oa_max > 0.0f) atomicMax(g.amax1, __float_as_uint(oa_max));
    }
}

template <int WM, int WN, int MB, int NB>
hipError_t launch_cfg(const GemmArgs& g, hipStream_t stream)
{
    constexpr int BM = WM * MB * 32, BN = WN * NB * 32;
    const int tiles_m = static_cast<int>((g.M + BM - 1) / BM), tiles_n = static_cast<int>((g.N + BN - 1) / BN);
    const int total = tiles_m * tiles_n;
    const int chunk = (total + 7) / 8;
    const dim3 grid(static_cast<unsigned>(chunk * 8)), block(64 * WM * WN);
    if (g.b_is_kn) {
        if (g.a_fmt == 0) gemm_fp8_kernel<WM, WN, MB, NB, true, 0><<<grid, block, 0, stream>>>(g, tiles_m, tiles_n, chunk);
        else gemm_fp8_kernel<WM, WN, MB, NB, true, 1><<<grid, block, 0, stream>>>(g, tiles_m, tiles_n, chunk);
    } else {
        if (g.a_fmt == 0) gemm_fp8_kernel<WM, WN, MB, NB, false, 0><<<grid, block, 0, stream>>>(g, tiles_m, tiles_n, chunk);
        else gemm_fp8_kernel<WM, WN, MB, NB, false, 1><<<grid, block, 0, stream>>>(g, tiles_m, tiles_n, chunk);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& g, hipStream_t stream)
{
    if (g.M <= 0 || g.N <= 0) return hipSuccess;
    // Large problems: 256x256 tiles, one workgroup per CU.  Small ones: 128x128 so that more
    // than a handful of CUs take part.
    const int64_t big_tiles = ((g.M + 255) / 256) * ((g.N + 255) / 256);
    if (big_tiles >= 128) return launch_cfg<2, 2, 4, 4>(g, stream);
    return launch_cfg<2, 2, 2, 2>(g, stream);
}

}  // namespace falqon
