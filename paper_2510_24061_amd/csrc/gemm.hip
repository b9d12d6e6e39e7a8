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
//     tiles go HBM/L2 -> LDS with global_load_lds (16 B per lane, no register staging) into
//     rings three (left operand) and two (right operand) stages deep: the fetches of step k+2
//     are issued while step k is multiplied.
//   - global_load_lds writes lanes to consecutive LDS addresses, so the bank-conflict
//     swizzle is applied on the global side: lane -> (row, physical chunk) is fixed, and
//     the lane fetches the logical chunk that belongs there.
//   - The [K,N] operand is read from LDS with ds_read_b64_tr_b8, which hands each lane
//     eight consecutive K for one N: exactly the matrix-core operand layout.
//   - Out-of-range rows and columns are clamped to the last valid one (their products land in
//     outputs that are never stored); the K tail is fetched from a 16-byte block of zeros.
//   - Workgroup ids are spread round-robin over the 8 XCDs by the hardware; the id -> tile
//     map hands each XCD a compact block of tiles so its L2 sees each operand panel once.
#include <type_traits>

#include "db_tile.h"
#include "falqon_internal.h"

namespace falqon {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

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

__device__ __forceinline__ const uint8_t* opaque_uniform(const uint8_t* p)
{
    const uint64_t u = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(u >> 32));
    return reinterpret_cast<const uint8_t*>((static_cast<uint64_t>(hi) << 32) | lo);
}

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits for every
// outstanding global access, which would drain the global_load_lds fetches that are meant to
// stay in flight across the barrier; their completion is awaited explicitly where needed.
__device__ __forceinline__ void barrier_lds_only()
{
    asm volatile("" ::: "memory");               // compiler-level: no LDS access moves across
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
}

// two fp32 -> two bf16 (round to nearest even) in one dword: v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef float v2f __attribute__((ext_vector_type(2)));
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    const v2f f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, v2bf));
}

// ---- side jobs of a 256x256 backbone tile ---------------------------------------------------------
// The adapter's two small products (O_A = x~ A~^T in the forward launch, dB = dy~^T O_A~ in the
// input-gradient launch) are 1.5 % of a step's flops.  Run as tiles of their own before the backbone
// tiles they cost a whole round of latency-bound workgroups, one per CU.  Instead every backbone
// workgroup takes a small share of them BEFORE its own tile, while the accumulation registers are
// still free: the share's operands are fetched straight into LDS together with the tile's first
// stage (so the two memory latencies overlap), multiplied, and written out as an fp32 partial that
// a later pass adds in a fixed order.  The partial's stores then drain, and leave the L2, under the
// tile's main loop; issued at the end of the kernel they would sit in front of its completion.
// LDS: the tile's first stage takes ring slot 0 of each operand; the share's operands take slots 1
// and 2 of the left ring (64 KB) and slot 1 of the right ring (32 KB), which the tile's second
// stage overwrites only after the share is done.
__device__ __forceinline__ void dma16_to_lds(const uint8_t* src, uint8_t* dst_wave_uniform)
{
    __builtin_amdgcn_global_load_lds(FQ_GLOBAL_PTR(src), FQ_LDS_PTR(dst_wave_uniform), 16, 0, 0);
}

// 32x32x64 operand of lane `lane` from a K-contiguous tile (128-byte rows, swizzle swz_kc)
__device__ __forceinline__ v8i read_kc_tile(const uint8_t* tile, int row, int kh, int lane)
{
    const int cb = kh * 4 + (lane >> 5) * 2;
    const int sw = swz_kc(row);
    const uint8_t* base = tile + row * BK;
    const v4i lo = *reinterpret_cast<const v4i*>(base + ((cb ^ sw) << 4));
    const v4i hi = *reinterpret_cast<const v4i*>(base + (((cb + 1) ^ sw) << 4));
    v8i r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return r;
}

// Forward: the tile columns of a tile row are taken in sets of Q (Q = t.row_parts, 1 or 2).  Set s
// < splits covers K-steps [s * steps_per_split, +steps_per_split); member h of the set multiplies
// token rows [h * 256 / Q, +256 / Q) of the tile row with the adapter rows over those K-steps and
// writes them to partial[s][token][rank] (rescaled).  Q = 2 halves the number of partials for the
// same work per workgroup.  LDS chunk: 2 Q K-steps of the 256 / Q token rows (64 KB in lds_x) and
// of up to 64 adapter rows (16 Q KB in lds_a).
static_assert(2 * 64 * BK * 2 <= 32 * 1024, "the adapter rows of a chunk fit one slot of the right ring");

__device__ __forceinline__ bool oa_side_active(const TailArgs& t, int tile_n) { return tile_n / t.row_parts < t.splits; }

template <int Q>
__device__ __forceinline__ void oa_side_fetch(const TailArgs& t, const GemmArgs& g, int64_t m0, int tile_n, int c,
                                              uint8_t* lds_x, uint8_t* lds_a, int wave, int lane)
{
    constexpr int ROWS = 256 / Q, STEPS = 2 * Q;                  // per chunk
    const int KT = static_cast<int>((g.K + BK - 1) / BK);
    const int set = tile_n / Q;
    int s_end = (set + 1) * t.steps_per_split;
    if (s_end > KT) s_end = KT;
    const int s0 = set * t.steps_per_split + c * STEPS;
    const int64_t row0 = m0 + (tile_n % Q) * ROWS;
    const int r = static_cast<int>(t.r);
#pragma unroll
    for (int j = 0; j < STEPS; ++j) {
        if (s0 + j >= s_end) break;
        const int64_t k0 = static_cast<int64_t>(s0 + j) * BK;
#pragma unroll
        for (int it = 0; it < ROWS / 8 / 4; ++it) {               // token rows, 8 per wave instruction
            const int i = it * 4 + wave;
            const int row = i * 8 + (lane >> 3);
            const int64_t gk = k0 + (((lane & 7) ^ swz_kc(row)) << 4);
            int64_t gr = row0 + row;
            if (gr >= g.M) gr = g.M - 1;
            dma16_to_lds(gk < g.K ? g.a + gr * g.lda + gk : g_zero16, lds_x + j * (ROWS * BK) + i * 1024);
        }
#pragma unroll
        for (int it = 0; it < 2; ++it) {                          // 64 adapter rows
            const int i = it * 4 + wave;
            const int row = i * 8 + (lane >> 3);
            const int64_t gk = k0 + (((lane & 7) ^ swz_kc(row)) << 4);
            const int rr = row < r ? row : r - 1;
            dma16_to_lds(gk < g.K ? t.side + rr * g.ldb + gk : g_zero16, lds_a + j * (64 * BK) + i * 1024);
        }
    }
}

// Chunk 0 has been issued by the caller, followed by the fetches of the tile's first stage; every
// further chunk is fetched here.
template <int Q>
__device__ __forceinline__ void oa_side_run(const TailArgs& t, const GemmArgs& g, int64_t m0, int tile_n, float inv,
                                            uint8_t* lds_x, uint8_t* lds_a, int wave, int lane)
{
    constexpr int ROWS = 256 / Q, STEPS = 2 * Q, MI = 4 / Q;      // a wave owns MI blocks of 32 rows and one of 32 ranks
    const int KT = static_cast<int>((g.K + BK - 1) / BK);
    const int set = tile_n / Q;
    const int s_begin = set * t.steps_per_split;
    int s_end = s_begin + t.steps_per_split;
    if (s_end > KT) s_end = KT;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = static_cast<int>(t.r);
    const bool live = wn * 32 < r;                                // wave-uniform: this wave's rank block exists
    v16f acc[MI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][v] = 0.0f;
    auto k_step = [&](int j) {
        const uint8_t* sx = lds_x + j * (ROWS * BK);
        const uint8_t* sa = lds_a + j * (64 * BK);
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            const v8i b = read_kc_tile(sa, wn * 32 + (lane & 31), kh, lane);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const v8i a = read_kc_tile(sx, wm * (MI * 32) + mi * 32 + (lane & 31), kh, lane);
                acc[mi] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b, a, acc[mi], 0, 0, 0, 0, 0, 0);
            }
        }
    };
    for (int c = 0; s_begin + c * STEPS < s_end; ++c) {
        if (c > 0) {
            __syncthreads();                                      // every wave has read the previous chunk
            oa_side_fetch<Q>(t, g, m0, tile_n, c, lds_x, lds_a, wave, lane);
        }
        __builtin_amdgcn_s_waitcnt(0);                            // this chunk (and the tile's first stage) has landed
        __syncthreads();                                          // ... for every wave
        const int steps = s_end - (s_begin + c * STEPS);
        if (live) {
            if (steps >= STEPS) {                                 // unrolled, so that LDS reads run ahead of the MFMAs
#pragma unroll
                for (int j = 0; j < STEPS; ++j) k_step(j);
            } else {
                for (int j = 0; j < steps; ++j) k_step(j);
            }
        }
    }
    if (live) {
        // lane l holds token row l % 32 of each 32-row block and runs of four consecutive ranks
        float* out = t.partial + static_cast<int64_t>(set) * g.M * r;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int64_t row = m0 + (tile_n % Q) * ROWS + wm * (MI * 32) + mi * 32 + (lane & 31);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = wn * 32 + q * 8 + (lane >> 5) * 4;
                if (row < g.M && col < r)
                    *reinterpret_cast<float4*>(out + row * r + col) =
                        make_float4(acc[mi][4 * q] * inv, acc[mi][4 * q + 1] * inv, acc[mi][4 * q + 2] * inv, acc[mi][4 * q + 3] * inv);
            }
        }
    }
    __syncthreads();                                              // the share's LDS reads are done: the tile may overwrite
}

// Input gradient: token tile rows are paired into groups of 512 tokens; the workgroups of a group
// divide the output features (the K dimension of this launch) among themselves in steps of 128.  A
// workgroup multiplies, per feature step, dy~[512 tokens][128 features] with O_A~[512 tokens][rank]
// over the tokens and writes raw sums to partial[group][feature][rank].  Both tiles sit in LDS as
// [token][feature] and are read with the transposing LDS read (dbt::read_tokens_of_feature).
constexpr int kDbTailTokens = 512, kDbTailGroupRows = 2;

struct DbTailGeom { int group, f_begin, f_end; int64_t t0, t_end; };

__device__ __forceinline__ DbTailGeom db_side_geom(const GemmArgs& g, int tile_m, int tile_n, int tiles_m, int tiles_n)
{
    DbTailGeom q;
    q.group = tile_m / kDbTailGroupRows;
    int rows = tiles_m - q.group * kDbTailGroupRows;
    if (rows > kDbTailGroupRows) rows = kDbTailGroupRows;
    const int F = static_cast<int>((g.K + 127) / 128);           // feature steps (K of this launch = m)
    const int W = rows * tiles_n;
    const int per = (F + W - 1) / W;
    const int w = (tile_m - q.group * kDbTailGroupRows) * tiles_n + tile_n;
    q.f_begin = w * per;
    q.f_end = q.f_begin + per < F ? q.f_begin + per : F;
    q.t0 = static_cast<int64_t>(q.group) * kDbTailTokens;
    q.t_end = q.t0 + kDbTailTokens < g.M ? q.t0 + kDbTailTokens : g.M;
    return q;
}

__device__ __forceinline__ void db_side_fetch(const TailArgs& t, const GemmArgs& g, const DbTailGeom& q, int c, bool with_oa,
                                              uint8_t* lds_dy, uint8_t* lds_oa, int wave, int lane)
{
    const int64_t i0 = static_cast<int64_t>(q.f_begin + c) * 128;
#pragma unroll
    for (int it = 0; it < kDbTailTokens / 8 / 4; ++it) {         // dy~: 8 token rows of 128 bytes per wave instruction
        const int i = it * 4 + wave;
        const int trow = i * 8 + (lane >> 3);
        const int64_t gt = q.t0 + trow, gi = i0 + (((lane & 7) ^ dbt::swz_t<8>(trow)) << 4);
        dma16_to_lds((gt < q.t_end && gi < g.K) ? g.a + gt * g.lda + gi : g_zero16, lds_dy + i * 1024);
    }
    if (!with_oa) return;
    const int64_t r = t.r;
#pragma unroll
    for (int it = 0; it < kDbTailTokens / 16 / 4; ++it) {        // O_A~: 16 token rows of 64 bytes per wave instruction
        const int i = it * 4 + wave;
        const int trow = i * 16 + (lane >> 2);
        const int64_t gt = q.t0 + trow, gp = ((lane & 3) ^ dbt::swz_t<4>(trow)) << 4;
        dma16_to_lds((gt < q.t_end && gp < r) ? t.side + gt * r + gp : g_zero16, lds_oa + i * 1024);
    }
}

// Step 0 (with O_A~) has been issued by the caller, followed by the tile's first stage.
__device__ __forceinline__ void db_side_run(const TailArgs& t, const GemmArgs& g, const DbTailGeom& q,
                                            uint8_t* lds_dy, uint8_t* lds_oa, int wave, int lane)
{
    const int64_t m = g.K, r = t.r;
    const int k_blocks = static_cast<int>((q.t_end - q.t0 + 63) / 64);
    float* out = t.partial + static_cast<int64_t>(q.group) * m * r;
    for (int c = 0; q.f_begin + c < q.f_end; ++c) {
        if (c > 0) {
            __syncthreads();                                      // every wave has read the previous feature step
            db_side_fetch(t, g, q, c, false, lds_dy, lds_oa, wave, lane);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        dbt::v16f acc[2];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][v] = 0.0f;
        // wave w owns features [32 w, 32 w + 32) of the step and both 32-wide rank blocks
        auto k_block = [&](int kb) {
            const dbt::v8i a = dbt::read_tokens_of_feature<8>(lds_dy, wave * 32, kb, lane);
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                if (b * 32 >= r) continue;
                const dbt::v8i bb = dbt::read_tokens_of_feature<4>(lds_oa, b * 32, kb, lane);
                acc[b] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, bb, acc[b], 1 /* E5M2 */, 0 /* E4M3 */, 0, 0, 0, 0);
            }
        };
        if (k_blocks == kDbTailTokens / 64) {                     // a full group: unrolled, so that LDS reads run ahead
#pragma unroll
            for (int kb = 0; kb < kDbTailTokens / 64; ++kb) k_block(kb);
        } else {
            for (int kb = 0; kb < k_blocks; ++kb) k_block(kb);
        }
        const int64_t i0 = static_cast<int64_t>(q.f_begin + c) * 128 + wave * 32;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int64_t p = b * 32 + (lane & 31);
            if (p >= r) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t i = i0 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                if (i < m) out[i * r + p] = acc[b][v];
            }
        }
    }
    __syncthreads();                                              // the share's LDS reads are done: the tile may overwrite
}

// LDS of one workgroup: operand rings, the left operand three stages deep, the right operand two
// (160 KB at 256x256).
template <int WM, int WN, int MB, int NB>
constexpr int gemm_lds_bytes() { return (3 * WM * MB + 2 * WN * NB) * 32 * BK; }

// One output tile.  `bid` is the workgroup's index in a grid of 8 * chunk workgroups whose index
// modulo 8 is the XCD it runs on, `split` its K split; `lds` is gemm_lds_bytes() of LDS, 1 KB aligned.
// TAIL selects what the workgroup does for the adapter besides its tile: 0 nothing; 1 a K slice of
// the adapter product O_A as a side job ahead of the tile (forward); 2 a slice of the adapter
// gradient dB as a side job ahead of the tile (input-gradient launch); 3, 4, 5: blocks of O_A formed
// inside the tile's own K-steps, one, two or four per wave, finished and written as bf16 with their
// maximum (forward).
template <int WM, int WN, int MB, int NB, bool B_KN, int A_FMT, int TAIL = 0>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, const int tiles_m, const int tiles_n, const int chunk,
                                          const int bid, const int split, uint8_t* const lds,
                                          const TailArgs* const tail = nullptr)
{
    static_assert(TAIL == 0 || (WM == 2 && WN == 2 && MB == 4 && NB == 4), "side jobs ride on the 256x256 tile only");
    static_assert((TAIL != 1 && TAIL != 3 && TAIL != 4 && TAIL != 5) || (!B_KN && A_FMT == 0), "the adapter product belongs to the forward product");
    static_assert(TAIL != 2 || (B_KN && A_FMT == 1), "the dB slice belongs to the input-gradient product");
    constexpr int BM = WM * MB * 32, BN = WN * NB * 32, NW = WM * WN;
    constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK;
    static_assert((BM / 8) % NW == 0 && (B_BYTES / 1024) % NW == 0, "loads must split evenly over waves");
    uint8_t* const lds_b = lds + 3 * A_BYTES;

    // ---- workgroup -> tile (XCD aware) ----------------------------------------------------
    // Hardware places workgroup b on XCD b % 8.  XCD x takes tiles [x*chunk, (x+1)*chunk) of a
    // raster that walks panels of 4 tile-rows, tile-column by tile-column.
    const int xcd = bid & 7, slot = bid >> 3;
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
    const int64_t M = g.M, N = g.N;
    // Split K: split `split` multiplies the K range [kbeg, kbeg + K) only and writes
    // its own copy of the output (fp32 partials, summed by a later pass).
    const int64_t kbeg = static_cast<int64_t>(split) * g.k_per_split;
    const int64_t K = (g.K - kbeg) < g.k_per_split ? (g.K - kbeg > 0 ? g.K - kbeg : 0) : g.k_per_split;
    const uint8_t* const ga = g.a + kbeg;
    const uint8_t* const gb = B_KN ? g.b + kbeg * g.ldb : g.b + kbeg;
    uint8_t* const c0p = static_cast<uint8_t*>(g.c0) +
                         static_cast<int64_t>(split) * M * g.ldc0 * (g.c0_is_f32 ? 4 : 2);
    // rescale factor: read here, where the two loads hide under the first operand fetches, and kept in
    // a scalar register (read at the top of the epilogue they cost every tile a memory round trip)
    const float inv = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(1.0f / ((*g.sa) * (*g.sb)))));

    // ---- global -> LDS ----------------------------------------------------------------------
    // Fast path (every K-step that lies fully inside K): address = uniform base + 32-bit lane
    // offset.  The lane offsets never change; only the scalar base advances with K.  Rows and
    // columns beyond the matrix are clamped to the last valid one: they load real bytes whose
    // products land in output elements that are never stored.  The K tail cannot be clamped
    // (it would add foreign terms to valid outputs); its step fetches out-of-range chunks from
    // a block of zeros instead (slow path, at most one step per tile).
    constexpr int IT_A = BM / 8 / NW, IT_B = B_BYTES / 1024 / NW;
    constexpr int CH = BN / 16;                               // [K][N] tile: chunks per K-row
    constexpr int RPI = 64 / CH;                              // [K][N] tile: K-rows per wave instruction
    const int rows_a = static_cast<int>((M - m0) < BM ? (M - m0) : BM);
    const int rows_b = static_cast<int>((N - n0) < BN ? (N - n0) : BN);   // rows of [N,K] / columns of [K,N]
    uint32_t off_a[IT_A], off_b[IT_B];
#pragma unroll
    for (int it = 0; it < IT_A; ++it) {
        const int row = (it * NW + wave) * 8 + (lane >> 3);
        const int c = (lane & 7) ^ swz_kc(row);
        const int rr = row < rows_a ? row : rows_a - 1;
        off_a[it] = static_cast<uint32_t>(rr) * static_cast<uint32_t>(g.lda) + c * 16;
    }
#pragma unroll
    for (int it = 0; it < IT_B; ++it) {
        if (!B_KN) {
            const int row = (it * NW + wave) * 8 + (lane >> 3);
            const int c = (lane & 7) ^ swz_kc(row);
            const int rr = row < rows_b ? row : rows_b - 1;
            off_b[it] = static_cast<uint32_t>(rr) * static_cast<uint32_t>(g.ldb) + c * 16;
        } else {
            const int krow = (it * NW + wave) * RPI + lane / CH;
            int c = (lane % CH) ^ swz_kn<CH>(krow);
            c = c * 16 < rows_b ? c : rows_b / 16 - 1;
            off_b[it] = static_cast<uint32_t>(krow) * static_cast<uint32_t>(g.ldb) + c * 16;
        }
    }
    const uint8_t* base_a = ga + m0 * g.lda;
    const uint8_t* base_b = B_KN ? gb + n0 : gb + n0 * g.ldb;
    const int64_t kstep_b = B_KN ? static_cast<int64_t>(BK) * g.ldb : BK;

    auto dma16 = [&](const uint8_t* src, uint8_t* dst_wave_uniform) {
        __builtin_amdgcn_global_load_lds(FQ_GLOBAL_PTR(src), FQ_LDS_PTR(dst_wave_uniform), 16, 0, 0);
    };
    // One 1 KB fetch of a stage that lies fully inside K (scalar base, opaque so that the lane
    // offset stays a separate 32-bit term).
    auto fetch_a_one = [&](const uint8_t* pa, uint8_t* dst, int j) { dma16(pa + off_a[j], dst + (j * NW + wave) * 1024); };
    auto fetch_b_one = [&](const uint8_t* pb, uint8_t* dst, int j) { dma16(pb + off_b[j], dst + (j * NW + wave) * 1024); };
    // All IT_A (IT_B) fetches of one operand tile of stage s, back to back: prologue and K tail.
    auto fetch_a_all = [&](int s, uint8_t* dst) {
        const int64_t k0 = static_cast<int64_t>(s) * BK;
        if (k0 + BK <= K) {
            const uint8_t* pa = opaque_uniform(base_a + k0);
#pragma unroll
            for (int it = 0; it < IT_A; ++it) fetch_a_one(pa, dst, it);
            return;
        }
#pragma unroll
        for (int it = 0; it < IT_A; ++it) {
            const int i = it * NW + wave;                     // 1 KB = 8 rows per wave instruction
            const int row = i * 8 + (lane >> 3);
            const int c = (lane & 7) ^ swz_kc(row);
            const int64_t gr = m0 + row, gk = k0 + c * 16;
            dma16((gr < M && gk < K) ? ga + gr * g.lda + gk : g_zero16, dst + i * 1024);
        }
    };
    auto fetch_b_all = [&](int s, uint8_t* dst) {
        const int64_t k0 = static_cast<int64_t>(s) * BK;
        if (k0 + BK <= K) {
            const uint8_t* pb = opaque_uniform(base_b + s * kstep_b);
#pragma unroll
            for (int it = 0; it < IT_B; ++it) fetch_b_one(pb, dst, it);
            return;
        }
#pragma unroll
        for (int it = 0; it < IT_B; ++it) {
            const int i = it * NW + wave;
            const uint8_t* src;
            if (!B_KN) {
                const int row = i * 8 + (lane >> 3);
                const int c = (lane & 7) ^ swz_kc(row);
                const int64_t gr = n0 + row, gk = k0 + c * 16;
                src = (gr < N && gk < K) ? gb + gr * g.ldb + gk : g_zero16;
            } else {
                const int krow = i * RPI + lane / CH;
                const int c = (lane % CH) ^ swz_kn<CH>(krow);
                const int64_t gk = k0 + krow, gn = n0 + c * 16;
                src = (gk < K && gn < N) ? gb + gk * g.ldb + gn : g_zero16;
            }
            dma16(src, dst + i * 1024);
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
    // The read is written as inline assembly: through the builtin the compiler cannot tell that
    // it does not touch the LDS slots that in-flight global_load_lds fetches are filling, and
    // makes every such read wait for all of them.  The price is that the compiler no longer
    // tracks its completion either: every consumer below is preceded by an explicit
    // s_waitcnt lgkmcnt(0).
    auto read_kn = [&](const uint8_t* tile, int ncol_base, int kh) -> v8i {
        v8i r;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int krow = kh * 64 + (lane >> 5) * 32 + t * 8 + ((lane & 15) >> 1);
            const int ncol = ncol_base + ((lane >> 4) & 1) * 16 + (lane & 1) * 8;
            const uint8_t* p = tile + krow * BN + ((((ncol >> 4) ^ swz_kn<CH>(krow)) << 4) | (ncol & 15));
            const uint32_t addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(FQ_LDS_PTR(p)));
            v2i d;
            asm volatile("ds_read_b64_tr_b8 %0, %1" : "=v"(d) : "v"(addr));
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
    // ---- main loop, software pipelined across K-steps -------------------------------------------
    // Step k multiplies stage k in two 64-deep halves.  A stage's left tile sits in ring slot
    // k % 3, its right tile in slot k % 2.
    //   half 0: MFMAs on operands already in registers.  Under them: read half 1's operands from
    //           LDS; fetch the LEFT tile of stage k+2 (its slot was last read in step k-1).
    //   wait until everything but those newest fetches has landed (stage k+1 is complete), barrier:
    //           now no wave reads the right tile of stage k any more.
    //   half 1: MFMAs.  Under them: fetch the RIGHT tile of stage k+2 into the slot just freed;
    //           read half 0's operands of stage k+1.
    // Fetches are spread one per MFMA: a wave that issues them back to back stalls on the CU's
    // 64 B/clk vector-memory path while the matrix core drains.  Left-tile fetches have a step and
    // a half to land, right-tile fetches a full half-step after the last one is issued.  The
    // barrier is reached with MFMAs still in flight, and no LDS latency is exposed.
    auto read_a = [&](const uint8_t* sA, int mi, int kh) -> v8i {
        return read_kc(sA, wm * MB * 32 + mi * 32 + (lane & 31), kh);
    };
    auto read_b = [&](const uint8_t* sB, int ni, int kh) -> v8i {
        if (!B_KN) return read_kc(sB, wn * NB * 32 + ni * 32 + (lane & 31), kh);
        return read_kn(sB, wn * NB * 32 + ni * 32, kh);
    };
    constexpr int N_MFMA = MB * NB, N_FRAG = MB + NB;
    constexpr int A_PER_SLOT = (IT_A + N_MFMA - 1) / N_MFMA, B_PER_SLOT = (IT_B + N_MFMA - 1) / N_MFMA;
    constexpr int FRAGS_PER_SLOT = (N_FRAG + N_MFMA - 1) / N_MFMA;
    // s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] | expcnt << 4 | lgkmcnt << 8 | vmcnt[5:4] << 14)
    constexpr int WAIT_ALL = 0;
    constexpr int WAIT_LDS = 0xC07F;                                                            // lgkmcnt 0 only
    constexpr int WAIT_BUT_A = (IT_A & 15) | (7 << 4) | ((IT_A >> 4) << 14);                    // lgkmcnt 0
    constexpr int WAIT_BUT_STAGE = ((IT_A + IT_B) & 15) | (7 << 4) | (((IT_A + IT_B) >> 4) << 14);

    v8i af[2][MB], bf[2][NB];
    // read fragment f (right-operand fragments first) of half kh from a stage
    auto read_frag = [&](const uint8_t* sA, const uint8_t* sB, int kh, int f) {
        if (f < NB) bf[kh][f] = read_b(sB, f, kh);
        else if (f < N_FRAG) af[kh][f - NB] = read_a(sA, f - NB, kh);
    };

    // ---- adapter product riding on the tile's own K-steps (TAIL == 3, 4) -------------------------
    // O_A of a tile row is 16 blocks of 16 token rows by r / 16 blocks of 16 ranks.  Wave w of tile
    // column c takes, of token rows [16 (u % 16), +16) of the tile row, u = 4 c + w, the RB rank
    // blocks from RB (u / 16) on (RB = 1, 2, 4 for TAIL == 3, 4, 5), over all of K.  Its token
    // operand is read from the left tile that sits in LDS for the tile's own product, its adapter
    // operands straight from memory one step ahead; RB 16x16x128 MFMAs per K-step and no partial
    // results.  Waves without a block run the same instructions on clamped rows and store nothing, so
    // the loop carries no branch for it.
    constexpr bool RIDE = TAIL == 3 || TAIL == 4 || TAIL == 5;
    constexpr int RB = TAIL == 5 ? 4 : TAIL == 4 ? 2 : 1;
    v4f accx[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j) accx[j] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
    float ride_max = 0.0f;
    v8i sb[RB];
    const int ride_u = tile_n * NW + wave;
    const int ride_row = (ride_u & 15) * 16 + (lane & 15);     // row of the left tile
    const int ride_blk0 = (ride_u >> 4) * RB;                  // first rank block of the wave
    // adapter operand of stage s: lane part of the address, and the wave's rank blocks (a block
    // beyond the rank is clamped to the last one)
    const uint8_t* ride_src = nullptr;
    int64_t ride_off[RB];
    if constexpr (RIDE) {
        const int nblk = static_cast<int>(tail->r) / 16;
        ride_src = tail->side + static_cast<int64_t>(lane & 15) * g.ldb + (lane >> 4) * 32;
#pragma unroll
        for (int j = 0; j < RB; ++j)
            ride_off[j] = static_cast<int64_t>(ride_blk0 + j < nblk ? ride_blk0 + j : nblk - 1) * 16 * g.ldb;
    }
    // `inside`: the stage lies fully inside K (otherwise chunks beyond K are zeros)
    auto ride_load = [&](int s, bool inside) {
        const int64_t gk = static_cast<int64_t>(s) * BK + (lane >> 4) * 32;
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            const uint8_t* p = ride_src + ride_off[j] + static_cast<int64_t>(s) * BK;
            const v4i lo = *reinterpret_cast<const v4i*>(inside || gk < g.K ? p : g_zero16);
            const v4i hi = *reinterpret_cast<const v4i*>(inside || gk + 16 < g.K ? p + 16 : g_zero16);
            sb[j][0] = lo[0]; sb[j][1] = lo[1]; sb[j][2] = lo[2]; sb[j][3] = lo[3];
            sb[j][4] = hi[0]; sb[j][5] = hi[1]; sb[j][6] = hi[2]; sb[j][7] = hi[3];
        }
    };
    auto ride_read = [&](const uint8_t* tile) -> v8i {         // lane l: row l % 16, K bytes [32 (l / 16), +32)
        const int cb = (lane >> 4) * 2;
        const int sw = swz_kc(ride_row);
        const uint8_t* base = tile + ride_row * BK;
        const v4i lo = *reinterpret_cast<const v4i*>(base + ((cb ^ sw) << 4));
        const v4i hi = *reinterpret_cast<const v4i*>(base + (((cb + 1) ^ sw) << 4));
        v8i x;
        x[0] = lo[0]; x[1] = lo[1]; x[2] = lo[2]; x[3] = lo[3];
        x[4] = hi[0]; x[5] = hi[1]; x[6] = hi[2]; x[7] = hi[3];
        return x;
    };
    v8i xa;
    // Written as assembly with the accumulator in ordinary vector registers: through the builtin it
    // is placed among the tile's accumulation registers, which the compiler then moves about in every
    // K-step.  (Both operands E4M3; the result is next read a whole K-step later.)
    auto ride_mfma = [&]() {
#pragma unroll
        for (int j = 0; j < RB; ++j)
            asm volatile("v_mfma_f32_16x16x128_f8f6f4 %0, %1, %2, %0" : "+v"(accx[j]) : "v"(sb[j]), "v"(xa));
    };
    if constexpr (RIDE) ride_load(0, false);

    // The side job's first operand fetches go out ahead of the tile's first stage; the job itself
    // runs while that stage is in flight or has landed, and ends with a barrier, after which the
    // second stage may overwrite the ring slots it used.
    if constexpr (TAIL == 1) {
        if (oa_side_active(*tail, tile_n)) {
            if (tail->row_parts == 2) oa_side_fetch<2>(*tail, g, m0, tile_n, 0, lds + A_BYTES, lds_b + B_BYTES, wave, lane);
            else oa_side_fetch<1>(*tail, g, m0, tile_n, 0, lds + A_BYTES, lds_b + B_BYTES, wave, lane);
            fetch_a_all(0, lds);
            fetch_b_all(0, lds_b);
            if (tail->row_parts == 2) oa_side_run<2>(*tail, g, m0, tile_n, inv, lds + A_BYTES, lds_b + B_BYTES, wave, lane);
            else oa_side_run<1>(*tail, g, m0, tile_n, inv, lds + A_BYTES, lds_b + B_BYTES, wave, lane);
        } else {
            fetch_a_all(0, lds);
            fetch_b_all(0, lds_b);
        }
    } else if constexpr (TAIL == 2) {
        const DbTailGeom q = db_side_geom(g, tile_m, tile_n, tiles_m, tiles_n);
        if (q.f_begin < q.f_end) {
            db_side_fetch(*tail, g, q, 0, true, lds + A_BYTES, lds_b + B_BYTES, wave, lane);
            fetch_a_all(0, lds);
            fetch_b_all(0, lds_b);
            db_side_run(*tail, g, q, lds + A_BYTES, lds_b + B_BYTES, wave, lane);
        } else {
            fetch_a_all(0, lds);
            fetch_b_all(0, lds_b);
        }
    } else {
        fetch_a_all(0, lds);
        fetch_b_all(0, lds_b);
    }
    if (KT > 1) {
        fetch_a_all(1, lds + A_BYTES);
        fetch_b_all(1, lds_b + B_BYTES);
        __builtin_amdgcn_s_waitcnt(WAIT_BUT_STAGE);           // stage 0 has landed
    } else {
        __builtin_amdgcn_s_waitcnt(WAIT_ALL);
    }
    barrier_lds_only();
#pragma unroll
    for (int f = 0; f < N_FRAG; ++f) read_frag(lds, lds_b, 0, f);
    if constexpr (RIDE) {
        xa = ride_read(lds);
        ride_mfma();
        if (KT > 1) ride_load(1, false);
    }
    __builtin_amdgcn_s_waitcnt(WAIT_LDS);

    int ia = 0;                                               // ring slot of stage kt's left tile
    // One K-step.  STEADY = true is the body for steps whose stage k+2 exists and lies fully inside
    // K: every "is there a next stage" test is resolved at compile time, so the steady-state loop
    // carries no branches between its MFMAs.
    auto k_step = [&](int kt, auto steady_tag) {
        constexpr bool STEADY = decltype(steady_tag)::value;
        const int ia1 = ia == 2 ? 0 : ia + 1, ia2 = ia1 == 2 ? 0 : ia1 + 1;
        const uint8_t* sA = lds + ia * A_BYTES;
        const uint8_t* sB = lds_b + (kt & 1) * B_BYTES;
        uint8_t* nA = lds + ia2 * A_BYTES;                     // destination of stage k+2, left
        uint8_t* nB = lds_b + (kt & 1) * B_BYTES;              // destination of stage k+2, right
        const bool fetch = STEADY || kt + 2 < KT;
        const bool fast = STEADY || (fetch && (static_cast<int64_t>(kt + 3) * BK <= K));
        const bool next = STEADY || kt + 1 < KT;
        const uint8_t* pa = opaque_uniform(base_a + static_cast<int64_t>(kt + 2) * BK);
        const uint8_t* pb = opaque_uniform(base_b + (kt + 2) * kstep_b);
        // ---- half 0 ----
        if (!STEADY && fetch && !fast) fetch_a_all(kt + 2, nA); // K tail: zero-filled slow path
#pragma unroll
        for (int mi = 0; mi < MB; ++mi) {
#pragma unroll
            for (int ni = 0; ni < NB; ++ni) {
                const int q = mi * NB + ni;
                // weight operand first: the accumulator then holds, per lane, one token row
                // and runs of four consecutive output columns (wide, row-contiguous stores)
                acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                    bf[0][ni], af[0][mi], acc[mi][ni], 0 /* E4M3 */, A_FMT, 0, 0, 0, 0);
                if (STEADY || fast) {
#pragma unroll
                    for (int u = 0; u < A_PER_SLOT; ++u)
                        if (q * A_PER_SLOT + u < IT_A) fetch_a_one(pa, nA, q * A_PER_SLOT + u);
                }
#pragma unroll
                for (int u = 0; u < FRAGS_PER_SLOT; ++u) read_frag(sA, sB, 1, q * FRAGS_PER_SLOT + u);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // half 1's operands are in registers and stage k+1 has landed (only the left-tile fetches
        // of stage k+2, issued last, may still be in flight)
        if (STEADY || fetch) __builtin_amdgcn_s_waitcnt(WAIT_BUT_A);
        else __builtin_amdgcn_s_waitcnt(WAIT_ALL);
        barrier_lds_only();                                    // ... for every wave
        // ---- half 1 ----
        const uint8_t* tA = lds + ia1 * A_BYTES;                // stage k+1
        const uint8_t* tB = lds_b + ((kt + 1) & 1) * B_BYTES;
        if (!STEADY && fetch && !fast) fetch_b_all(kt + 2, nB);
#pragma unroll
        for (int mi = 0; mi < MB; ++mi) {
#pragma unroll
            for (int ni = 0; ni < NB; ++ni) {
                const int q = mi * NB + ni;
                if (RIDE && (STEADY || next)) {                    // the adapter product's share of stage k+1
                    if (q == N_FRAG) xa = ride_read(tA);           // behind the reads of the next half-step's operands
                    if (q == N_FRAG + 4) {
                        ride_mfma();
                        if (STEADY || fetch) ride_load(kt + 2, STEADY);
                    }
                }
                acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                    bf[1][ni], af[1][mi], acc[mi][ni], 0 /* E4M3 */, A_FMT, 0, 0, 0, 0);
                if (STEADY || fast) {
#pragma unroll
                    for (int u = 0; u < B_PER_SLOT; ++u)
                        if (q * B_PER_SLOT + u < IT_B) fetch_b_one(pb, nB, q * B_PER_SLOT + u);
                }
                if (STEADY || next) {
#pragma unroll
                    for (int u = 0; u < FRAGS_PER_SLOT; ++u) read_frag(tA, tB, 0, q * FRAGS_PER_SLOT + u);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __builtin_amdgcn_s_waitcnt(WAIT_LDS);                 // next half 0's operands are in registers
        ia = ia1;
    };
    const int steady_steps = static_cast<int>(K / BK) - 2;     // steps whose stage k+2 is a full stage
    int kt = 0;
    for (; kt < steady_steps; ++kt) k_step(kt, std::true_type{});
    for (; kt < KT; ++kt) k_step(kt, std::false_type{});
    __builtin_amdgcn_s_waitcnt(WAIT_ALL);
    if constexpr (RIDE) {
        // lane l holds token row l % 16 of the block and ranks [4 (l / 16), +4)
        const int r = static_cast<int>(tail->r);
        const int64_t row = m0 + (ride_u & 15) * 16 + (lane & 15);
#pragma unroll
        for (int j = 0; j < RB; ++j) {
            const int col = (ride_blk0 + j) * 16 + (lane >> 4) * 4;
            if (row < M && col < r) {
                uint2 pk;
                pk.x = pack_bf16x2(accx[j][0] * inv, accx[j][1] * inv);
                pk.y = pack_bf16x2(accx[j][2] * inv, accx[j][3] * inv);
                *reinterpret_cast<uint2*>(static_cast<uint16_t*>(g.c1) + row * g.ldc1 + col) = pk;
                ride_max = fmaxf(ride_max,
                                 fmaxf(fmaxf(fabsf(__uint_as_float(pk.x << 16)), fabsf(__uint_as_float(pk.x & 0xffff0000u))),
                                       fmaxf(fabsf(__uint_as_float(pk.y << 16)), fabsf(__uint_as_float(pk.y & 0xffff0000u)))));
            }
        }
        for (int off = 32; off > 0; off >>= 1) ride_max = fmaxf(ride_max, __shfl_xor(ride_max, off, 64));
    }

    // ---- epilogue: rescale, convert, stage through LDS, split, store ----------------------------
    // Accumulator layout of a 32x32 block (weight operand first): lane l holds token row l % 32;
    // register v holds column 8*(v/4) + 4*(l/32) + v%4 of the block.  One pass per 32-row block
    // index mi: every wave parks its 32 x (NB*32) strip in LDS, then the workgroup streams the
    // WM*32 rows out with 16 bytes per lane, row-contiguous.
    float oa_max = 0.0f;
    __syncthreads();                                              // all operand reads are done
    // the waves' maxima of |O_A| meet in the last bytes of the rings, beyond the staging rows
    float* const ride_max_slot = reinterpret_cast<float*>(lds + gemm_lds_bytes<WM, WN, MB, NB>() - 64);
    if constexpr (RIDE) {
        if (lane == 0) ride_max_slot[wave] = ride_max;
    }
    // the output type is a run-time argument; each of the two bodies is compiled with it fixed
    auto epilogue = [&](auto is_f32) {
        constexpr bool F32 = decltype(is_f32)::value;
        constexpr int ES = F32 ? 4 : 2;
        constexpr int PITCH = BN * ES + 16;                       // +16 B: rows start on different banks
        constexpr int SEGS = BN * ES / 16, COLS_PER_SEG = 16 / ES;
#pragma unroll
        for (int mi = 0; mi < MB; ++mi) {
            uint8_t* srow = lds + (wm * 32 + (lane & 31)) * PITCH;
#pragma unroll
            for (int ni = 0; ni < NB; ++ni) {
                // One block at a time leaves the accumulation registers (the empty asm pins the copy
                // here; left to itself the compiler moves all 256 up front and spills).
                v16f t = acc[mi][ni];
                asm volatile("" : "+v"(t));
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c = wn * NB * 32 + ni * 32 + q * 8 + (lane >> 5) * 4;
                    const float v0 = t[4 * q] * inv, v1 = t[4 * q + 1] * inv;
                    const float v2 = t[4 * q + 2] * inv, v3 = t[4 * q + 3] * inv;
                    if (F32) {
                        *reinterpret_cast<float4*>(srow + c * 4) = make_float4(v0, v1, v2, v3);
                    } else {
                        uint2 pk;
                        pk.x = pack_bf16x2(v0, v1);
                        pk.y = pack_bf16x2(v2, v3);
                        *reinterpret_cast<uint2*>(srow + c * 2) = pk;
                    }
                }
            }
            __syncthreads();
#pragma unroll
            for (int it = 0; it < WM * 32 * SEGS / (64 * NW); ++it) {
                const int sidx = it * 64 * NW + threadIdx.x;
                const int srw = sidx / SEGS, seg = sidx % SEGS;
                const int64_t row = m0 + (srw >> 5) * (MB * 32) + mi * 32 + (srw & 31);
                const int64_t col = n0 + seg * COLS_PER_SEG;
                if (row < M && col < N) {
                    const uint4 d = *reinterpret_cast<const uint4*>(lds + srw * PITCH + seg * 16);
                    if (col < g.n_split) {
                        // streaming store: every workgroup writes 512-byte row segments of its tile at
                        // the same time; the output is not read again by this layer
                        typedef unsigned v4u __attribute__((ext_vector_type(4)));
                        const v4u dd = {d.x, d.y, d.z, d.w};
                        __builtin_nontemporal_store(dd, reinterpret_cast<v4u*>(c0p + (row * g.ldc0 + col) * ES));
                    } else {
                        uint16_t* dst = static_cast<uint16_t*>(g.c1) + row * g.ldc1 + (col - g.n_split);
                        const uint32_t w[4] = {d.x, d.y, d.z, d.w};
                        if (F32) {                                 // four fp32 -> four bf16
                            uint2 pk;
                            pk.x = pack_bf16x2(__uint_as_float(w[0]), __uint_as_float(w[1]));
                            pk.y = pack_bf16x2(__uint_as_float(w[2]), __uint_as_float(w[3]));
                            *reinterpret_cast<uint2*>(dst) = pk;
                            oa_max = fmaxf(oa_max, fmaxf(fmaxf(fabsf(__uint_as_float(pk.x << 16)),
                                                               fabsf(__uint_as_float(pk.x & 0xffff0000u))),
                                                         fmaxf(fabsf(__uint_as_float(pk.y << 16)),
                                                               fabsf(__uint_as_float(pk.y & 0xffff0000u)))));
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
    };
    if (g.c0_is_f32) epilogue(std::true_type{});
    else epilogue(std::false_type{});
    if constexpr (RIDE) {                                         // (the epilogue ends with a barrier)
        if (g.amax1 && threadIdx.x == 0) {
            float mx = ride_max_slot[0];
            for (int w = 1; w < NW; ++w) mx = fmaxf(mx, ride_max_slot[w]);
            if (mx > 0.0f) atomicMax(g.amax1, __float_as_uint(mx));
        }
    }
    if (g.amax1 && n0 + BN > g.n_split) {
        for (int off = 32; off > 0; off >>= 1) oa_max = fmaxf(oa_max, __shfl_xor(oa_max, off, 64));
        // non-negative floats order like their bit patterns
        if (lane == 0 && oa_max > 0.0f) atomicMax(g.amax1, __float_as_uint(oa_max));
    }
}

template <int WM, int WN, int MB, int NB, bool B_KN, int A_FMT>
__global__ void __launch_bounds__(64 * WM * WN)
gemm_fp8_kernel(const GemmArgs g, const int tiles_m, const int tiles_n, const int chunk)
{
    __shared__ __attribute__((aligned(1024))) uint8_t lds[gemm_lds_bytes<WM, WN, MB, NB>()];
    gemm_tile<WM, WN, MB, NB, B_KN, A_FMT>(g, tiles_m, tiles_n, chunk, blockIdx.x, blockIdx.y, lds);
}

// The backbone product with the adapter's share as a side job of every tile (TailArgs).
__global__ void __launch_bounds__(256)
gemm_fwd_tail_kernel(const GemmArgs g, const int tiles_m, const int tiles_n, const int chunk, const TailArgs t)
{
    __shared__ __attribute__((aligned(1024))) uint8_t lds[gemm_lds_bytes<2, 2, 4, 4>()];
    gemm_tile<2, 2, 4, 4, false, 0, 1>(g, tiles_m, tiles_n, chunk, blockIdx.x, 0, lds, &t);
}

// The same product with the adapter product riding on the K-steps of the tiles themselves: writes
// O_A (bf16) and its running maximum, no partial results.
template <int RB>
__global__ void __launch_bounds__(256)
gemm_fwd_ride_kernel(const GemmArgs g, const int tiles_m, const int tiles_n, const int chunk, const TailArgs t)
{
    __shared__ __attribute__((aligned(1024))) uint8_t lds[gemm_lds_bytes<2, 2, 4, 4>()];
    gemm_tile<2, 2, 4, 4, false, 0, RB == 4 ? 5 : RB == 2 ? 4 : 3>(g, tiles_m, tiles_n, chunk, blockIdx.x, 0, lds, &t);
}

__global__ void __launch_bounds__(256)
gemm_dx_tail_kernel(const GemmArgs g, const int tiles_m, const int tiles_n, const int chunk, const TailArgs t)
{
    __shared__ __attribute__((aligned(1024))) uint8_t lds[gemm_lds_bytes<2, 2, 4, 4>()];
    gemm_tile<2, 2, 4, 4, true, 1, 2>(g, tiles_m, tiles_n, chunk, blockIdx.x, 0, lds, &t);
}

// Forward product and the adapter's split-K product in one launch.  Both read only x~ and the
// concatenated weight, so nothing orders them; as two launches the second costs a dispatch, a
// ramp-up and a drain of its own (about 4 us on this chip) on top of its few microseconds of work.
// The first n_side workgroups take the adapter tiles (128x128, K split), the rest the backbone
// tiles (256x256); n_side is a multiple of 8, so workgroup index modulo 8 is still the XCD.
__global__ void __launch_bounds__(256)
gemm_fwd_pair_kernel(const GemmArgs g, const int tiles_m, const int tiles_n, const int chunk,
                     const GemmArgs h, const int h_tiles_m, const int h_tiles_n, const int h_chunk, const int n_side)
{
    __shared__ __attribute__((aligned(1024))) uint8_t lds[gemm_lds_bytes<2, 2, 4, 4>()];
    static_assert(gemm_lds_bytes<2, 2, 2, 2>() <= gemm_lds_bytes<2, 2, 4, 4>(), "the small tile fits in the large tile's LDS");
    const int b = blockIdx.x;
    if (b < n_side) {
        const int per_split = 8 * h_chunk;
        gemm_tile<2, 2, 2, 2, false, 0>(h, h_tiles_m, h_tiles_n, h_chunk, b % per_split, b / per_split, lds);
    } else {
        gemm_tile<2, 2, 4, 4, false, 0>(g, tiles_m, tiles_n, chunk, b - n_side, 0, lds);
    }
}

// Input-gradient product and the partial pass of the adapter gradient in one launch, for the same
// reason: the first n_side workgroups take the adapter-gradient tiles, the rest the 256x256 tiles
// of dX = dy~ W~.
__global__ void __launch_bounds__(256)
gemm_dx_db_pair_kernel(const GemmArgs g, const int tiles_m, const int tiles_n, const int chunk,
                       const DbArgs d, const int n_side)
{
    __shared__ __attribute__((aligned(1024))) uint8_t lds[gemm_lds_bytes<2, 2, 4, 4>()];
    static_assert(dbt::kDbLdsBytes <= static_cast<size_t>(gemm_lds_bytes<2, 2, 4, 4>()), "the dB tiles fit in the GEMM's LDS");
    static_assert(dbt::kThreads == 256, "one workgroup shape for both kinds of tile");
    const int b = blockIdx.x;
    if (b < n_side) {
        if (b >= d.i_tiles * d.splits * d.p_tiles) return;               // padding up to a multiple of 8
        const int bi = b % d.i_tiles, rest = b / d.i_tiles;
        dbt::db_partial_tile(d, bi, rest % d.splits, rest / d.splits, lds, g_zero16);
    } else {
        gemm_tile<2, 2, 4, 4, true, 1>(g, tiles_m, tiles_n, chunk, b - n_side, 0, lds);
    }
}

template <int WM, int WN, int MB, int NB>
hipError_t launch_cfg(const GemmArgs& g, hipStream_t stream)
{
    constexpr int BM = WM * MB * 32, BN = WN * NB * 32;
    const int tiles_m = static_cast<int>((g.M + BM - 1) / BM), tiles_n = static_cast<int>((g.N + BN - 1) / BN);
    const int total = tiles_m * tiles_n;
    const int chunk = (total + 7) / 8;
    const dim3 grid(static_cast<unsigned>(chunk * 8), static_cast<unsigned>(g.splits)), block(64 * WM * WN);
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

static bool use_big_tiles(int64_t M, int64_t N)
{
    // Large problems: 256x256 tiles, one workgroup per CU.  Small ones: 128x128 so that more
    // than a handful of CUs take part.
    return ((M + 255) / 256) * ((N + 255) / 256) >= 128;
}

int64_t gemm_tile_n(int64_t M, int64_t N) { return use_big_tiles(M, N) ? 256 : 128; }

bool gemm_fwd_pair_supported(const GemmArgs& g, const GemmArgs& h)
{
    return use_big_tiles(g.M, g.N) && g.splits == 1 && !g.b_is_kn && !h.b_is_kn && g.a_fmt == 0 && h.a_fmt == 0;
}

hipError_t launch_gemm_fwd_pair(const GemmArgs& g, const GemmArgs& h, hipStream_t stream)
{
    const int tiles_m = static_cast<int>((g.M + 255) / 256), tiles_n = static_cast<int>((g.N + 255) / 256);
    const int chunk = (tiles_m * tiles_n + 7) / 8;
    const int h_tiles_m = static_cast<int>((h.M + 127) / 128), h_tiles_n = static_cast<int>((h.N + 127) / 128);
    const int h_chunk = (h_tiles_m * h_tiles_n + 7) / 8;
    const int n_side = 8 * h_chunk * h.splits;
    gemm_fwd_pair_kernel<<<dim3(static_cast<unsigned>(n_side + 8 * chunk)), dim3(256), 0, stream>>>(
        g, tiles_m, tiles_n, chunk, h, h_tiles_m, h_tiles_n, h_chunk, n_side);
    return hipGetLastError();
}

// ---- tiles that also work for the adapter: plans and launches ------------------------------------
// Forward.  Where the waves of a tile row (four per tile column) can take the 16x16 blocks of its
// O_A (16 r / 16 of them) at one, two or four blocks each, the blocks ride on the tiles' own K-steps and
// the launch writes O_A itself (splits = 0, row_parts = 0, steps_per_split = blocks per wave: no
// partials, no sum pass).  Otherwise, for ranks up to 64, the
// side job: the tile columns of a tile row in sets of two (one where a tile row has a single tile),
// one K slice per set, at most 8 slices, each a whole number of K-steps and none empty; used when a
// slice is at most four chunks (beyond that the exposed fetch round trips outweigh the saved round
// of tiles).
OaTailPlan plan_oa_tail(int64_t T, int64_t n, int64_t m, int64_t r)
{
    OaTailPlan p{false, 0, 0, 1};
    if (!use_big_tiles(T, m)) return p;
    const int tiles_n = static_cast<int>((m + 255) / 256);
    const int KT = static_cast<int>((n + BK - 1) / BK);
    const int rank_blocks = static_cast<int>((r + 15) / 16);
    for (int rb = 1; rb <= 4; rb *= 2) {
        // wave u of a tile row takes token block u % 16 and the rank blocks from rb (u / 16) on: the
        // 4 tiles_n waves must reach every token block for every group of rb rank blocks
        if (4 * tiles_n >= 16 * ((rank_blocks + rb - 1) / rb)) {
            p.use = true;
            p.splits = 0;
            p.steps_per_split = rb;                                       // rank blocks per wave
            p.row_parts = 0;
            return p;
        }
    }
    if (r > 64) return p;
    p.row_parts = tiles_n >= 2 ? 2 : 1;
    int s0 = tiles_n / p.row_parts < 8 ? tiles_n / p.row_parts : 8;
    if (s0 > KT) s0 = KT;
    p.steps_per_split = (KT + s0 - 1) / s0;
    p.splits = (KT + p.steps_per_split - 1) / p.steps_per_split;
    p.use = p.steps_per_split <= 4 * 2 * p.row_parts;
    return p;
}

// Input gradient: groups of two token tile rows; at most kDbSplitMax groups, four feature steps per
// workgroup of a full group and eight in a last group of a single tile row.
DbTailPlan plan_db_tail(int64_t T, int64_t n, int64_t m, int64_t r)
{
    DbTailPlan p{false, 0};
    if (!use_big_tiles(T, n) || r > 64) return p;
    const int tiles_m = static_cast<int>((T + 255) / 256), tiles_n = static_cast<int>((n + 255) / 256);
    p.groups = (tiles_m + kDbTailGroupRows - 1) / kDbTailGroupRows;
    const int F = static_cast<int>((m + 127) / 128);
    const int per_full = (F + kDbTailGroupRows * tiles_n - 1) / (kDbTailGroupRows * tiles_n);
    const int per_last = (tiles_m % kDbTailGroupRows) ? (F + tiles_n - 1) / tiles_n : per_full;
    p.use = p.groups <= kDbSplitMax && per_full <= 4 && per_last <= 8;
    return p;
}

hipError_t launch_gemm_fwd_tail(const GemmArgs& g, const TailArgs& t, hipStream_t stream)
{
    const int tiles_m = static_cast<int>((g.M + 255) / 256), tiles_n = static_cast<int>((g.N + 255) / 256);
    const int chunk = (tiles_m * tiles_n + 7) / 8;
    if (t.row_parts == 0 && t.steps_per_split == 4)
        gemm_fwd_ride_kernel<4><<<dim3(static_cast<unsigned>(8 * chunk)), dim3(256), 0, stream>>>(g, tiles_m, tiles_n, chunk, t);
    else if (t.row_parts == 0 && t.steps_per_split == 2)
        gemm_fwd_ride_kernel<2><<<dim3(static_cast<unsigned>(8 * chunk)), dim3(256), 0, stream>>>(g, tiles_m, tiles_n, chunk, t);
    else if (t.row_parts == 0)
        gemm_fwd_ride_kernel<1><<<dim3(static_cast<unsigned>(8 * chunk)), dim3(256), 0, stream>>>(g, tiles_m, tiles_n, chunk, t);
    else
        gemm_fwd_tail_kernel<<<dim3(static_cast<unsigned>(8 * chunk)), dim3(256), 0, stream>>>(g, tiles_m, tiles_n, chunk, t);
    return hipGetLastError();
}

hipError_t launch_gemm_dx_tail(const GemmArgs& g, const TailArgs& t, hipStream_t stream)
{
    const int tiles_m = static_cast<int>((g.M + 255) / 256), tiles_n = static_cast<int>((g.N + 255) / 256);
    const int chunk = (tiles_m * tiles_n + 7) / 8;
    gemm_dx_tail_kernel<<<dim3(static_cast<unsigned>(8 * chunk)), dim3(256), 0, stream>>>(g, tiles_m, tiles_n, chunk, t);
    return hipGetLastError();
}

bool gemm_dx_db_pair_supported(const GemmArgs& g)
{
    return use_big_tiles(g.M, g.N) && g.splits == 1 && g.b_is_kn && g.a_fmt == 1;
}

hipError_t launch_gemm_dx_db_pair(const GemmArgs& g, const DbArgs& d, hipStream_t stream)
{
    const int tiles_m = static_cast<int>((g.M + 255) / 256), tiles_n = static_cast<int>((g.N + 255) / 256);
    const int chunk = (tiles_m * tiles_n + 7) / 8;
    const int n_side = (d.i_tiles * d.splits * d.p_tiles + 7) / 8 * 8;
    gemm_dx_db_pair_kernel<<<dim3(static_cast<unsigned>(n_side + 8 * chunk)), dim3(256), 0, stream>>>(
        g, tiles_m, tiles_n, chunk, d, n_side);
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& g, hipStream_t stream)
{
    if (g.M <= 0 || g.N <= 0) return hipSuccess;
    if (use_big_tiles(g.M, g.N)) return launch_cfg<2, 2, 4, 4>(g, stream);
    return launch_cfg<2, 2, 2, 2>(g, stream);
}

}  // namespace falqon
