// Variant of the adapter gradient (modified LoRA-backward equation) that keeps the saved O_A = A x
// at its 16-bit precision instead of casting it to E4M3:
//
//   dB[i,p] = ( sum_t value5(dyq[t,i]) * o_a[t,p] ) / s_dy
//
// An E5M2 value has two mantissa bits and a five-bit exponent, so it is exactly representable in
// bf16; the product therefore runs on the bf16 matrix cores with nothing rounded before the fp32
// accumulation.  The same kernel with E4M3 codes on the left (three mantissa bits: exact in bf16
// too) forms the second product of the gradient of the adapter factor A (LoRA backward equation),
//   dA^T[j,p] = ( sum_t value4(xq[t,j]) * g[t,p] ) / s_x.  Same split into fp32 partials over token ranges and the same ordered second pass
// as the FP8 variant.
//
// Operands for a contraction over tokens (the strided dimension of both tensors):
//   dy~  stays bytes in a [token][feature] LDS tile; ds_read_b64_tr_b8 hands each lane eight
//        consecutive tokens of one feature, which are widened to bf16 in registers;
//   O_A  is written to LDS transposed, [rank][token], two tokens per 32-bit store, so that a lane
//        reads its eight consecutive tokens with one 16-byte load.
#include "db_tile.h"

namespace falqon {
namespace {

using namespace dbt;

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kWideTiles = 4;                                          // token tiles fetched per round trip
constexpr int kWideTileBytes = BT * BI + BP * BT * 2;                  // dyq tile + transposed O_A tile (bf16)
constexpr size_t kWideLdsBytes = static_cast<size_t>(kWideTiles) * kWideTileBytes;

__device__ __attribute__((aligned(16))) uint8_t g_wide_zero16[16];

// two FP8 codes (the selected 16-bit half of w; E5M2 if LEFT_E5M2, else E4M3) -> two bf16 in one
// dword, first code in the low half
template <bool LEFT_E5M2>
__device__ __forceinline__ int widen2(int w, bool upper_half)
{
    v2f f;
    if (LEFT_E5M2) f = upper_half ? __builtin_amdgcn_cvt_pk_f32_bf8(w, true) : __builtin_amdgcn_cvt_pk_f32_bf8(w, false);
    else f = upper_half ? __builtin_amdgcn_cvt_pk_f32_fp8(w, true) : __builtin_amdgcn_cvt_pk_f32_fp8(w, false);
    // the value has at most four significant bits: the upper half of the fp32 pattern is the bf16
    return static_cast<int>(__builtin_amdgcn_perm(__float_as_uint(f[1]), __float_as_uint(f[0]), 0x07060302u));
}

// chunk (16 bytes = 8 tokens) c of rank row p sits at c ^ (p % 16)
__device__ __forceinline__ int oat_offset(int p, int token)
{
    return p * (BT * 2) + ((((token >> 3) ^ (p & 15)) << 4) | ((token & 7) << 1));
}

template <bool LEFT_E5M2>
__global__ void __launch_bounds__(kThreads)
db_wide_partial_kernel(const DbArgs d)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t s_tiles[];
    constexpr int CH_DY = BI / 16;
    const uint8_t* const zero16 = g_wide_zero16;
    const uint8_t* const dyq = d.dyq;
    const uint16_t* const o_a = d.o_a;
    const int64_t T = d.T, m = d.m, r = d.r;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t i0 = static_cast<int64_t>(blockIdx.x) * BI;
    const int64_t p0 = static_cast<int64_t>(blockIdx.z) * BP;
    const int64_t t_begin = static_cast<int64_t>(blockIdx.y) * d.tokens_per_split;
    int64_t t_end = t_begin + d.tokens_per_split;
    if (t_end > T) t_end = T;

    v16f acc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.0f;

    for (int64_t tg = t_begin; tg < t_end; tg += kWideTiles * BT) {
        __syncthreads();                       // the previous group's operand reads are done
        // dy~ tiles: as in the FP8 variant (rows, features and tiles out of range come from a block of zeros)
#pragma unroll
        for (int tl = 0; tl < kWideTiles; ++tl) {
            const int64_t t0 = tg + tl * BT;
#pragma unroll
            for (int it = 0; it < BT * BI / 1024 / 4; ++it) {
                const int q = it * 4 + wave;
                const int trow = q * 8 + (lane >> 3);
                const int c = (lane & 7) ^ swz_t<CH_DY>(trow);
                const int64_t gt = t0 + trow, gi = i0 + c * 16;
                const uint8_t* src = (gt < t_end && gi < m) ? dyq + gt * m + gi : zero16;
                __builtin_amdgcn_global_load_lds(FQ_GLOBAL_PTR(src), FQ_LDS_PTR(s_tiles + tl * kWideTileBytes + q * 1024), 16, 0, 0);
            }
        }
        // O_A tiles: thread -> (token pair, eight ranks), two such items per tile
        const int oct = threadIdx.x & 7;
        uint4 w[kWideTiles][2][2];
#pragma unroll
        for (int tl = 0; tl < kWideTiles; ++tl)
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int64_t gt = tg + tl * BT + 2 * ((threadIdx.x >> 3) + 32 * h) + e;
                    const int64_t gp = p0 + oct * 8;
                    const void* src = (gt < t_end && gp < r) ? static_cast<const void*>(o_a + gt * r + gp)
                                                             : static_cast<const void*>(zero16);
                    w[tl][h][e] = *reinterpret_cast<const uint4*>(src);
                }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int tl = 0; tl < kWideTiles; ++tl) {
            uint8_t* s_oat = s_tiles + tl * kWideTileBytes + BT * BI;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int token = 2 * ((threadIdx.x >> 3) + 32 * h);
                const uint32_t lo[4] = {w[tl][h][0].x, w[tl][h][0].y, w[tl][h][0].z, w[tl][h][0].w};   // token
                const uint32_t hi[4] = {w[tl][h][1].x, w[tl][h][1].y, w[tl][h][1].z, w[tl][h][1].w};   // token + 1
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // ranks 8 oct + 2 e and + 2 e + 1: (token, token + 1) pairs
                    const uint32_t even = __builtin_amdgcn_perm(hi[e], lo[e], 0x05040100u);
                    const uint32_t odd = __builtin_amdgcn_perm(hi[e], lo[e], 0x07060302u);
                    *reinterpret_cast<uint32_t*>(s_oat + oat_offset(oct * 8 + 2 * e, token)) = even;
                    *reinterpret_cast<uint32_t*>(s_oat + oat_offset(oct * 8 + 2 * e + 1, token)) = odd;
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        // wave w owns features [32 w, 32 w + 32) of the tile and both 32-wide rank blocks;
        // one matrix-core step covers 16 tokens: lanes 0-31 the first eight, lanes 32-63 the next eight
#pragma unroll
        for (int tl = 0; tl < kWideTiles; ++tl) {
            if (tg + tl * BT >= t_end) break;                               // tiles beyond the range hold zeros
            const uint8_t* s_dy = s_tiles + tl * kWideTileBytes;
            const uint8_t* s_oat = s_dy + BT * BI;
#pragma unroll
            for (int ks = 0; ks < BT / 16; ++ks) {
                const int tok = ks * 16 + (lane >> 5) * 8;
                // lane s of a 16-lane group supplies token row (s % 16) / 2, feature block 8 (s % 2);
                // lane L receives feature L % 32 of the wave's span, eight tokens in eight bytes
                const int trow = tok + ((lane & 15) >> 1);
                const int feat = wave * 32 + ((lane >> 4) & 1) * 16 + (lane & 1) * 8;
                const uint8_t* pa = s_dy + trow * BI + ((((feat >> 4) ^ swz_t<CH_DY>(trow)) << 4) | (feat & 15));
                const v2i c8 = __builtin_amdgcn_ds_read_tr8_b64_v2i32((v2i __attribute__((address_space(3)))*)(pa));
                v4i aw;
                aw[0] = widen2<LEFT_E5M2>(c8[0], false); aw[1] = widen2<LEFT_E5M2>(c8[0], true);
                aw[2] = widen2<LEFT_E5M2>(c8[1], false); aw[3] = widen2<LEFT_E5M2>(c8[1], true);
                const v8bf a = __builtin_bit_cast(v8bf, aw);
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const v4i bw = *reinterpret_cast<const v4i*>(s_oat + oat_offset(b * 32 + (lane & 31), tok));
                    acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(v8bf, bw), acc[b], 0, 0, 0);
                }
            }
        }
    }

    float* out = d.partial + static_cast<int64_t>(blockIdx.y) * m * r;
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

}  // namespace

template <bool LEFT_E5M2>
static hipError_t launch_wide(const DbArgs& d, hipStream_t stream)
{
    const dim3 grid(static_cast<unsigned>(d.i_tiles), static_cast<unsigned>(d.splits), static_cast<unsigned>(d.p_tiles));
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&db_wide_partial_kernel<LEFT_E5M2>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kWideLdsBytes));
    if (e != hipSuccess) return e;
    db_wide_partial_kernel<LEFT_E5M2><<<grid, kThreads, kWideLdsBytes, stream>>>(d);
    return hipGetLastError();
}

hipError_t launch_db_wide_partial(const DbArgs& d, hipStream_t stream, bool left_e5m2)
{
    return left_e5m2 ? launch_wide<true>(d, stream) : launch_wide<false>(d, stream);
}

}  // namespace falqon
