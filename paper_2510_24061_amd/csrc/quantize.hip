// Per-tensor FP8 quantizer Q_fp8 for gfx950: absolute-maximum reduction, then scale and cast.
//
// Follows the quantization equation of the paper's "Low-precision floating-point
// quantization" section, read as s = max(FP8) / max|X| (the scale multiplies up to the
// format's range; the rescale of the FP8 product divides by it).
//
// Both passes stream the tensor with 16-byte accesses per lane.  The reduction leaves one
// partial maximum per workgroup; the cast pass folds them itself, so there is no atomic,
// no counter to clear and no host round trip between the passes.  The tensor (tens of MB)
// stays in the 256 MB last-level cache between the passes, so HBM sees about one read.
#include "falqon_internal.h"

namespace falqon {
namespace {

constexpr int kThreads = 256;
constexpr int kVec = 16;          // elements per lane per step

__device__ __forceinline__ float wave_max(float v)
{
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ __forceinline__ float block_max(float v, float* smem /* [kThreads/64] */)
{
    v = wave_max(v);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    __syncthreads();
    if (lane == 0) smem[wave] = v;
    __syncthreads();
    float r = smem[0];
    for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, smem[w]);
    return r;
}

// 16 consecutive elements -> fp32
__device__ __forceinline__ void load16(const uint16_t* p /* bf16 bits */, float (&f)[kVec])
{
    const uint4 a = *reinterpret_cast<const uint4*>(p);
    const uint4 b = *reinterpret_cast<const uint4*>(p + 8);
    const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);            // bf16 -> fp32 is exact
        f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

__device__ __forceinline__ void load16(const float* p, float (&f)[kVec])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float4 v = *reinterpret_cast<const float4*>(p + 4 * i);
        f[4 * i] = v.x; f[4 * i + 1] = v.y; f[4 * i + 2] = v.z; f[4 * i + 3] = v.w;
    }
}

// Saturating round-to-nearest-even cast of four fp32 values to one dword of FP8 codes.
// The hardware conversion rounds to nearest even but turns out-of-range inputs into
// NaN (E4M3) or Inf (E5M2), so the value is clamped to the largest finite one first.
template <int FMT>
__device__ __forceinline__ uint32_t cast4(float a, float b, float c, float d)
{
    constexpr float mx = FMT == FALQON_E4M3 ? 448.0f : 57344.0f;
    a = __builtin_amdgcn_fmed3f(a, -mx, mx);
    b = __builtin_amdgcn_fmed3f(b, -mx, mx);
    c = __builtin_amdgcn_fmed3f(c, -mx, mx);
    d = __builtin_amdgcn_fmed3f(d, -mx, mx);
    int w = 0;
    if (FMT == FALQON_E4M3) {
        w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, w, false);
        w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
    } else {
        w = __builtin_amdgcn_cvt_pk_bf8_f32(a, b, w, false);
        w = __builtin_amdgcn_cvt_pk_bf8_f32(c, d, w, true);
    }
    return static_cast<uint32_t>(w);
}

// vector v (16 elements) of a [rows, cols] tensor with row stride ld -> element offset
__device__ __forceinline__ int64_t vec_offset(int64_t v, int64_t vecs_per_row, int64_t ld)
{
    if (vecs_per_row * kVec == ld) return v * kVec;        // dense: flat
    const int64_t row = v / vecs_per_row;
    return row * ld + (v - row * vecs_per_row) * kVec;
}

template <typename T>
__global__ void __launch_bounds__(kThreads)
amax_partial_kernel(const T* __restrict__ x, int64_t n_vecs, int64_t vecs_per_row, int64_t ld_x,
                    float* __restrict__ partials)
{
    __shared__ float smem[kThreads / 64];
    float m = 0.0f;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; v < n_vecs; v += stride) {
        float f[kVec];
        load16(x + vec_offset(v, vecs_per_row, ld_x), f);
#pragma unroll
        for (int i = 0; i < kVec; ++i) m = fmaxf(m, fabsf(f[i]));
    }
    m = block_max(m, smem);
    if (threadIdx.x == 0) partials[blockIdx.x] = m;
}

template <typename T, int FMT>
__global__ void __launch_bounds__(kThreads)
scale_cast_kernel(const T* __restrict__ x, int64_t n_vecs, int64_t vecs_per_row, int64_t ld_x,
                  const float* __restrict__ partials, int n_partials, const float* __restrict__ scale_in,
                  uint8_t* __restrict__ q, int64_t ld_q, float* __restrict__ scale_out,
                  float* __restrict__ amax_out, uint32_t* __restrict__ zero_word, const SideCast side, int side_blocks)
{
    __shared__ float smem[kThreads / 64];
    // The last side_blocks workgroups cast a second, small bf16 tensor whose maximum is already
    // known (the saved O_A of the layer, for the adapter gradient): s = 448 / max(amax, 1e-12f),
    // one fp32 multiply, then the E4M3 cast.  It rides in this launch so that no launch, and no
    // reduction pass, exists for it alone.
    if (static_cast<int>(blockIdx.x) >= static_cast<int>(gridDim.x) - side_blocks) {
        const int b = static_cast<int>(blockIdx.x) - (static_cast<int>(gridDim.x) - side_blocks);
        const float s2 = 448.0f / fmaxf(*side.amax, 1e-12f);
        const int64_t vecs = side.count / kVec;
        for (int64_t v = static_cast<int64_t>(b) * kThreads + threadIdx.x; v < vecs; v += static_cast<int64_t>(side_blocks) * kThreads) {
            float f[kVec];
            load16(side.x + v * kVec, f);
#pragma unroll
            for (int i = 0; i < kVec; ++i) f[i] = __fmul_rn(f[i], s2);
            uint4 o;
            o.x = cast4<FALQON_E4M3>(f[0], f[1], f[2], f[3]);
            o.y = cast4<FALQON_E4M3>(f[4], f[5], f[6], f[7]);
            o.z = cast4<FALQON_E4M3>(f[8], f[9], f[10], f[11]);
            o.w = cast4<FALQON_E4M3>(f[12], f[13], f[14], f[15]);
            *reinterpret_cast<uint4*>(side.q + v * kVec) = o;
        }
        return;
    }
    const int main_blocks = static_cast<int>(gridDim.x) - side_blocks;
    float m = 0.0f;
    for (int i = threadIdx.x; i < n_partials; i += kThreads) m = fmaxf(m, partials[i]);
    const float amax = block_max(m, smem);
    constexpr float mx = FMT == FALQON_E4M3 ? 448.0f : 57344.0f;
    // IEEE fp32 division (hipcc's default for '/' is the correctly rounded one)
    const float s = scale_in ? *scale_in : mx / fmaxf(amax, 1e-12f);

    const int64_t stride = static_cast<int64_t>(main_blocks) * kThreads;
    for (int64_t v = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; v < n_vecs; v += stride) {
        float f[kVec];
        load16(x + vec_offset(v, vecs_per_row, ld_x), f);
#pragma unroll
        for (int i = 0; i < kVec; ++i) f[i] = __fmul_rn(f[i], s);
        uint4 o;
        o.x = cast4<FMT>(f[0], f[1], f[2], f[3]);
        o.y = cast4<FMT>(f[4], f[5], f[6], f[7]);
        o.z = cast4<FMT>(f[8], f[9], f[10], f[11]);
        o.w = cast4<FMT>(f[12], f[13], f[14], f[15]);
        *reinterpret_cast<uint4*>(q + vec_offset(v, vecs_per_row, ld_q)) = o;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *scale_out = s;
        if (amax_out) *amax_out = amax;
        if (zero_word) *zero_word = 0u;
    }
}

__global__ void zero_word_kernel(uint32_t* w) { *w = 0u; }

template <typename T>
hipError_t run(const T* x, int64_t rows, int64_t cols, int64_t ld_x, falqon_fmt fmt, const float* scale_in,
               uint8_t* q, int64_t ld_q, float* scale_out, float* amax_out, float* partials,
               uint32_t* zero_word, const SideCast* side_job, hipStream_t stream)
{
    SideCast side{nullptr, nullptr, nullptr, 0};
    int side_blocks = 0;
    if (side_job && side_job->count > 0) {
        side = *side_job;
        const int64_t want = (side.count / kVec + kThreads - 1) / kThreads;
        side_blocks = static_cast<int>(want < 64 ? want : 64);
    }
    const int64_t vecs_per_row = cols / kVec;
    const int64_t n_vecs = rows * vecs_per_row;
    // The amax pass wants few, long-running workgroups (one partial each); the cast pass
    // is a plain grid-stride stream.
    int n_partials = 0;
    if (n_vecs > 0) {
        const int64_t want = (n_vecs + kThreads * 4 - 1) / (kThreads * 4);
        n_partials = static_cast<int>(want < kMaxAmaxBlocks ? want : kMaxAmaxBlocks);
        amax_partial_kernel<T><<<n_partials, kThreads, 0, stream>>>(x, n_vecs, vecs_per_row, ld_x, partials);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    int64_t blocks = (n_vecs + kThreads * 2 - 1) / (kThreads * 2);
    if (blocks < 1) blocks = 1;
    if (blocks > 256 * 16) blocks = 256 * 16;
    const dim3 grid(static_cast<unsigned>(blocks + side_blocks));
    if (fmt == FALQON_E4M3)
        scale_cast_kernel<T, FALQON_E4M3><<<grid, kThreads, 0, stream>>>(
            x, n_vecs, vecs_per_row, ld_x, partials, n_partials, scale_in, q, ld_q, scale_out, amax_out, zero_word,
            side, side_blocks);
    else
        scale_cast_kernel<T, FALQON_E5M2><<<grid, kThreads, 0, stream>>>(
            x, n_vecs, vecs_per_row, ld_x, partials, n_partials, scale_in, q, ld_q, scale_out, amax_out, zero_word,
            side, side_blocks);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_zero_word(uint32_t* w, hipStream_t stream)
{
    zero_word_kernel<<<1, 1, 0, stream>>>(w);
    return hipGetLastError();
}

hipError_t launch_quantize(const void* x, falqon_dtype xt, int64_t rows, int64_t cols, int64_t ld_x,
                           falqon_fmt fmt, const float* scale_in, uint8_t* q, int64_t ld_q,
                           float* scale_out, float* amax_out, float* partials, uint32_t* zero_word,
                           hipStream_t stream, const SideCast* side)
{
    if (xt == FALQON_BF16)
        return run(static_cast<const uint16_t*>(x), rows, cols, ld_x, fmt, scale_in, q, ld_q, scale_out,
                   amax_out, partials, zero_word, side, stream);
    return run(static_cast<const float*>(x), rows, cols, ld_x, fmt, scale_in, q, ld_q, scale_out, amax_out,
               partials, zero_word, side, stream);
}

}  // namespace falqon
