// Sum of split-K partial products into the bf16 O_A = A x block of the merged forward output
// (merged-output equation), and its absolute maximum.
//
// The r adapter columns would spoil the tiling of the main forward product (4096 + 64 columns
// are 16.25 tiles of 256: a seventeenth, almost empty tile column would run as a second wave
// over the CUs).  They are instead formed by the same GEMM kernel as a separate, small launch,
// split along K so that it fills the chip; this pass adds the fp32 partials in a fixed order
// (bitwise reproducible, no floating-point atomics).
#include "falqon_internal.h"

namespace falqon {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ uint16_t bf16_bits_rne(float v)
{
    uint32_t u = __float_as_uint(v);
    u += 0x7fffu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

// Adds `splits` partials in ascending order, eight loads in flight at a time.
__device__ __forceinline__ float4 ordered_sum(const float* __restrict__ partial, int splits, int64_t count, int64_t e)
{
    constexpr int B = 8;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int sp0 = 0; sp0 < splits; sp0 += B) {
        float4 v[B];
#pragma unroll
        for (int u = 0; u < B; ++u) {
            const int sp = sp0 + u < splits ? sp0 + u : splits - 1;      // beyond the range: a valid address, value unused
            v[u] = *reinterpret_cast<const float4*>(partial + sp * count + e);
        }
#pragma unroll
        for (int u = 0; u < B; ++u) {
            if (sp0 + u == 0) s = v[u];
            else if (sp0 + u < splits) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
        }
    }
    return s;
}

__global__ void __launch_bounds__(kThreads)
sum_partials_bf16_kernel(const float* __restrict__ partial, int splits, int64_t count,
                         uint16_t* __restrict__ out, uint32_t* __restrict__ amax)
{
    float mx = 0.0f;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads * 4;
    for (int64_t e = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4; e < count; e += stride) {
        const float4 s = ordered_sum(partial, splits, count, e);
        const uint16_t b0 = bf16_bits_rne(s.x), b1 = bf16_bits_rne(s.y), b2 = bf16_bits_rne(s.z), b3 = bf16_bits_rne(s.w);
        uint2 pk;
        pk.x = b0 | (static_cast<uint32_t>(b1) << 16);
        pk.y = b2 | (static_cast<uint32_t>(b3) << 16);
        *reinterpret_cast<uint2*>(out + e) = pk;
        mx = fmaxf(mx, fmaxf(fmaxf(fabsf(__uint_as_float(static_cast<uint32_t>(b0) << 16)),
                                   fabsf(__uint_as_float(static_cast<uint32_t>(b1) << 16))),
                             fmaxf(fabsf(__uint_as_float(static_cast<uint32_t>(b2) << 16)),
                                   fabsf(__uint_as_float(static_cast<uint32_t>(b3) << 16)))));
    }
    // one atomic per workgroup: a thousand waves hitting one address would serialise in the L2
    __shared__ float s_max[kThreads / 64];
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if ((threadIdx.x & 63) == 0) s_max[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kThreads / 64; ++w) mx = fmaxf(mx, s_max[w]);
        // non-negative floats order like their bit patterns
        if (mx > 0.0f) atomicMax(amax, __float_as_uint(mx));
    }
}

}  // namespace

hipError_t launch_sum_partials_bf16(const float* partial, int splits, int64_t count, uint16_t* out, uint32_t* amax,
                                    hipStream_t stream)
{
    int64_t blocks = (count / 4 + kThreads - 1) / kThreads;
    if (blocks > 128) blocks = 128;                               // grid-stride: few workgroups, few atomics
    if (blocks < 1) blocks = 1;
    if (splits < 1) return hipErrorInvalidValue;
    sum_partials_bf16_kernel<<<static_cast<unsigned>(blocks), kThreads, 0, stream>>>(partial, splits, count, out, amax);
    return hipGetLastError();
}

}  // namespace falqon
