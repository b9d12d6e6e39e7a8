// Optimizer step into the proxy buffer ("DeltaBuffer <- Optimizer(dL/dB, lr)", second line of
// the loop of the backward-and-update algorithm) with the optimizer the paper's experiments name:
// AdamW under gradient-norm clipping.  B is never stored, only its change, so the decoupled
// weight decay has nothing to act on; what remains is Adam with bias correction, writing the
// change of B into the buffer.
//
// Both kernels stream a few MB once: HBM/launch bound, 16-byte accesses per lane.  The sum of
// squares is formed in fp64 with a fixed assignment of elements to threads and fixed reduction
// trees, so it is bitwise reproducible (no floating-point atomics).
#include "falqon_internal.h"

namespace falqon {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxNormBlocks = 256;     // partial sums of squares (doubles) in the workspace

__global__ void __launch_bounds__(kThreads)
sqnorm_partial_kernel(const float* __restrict__ g, int64_t count, double* __restrict__ partial)
{
    __shared__ double s_sum[kThreads];
    double acc = 0.0;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads * 4;
    for (int64_t e = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4; e < count; e += stride) {
        const float4 v = *reinterpret_cast<const float4*>(g + e);
        acc += static_cast<double>(v.x) * v.x;
        acc += static_cast<double>(v.y) * v.y;
        acc += static_cast<double>(v.z) * v.z;
        acc += static_cast<double>(v.w) * v.w;
    }
    s_sum[threadIdx.x] = acc;
    __syncthreads();
    for (int half = kThreads / 2; half > 0; half >>= 1) {             // fixed tree
        if (threadIdx.x < half) s_sum[threadIdx.x] += s_sum[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = s_sum[0];
}

// one workgroup: partials added in a fixed tree, result added to the accumulator
__global__ void __launch_bounds__(kMaxNormBlocks)
sqnorm_final_kernel(const double* __restrict__ partial, int n_partials, double* sum_sq)
{
    __shared__ double s_sum[kMaxNormBlocks];
    s_sum[threadIdx.x] = static_cast<int>(threadIdx.x) < n_partials ? partial[threadIdx.x] : 0.0;
    __syncthreads();
    for (int half = kMaxNormBlocks / 2; half > 0; half >>= 1) {
        if (static_cast<int>(threadIdx.x) < half) s_sum[threadIdx.x] += s_sum[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) *sum_sq += s_sum[0];
}

__global__ void __launch_bounds__(kThreads)
adamw_delta_kernel(const float* __restrict__ d_b, float* __restrict__ exp_avg, float* __restrict__ exp_avg_sq,
                   float* __restrict__ delta_buf, int64_t count, const AdamFactors f,
                   const double* __restrict__ sum_sq)
{
    float c = 1.0f;
    if (sum_sq) {
        const double cc = f.max_norm / (sqrt(*sum_sq) + 1e-6);
        c = cc < 1.0 ? static_cast<float>(cc) : 1.0f;
    }
    const float beta1 = f.beta1, omb1 = f.one_minus_beta1, beta2 = f.beta2, omb2 = f.one_minus_beta2;
    const float eps = f.eps, step_size = f.step_size, inv_sqrt_bias2 = f.inv_sqrt_bias2;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads * 4;
    for (int64_t e = (static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4; e < count; e += stride) {
        const float4 g4 = *reinterpret_cast<const float4*>(d_b + e);
        float4 m4 = *reinterpret_cast<const float4*>(exp_avg + e);
        float4 v4 = *reinterpret_cast<const float4*>(exp_avg_sq + e);
        float4 b4 = *reinterpret_cast<const float4*>(delta_buf + e);
        const float g[4] = {g4.x, g4.y, g4.z, g4.w};
        float m[4] = {m4.x, m4.y, m4.z, m4.w}, v[4] = {v4.x, v4.y, v4.z, v4.w}, b[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float gi = c * g[i];
            m[i] = beta1 * m[i] + omb1 * gi;
            v[i] = beta2 * v[i] + omb2 * gi * gi;
            const float denom = sqrtf(v[i]) * inv_sqrt_bias2 + eps;
            b[i] += -step_size * m[i] / denom;
        }
        *reinterpret_cast<float4*>(exp_avg + e) = make_float4(m[0], m[1], m[2], m[3]);
        *reinterpret_cast<float4*>(exp_avg_sq + e) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(delta_buf + e) = make_float4(b[0], b[1], b[2], b[3]);
    }
}

unsigned blocks_for(int64_t count, int64_t cap)
{
    int64_t b = (count / 4 + kThreads - 1) / kThreads;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return static_cast<unsigned>(b);
}

}  // namespace

hipError_t launch_grad_sqnorm(const float* g, int64_t count, double* sum_sq, double* partials, hipStream_t stream)
{
    const unsigned nb = blocks_for(count, kMaxNormBlocks);
    sqnorm_partial_kernel<<<nb, kThreads, 0, stream>>>(g, count, partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    sqnorm_final_kernel<<<1, kMaxNormBlocks, 0, stream>>>(partials, static_cast<int>(nb), sum_sq);
    return hipGetLastError();
}

hipError_t launch_adamw_delta(const float* d_b, float* exp_avg, float* exp_avg_sq, float* delta_buf, int64_t count,
                              const AdamFactors& f, const double* sum_sq, hipStream_t stream)
{
    adamw_delta_kernel<<<blocks_for(count, 4096), kThreads, 0, stream>>>(d_b, exp_avg, exp_avg_sq, delta_buf, count, f,
                                                                         sum_sq);
    return hipGetLastError();
}

}  // namespace falqon
