// Measurement aid: a register-only FP8 matrix-core loop.  Every wave keeps 16 accumulator blocks
// of the same 32x32x64 instruction the products use and feeds them from registers that were filled
// once from the caller's FP8 codes, so the loop has no LDS, cache or HBM traffic at all.  Its rate
// is what the chip sustains on matrix cores alone for that operand data; a product kernel is to be
// read against it as well as against the nominal peak, because the clock under matrix-core load
// depends on how much the operand bits toggle.
#include "falqon_internal.h"

namespace falqon {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kBlocks = 16;                // accumulator blocks per wave: a 128x128 wave tile

__global__ void __launch_bounds__(kThreads)
mfma_probe_kernel(const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ b_codes, int iters,
                  float* __restrict__ sink)
{
    // lane t of every wave takes bytes [128 t, 128 t + 128) of each operand: four 32-byte fragments
    v8i a[4], b[4];
    const int t = threadIdx.x & 63;
    const v8i* pa = reinterpret_cast<const v8i*>(a_codes + 128 * t);
    const v8i* pb = reinterpret_cast<const v8i*>(b_codes + 128 * t);
#pragma unroll
    for (int i = 0; i < 4; ++i) { a[i] = pa[i]; b[i] = pb[i]; }
    v16f acc[kBlocks];
#pragma unroll
    for (int i = 0; i < kBlocks; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kBlocks; ++i)
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i & 3], b[i >> 2], acc[i], 0 /* E4M3 */,
                                                                      0 /* E4M3 */, 0, 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < kBlocks; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[i][j];
    sink[static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_mfma_probe(const uint8_t* a_codes, const uint8_t* b_codes, int workgroups, int iters, float* sink,
                             hipStream_t stream)
{
    mfma_probe_kernel<<<static_cast<unsigned>(workgroups), kThreads, 0, stream>>>(a_codes, b_codes, iters, sink);
    return hipGetLastError();
}

}  // namespace falqon
