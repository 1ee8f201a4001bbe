// Measurement aid: what the fp32 matrix pipes of this chip sustain right now.
//
// The roofline the convolution kernels are held against is 256 CUs x 4 SIMDs x 64 flop
// per clock (v_mfma_f32_32x32x2_f32: 4096 flop per 64-clock instruction) x the shader
// clock, 157.3 TFLOP/s at the nominal 2.4 GHz.  Under a saturated matrix load the chip
// does not hold exactly that clock, so a benchmark that states a fraction of the nominal
// peak should also state the clock of the run.  This kernel is nothing but independent
// MFMA chains on every SIMD (two waves per SIMD, seven accumulator blocks each, operands
// that differ per lane so that the data path toggles as in real work): its flop rate
// divided by 65536 flop per clock is the clock under such a load, and each workgroup also
// records the shader-clock and constant-rate counters around its loop.
#include <hip/hip_runtime.h>

#include "layout.h"

namespace convd {

typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(256, 2) mfma_probe_kernel(float *sums, long long *ticks, int iters)
{
    constexpr int NACC = 7;
    probe_floatx16 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    float av[8], bv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        // values in [-1, 1) that differ from lane to lane and from step to step
        const unsigned u = (threadIdx.x * 16u + i) * 2654435761u, t = (threadIdx.x * 16u + 8u + i + blockIdx.x) * 2246822519u;
        av[i] = (float)(int)(u >> 8) * (1.f / 8388608.f) - 1.f;
        bv[i] = (float)(int)(t >> 8) * (1.f / 8388608.f) - 1.f;
    }
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < NACC; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u], bv[(u + i) & 7], acc[i], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    sums[blockIdx.x * 256 + threadIdx.x] = s;
    if (threadIdx.x == 0) {
        ticks[2 * blockIdx.x] = c1 - c0;
        ticks[2 * blockIdx.x + 1] = w1 - w0;
    }
}

hipError_t launch_mfma_probe(float *sums, long long *ticks, int iters, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(PROBE_BLOCKS), dim3(256), 0, stream, sums, ticks, iters);
    return hipGetLastError();
}

}  // namespace convd
