// Roofline calibration kernels: what this GPU sustains on the two limits the layer kernels
// are priced against - a register-resident fp32 MFMA loop (no memory traffic at all) and a
// plain streaming copy.  They compute nothing of the method.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/chebykan_tools.h"
#include "launch.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int CAL_THREADS = 256;
constexpr int CAL_ACCS = 4;            // independent accumulators per wave, as in the 128x128 tiles
constexpr int CAL_UNROLL = 8;          // MFMA rounds per loop trip

// Each wave issues iterations * CAL_UNROLL * CAL_ACCS v_mfma_f32_32x32x2_f32 on register operands.
__global__ void __launch_bounds__(CAL_THREADS, 2) mfma_loop_kernel(float* __restrict__ sink, int iterations)
{
    floatx16 acc[CAL_ACCS];
#pragma unroll
    for (int q = 0; q < CAL_ACCS; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[q][r] = 0.0f;
    float a = 1.0f + (float)threadIdx.x * 1e-6f, b = 1.0f - (float)threadIdx.x * 1e-6f;
    for (int it = 0; it < iterations; ++it) {
#pragma unroll
        for (int u = 0; u < CAL_UNROLL; ++u)
#pragma unroll
            for (int q = 0; q < CAL_ACCS; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[q], 0, 0, 0);
        a = -a;   // keeps the sums bounded
    }
    float total = 0.0f;
#pragma unroll
    for (int q = 0; q < CAL_ACCS; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) total += acc[q][r];
    // one float per thread, so that the loop cannot be removed
    sink[(size_t)blockIdx.x * CAL_THREADS + threadIdx.x] = total;
}

// dst[i] = src[i], 16 bytes per thread and trip, grid-stride.
__global__ void __launch_bounds__(CAL_THREADS) copy_kernel(floatx4* __restrict__ dst, const floatx4* __restrict__ src,
                                                           int64_t n_vec)
{
    const int64_t stride = (int64_t)gridDim.x * CAL_THREADS;
    for (int64_t i = (int64_t)blockIdx.x * CAL_THREADS + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

}  // namespace

extern "C" {

chebykan_status chebykan_calibrate_mfma(float* sink, int workgroups, int iterations, double* flops,
                                        chebykan_stream_t stream)
{
    if (!sink) return CHEBYKAN_ERR_NULL;
    if (workgroups <= 0 || workgroups > 65536 || iterations <= 0) return CHEBYKAN_ERR_SHAPE;
    chebykan::launch<mfma_loop_kernel>(dim3((unsigned)workgroups), dim3(CAL_THREADS), 0, static_cast<hipStream_t>(stream),
                                       sink, iterations);
    if (hipGetLastError() != hipSuccess) return CHEBYKAN_ERR_LAUNCH;
    if (flops)
        *flops = (double)workgroups * (CAL_THREADS / 64) * (double)iterations * CAL_UNROLL * CAL_ACCS * (32.0 * 32 * 2 * 2);
    return CHEBYKAN_OK;
}

chebykan_status chebykan_calibrate_copy(float* dst, const float* src, int64_t n, chebykan_stream_t stream)
{
    if (!dst || !src) return CHEBYKAN_ERR_NULL;
    if (n <= 0 || n % 4 != 0 || (reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) % 16 != 0)
        return CHEBYKAN_ERR_SHAPE;
    chebykan::launch<copy_kernel>(dim3(256 * 16), dim3(CAL_THREADS), 0, static_cast<hipStream_t>(stream),
                                  reinterpret_cast<floatx4*>(dst), reinterpret_cast<const floatx4*>(src), n / 4);
    if (hipGetLastError() != hipSuccess) return CHEBYKAN_ERR_LAUNCH;
    return CHEBYKAN_OK;
}

}  // extern "C"
