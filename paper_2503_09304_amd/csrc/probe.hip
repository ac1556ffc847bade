// Yardstick for the MFMA-bound kernels' profiles (no part of the method): a loop of bf16 MFMAs on
// register operands only, no memory traffic inside the loop, one wave per SIMD like the expert
// kernels.  Its rate, MFMA-busy fraction and clock under rocprofv3 counters say what the chip
// sustains on operands with the workload's bit patterns, which is what the expert kernels' own
// figures are to be read against.
#include <hip/hip_runtime.h>

#include "qmoe_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Every lane takes 4 A fragments and 2 B fragments (8 bf16 each) from the caller's tensors, then runs
// `iters` rounds of the 8 MFMAs a[i] x b[j]: 8 independent accumulator tiles, back-to-back issue.
__global__ __launch_bounds__(256) void mfma_probe(const bf16x8 *__restrict__ a_src, const bf16x8 *__restrict__ b_src, int iters,
                                                  float *__restrict__ sink) {
    const int t = threadIdx.x;
    bf16x8 a[4], b[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = a_src[(i * 256 + t) & 511];
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = b_src[(j * 256 + t) & 511];
    f32x16 acc[8];
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i * 2 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i * 2 + j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[q][r];
    if (s == 12345.678f) sink[0] = s;      // keeps the loop alive; practically never true
}

}  // namespace

extern "C" int32_t moe_probe_mfma(const void *a_bf16, const void *b_bf16, int32_t iters, int32_t workgroups, float *sink,
                                  void *stream) {
    if (!a_bf16 || !b_bf16 || !sink || iters < 1 || workgroups < 1 || workgroups > (1 << 20))
        return qmoe::set_error(MOE_E_ARG, "moe_probe_mfma: bad argument");
    hipLaunchKernelGGL(mfma_probe, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream, (const bf16x8 *)a_bf16,
                       (const bf16x8 *)b_bf16, iters, sink);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return qmoe::set_error(MOE_E_HIP, "moe_probe_mfma: %s", hipGetErrorString(e));
    return MOE_OK;
}
