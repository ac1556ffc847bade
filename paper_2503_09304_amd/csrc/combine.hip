// Gate-weighted combine of complete tokens (Sec. 3.1, "Top-k expert selection": finished expert
// outputs are tracked as state and only fully processed tokens feed the next layer).
//   y[n,:] = sum_j w[n,j] * out[inv[n*k+j], :],  j = 0..k-1 in slot order, fp32 fma chain from 0,
// one rounding to the output type.  HBM-bound gather-reduce: one workgroup per token, 16-byte
// loads along the hidden dimension.
#include <hip/hip_runtime.h>

#include "qmoe_internal.h"

namespace qmoe {
namespace {

template <bool BF16>
__global__ __launch_bounds__(256) void combine_rows(const float *__restrict__ out, const float *__restrict__ topk_w,
                                                    const int32_t *__restrict__ inv, const uint8_t *__restrict__ cls,
                                                    void *__restrict__ y, int N, int H, int k, int class_mask) {
    const int n = blockIdx.x;
    if (n >= N) return;
    const int bit = cls[n] == 0 ? MOE_CLASS_LS : MOE_CLASS_BE;
    if (!(class_mask & bit)) return;
    __shared__ float sw[kMaxTopK];
    __shared__ int32_t sp[kMaxTopK];
    if (threadIdx.x < k) {
        sw[threadIdx.x] = topk_w[(long)n * k + threadIdx.x];
        sp[threadIdx.x] = inv[(long)n * k + threadIdx.x];
    }
    __syncthreads();
    if ((H & 3) == 0) {
        for (int h = threadIdx.x * 4; h < H; h += 1024) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int j = 0; j < k; ++j) {
                const float4 v = *reinterpret_cast<const float4 *>(out + (long)sp[j] * H + h);
                const float wj = sw[j];
                acc.x = fmaf(wj, v.x, acc.x);
                acc.y = fmaf(wj, v.y, acc.y);
                acc.z = fmaf(wj, v.z, acc.z);
                acc.w = fmaf(wj, v.w, acc.w);
            }
            if (BF16) {
                __bf16 r[4] = {(__bf16)acc.x, (__bf16)acc.y, (__bf16)acc.z, (__bf16)acc.w};
                *reinterpret_cast<uint2 *>((uint16_t *)y + (long)n * H + h) = *reinterpret_cast<uint2 *>(r);
            } else {
                *reinterpret_cast<float4 *>((float *)y + (long)n * H + h) = acc;
            }
        }
    } else {
        for (int h = threadIdx.x; h < H; h += 256) {
            float acc = 0.f;
            for (int j = 0; j < k; ++j) acc = fmaf(sw[j], out[(long)sp[j] * H + h], acc);
            if (BF16) ((__bf16 *)y)[(long)n * H + h] = (__bf16)acc;
            else ((float *)y)[(long)n * H + h] = acc;
        }
    }
}

}  // namespace

hipError_t launch_combine(const CombineArgs &a, hipStream_t s) {
    if (a.N <= 0) return hipSuccess;
    if (a.dtype == MOE_BF16)
        hipLaunchKernelGGL(combine_rows<true>, dim3(a.N), dim3(256), 0, s, a.out, a.topk_w, a.inv, a.cls, a.y, a.N, a.H,
                           a.k, a.class_mask);
    else
        hipLaunchKernelGGL(combine_rows<false>, dim3(a.N), dim3(256), 0, s, a.out, a.topk_w, a.inv, a.cls, a.y, a.N, a.H,
                           a.k, a.class_mask);
    return hipGetLastError();
}

}  // namespace qmoe
