// Gate-weighted combine of complete tokens (Sec. 3.1, "Top-k expert selection": finished expert
// outputs are tracked as state and only fully processed tokens feed the next layer).
//   y[n,:] = sum_j w[n,j] * out[inv[n*k+j], :],  j = 0..k-1 in slot order, fp32 fma chain from 0,
// one rounding to the output type.  HBM-bound gather-reduce: one workgroup per token, 16-byte
// loads along the hidden dimension.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "qmoe_internal.h"

namespace qmoe {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// One 16-byte piece of an expert output row.  KS > 1: the down projection left KS partial planes
// (K ranges); they are added here in the fixed order ((p0 + p1) + p2) + p3, so the value is the one a
// separate reduction pass would have stored.  Read once: non-temporal.
template <int KS>
__device__ __forceinline__ f32x4 load_out(const float *__restrict__ p, long plane) {
    f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    if constexpr (KS > 1) {
#pragma unroll
        for (int q = 1; q < KS; ++q) {
            const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p + q * plane));
            v[0] = v[0] + t[0]; v[1] = v[1] + t[1]; v[2] = v[2] + t[2]; v[3] = v[3] + t[3];
        }
    }
    return v;
}

// done == nullptr: tokens are selected by class (the host has checked that the class is finished).
// done != nullptr: a token is selected when done[] is set for all k of its sorted positions;
// complete[n] (if given) reports the selection.
template <bool BF16, int KS>
__global__ __launch_bounds__(256) void combine_rows(const float *__restrict__ out, long plane, const float *__restrict__ topk_w,
                                                    const int32_t *__restrict__ inv, const uint8_t *__restrict__ cls,
                                                    const uint8_t *__restrict__ done, uint8_t *__restrict__ complete,
                                                    void *__restrict__ y, int N, int H, int k, int class_mask) {
    const int n = blockIdx.x;
    if (n >= N) return;
    if (done == nullptr) {
        const int bit = cls[n] == 0 ? MOE_CLASS_LS : MOE_CLASS_BE;
        if (!(class_mask & bit)) return;
    }
    __shared__ float sw[kMaxTopK];
    __shared__ int32_t sp[kMaxTopK];
    __shared__ int missing;
    if (threadIdx.x == 0) missing = 0;
    __syncthreads();
    if (threadIdx.x < k) {
        const int32_t p = inv[(long)n * k + threadIdx.x];
        sw[threadIdx.x] = topk_w[(long)n * k + threadIdx.x];
        sp[threadIdx.x] = p;
        if (done != nullptr && done[p] == 0) missing = 1;     // any writer stores the same value
    }
    __syncthreads();
    if (done != nullptr) {
        if (complete != nullptr && threadIdx.x == 0) complete[n] = missing ? 0 : 1;
        if (missing) return;
    }
    if ((H & 3) == 0) {
        for (int h = threadIdx.x * 4; h < H; h += 1024) {
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int j = 0; j < k; ++j) {
                const f32x4 v = load_out<KS>(out + (long)sp[j] * H + h, plane);
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
            for (int j = 0; j < k; ++j) {
                float v = out[(long)sp[j] * H + h];
#pragma unroll
                for (int q = 1; q < KS; ++q) v = v + out[q * plane + (long)sp[j] * H + h];
                acc = fmaf(sw[j], v, acc);
            }
            if (BF16) ((__bf16 *)y)[(long)n * H + h] = (__bf16)acc;
            else ((float *)y)[(long)n * H + h] = acc;
        }
    }
}

// done[row] = 1 for the rows of up to kMaxSegs row ranges: one workgroup per range.
struct MarkArgs {
    int n;
    Seg seg[kMaxSegs];
};

__global__ __launch_bounds__(256) void mark_rows(const MarkArgs m, uint8_t *__restrict__ done) {
    const Seg g = m.seg[blockIdx.x];
    for (int r = threadIdx.x; r < g.rows; r += 256) done[g.row0 + r] = 1;
}

__global__ __launch_bounds__(256) void clear_bytes(uint8_t *__restrict__ p, long n) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) p[i] = 0;
}

__global__ void gate_kernel(const int32_t *__restrict__ stop_host, int32_t *__restrict__ go, int g) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int prev_open = g == 0 ? 1 : go[g - 1];
    const int stop = __hip_atomic_load(stop_host, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    go[g] = (prev_open && stop == 0) ? 1 : 0;
}

struct ReportArgs {
    int n;
    Seg seg[kMaxSegs];
};

__global__ __launch_bounds__(256) void report_ranges(const ReportArgs r, const int32_t *__restrict__ cnt_dn,
                                                     int32_t *__restrict__ ok_host, int dtype, int H, int ksplit) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= r.n) return;
    const Seg g = r.seg[i];
    const int ok = cnt_dn[g.row0] == down_wgs_of_range(dtype, H, ksplit, g.rows) ? 1 : 0;
    __hip_atomic_store(ok_host + i, ok, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ __launch_bounds__(256) void clear_words(int32_t *__restrict__ p, long n) {
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) p[i] = 0;
}

}  // namespace

hipError_t launch_gate(const int32_t *stop_host, int32_t *go, int g, hipStream_t s) {
    hipLaunchKernelGGL(gate_kernel, dim3(1), dim3(64), 0, s, stop_host, go, g);
    return hipGetLastError();
}

hipError_t launch_report(const Seg *ranges, int n, const int32_t *cnt_dn, int32_t *ok_host, int dtype, int H, int ksplit,
                         hipStream_t s) {
    for (int i = 0; i < n; i += kMaxSegs) {
        ReportArgs r{};
        r.n = std::min(kMaxSegs, n - i);
        std::copy(ranges + i, ranges + i + r.n, r.seg);
        hipLaunchKernelGGL(report_ranges, dim3((r.n + 255) / 256), dim3(256), 0, s, r, cnt_dn, ok_host + i, dtype, H, ksplit);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_clear_words(int32_t *p, long n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<long>((n + 255) / 256, 1024);
    hipLaunchKernelGGL(clear_words, dim3(blocks), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

template <bool BF16, int KS>
static void launch_combine_ks(const CombineArgs &a, hipStream_t s) {
    hipLaunchKernelGGL((combine_rows<BF16, KS>), dim3(a.N), dim3(256), 0, s, a.out, a.plane, a.topk_w, a.inv, a.cls, a.done,
                       a.complete, a.y, a.N, a.H, a.k, a.class_mask);
}

hipError_t launch_combine(const CombineArgs &a, hipStream_t s) {
    if (a.N <= 0) return hipSuccess;
    const bool bf = a.dtype == MOE_BF16;
    if (a.ksplit == 4) { if (bf) launch_combine_ks<true, 4>(a, s); else launch_combine_ks<false, 4>(a, s); }
    else if (a.ksplit == 2) { if (bf) launch_combine_ks<true, 2>(a, s); else launch_combine_ks<false, 2>(a, s); }
    else { if (bf) launch_combine_ks<true, 1>(a, s); else launch_combine_ks<false, 1>(a, s); }
    return hipGetLastError();
}

hipError_t launch_clear_done(uint8_t *done, long n, hipStream_t s) {
    if (n <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)std::min<long>((n + 255) / 256, 1024);
    hipLaunchKernelGGL(clear_bytes, dim3(blocks), dim3(256), 0, s, done, n);
    return hipGetLastError();
}

hipError_t launch_mark_done(const Seg *segs, int n, uint8_t *done, hipStream_t s) {
    for (int i = 0; i < n; i += kMaxSegs) {
        MarkArgs m{};
        m.n = std::min(kMaxSegs, n - i);
        std::copy(segs + i, segs + i + m.n, m.seg);
        hipLaunchKernelGGL(mark_rows, dim3(m.n), dim3(256), 0, s, m, done);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace qmoe
