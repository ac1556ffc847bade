// Router kernels: gate GEMM (fp32 logits), then per-token top-k with renormalised softmax
// weights.  Follows the paper's description of the MoE router (Sec. 2.1, Sec. 2.2): each token is
// assigned to its k most relevant experts.
//
// bf16: logits come from 16x16x32 bf16 MFMA tiles (16 tokens x 16 experts per tile), fp32
// accumulation.  Wg is [H,E] with E contiguous, the wrong majorness for MFMA operands, so a
// small kernel first writes it transposed (and padded to a multiple of 16 experts) into scratch.
// A workgroup owns 16 tokens; its 8 waves split the hidden dimension into 8 contiguous ranges and
// add their partial tiles through LDS in wave order, so the summation order is fixed; the same
// workgroup then selects the experts (fused, no second launch).
// fp32: one wave per token, lanes stride the hidden dimension, butterfly reduction; separate top-k.
// top-k: one wave per token.  bf16: every lane ranks its experts against the whole row of logits in
// LDS (order: logit desc, index asc).  fp32: k rounds of a wave-wide arg-max over the same order.
#include <hip/hip_runtime.h>

#include <mutex>

#include "qmoe_internal.h"

// Scratch of moe_route_noalloc: the router weight transposed and padded, bf16 [ceil16(E)][H].  One
// copy per GPU the library runs on, held until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels get the device address that call returns.
constexpr size_t kRouteScratchBytes = 2u << 20;
static __device__ __align__(256) unsigned char scratch[kRouteScratchBytes];

namespace qmoe {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void wg_transpose_bf16(const uint16_t *__restrict__ Wg, uint16_t *__restrict__ WgT,
                                                         int H, int E, int E16) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= (long)E16 * H) return;
    const int e = (int)(i / H), h = (int)(i % H);
    WgT[i] = e < E ? Wg[(long)h * E + e] : (uint16_t)0;
}

// Wave-wide top-k of one token's logits: lane l holds the logits of experts l, l+64, l+128, l+192
// in v[]; k rounds of an arg-max over (logit descending, expert index ascending), butterfly
// shuffles; lane j ends up with slot j; weights = softmax over the k selected logits.
constexpr int kSlots = kMaxExperts / 64;
__device__ __forceinline__ void wave_topk(const float (&v)[kSlots], int l, int E, int k, int32_t *__restrict__ idx_out,
                                          float *__restrict__ w_out) {
    unsigned picked = 0;
    float my_v = 0.f;
    int my_e = 0;
    for (int j = 0; j < k; ++j) {
        float bv = -INFINITY;
        int be = 0x7fffffff;
#pragma unroll
        for (int c = 0; c < kSlots; ++c) {
            const int e = l + 64 * c;
            const bool ok = e < E && !((picked >> c) & 1u);
            if (ok && (be == 0x7fffffff || v[c] > bv)) { bv = v[c]; be = e; }   // ascending e: '>' keeps the lowest index
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float ov = __shfl_xor(bv, o, 64);
            const int oe = __shfl_xor(be, o, 64);
            const bool take = (oe != 0x7fffffff) && (be == 0x7fffffff || ov > bv || (ov == bv && oe < be));
            if (take) { bv = ov; be = oe; }
        }
        if ((be & 63) == l) picked |= 1u << (be >> 6);
        if (l == j) { my_v = bv; my_e = be; }
    }
    const float top = __shfl(my_v, 0, 64);
    const float p = l < k ? expf(my_v - top) : 0.f;
    float s = p;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (l < k) {
        idx_out[l] = my_e;
        w_out[l] = p / s;
    }
}

// Top-k by ranking, for logits that sit in LDS: lane l counts, for each of its experts l, l+64, ...,
// how many experts precede it in the order (logit descending, index ascending); an expert of rank
// < k is the token's slot `rank`.  No chain of dependent shuffles: the E reads of the row are
// broadcasts.  The selected logits go through `slot_v` / `slot_e` (k entries of LDS, private to the
// wave) so that lane j holds slot j, and the weights are the same softmax, summed in the same
// butterfly order, as wave_topk computes.
template <int NT>
__device__ __forceinline__ void wave_topk_rank(const float *const (&row)[NT], float (*__restrict__ slot_v)[kMaxTopK],
                                               int32_t (*__restrict__ slot_e)[kMaxTopK], int l, int E, int k,
                                               int32_t *const (&idx_out)[NT], float *const (&w_out)[NT]) {
    // NT tokens of the wave side by side: their LDS reads and shuffles overlap.  idx_out[h] == nullptr:
    // token h is past the end of the batch (its row holds a copy of the last token) and stores nothing.
    float mine[NT][kSlots];
    int rank[NT][kSlots];
#pragma unroll
    for (int h = 0; h < NT; ++h)
#pragma unroll
        for (int c = 0; c < kSlots; ++c) {
            const int e = l + 64 * c;
            mine[h][c] = e < E ? row[h][e] : 0.f;
            rank[h][c] = 0;
        }
    const int nslots = (E + 63) >> 6;
    const int E8 = E & ~7;
    for (int o0 = 0; o0 < E8; o0 += 8) {                 // 8 broadcast reads per token in flight at a time
        float ov[NT][8];
#pragma unroll
        for (int h = 0; h < NT; ++h)
#pragma unroll
            for (int i = 0; i < 8; ++i) ov[h][i] = row[h][o0 + i];
#pragma unroll
        for (int c = 0; c < kSlots; ++c) {
            if (c < nslots) {
                const int e = l + 64 * c;
#pragma unroll
                for (int h = 0; h < NT; ++h)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        rank[h][c] += (ov[h][i] > mine[h][c] || (ov[h][i] == mine[h][c] && o0 + i < e)) ? 1 : 0;
            }
        }
    }
    for (int o = E8; o < E; ++o) {
#pragma unroll
        for (int h = 0; h < NT; ++h) {
            const float ov = row[h][o];
#pragma unroll
            for (int c = 0; c < kSlots; ++c) {
                const int e = l + 64 * c;
                if (c < nslots) rank[h][c] += (ov > mine[h][c] || (ov == mine[h][c] && o < e)) ? 1 : 0;
            }
        }
    }
#pragma unroll
    for (int h = 0; h < NT; ++h)
#pragma unroll
        for (int c = 0; c < kSlots; ++c) {
            const int e = l + 64 * c;
            if (e < E && rank[h][c] < k) { slot_v[h][rank[h][c]] = mine[h][c]; slot_e[h][rank[h][c]] = e; }
        }
    __builtin_amdgcn_s_waitcnt(0xc07f);      // this wave's LDS writes have landed
    __builtin_amdgcn_wave_barrier();
    float my_v[NT], p[NT], s[NT];
    int my_e[NT];
#pragma unroll
    for (int h = 0; h < NT; ++h) {
        my_v[h] = l < k ? slot_v[h][l] : 0.f;
        my_e[h] = l < k ? slot_e[h][l] : 0;
        const float top = __shfl(my_v[h], 0, 64);
        p[h] = l < k ? expf(my_v[h] - top) : 0.f;
        s[h] = p[h];
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
#pragma unroll
        for (int h = 0; h < NT; ++h) s[h] += __shfl_xor(s[h], o, 64);
#pragma unroll
    for (int h = 0; h < NT; ++h)
        if (l < k && idx_out[h] != nullptr) {
            idx_out[h][l] = my_e[h];
            w_out[h][l] = p[h] / s[h];
        }
}

// Gate GEMM and top-k of 16 tokens per workgroup.  NB = number of 16-expert blocks held in
// registers (E16 <= 16*NB).  The 8 waves split the hidden dimension into 8 contiguous ranges (loads
// issued 8, 4 or 2 k-steps at a time: few enough registers that at least two workgroups share a CU,
// which halves the router's time on 8192 tokens x 64 experts), add their partial tiles through LDS
// in wave order, and then each wave selects the experts of 2 of the 16 tokens.
template <int NB>
__global__ __launch_bounds__(512) void gate_topk_bf16(const uint16_t *__restrict__ x, const uint16_t *__restrict__ WgT,
                                                      const float *__restrict__ bias, float *__restrict__ logits,
                                                      int32_t *__restrict__ topk_idx, float *__restrict__ topk_w, int N, int H,
                                                      int E, int nb, int k) {
    __shared__ float red[8][NB][4][64];
    __shared__ float lt[16][NB * 16 + 1];
    __shared__ float sbias[NB * 16];
    __shared__ float slot_v[8][2][kMaxTopK];
    __shared__ int32_t slot_e[8][2][kMaxTopK];
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    const int t16 = l & 15, q = l >> 4;
    int tok = blockIdx.x * 16 + t16;
    if (tok > N - 1) tok = N - 1;
    if (tid < NB * 16) sbias[tid] = (bias && tid < E) ? bias[tid] : 0.f;   // read after the first barrier
    const int steps = H / 32;
    const int per = (steps + 7) / 8;
    const int s0 = w * per, s1 = min(steps, s0 + per);
    f32x4 acc[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = f32x4{0.f, 0.f, 0.f, 0.f};
    const uint16_t *xa = x + (long)tok * H + q * 8;
    const uint16_t *wb = WgT + (long)t16 * H + q * 8;
    constexpr int CH = NB == 1 ? 8 : (NB == 2 ? 4 : 2);   // k-steps whose loads are issued together
    for (int s = s0; s < s1; s += CH) {
        bf16x8 a[CH], bv[CH][NB];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int sc = min(s + c, s1 - 1);
            a[c] = *reinterpret_cast<const bf16x8 *>(xa + sc * 32);
#pragma unroll
            for (int b = 0; b < NB; ++b)
                bv[c][b] = *reinterpret_cast<const bf16x8 *>(wb + (long)min(b, nb - 1) * 16 * H + sc * 32);
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            if (s + c < s1) {
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    if (b < nb) acc[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[c], bv[c][b], acc[b], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[w][b][r][l] = acc[b][r];
    __syncthreads();
    // The NB*4 (expert block, D register) pairs are dealt to the 8 waves; each sum runs over the waves'
    // partial tiles in wave order.
#pragma unroll
    for (int j = 0; j < (NB * 4 + 7) / 8; ++j) {
        const int pr = w + 8 * j;
        const int b = pr >> 2, r = pr & 3;
        if (pr < NB * 4 && b < nb) {
            float v = red[0][b][r][l];
#pragma unroll
            for (int ww = 1; ww < 8; ++ww) v += red[ww][b][r][l];
            const int e = b * 16 + t16;                 // D: column = expert
            const int tl = q * 4 + r;                   // D: row = token (within the 16)
            const int t = blockIdx.x * 16 + tl;
            const float lv = v + sbias[e];
            lt[tl][e] = lv;
            if (e < E && t < N) logits[(long)t * E + e] = lv;
        }
    }
    __syncthreads();
    const int t0 = blockIdx.x * 16 + w * 2;             // this wave's two tokens
    if (t0 < N) {
        const float *const rows[2] = {lt[w * 2], lt[w * 2 + 1]};
        int32_t *const io[2] = {topk_idx + (long)t0 * k, t0 + 1 < N ? topk_idx + (long)(t0 + 1) * k : nullptr};
        float *const wo[2] = {topk_w + (long)t0 * k, t0 + 1 < N ? topk_w + (long)(t0 + 1) * k : nullptr};
        wave_topk_rank<2>(rows, slot_v[w], slot_e[w], l, E, k, io, wo);
    }
}

// One wave per token, 8 experts at a time.
__global__ __launch_bounds__(256) void gate_logits_f32(const float *__restrict__ x, const float *__restrict__ Wg,
                                                       const float *__restrict__ bias, float *__restrict__ logits,
                                                       int N, int H, int E) {
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    const int tok = blockIdx.x * 4 + w;
    if (tok >= N) return;
    for (int e0 = 0; e0 < E; e0 += 8) {
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        for (int h = l; h < H; h += 64) {
            const float xv = x[(long)tok * H + h];
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (e0 + j < E) acc[j] = fmaf(xv, Wg[(long)h * E + e0 + j], acc[j]);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float v = acc[j];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
            if (l == 0 && e0 + j < E) logits[(long)tok * E + e0 + j] = v + (bias ? bias[e0 + j] : 0.f);
        }
    }
}

// One wave per token (fp32 path).
__global__ __launch_bounds__(256) void topk_softmax(const float *__restrict__ logits, int32_t *__restrict__ topk_idx,
                                                    float *__restrict__ topk_w, int N, int E, int k) {
    const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
    const int tok = blockIdx.x * 4 + w;
    if (tok >= N) return;
    float v[kSlots];
#pragma unroll
    for (int c = 0; c < kSlots; ++c) {
        const int e = l + 64 * c;
        v[c] = e < E ? logits[(long)tok * E + e] : -INFINITY;
    }
    wave_topk(v, l, E, k, topk_idx + (long)tok * k, topk_w + (long)tok * k);
}

}  // namespace

hipError_t launch_pack_gate(const void *Wg, void *WgT, int H, int E, hipStream_t s) {
    const int E16 = (E + 15) / 16 * 16;
    const long tot = (long)E16 * H;
    hipLaunchKernelGGL(wg_transpose_bf16, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, s, (const uint16_t *)Wg,
                       (uint16_t *)WgT, H, E, E16);
    return hipGetLastError();
}

hipError_t launch_route(const RouteArgs &a, hipStream_t s) {
    if (a.N <= 0) return hipSuccess;
    if (a.dtype == MOE_BF16) {
        const int E16 = (a.E + 15) / 16 * 16, nb = E16 / 16;
        const long tot = (long)E16 * a.H;
        if (!a.packed)
            hipLaunchKernelGGL(wg_transpose_bf16, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, s,
                               (const uint16_t *)a.Wg, (uint16_t *)a.WgT, a.H, a.E, E16);
        const dim3 g((a.N + 15) / 16), b(512);
        const uint16_t *x = (const uint16_t *)a.x, *wt = (const uint16_t *)(a.packed ? a.Wg : a.WgT);
#define QMOE_GATE(NBV) hipLaunchKernelGGL(gate_topk_bf16<NBV>, g, b, 0, s, x, wt, a.bias, a.logits, a.topk_idx, a.topk_w, a.N, a.H, a.E, nb, a.k)
        if (nb <= 1) QMOE_GATE(1);
        else if (nb <= 2) QMOE_GATE(2);
        else if (nb <= 4) QMOE_GATE(4);
        else if (nb <= 8) QMOE_GATE(8);
        else QMOE_GATE(16);
#undef QMOE_GATE
    } else {
        hipLaunchKernelGGL(gate_logits_f32, dim3((a.N + 3) / 4), dim3(256), 0, s, (const float *)a.x,
                           (const float *)a.Wg, a.bias, a.logits, a.N, a.H, a.E);
        hipLaunchKernelGGL(topk_softmax, dim3((a.N + 3) / 4), dim3(256), 0, s, (const float *)a.logits, a.topk_idx,
                           a.topk_w, a.N, a.E, a.k);
    }
    return hipGetLastError();
}

}  // namespace qmoe

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, once looked up
}  // namespace

extern "C" int32_t moe_route_noalloc(const moe_config *cfg, const void *x, int32_t n_tokens, const void *Wg,
                                     const float *logit_bias, float *logits, int32_t *topk_idx, float *topk_w, void *stream) {
    using qmoe::set_error;
    if (!cfg) return set_error(MOE_E_ARG, "moe_route_noalloc: null config");
    if (cfg->E < 1 || cfg->E > qmoe::kMaxExperts || cfg->k < 1 || cfg->k > cfg->E || cfg->k > qmoe::kMaxTopK || cfg->H < 1 ||
        (cfg->dtype != MOE_F32 && cfg->dtype != MOE_BF16) || (cfg->dtype == MOE_BF16 && cfg->H % 64))
        return set_error(MOE_E_ARG, "moe_route_noalloc: bad configuration (E 1..256, k 1..min(E,32), bf16 needs H a multiple of 64)");
    if (n_tokens < 0 || (int64_t)n_tokens * cfg->k >= (int64_t)1 << 31) return set_error(MOE_E_ARG, "moe_route_noalloc: n_tokens out of range");
    if (!Wg || !logits || !topk_idx || !topk_w || (n_tokens > 0 && !x)) return set_error(MOE_E_ARG, "moe_route_noalloc: null pointer");
    const size_t need = cfg->dtype == MOE_BF16 ? (size_t)((cfg->E + 15) / 16 * 16) * (size_t)cfg->H * 2 : 0;
    if (need > kRouteScratchBytes)
        return set_error(MOE_E_ARG, "moe_route_noalloc: ceil16(E)*H*2 = %zu bytes exceed the %zu-byte static scratch", need,
                         (size_t)kRouteScratchBytes);
    if (n_tokens == 0) return MOE_OK;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return set_error(MOE_E_HIP, "moe_route_noalloc: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return set_error(MOE_E_ARG, "moe_route_noalloc: device %d out of range", dev);
    void *ptr;
    {
        std::lock_guard<std::mutex> lk(g_scratch_mu);
        if (!g_scratch_ptr[dev]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !p)
                return set_error(MOE_E_HIP, "moe_route_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(e));
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    qmoe::RouteArgs a{};
    a.x = x; a.Wg = Wg; a.bias = logit_bias;
    a.WgT = ptr;                  // every element the kernels read is rewritten by this call's transpose first
    a.logits = logits; a.topk_idx = topk_idx; a.topk_w = topk_w;
    a.N = n_tokens; a.H = cfg->H; a.E = cfg->E; a.k = cfg->k; a.dtype = cfg->dtype;
    a.packed = false;
    e = qmoe::launch_route(a, (hipStream_t)stream);
    if (e != hipSuccess) return set_error(MOE_E_HIP, "moe_route_noalloc: launch: %s", hipGetErrorString(e));
    return MOE_OK;
}
