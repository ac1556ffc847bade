// Per-expert priority queues as a stable counting sort (Sec. 3.3: per-expert FIFO queues;
// Sec. 3.2 / Algorithm 1: latency-sensitive work before best-effort work).
//
// Assignment a = n*k + slot has bucket key 2*expert + (LS ? 0 : 1).  Sorting the assignments by
// (key, a) gives, per expert, its LS tokens in arrival order followed by its BE tokens in arrival
// order.  Small batches run the whole sort in one workgroup (perm_fused); larger ones take three
// kernels, integer work only:
//   perm_rank    every wave finds, with one ballot per key bit, the lanes that share its key
//                (rank inside the wave = popcount of the lower lanes); the 16 waves of a workgroup
//                are chained through LDS counters -> rank inside the 1024-assignment block, and
//                the block's per-bucket totals.
//   perm_scan    one workgroup: running totals over blocks per bucket, bucket offsets, and the
//                work-unit list (phase LS then BE; experts ascending; chunks of C rows).
//   perm_scatter position = bucket offset + block offset + rank; writes perm and inv.
#include <hip/hip_runtime.h>

#include "qmoe_internal.h"

namespace qmoe {
namespace {

__global__ __launch_bounds__(kPermBlock) void perm_rank(const int32_t *__restrict__ topk_idx,
                                                        const uint8_t *__restrict__ prio, int A, int k, int nb,
                                                        int nbits, int32_t *__restrict__ rank,
                                                        int32_t *__restrict__ blockcnt, uint8_t *__restrict__ cls) {
    extern __shared__ int32_t wavecnt[];  // [16][nb]
    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    for (int i = tid; i < 16 * nb; i += kPermBlock) wavecnt[i] = 0;
    __syncthreads();
    const int a = blockIdx.x * kPermBlock + tid;
    const bool valid = a < A;
    int key = 0;
    if (valid) {
        const int n = a / k;
        const int c = prio[n] ? 0 : 1;
        key = topk_idx[a] * 2 + c;
        if (a - n * k == 0) cls[n] = (uint8_t)c;
    }
    unsigned long long m = __ballot(valid);
    for (int b = 0; b < nbits; ++b) {
        const bool bit = (key >> b) & 1;
        const unsigned long long bal = __ballot(valid && bit);
        m &= bit ? bal : ~bal;
    }
    const int r_in_wave = __popcll(m & ((1ull << l) - 1ull));
    if (valid && r_in_wave == 0) wavecnt[w * nb + key] = __popcll(m);
    __syncthreads();
    for (int b = tid; b < nb; b += kPermBlock) {
        int run = 0;
        for (int ww = 0; ww < 16; ++ww) {
            const int c = wavecnt[ww * nb + b];
            wavecnt[ww * nb + b] = run;
            run += c;
        }
        blockcnt[(long)blockIdx.x * nb + b] = run;
    }
    __syncthreads();
    if (valid) rank[a] = wavecnt[w * nb + key] + r_in_wave;
}

// Exclusive scan of v[0..n) held in LDS (n <= 1024), result in place, returns the total.
__device__ int block_excl_scan(int32_t *v, int32_t *tmp, int n) {
    const int tid = threadIdx.x;
    int32_t *src = v, *dst = tmp;
    for (int d = 1; d < n; d <<= 1) {
        for (int i = tid; i < n; i += blockDim.x) dst[i] = src[i] + (i >= d ? src[i - d] : 0);
        __syncthreads();
        int32_t *t = src; src = dst; dst = t;
    }
    // src holds the inclusive scan
    const int total = n > 0 ? src[n - 1] : 0;
    __syncthreads();
    for (int i = tid; i < n; i += blockDim.x) dst[i] = i ? src[i - 1] : 0;
    __syncthreads();
    if (dst != v)
        for (int i = tid; i < n; i += blockDim.x) v[i] = dst[i];
    __syncthreads();
    return total;
}

// The engine's report to the scheduler after the router stage (Sec. 3.2): the queue lengths and the
// unit count go straight into host memory as soon as they are known, before the ranking work, and the
// sequence word is stored last, after a system-scope fence, so a host that sees the sequence number
// sees the report.  Called by every thread of the one workgroup that knows the totals.
__device__ __forceinline__ void report_to_host(int32_t *__restrict__ report, int32_t seq, const int32_t *tot, int nb, int nu) {
    for (int b = threadIdx.x; b < nb; b += blockDim.x) report[b] = tot[b];
    if (threadIdx.x == 0) report[nb] = nu;
    __threadfence_system();
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(report + nb + 1, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ __launch_bounds__(1024) void perm_scan(int32_t *__restrict__ blockcnt, int nblocks, int E, int C,
                                                  int32_t *__restrict__ cnt, int32_t *__restrict__ off,
                                                  moe_unit *__restrict__ units, int32_t *__restrict__ n_units,
                                                  int max_units, int32_t *__restrict__ report, int32_t seq) {
    __shared__ int32_t tot[2 * kMaxExperts];
    __shared__ int32_t boff[2 * kMaxExperts];
    __shared__ int32_t ustart[2 * kMaxExperts];
    __shared__ int32_t tmp[2 * kMaxExperts];
    const int nb = 2 * E, tid = threadIdx.x;
    // Per bucket, the exclusive prefix over the blocks.  The 1024 threads cut the blocks into
    // `slices` ranges per bucket (thread = (slice, bucket)): sums of the ranges, their prefix through
    // LDS, then each thread rewrites its range; the loads of a range do not depend on one another.
    __shared__ int32_t part[1024];
    const int slices = blockDim.x / nb > 0 ? blockDim.x / nb : 1;
    const int per = (nblocks + slices - 1) / slices;
    for (int b0 = 0; b0 < nb; b0 += blockDim.x) {            // one pass unless there are more buckets than threads
        const int sl = slices > 1 ? tid / nb : 0;
        const int b = b0 + (slices > 1 ? tid - sl * nb : tid);
        const bool active = b < nb && sl < slices;
        const int blk0 = sl * per, blk1 = min(nblocks, blk0 + per);
        int sum = 0;
        if (active)
            for (int blk = blk0; blk < blk1; ++blk) sum += blockcnt[(long)blk * nb + b];
        if (active && slices > 1) part[sl * nb + (b - b0)] = sum;
        __syncthreads();
        int run = 0;
        if (active && slices > 1) {
            int total = 0;
            for (int q = 0; q < slices; ++q) {
                const int v = part[q * nb + (b - b0)];
                if (q < sl) run += v;
                total += v;
            }
            sum = total;
        }
        if (active) {
            for (int blk = blk0; blk < blk1; ++blk) {
                const int c = blockcnt[(long)blk * nb + b];
                blockcnt[(long)blk * nb + b] = run;
                run += c;
            }
            if (sl == 0) { tot[b] = sum; boff[b] = sum; }
        }
        __syncthreads();
    }
    const int total = block_excl_scan(boff, tmp, nb);
    for (int b = tid; b < nb; b += blockDim.x) {
        cnt[b] = tot[b];
        off[b] = boff[b];
    }
    if (tid == 0) off[nb] = total;
    // unit list: order index q = cls*E + e
    for (int q = tid; q < nb; q += blockDim.x) {
        const int cl = q / E, e = q - cl * E;
        ustart[q] = (tot[2 * e + cl] + C - 1) / C;
    }
    __syncthreads();
    const int nu = block_excl_scan(ustart, tmp, nb);
    if (tid == 0) *n_units = nu;
    report_to_host(report, seq, tot, nb, nu);
    for (int q = tid; q < nb; q += blockDim.x) {
        const int cl = q / E, e = q - cl * E;
        const int len = tot[2 * e + cl], first = boff[2 * e + cl];
        int u = ustart[q];
        for (int r = 0; r < len; r += C, ++u) {
            if (u < max_units) {
                moe_unit v;
                v.expert = e; v.cls = cl; v.row0 = first + r; v.rows = len - r < C ? len - r : C;
                units[u] = v;
            }
        }
    }
}

__global__ __launch_bounds__(256) void perm_scatter(const int32_t *__restrict__ topk_idx, const uint8_t *__restrict__ prio,
                                                    int A, int k, int nb, const int32_t *__restrict__ rank,
                                                    const int32_t *__restrict__ blockoff, const int32_t *__restrict__ off,
                                                    int32_t *__restrict__ perm, int32_t *__restrict__ inv) {
    const int a = blockIdx.x * 256 + threadIdx.x;
    if (a >= A) return;
    const int n = a / k;
    const int key = topk_idx[a] * 2 + (prio[n] ? 0 : 1);
    const int pos = off[key] + blockoff[(long)(a / kPermBlock) * nb + key] + rank[a];
    perm[pos] = a;
    inv[a] = pos;
}

// The whole sort in one workgroup, for batches of at most kPermFusedMax assignments (latency
// matters more than parallelism there): LDS-atomic histogram, bucket scan and unit list, then the
// blocks of 1024 assignments ranked one after the other with running per-bucket counters.
constexpr int kPermFusedMax = 8192;

__global__ __launch_bounds__(kPermBlock) void perm_fused(const int32_t *__restrict__ topk_idx, const uint8_t *__restrict__ prio,
                                                         int A, int k, int E, int C, int nbits, int32_t *__restrict__ cnt,
                                                         int32_t *__restrict__ off, int32_t *__restrict__ perm,
                                                         int32_t *__restrict__ inv, uint8_t *__restrict__ cls,
                                                         moe_unit *__restrict__ units, int32_t *__restrict__ n_units,
                                                         int max_units, int32_t *__restrict__ report, int32_t seq) {
    extern __shared__ int32_t sm[];
    const int nb = 2 * E, tid = threadIdx.x, w = tid >> 6, l = tid & 63;
    int32_t *tot = sm, *boff = sm + nb, *ustart = sm + 2 * nb, *tmp = sm + 3 * nb, *running = sm + 4 * nb;
    int32_t *wavecnt = sm + 5 * nb;  // [16][nb]
    for (int b = tid; b < nb; b += kPermBlock) { tot[b] = 0; running[b] = 0; }
    __syncthreads();
    for (int a = tid; a < A; a += kPermBlock) {
        const int n = a / k;
        const int c = prio[n] ? 0 : 1;
        atomicAdd(&tot[topk_idx[a] * 2 + c], 1);
        if (a - n * k == 0) cls[n] = (uint8_t)c;
    }
    __syncthreads();
    // The report leaves as soon as the histogram is complete: wave 0 writes the counts and the number
    // of units they imply, fences, and stores the sequence word, while the other waves go on.
    if (w == 0) {
        int nu_part = 0;
        for (int b = l; b < nb; b += 64) {
            report[b] = tot[b];
            nu_part += (tot[b] + C - 1) / C;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) nu_part += __shfl_xor(nu_part, o, 64);
        if (l == 0) report[nb] = nu_part;
        __threadfence_system();
        if (l == 0) __hip_atomic_store(report + nb + 1, seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    for (int b = tid; b < nb; b += kPermBlock) boff[b] = tot[b];
    __syncthreads();
    const int total = block_excl_scan(boff, tmp, nb);
    for (int b = tid; b < nb; b += kPermBlock) { cnt[b] = tot[b]; off[b] = boff[b]; }
    if (tid == 0) off[nb] = total;
    for (int q = tid; q < nb; q += kPermBlock) {
        const int cl = q / E, e = q - cl * E;
        ustart[q] = (tot[2 * e + cl] + C - 1) / C;
    }
    __syncthreads();
    const int nu = block_excl_scan(ustart, tmp, nb);
    if (tid == 0) *n_units = nu;
    for (int q = tid; q < nb; q += kPermBlock) {
        const int cl = q / E, e = q - cl * E;
        const int len = tot[2 * e + cl], first = boff[2 * e + cl];
        int u = ustart[q];
        for (int r = 0; r < len; r += C, ++u) {
            if (u < max_units) {
                moe_unit v;
                v.expert = e; v.cls = cl; v.row0 = first + r; v.rows = len - r < C ? len - r : C;
                units[u] = v;
            }
        }
    }
    // stable ranks, block by block
    for (int base = 0; base < A; base += kPermBlock) {
        for (int i = tid; i < 16 * nb; i += kPermBlock) wavecnt[i] = 0;
        __syncthreads();
        const int a = base + tid;
        const bool valid = a < A;
        int key = 0;
        if (valid) key = topk_idx[a] * 2 + (prio[a / k] ? 0 : 1);
        unsigned long long m = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {
            const bool bit = (key >> b) & 1;
            const unsigned long long bal = __ballot(valid && bit);
            m &= bit ? bal : ~bal;
        }
        const int r_in_wave = __popcll(m & ((1ull << l) - 1ull));
        if (valid && r_in_wave == 0) wavecnt[w * nb + key] = __popcll(m);
        __syncthreads();
        for (int b = tid; b < nb; b += kPermBlock) {
            int run = running[b];
            for (int ww = 0; ww < 16; ++ww) {
                const int c = wavecnt[ww * nb + b];
                wavecnt[ww * nb + b] = run;
                run += c;
            }
            running[b] = run;
        }
        __syncthreads();
        if (valid) {
            const int pos = boff[key] + wavecnt[w * nb + key] + r_in_wave;
            perm[pos] = a;
            inv[a] = pos;
        }
        __syncthreads();
    }
}

}  // namespace

hipError_t launch_permute(const PermuteArgs &a, hipStream_t s) {
    const int A = a.N * a.k;
    if (A <= 0) return hipSuccess;
    const int nb = 2 * a.E;
    int nbits = 0;
    while ((1 << nbits) < nb) ++nbits;
    const int nblocks = (A + kPermBlock - 1) / kPermBlock;
    if (A <= kPermFusedMax) {
        hipLaunchKernelGGL(perm_fused, dim3(1), dim3(kPermBlock), (size_t)(5 + 16) * nb * sizeof(int32_t), s, a.topk_idx,
                           a.prio, A, a.k, a.E, a.C, nbits, a.cnt, a.off, a.perm, a.inv, a.cls, a.units, a.n_units,
                           a.max_units, a.report, a.seq);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(perm_rank, dim3(nblocks), dim3(kPermBlock), (size_t)16 * nb * sizeof(int32_t), s, a.topk_idx,
                       a.prio, A, a.k, nb, nbits, a.rank, a.blockoff, a.cls);
    hipLaunchKernelGGL(perm_scan, dim3(1), dim3(1024), 0, s, a.blockoff, nblocks, a.E, a.C, a.cnt, a.off, a.units,
                       a.n_units, a.max_units, a.report, a.seq);
    hipLaunchKernelGGL(perm_scatter, dim3((A + 255) / 256), dim3(256), 0, s, a.topk_idx, a.prio, A, a.k, nb, a.rank,
                       (const int32_t *)a.blockoff, (const int32_t *)a.off, a.perm, a.inv);
    return hipGetLastError();
}

}  // namespace qmoe
