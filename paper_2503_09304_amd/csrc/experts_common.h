// Shared by the expert kernels' translation units: kernel arguments and the profiling scope.
#pragma once

#include <hip/hip_runtime.h>

#include "qmoe_internal.h"

namespace qmoe {

struct KArgs {
    const void *a_src;      // x [N,H] (gate-up) or act [A,F] (down)
    const int32_t *perm;    // gate-up: sorted row -> assignment id; down: nullptr
    const void *b0, *b1;    // gate-up: W1, W3; down: W2, unused
    const void *s0, *s1;    // 4-bit weights: the block scales of b0, b1 (else nullptr)
    void *dst;              // gate-up: act; down: out (fp32)
    const moe_unit *units;
    long b_estride;         // elements per expert in b0/b1
    int lda, K, ncols, ldd, kdiv;
    unsigned u0;
    int nu;                 // units in this launch
    int col_tiles;
    int cw;                 // bf16 gate-up: output columns per wave (32, or 28 .. 16 in steps of 4)
    // Launches of an enqueued, stoppable sequence (nullptr / 0 otherwise): see wg_may_run.
    int32_t *go;              // [device] gate word of the launch: 0 = the sequence was stopped (before this launch, or by a
                              // workgroup of it that saw the stop word: the ones that start later leave at once)
    const int32_t *stop;      // [host memory mapped into the device] the context's stop word
    int32_t *cnt_self;        // [device] workgroups of this kernel that ran, per row range, indexed by its first sorted row
    const int32_t *cnt_need;  // down projection: the gate-up kernel's counters (the activation rows must be complete)
    int need;                 // gate-up workgroups per 64-row tile (fp32) or per row range (bf16) that make them complete
};

// Entry protocol of a workgroup of a stoppable launch; the same answer for every thread of the
// workgroup (one thread decides, LDS and a barrier hand the decision to the others: threads reading
// the host's stop word on their own could see different values).  The workgroup runs, and is counted,
// unless the launch's gate is closed, the stop word is set, or (down projection) the gate-up
// workgroups of its row range did not all run.  Nothing waits: a workgroup that may not run returns.
// row0: first sorted row of the row range; tiles: how many `need`-sized groups of gate-up workgroups
// cover it.
// The bf16 kernels split it in two so that the read of the host's stop word (a trip over the bus)
// overlaps with the loads of their prologue: wg_probe issues the reads at the start of the
// workgroup, wg_decide turns them into the decision in front of the prologue's barrier, and the
// workgroup leaves behind that barrier if *s_run is 0 (nothing has been stored by then).
struct WgProbe { int stop, have; };
__device__ __forceinline__ WgProbe wg_probe(const KArgs &p, int row0) {
    WgProbe v{0, 0};
    if (p.go != nullptr && threadIdx.x == 0) {
        v.stop = __hip_atomic_load(p.stop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
        v.have = p.cnt_need != nullptr ? p.cnt_need[row0] : 0;
    }
    return v;
}
__device__ __forceinline__ void wg_decide(const KArgs &p, int row0, int tiles, const WgProbe &v, int *s_run) {
    if (p.go != nullptr && threadIdx.x == 0) {
        const bool ok = v.stop == 0 && (p.cnt_need == nullptr || v.have == p.need * tiles);
        if (ok) atomicAdd(p.cnt_self + row0, 1);
        if (v.stop != 0) __hip_atomic_store(p.go, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // close the launch for the rest
        *s_run = ok ? 1 : 0;
    }
}

__device__ __forceinline__ bool wg_may_run(const KArgs &p, int row0, int tiles, int *s_run) {
    if (p.go == nullptr) return true;
    if (threadIdx.x == 0) {
        bool ok = __hip_atomic_load(p.go, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
        if (ok && __hip_atomic_load(p.stop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != 0) {
            __hip_atomic_store(p.go, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // close the launch for the rest
            ok = false;
        }
        if (ok && p.cnt_need != nullptr) ok = p.cnt_need[row0] == p.need * tiles;
        if (ok) atomicAdd(p.cnt_self + row0, 1);
        *s_run = ok ? 1 : 0;
    }
    __syncthreads();
    return *s_run != 0;
}

struct Scope {
    Profiler *p; hipStream_t s;
    Scope(Profiler *p_, int kind, hipStream_t s_) : p(p_), s(s_) { if (p) p->begin(kind, s); }
    ~Scope() { if (p) p->end(s); }
};

void launch_experts_f32(const ExpertArgs &a, const KArgs &gu, const KArgs &dn, hipStream_t s);
void launch_experts_bf16(const ExpertArgs &a, const KArgs &gu, const KArgs &dn, hipStream_t s);

}  // namespace qmoe
