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
    const int32_t *go;      // gated launches: the workgroups do nothing unless *go != 0 (nullptr: not gated)
};

struct Scope {
    Profiler *p; hipStream_t s;
    Scope(Profiler *p_, int kind, hipStream_t s_) : p(p_), s(s_) { if (p) p->begin(kind, s); }
    ~Scope() { if (p) p->end(s); }
};

void launch_experts_f32(const ExpertArgs &a, const KArgs &gu, const KArgs &dn, hipStream_t s);
void launch_experts_bf16(const ExpertArgs &a, const KArgs &gu, const KArgs &dn, hipStream_t s);

}  // namespace qmoe
