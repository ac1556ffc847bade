// Expert work dispatch: for every row r of a work unit of expert e (token n = perm[r] / k)
//     act[r,:] = silu(W1[e] x[n,:]) (.) (W3[e] x[n,:])        ("gate-up" kernel, SwiGLU fused)
//     out[r,:] = W2[e] act[r,:]                               ("down" kernel)
// Independent per-expert execution over the per-expert queues (Introduction, "Novel MoE Layer
// Design"; Sec. 3.3), one call covering the row segments (or the range [u0, u0+nu) of the device unit
// list) handed over by the host.
#include <hip/hip_runtime.h>

#include "experts_common.h"

namespace qmoe {

hipEvent_t Profiler::get() {
    hipEvent_t e = nullptr;
    if (!pool.empty()) { e = pool.back(); pool.pop_back(); }
    else (void)hipEventCreate(&e);
    return e;
}
void Profiler::begin(int kind, hipStream_t s) {
    live = (kinds >> kind) & 1;
    if (!live) return;
    Span sp{kind, get(), get()};
    (void)hipEventRecord(sp.a, s);
    spans.push_back(sp);
}
void Profiler::end(hipStream_t s) {
    if (live) (void)hipEventRecord(spans.back().b, s);
    live = false;
}

hipError_t launch_experts(const ExpertArgs &a, hipStream_t s) {
    if (a.nu == 0 && a.nseg == 0) return hipSuccess;
    KArgs gu{};
    gu.a_src = a.x; gu.perm = a.perm; gu.b0 = a.W1; gu.b1 = a.W3; gu.dst = a.act; gu.units = a.units;
    gu.b_estride = (long)a.F * a.H; gu.lda = a.H; gu.K = a.H; gu.ncols = a.F; gu.ldd = a.F; gu.kdiv = a.k;
    gu.s0 = a.S1; gu.s1 = a.S3;
    gu.go = a.go; gu.stop = a.stop; gu.cnt_self = a.cnt_gu; gu.cnt_need = nullptr; gu.need = 0;
    gu.u0 = a.u0; gu.nu = (int)a.nu;
    KArgs dn{};
    dn.a_src = a.act; dn.perm = nullptr; dn.b0 = a.W2; dn.b1 = nullptr; dn.dst = a.out; dn.units = a.units;
    dn.b_estride = (long)a.H * a.F; dn.lda = a.F; dn.K = a.F; dn.ncols = a.H; dn.ldd = a.H; dn.kdiv = 1;
    dn.s0 = a.S2; dn.s1 = nullptr;
    dn.go = a.go; dn.stop = a.stop; dn.cnt_self = a.cnt_dn; dn.cnt_need = a.go ? a.cnt_gu : nullptr; dn.need = 0;   // need: set by the launcher
    dn.u0 = a.u0; dn.nu = (int)a.nu;
    if (a.dtype == MOE_F32) launch_experts_f32(a, gu, dn, s);
    else launch_experts_bf16(a, gu, dn, s);
    return hipGetLastError();
}

}  // namespace qmoe
