// Recording stand-ins for the kernel launchers of libqmoe (see hip/hip_runtime.h in this folder).
// The permutation "kernel" reports the queue lengths the test planted; the expert launcher records
// the row ranges it was asked to run; the report "kernel" of an enqueued sequence marks as complete
// the ranges the test says ran.  Nothing here computes layer values.
#include <algorithm>
#include <vector>

#include "qmoe_internal.h"
#include "stub_hooks.h"

namespace {
std::vector<int32_t> g_counts;                 // [E][2], planted by the test
std::vector<StubLaunch> g_launches;            // every expert launch since the last reset
int g_complete_first = -1;                     // report: ranges [0, n) complete; -1 = all
}  // namespace

extern "C" {
void stub_set_counts(const int32_t *cnt, int n) { g_counts.assign(cnt, cnt + n); }
void stub_reset_launches(void) { g_launches.clear(); }
int stub_n_launches(void) { return (int)g_launches.size(); }
const StubLaunch *stub_launch(int i) { return &g_launches[(size_t)i]; }
void stub_complete_first(int n) { g_complete_first = n; }
}

namespace qmoe {

hipEvent_t Profiler::get() { return nullptr; }
void Profiler::begin(int, hipStream_t) {}
void Profiler::end(hipStream_t) {}

hipError_t launch_route(const RouteArgs &, hipStream_t) { return hipSuccess; }

hipError_t launch_permute(const PermuteArgs &a, hipStream_t) {
    // what the real kernel stores into host memory: 2E counts, the unit count, then the sequence word
    int32_t n_units = 0;
    for (int i = 0; i < 2 * a.E; ++i) {
        const int32_t c = i < (int)g_counts.size() ? g_counts[(size_t)i] : 0;
        a.report[i] = c;
        a.cnt[i] = c;
        n_units += (c + a.C - 1) / a.C;
    }
    a.report[2 * a.E] = n_units;
    *a.n_units = n_units;
    // the device unit list, in the documented order (phase LS then BE, experts ascending, chunks of C)
    int n = 0;
    for (int cls = 0; cls < 2; ++cls) {
        int seg = 0;
        for (int e = 0; e < a.E; ++e) {
            const int ls = a.cnt[2 * e], be = a.cnt[2 * e + 1];
            const int first = seg + (cls ? ls : 0), len = cls ? be : ls;
            for (int r = 0; r < len; r += a.C)
                if (n < a.max_units) a.units[n++] = moe_unit{e, cls, first + r, std::min(a.C, len - r)};
            seg += ls + be;
        }
    }
    a.report[2 * a.E + 1] = a.seq;
    return hipSuccess;
}

hipError_t launch_experts(const ExpertArgs &a, hipStream_t) {
    StubLaunch L{};
    L.gated = a.go != nullptr;
    L.nseg = a.nseg;
    L.u0 = a.u0;
    L.nu = a.nu;
    L.max_rows = a.max_rows;
    for (int i = 0; i < a.nseg && i < STUB_MAX_SEGS; ++i) {
        L.row0[i] = a.segs[i].row0;
        L.rows[i] = a.segs[i].rows;
        L.expert[i] = a.segs[i].expert;
    }
    g_launches.push_back(L);
    return hipSuccess;
}

hipError_t launch_pack(const void *, void *, int, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_pack_mxfp4(const void *, const void *, void *, void *, int, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_pack_gate(const void *, void *, int, int, hipStream_t) { return hipSuccess; }
hipError_t launch_reduce_planes(const Seg *, int, const float *, float *, int, int, long, hipStream_t) { return hipSuccess; }
hipError_t launch_combine(const CombineArgs &, hipStream_t) { return hipSuccess; }
hipError_t launch_gate(const int32_t *, int32_t *go, int g, hipStream_t) { go[g] = 1; return hipSuccess; }
hipError_t launch_report(const Seg *, int n, const int32_t *, int32_t *ok_host, int, int, int, hipStream_t) {
    for (int i = 0; i < n; ++i) ok_host[i] = (g_complete_first < 0 || i < g_complete_first) ? 1 : 0;
    return hipSuccess;
}
hipError_t launch_clear_words(int32_t *p, long n, hipStream_t) { std::fill(p, p + n, 0); return hipSuccess; }
hipError_t launch_clear_done(uint8_t *p, long n, hipStream_t) { std::fill(p, p + n, (uint8_t)0); return hipSuccess; }
hipError_t launch_mark_done(const Seg *segs, int n, uint8_t *done, hipStream_t) {
    for (int i = 0; i < n; ++i) std::fill(done + segs[i].row0, done + segs[i].row0 + segs[i].rows, (uint8_t)1);
    return hipSuccess;
}

}  // namespace qmoe
