// Internal declarations shared by the host API and the kernel translation units of libqmoe.
// Not part of the public ABI (that is include/qmoe.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "qmoe.h"

namespace qmoe {

constexpr int kPermBlock = 1024;  // assignments ranked by one workgroup of the counting sort
constexpr int kMaxExperts = 256;  // 2*E bucket counters of a 16-wave workgroup must fit in LDS
constexpr int kMaxTopK = 32;
constexpr int kMaxChunkRows = 256;

// A launch of at most this many row segments carries them in its kernel arguments (and may merge
// row-adjacent units of one expert into one segment); larger launches read the device unit list.
constexpr int kMaxSegs = 384;

// Rows [row0, row0+rows) of the sorted order, all of one expert: what one workgroup column works on.
struct Seg {
    uint32_t row0;
    uint16_t rows;    // 1..256
    uint16_t expert;
};

struct RouteArgs {
    const void *x;
    const void *Wg;
    const float *bias;
    void *WgT;  // scratch: bf16 [E16][H], Wg transposed and padded to a multiple of 16 experts
    float *logits;
    int32_t *topk_idx;
    float *topk_w;
    int N, H, E, k, dtype;
    bool packed;  // Wg already transposed and padded ([E16][H])
};
hipError_t launch_route(const RouteArgs &a, hipStream_t s);

// Records the text moe_last_error() returns on this thread and hands `code` back (printf-style).
int32_t set_error(int32_t code, const char *fmt, ...);

struct PermuteArgs {
    const int32_t *topk_idx;
    const uint8_t *prio;
    int N, E, k, C;
    int32_t *cnt;       // [E][2]
    int32_t *off;       // [2E+1]
    int32_t *perm;      // [A]
    int32_t *inv;       // [A]
    int32_t *rank;      // scratch [A]
    int32_t *blockoff;  // scratch [nblocks][2E]
    uint8_t *cls;       // [N] 0 = LS, 1 = BE
    moe_unit *units;    // device unit list
    int32_t *n_units;   // device scalar
    int32_t max_units;
    int32_t *report;    // host memory mapped into the device: counts [2E], unit count, sequence word
    int32_t seq;        // value the kernel stores into the sequence word once the report is written
};
hipError_t launch_permute(const PermuteArgs &a, hipStream_t s);

// Optional event bracketing of the expert launches (benchmarks only).
struct Profiler {
    struct Span { int kind; hipEvent_t a, b; };
    std::vector<Span> spans;        // recorded since the last read
    std::vector<hipEvent_t> pool;   // events free for reuse
    int kinds = 0;                  // bit mask of the kernel kinds to bracket
    bool live = false;              // the span opened by the last begin() is being recorded
    hipEvent_t get();
    void begin(int kind, hipStream_t s);
    void end(hipStream_t s);
};

struct ExpertArgs {
    const void *x;
    const void *W1, *W3, *W2;
    const int32_t *perm;
    const moe_unit *units;  // device list
    void *act;              // [A,F] dtype
    float *out;             // [A,H]
    int H, F, k, dtype;
    uint32_t u0, nu;        // units [u0, u0+nu)
    int max_rows;           // largest rows among the segments (or units) of the launch
    Profiler *prof;             // nullptr unless timing is on
    int wfmt;                   // expert weights: 0 bf16 row-major, 1 bf16 in MFMA-ordered blocks, 2 4-bit blocks
    const void *S1, *S3, *S2;   // 4-bit weights: block scales
    const Seg *segs;            // host array [nseg] (nseg <= kMaxSegs), or nullptr: use the unit list
    int nseg;
    int ksplit;                 // 1, 2 or 4 K ranges (down projection; fixed per context)
    int wave_cols;              // bf16 gate-up: columns per wave, 0 = chosen per launch
    float *partial;             // [ksplit][A][H] fp32 partial planes of the K-split down projection, or nullptr
                                // (they stay as they are: moe_combine adds them, launch_reduce_planes on request)
    long plane;                 // elements per plane
    // launches of an enqueued, stoppable sequence (all nullptr otherwise; see launch_gate, launch_report)
    int32_t *go;                // [device] gate word of this launch
    const int32_t *stop;        // [host, mapped] the context's stop word
    int32_t *cnt_gu, *cnt_dn;   // [device] workgroups that ran per row range (indexed by first sorted row): gate-up, down
};

// Workgroups of the down projection that cover a row range of `rows` rows: what its counter reads
// when the range is complete.
__host__ __device__ inline int down_wgs_of_range(int dtype, int H, int ksplit, int rows) {
    return dtype == MOE_BF16 ? ((H + 255) / 256) * ksplit : ((H + 63) / 64) * ((rows + 63) / 64);
}
hipError_t launch_experts(const ExpertArgs &a, hipStream_t s);

// out[r,:] = ((p0 + p1) + p2) + p3 (p0 + p1 with two planes) for the rows of the segments: what
// moe_combine computes on the fly, materialised for a caller that asks for the expert outputs.
hipError_t launch_reduce_planes(const Seg *segs, int nseg, const float *partial, float *out, int H, int ksplit, long plane,
                                hipStream_t s);

// Re-layout of one [E][R][K] bf16 tensor into the packed block order (see MOE_W_PACKED).
hipError_t launch_pack(const void *src, void *dst, int E, int R, int K, hipStream_t s);
// Re-layout of 4-bit codes [E][R][K/2] and scales [E][R][K/32] into the MOE_W_MXFP4 block order.
hipError_t launch_pack_mxfp4(const void *codes, const void *scales, void *dcodes, void *dscales, int E, int R, int K,
                             hipStream_t s);
hipError_t launch_pack_gate(const void *Wg, void *WgT, int H, int E, hipStream_t s);

struct CombineArgs {
    const float *out;      // [A,H]; with ksplit > 1: the first of ksplit partial planes, `plane` elements apart
    int ksplit;            // 1, 2 or 4
    long plane;
    const float *topk_w;   // [N,k]
    const int32_t *inv;    // [A]
    const uint8_t *cls;    // [N]
    const uint8_t *done;   // [A] per sorted row, or nullptr: select by class_mask
    uint8_t *complete;     // [N] out (with done), or nullptr
    void *y;               // [N,H] dtype
    int N, H, k, dtype, class_mask;
};
hipError_t launch_combine(const CombineArgs &a, hipStream_t s);
// Gate in front of launch g of an enqueued sequence (moe_expert_enqueue): one thread,
// go[g] = (g == 0 || go[g-1]) && *stop == 0.  Once a gate closes every later one stays closed, so the
// workgroups of the launches behind a stop leave after one read of device memory.
hipError_t launch_gate(const int32_t *stop_host, int32_t *go, int g, hipStream_t s);
// Behind the last launch of the sequence: ok_host[i] (host memory, mapped) = 1 if all `need(rows)`
// down-projection workgroups of row range i ran (cnt_dn[row0] == down_wgs_of_range), else 0.
hipError_t launch_report(const Seg *ranges, int n, const int32_t *cnt_dn, int32_t *ok_host, int dtype, int H, int ksplit,
                         hipStream_t s);
hipError_t launch_clear_words(int32_t *p, long n, hipStream_t s);
// Completion flags per sorted row (used by moe_combine_complete): clear all, set the rows of segments.
hipError_t launch_clear_done(uint8_t *done, long n, hipStream_t s);
hipError_t launch_mark_done(const Seg *segs, int n, uint8_t *done, hipStream_t s);

}  // namespace qmoe
