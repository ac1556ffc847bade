// Host side of libqmoe: context object, workspace carving, call-order state machine, the
// work-unit list and the cursor.  Every arithmetic step runs in the kernels of the other
// translation units; nothing here computes layer values.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <atomic>
#include <chrono>
#include <climits>
#include <cstring>
#include <new>
#include <vector>

#include "qmoe_internal.h"

namespace {

thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int32_t hip_fail(hipError_t e, const char *what) {
    return fail(MOE_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

constexpr size_t kAlign = 256;
constexpr int kReportSpinMs = 200;   // how long moe_permute polls for the kernel's report before it waits for the stream
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

bool config_ok(const moe_config *c, const char **why) {
    *why = "";
    if (!c) { *why = "null config"; return false; }
    if (c->E < 1 || c->E > qmoe::kMaxExperts) { *why = "E out of range (1..256)"; return false; }
    if (c->k < 1 || c->k > c->E || c->k > qmoe::kMaxTopK) { *why = "k out of range (1..min(E,32))"; return false; }
    if (c->H < 1 || c->F < 1) { *why = "H and F must be positive"; return false; }
    if (c->dtype != MOE_F32 && c->dtype != MOE_BF16) { *why = "unknown dtype"; return false; }
    if (c->dtype == MOE_BF16 && (c->H % 64 || c->F % 64)) { *why = "bf16 needs H and F multiples of 64"; return false; }
    if (c->chunk_rows < 1 || c->chunk_rows > qmoe::kMaxChunkRows) { *why = "chunk_rows out of range (1..256)"; return false; }
    if (c->max_tokens < 0) { *why = "max_tokens negative"; return false; }
    if (c->down_ksplit != 0 && c->down_ksplit != 1 && c->down_ksplit != 2 && c->down_ksplit != 4) { *why = "down_ksplit must be 0, 1, 2 or 4"; return false; }
    if (c->down_ksplit > 1 && (c->dtype != MOE_BF16 || c->F % (64 * c->down_ksplit))) { *why = "down_ksplit 2 or 4 needs bf16 and F a multiple of 64 * down_ksplit"; return false; }
    if ((int64_t)c->max_tokens * c->k >= (int64_t)1 << 31) { *why = "max_tokens*k must be below 2^31"; return false; }
    if (c->dtype == MOE_BF16 && ((int64_t)c->max_tokens * c->H * 2 >= (int64_t)1 << 36 ||
                                 (int64_t)c->max_tokens * c->k * c->F * 2 >= (int64_t)1 << 36)) {
        *why = "bf16: x (max_tokens*H) and the activation (max_tokens*k*F) must each stay below 64 GiB";
        return false;
    }
    return true;
}

// Offsets of the workspace regions, computed the same way for sizing and for carving.
struct Layout {
    size_t logits, topk_idx, topk_w, cnt, off, n_units, perm, inv, rank, blockoff, cls, done, go, prog, units, wgt, act, out, partial, total;
    bool has_partial;
    int ksplit;            // 1, 2 or 4: K ranges of the down projection, one partial plane each
    uint32_t max_units;
};

int down_ksplit(const moe_config &c) {
    if (c.down_ksplit) return c.down_ksplit;
    if (c.dtype != MOE_BF16 || (int64_t)c.max_tokens * c.k > (int64_t)256 * c.E) return 1;
    // Weight-streaming shapes: a launch has one workgroup per (expert, 256 columns, K range).  The
    // fewest ranges that give each of the 256 CUs a workgroup: more ranges only add partial planes
    // (Mixtral shape, 512 tokens: 2 ranges 0.17 ms, 4 ranges 0.19-0.20 ms, none 0.26 ms).
    const int64_t wgs = (int64_t)c.E * ((c.H + 255) / 256);
    if (wgs >= 256) return 1;
    if (2 * wgs >= 256 && c.F % 128 == 0) return 2;
    return c.F % 256 == 0 ? 4 : (c.F % 128 == 0 ? 2 : 1);
}

Layout make_layout(const moe_config &c) {
    Layout L{};
    const size_t N = (size_t)c.max_tokens, A = N * (size_t)c.k, E = (size_t)c.E;
    const size_t es = c.dtype == MOE_BF16 ? 2 : 4;
    const size_t nblocks = (A + qmoe::kPermBlock - 1) / qmoe::kPermBlock;
    L.max_units = (uint32_t)(2 * E + (A + (size_t)c.chunk_rows - 1) / (size_t)c.chunk_rows);
    size_t p = 0;
    auto take = [&](size_t bytes) { size_t at = p; p = align_up(p + bytes); return at; };
    L.logits = take(N * E * 4);
    L.topk_idx = take(A * 4);
    L.topk_w = take(A * 4);
    L.cnt = take((2 * E + 1) * 4);      // counts [E][2], then the unit count: read back in one copy
    L.n_units = L.cnt + 2 * E * 4;
    L.off = take((2 * E + 1) * 4);
    L.perm = take(A * 4);
    L.inv = take(A * 4);
    L.rank = take(A * 4);
    L.blockoff = take((nblocks ? nblocks : 1) * 2 * E * 4);
    L.cls = take(N ? N : 1);
    L.done = take(A ? A : 1);           // completion flag per sorted row (moe_combine_complete)
    L.go = take(((size_t)L.max_units + 1) * 4);   // gate words of an enqueued launch sequence
    L.prog = take((A ? 2 * A : 1) * 4);           // its progress: workgroups that ran per row range, gate-up [A] then down [A]
    L.units = take((size_t)L.max_units * sizeof(moe_unit));
    L.wgt = take(((E + 15) / 16 * 16) * (size_t)c.H * 2);
    L.act = take(A * (size_t)c.F * es);
    L.out = take(A * (size_t)c.H * 4);
    // K-split down projection: one partial plane shaped like `out` per K range
    L.ksplit = down_ksplit(c);
    L.has_partial = L.ksplit > 1;
    L.partial = L.has_partial ? take((size_t)L.ksplit * A * (size_t)c.H * 4) : 0;
    L.total = p ? p : kAlign;
    return L;
}

enum State { ST_CREATED = 0, ST_ROUTED = 1, ST_PERMUTED = 2 };

}  // namespace

namespace qmoe {
int32_t set_error(int32_t code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}
}  // namespace qmoe

struct moe_ctx {
    moe_config cfg;
    Layout lay;
    char *ws;
    int state;
    int32_t N;
    uint32_t next_unit, n_units, n_ls_units;   // next_unit: first unit that has not run
    uint32_t n_done, n_ls_done;                // executed units, and how many of them are LS units
    std::vector<moe_unit> units;
    std::vector<uint8_t> executed;             // per unit
    std::vector<uint32_t> unmarked;            // executed units whose rows are not yet flagged on the device
    std::vector<uint32_t> unreduced;           // K-split contexts: executed units whose partial planes have not been added into `out`
    hipStream_t last_stream;                   // stream of the last expert launch (moe_get adds the planes there)
    bool done_valid;                           // the device flags of this layer-batch have been cleared
    bool pending;                              // an enqueued launch sequence has not been collected yet
    std::vector<uint32_t> plan;                // the units of that sequence
    std::vector<qmoe::Seg> plan_ranges;        // the row ranges its launches worked on, in the order of the device's report
    std::vector<int32_t> cnt;
    int32_t *pinned;  // 2E counts, unit count, sequence word, stop word, a spare word, then one completion flag per row
                      // range of an enqueued sequence (at most max_units): pinned host memory mapped into the device
                      // (allocated at first route); the permutation and report kernels write it directly
    int32_t *pinned_dev;   // the device's address of the same memory
    int32_t seq;           // sequence number of the last report asked for
    int spin_ms;           // how long moe_permute polls for the report before it waits for the stream
    int wave_cols;         // 0: the launch policy picks the gate-up wave width; else forced (tests)
    const void *x;
    moe_weights w;
    qmoe::Profiler prof;
    bool prof_on;
};

namespace {
template <class T>
T *at(moe_ctx *c, size_t off) { return reinterpret_cast<T *>(c->ws + off); }
}  // namespace

extern "C" {

const char *moe_last_error(void) { return g_err; }

size_t moe_workspace_bytes(const moe_config *cfg) {
    const char *why;
    if (!config_ok(cfg, &why)) { fail(MOE_E_ARG, "moe_workspace_bytes: %s", why); return 0; }
    return make_layout(*cfg).total;
}

int32_t moe_plan_units(const int32_t *cnt, int32_t E, int32_t chunk_rows, moe_unit *out, uint32_t cap,
                       uint32_t *n_units) {
    if (!cnt || !n_units || E < 1 || chunk_rows < 1 || (cap && !out))
        return fail(MOE_E_ARG, "moe_plan_units: bad argument");
    // Sorted rows are laid out expert-major (LS rows of an expert, then its BE rows); the list
    // walks them priority-major: every LS chunk of every expert, then every BE chunk.
    uint32_t n = 0;
    for (int cls = 0; cls < 2; ++cls) {
        int64_t seg = 0;
        for (int e = 0; e < E; ++e) {
            const int32_t ls = cnt[2 * e], be = cnt[2 * e + 1];
            if (ls < 0 || be < 0) return fail(MOE_E_ARG, "moe_plan_units: negative count");
            const int64_t first = seg + (cls ? ls : 0);
            const int32_t len = cls ? be : ls;
            for (int32_t r = 0; r < len; r += chunk_rows) {
                if (n < cap) {
                    out[n].expert = e;
                    out[n].cls = cls;
                    out[n].row0 = (int32_t)(first + r);
                    out[n].rows = len - r < chunk_rows ? len - r : chunk_rows;
                }
                ++n;
            }
            seg += (int64_t)ls + be;
        }
    }
    *n_units = n;
    return MOE_OK;
}

int32_t moe_pack_weights(const moe_config *cfg, const moe_weights *src, moe_weights *dst, void *stream) {
    const char *why;
    if (!config_ok(cfg, &why)) return fail(MOE_E_ARG, "moe_pack_weights: %s", why);
    if (cfg->dtype != MOE_BF16) return fail(MOE_E_ARG, "moe_pack_weights: bf16 only");
    if (!src || !dst || !src->Wg || !src->W1 || !src->W3 || !src->W2 || !dst->Wg || !dst->W1 || !dst->W3 || !dst->W2)
        return fail(MOE_E_ARG, "moe_pack_weights: null pointer");
    if (src->layout != MOE_W_ROWMAJOR && src->layout != MOE_W_MXFP4_ROWMAJOR)
        return fail(MOE_E_ARG, "moe_pack_weights: source must be row-major (bf16 or 4-bit)");
    if (src->W1 == dst->W1 || src->W3 == dst->W3 || src->W2 == dst->W2 || src->Wg == dst->Wg)
        return fail(MOE_E_ARG, "moe_pack_weights: cannot pack in place");
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (src->layout == MOE_W_MXFP4_ROWMAJOR) {
        if (!src->S1 || !src->S3 || !src->S2 || !dst->S1 || !dst->S3 || !dst->S2)
            return fail(MOE_E_ARG, "moe_pack_weights: 4-bit weights need the scale pointers S1, S3, S2");
        if (src->S1 == dst->S1 || src->S3 == dst->S3 || src->S2 == dst->S2)
            return fail(MOE_E_ARG, "moe_pack_weights: cannot pack in place");
        e = qmoe::launch_pack_mxfp4(src->W1, src->S1, const_cast<void *>(dst->W1), const_cast<void *>(dst->S1), cfg->E, cfg->F, cfg->H, s);
        if (e == hipSuccess) e = qmoe::launch_pack_mxfp4(src->W3, src->S3, const_cast<void *>(dst->W3), const_cast<void *>(dst->S3), cfg->E, cfg->F, cfg->H, s);
        if (e == hipSuccess) e = qmoe::launch_pack_mxfp4(src->W2, src->S2, const_cast<void *>(dst->W2), const_cast<void *>(dst->S2), cfg->E, cfg->H, cfg->F, s);
    } else {
        e = qmoe::launch_pack(src->W1, const_cast<void *>(dst->W1), cfg->E, cfg->F, cfg->H, s);
        if (e == hipSuccess) e = qmoe::launch_pack(src->W3, const_cast<void *>(dst->W3), cfg->E, cfg->F, cfg->H, s);
        if (e == hipSuccess) e = qmoe::launch_pack(src->W2, const_cast<void *>(dst->W2), cfg->E, cfg->H, cfg->F, s);
    }
    if (e == hipSuccess) e = qmoe::launch_pack_gate(src->Wg, const_cast<void *>(dst->Wg), cfg->H, cfg->E, s);
    if (e != hipSuccess) return hip_fail(e, "moe_pack_weights: launch");
    dst->layout = src->layout == MOE_W_MXFP4_ROWMAJOR ? MOE_W_MXFP4 : MOE_W_PACKED;
    return MOE_OK;
}

int32_t moe_create(const moe_config *cfg, void *workspace, size_t workspace_bytes, moe_ctx **out) {
    const char *why;
    if (!out) return fail(MOE_E_ARG, "moe_create: null out pointer");
    *out = nullptr;
    if (!config_ok(cfg, &why)) return fail(MOE_E_ARG, "moe_create: %s", why);
    if (!workspace) return fail(MOE_E_ARG, "moe_create: null workspace");
    Layout lay = make_layout(*cfg);
    if ((uintptr_t)workspace % kAlign) return fail(MOE_E_WORKSPACE, "moe_create: workspace not 256-byte aligned");
    if (workspace_bytes < lay.total)
        return fail(MOE_E_WORKSPACE, "moe_create: workspace has %zu bytes, %zu needed", workspace_bytes, lay.total);
    moe_ctx *c = new (std::nothrow) moe_ctx();
    if (!c) return fail(MOE_E_ARG, "moe_create: out of host memory");
    c->cfg = *cfg;
    c->lay = lay;
    c->ws = static_cast<char *>(workspace);
    c->state = ST_CREATED;
    c->N = 0;
    c->next_unit = c->n_units = c->n_ls_units = c->n_done = c->n_ls_done = 0;
    c->done_valid = false;
    c->pending = false;
    c->last_stream = nullptr;
    c->pinned = nullptr;
    c->pinned_dev = nullptr;
    c->seq = 0;
    c->spin_ms = kReportSpinMs;
    if (const char *v = getenv("QMOE_REPORT_SPIN_MS")) {      // for tests of the fall-back: 0 = do not poll at all
        const long ms = strtol(v, nullptr, 10);
        if (ms >= 0 && ms <= 60000) c->spin_ms = (int)ms;
    }
    c->wave_cols = 0;
    if (const char *v = getenv("QMOE_GATE_UP_WAVE_COLUMNS")) {   // for tests: every bf16 gate-up launch uses this width
        const long cw = strtol(v, nullptr, 10);
        if (cw >= 16 && cw <= 32 && cw % 4 == 0) c->wave_cols = (int)cw;
    }
    c->prof_on = false;
    c->x = nullptr;
    c->w = moe_weights{};
    *out = c;
    return MOE_OK;
}

int32_t moe_destroy(moe_ctx *ctx) {
    if (!ctx) return fail(MOE_E_ARG, "moe_destroy: null context");
    // the gate kernels of an enqueued sequence read the stop word and store the completed count in
    // the pinned buffer: it must not be freed under them
    if (ctx->pending) return fail(MOE_E_STATE, "moe_destroy: an enqueued launch sequence is pending; call moe_expert_collect first");
    if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    for (auto &sp : ctx->prof.spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    for (auto e : ctx->prof.pool) (void)hipEventDestroy(e);
    delete ctx;
    return MOE_OK;
}

int32_t moe_route(moe_ctx *ctx, const void *x, int32_t n_tokens, const moe_weights *w, const float *logit_bias,
                  void *stream) {
    if (!ctx) return fail(MOE_E_ARG, "moe_route: null context");
    if (ctx->pending) return fail(MOE_E_STATE, "moe_route: an enqueued launch sequence is pending; call moe_expert_collect first");
    if (n_tokens < 0 || n_tokens > ctx->cfg.max_tokens)
        return fail(MOE_E_ARG, "moe_route: n_tokens %d outside 0..%d", n_tokens, ctx->cfg.max_tokens);
    if (!w || !w->Wg || !w->W1 || !w->W3 || !w->W2) return fail(MOE_E_ARG, "moe_route: null weight pointer");
    if (w->layout != MOE_W_ROWMAJOR && w->layout != MOE_W_PACKED && w->layout != MOE_W_MXFP4)
        return fail(MOE_E_ARG, "moe_route: weight layout %d is not one the kernels read (row-major 4-bit weights go through moe_pack_weights)", w->layout);
    if (w->layout != MOE_W_ROWMAJOR && ctx->cfg.dtype != MOE_BF16) return fail(MOE_E_ARG, "moe_route: packed weights are bf16 only");
    if (w->layout == MOE_W_MXFP4 && (!w->S1 || !w->S3 || !w->S2)) return fail(MOE_E_ARG, "moe_route: 4-bit weights need the scale pointers S1, S3, S2");
    if (n_tokens > 0 && !x) return fail(MOE_E_ARG, "moe_route: null x");
    if (!ctx->pinned) {
        const size_t words = 2 * (size_t)ctx->cfg.E + 4 + ctx->lay.max_units;   // counts, unit count, sequence word, stop word, spare, range flags
        hipError_t e = hipHostMalloc((void **)&ctx->pinned, words * sizeof(int32_t), hipHostMallocMapped | hipHostMallocCoherent);
        if (e != hipSuccess) { ctx->pinned = nullptr; return hip_fail(e, "moe_route: hipHostMalloc"); }
        e = hipHostGetDevicePointer((void **)&ctx->pinned_dev, ctx->pinned, 0);
        if (e != hipSuccess) {
            (void)hipHostFree(ctx->pinned);
            ctx->pinned = nullptr;
            return hip_fail(e, "moe_route: hipHostGetDevicePointer");
        }
        memset(ctx->pinned, 0, words * sizeof(int32_t));
    }
    if (n_tokens > 0) {
        qmoe::RouteArgs a{};
        a.x = x; a.Wg = w->Wg; a.bias = logit_bias;
        a.WgT = at<void>(ctx, ctx->lay.wgt);
        a.logits = at<float>(ctx, ctx->lay.logits);
        a.topk_idx = at<int32_t>(ctx, ctx->lay.topk_idx);
        a.topk_w = at<float>(ctx, ctx->lay.topk_w);
        a.N = n_tokens; a.H = ctx->cfg.H; a.E = ctx->cfg.E; a.k = ctx->cfg.k; a.dtype = ctx->cfg.dtype;
        a.packed = w->layout != MOE_W_ROWMAJOR;      // Wg transposed and padded
        hipError_t e = qmoe::launch_route(a, (hipStream_t)stream);
        if (e != hipSuccess) return hip_fail(e, "moe_route: launch");
    }
    ctx->N = n_tokens;
    ctx->x = x;
    ctx->w = *w;
    ctx->state = ST_ROUTED;
    ctx->next_unit = ctx->n_units = ctx->n_ls_units = ctx->n_done = ctx->n_ls_done = 0;
    ctx->units.clear();
    ctx->executed.clear();
    ctx->unmarked.clear();
    ctx->unreduced.clear();
    ctx->done_valid = false;
    ctx->cnt.assign(2 * (size_t)ctx->cfg.E, 0);
    return MOE_OK;
}

int32_t moe_permute(moe_ctx *ctx, const uint8_t *prio, moe_cursor *cursor, void *stream) {
    if (!ctx) return fail(MOE_E_ARG, "moe_permute: null context");
    if (!cursor) return fail(MOE_E_ARG, "moe_permute: null cursor");
    if (ctx->state != ST_ROUTED) return fail(MOE_E_STATE, "moe_permute: call moe_route first (once per layer-batch)");
    if (ctx->N > 0 && !prio) return fail(MOE_E_ARG, "moe_permute: null prio");
    const int E = ctx->cfg.E;
    hipStream_t s = (hipStream_t)stream;
    if (ctx->N > 0) {
        qmoe::PermuteArgs a{};
        a.topk_idx = at<int32_t>(ctx, ctx->lay.topk_idx);
        a.prio = prio;
        a.N = ctx->N; a.E = E; a.k = ctx->cfg.k; a.C = ctx->cfg.chunk_rows;
        a.cnt = at<int32_t>(ctx, ctx->lay.cnt);
        a.off = at<int32_t>(ctx, ctx->lay.off);
        a.perm = at<int32_t>(ctx, ctx->lay.perm);
        a.inv = at<int32_t>(ctx, ctx->lay.inv);
        a.rank = at<int32_t>(ctx, ctx->lay.rank);
        a.blockoff = at<int32_t>(ctx, ctx->lay.blockoff);
        a.cls = at<uint8_t>(ctx, ctx->lay.cls);
        a.units = at<moe_unit>(ctx, ctx->lay.units);
        a.n_units = at<int32_t>(ctx, ctx->lay.n_units);
        a.max_units = (int32_t)ctx->lay.max_units;
        ctx->seq = ctx->seq == INT32_MAX ? 1 : ctx->seq + 1;
        a.report = ctx->pinned_dev;
        a.seq = ctx->seq;
        hipError_t e = qmoe::launch_permute(a, s);
        if (e != hipSuccess) return hip_fail(e, "moe_permute: launch");
        // The kernel stores the counts, the unit count and then the sequence word into host memory as
        // soon as it knows them; wait for that word (bounded: after kReportSpinMs fall back to waiting
        // for the stream, which also surfaces a failed launch).
        volatile int32_t *word = ctx->pinned + 2 * E + 1;
        const auto t0 = std::chrono::steady_clock::now();
        bool seen = false;
        for (unsigned spins = 0; ctx->spin_ms > 0; ++spins) {
            if (*word == ctx->seq) { seen = true; break; }
            if ((spins & 1023u) == 1023u &&
                std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(ctx->spin_ms)) break;
        }
        if (!seen) {
            e = hipStreamSynchronize(s);
            if (e != hipSuccess) return hip_fail(e, "moe_permute: waiting for the counts");
            if (*word != ctx->seq) return fail(MOE_E_HIP, "moe_permute: the permutation kernel did not report its counts");
        }
        std::atomic_thread_fence(std::memory_order_acquire);
        ctx->cnt.assign(ctx->pinned, ctx->pinned + 2 * E);
    } else {
        hipError_t e = hipMemsetAsync(at<void>(ctx, ctx->lay.cnt), 0, (2 * (size_t)E + 1) * 4, s);
        if (e == hipSuccess) e = hipMemsetAsync(at<void>(ctx, ctx->lay.off), 0, (2 * (size_t)E + 1) * 4, s);
        if (e != hipSuccess) return hip_fail(e, "moe_permute: clearing the counts");
        ctx->cnt.assign(2 * (size_t)E, 0);
    }
    uint32_t n = 0;
    ctx->units.resize(ctx->lay.max_units);
    int32_t rc = moe_plan_units(ctx->cnt.data(), E, ctx->cfg.chunk_rows, ctx->units.data(), ctx->lay.max_units, &n);
    if (rc != MOE_OK) return rc;
    if (n > ctx->lay.max_units) return fail(MOE_E_HIP, "moe_permute: %u units exceed the bound %u", n, ctx->lay.max_units);
    if (ctx->N > 0 && (int32_t)n != ctx->pinned[2 * E])
        return fail(MOE_E_HIP, "moe_permute: device built %d units, host %u", ctx->pinned[2 * E], n);
    ctx->units.resize(n);
    ctx->n_units = n;
    ctx->n_ls_units = 0;
    for (const moe_unit &u : ctx->units) ctx->n_ls_units += u.cls == 0;
    ctx->next_unit = 0;
    ctx->n_done = ctx->n_ls_done = 0;
    ctx->executed.assign(n, 0);
    ctx->unmarked.clear();
    ctx->unreduced.clear();
    ctx->done_valid = false;
    ctx->state = ST_PERMUTED;
    cursor->next_unit = 0;
    cursor->n_units = n;
    return MOE_OK;
}

// Launches the expert kernels for the listed units (already validated: in range, distinct, not
// yet executed).  go: gate word of the launch on the device for a launch of an enqueued, stoppable
// sequence (its workgroups then also watch the stop word and count themselves per row range), or
// nullptr.  ranges (may be null) receives the row ranges the launches work on.
static int32_t launch_unit_list(moe_ctx *ctx, const void *x, const moe_weights *w, const std::vector<uint32_t> &ids,
                                int32_t *go, std::vector<qmoe::Seg> *ranges, hipStream_t stream, const char *who) {
    if (ids.empty()) return MOE_OK;
    ctx->last_stream = stream;
    qmoe::ExpertArgs a{};
    a.go = go;
    if (go != nullptr) {
        a.stop = ctx->pinned_dev + 2 * ctx->cfg.E + 2;
        a.cnt_gu = at<int32_t>(ctx, ctx->lay.prog);
        a.cnt_dn = a.cnt_gu + (size_t)ctx->N * ctx->cfg.k;
    }
    a.x = x; a.W1 = w->W1; a.W3 = w->W3; a.W2 = w->W2;
    a.perm = at<int32_t>(ctx, ctx->lay.perm);
    a.units = at<moe_unit>(ctx, ctx->lay.units);
    a.act = at<void>(ctx, ctx->lay.act);
    a.out = at<float>(ctx, ctx->lay.out);
    a.H = ctx->cfg.H; a.F = ctx->cfg.F; a.k = ctx->cfg.k; a.dtype = ctx->cfg.dtype;
    a.prof = ctx->prof_on ? &ctx->prof : nullptr;
    a.wfmt = w->layout == MOE_W_MXFP4 ? 2 : (w->layout == MOE_W_PACKED ? 1 : 0);
    a.S1 = w->S1; a.S3 = w->S3; a.S2 = w->S2;
    a.ksplit = ctx->lay.ksplit;
    a.wave_cols = ctx->wave_cols;
    a.partial = ctx->lay.has_partial ? at<float>(ctx, ctx->lay.partial) : nullptr;
    a.plane = (long)ctx->cfg.max_tokens * ctx->cfg.k * ctx->cfg.H;
    const moe_unit *un = ctx->units.data();
    bool contiguous = true;                       // ids = u0, u0+1, ..., a range of the device unit list
    for (size_t i = 1; i < ids.size(); ++i) contiguous = contiguous && ids[i] == ids[i - 1] + 1;
    hipError_t e = hipSuccess;
    if (ctx->cfg.dtype == MOE_BF16) {
        // Row segments: units sorted by (expert, row), row-adjacent units of one expert (its LS part
        // and the start of its BE part, or consecutive chunks) merged while they fit 256 rows, so
        // that one pass over the expert's weights serves them all.  Which rows share a workgroup
        // never changes what is computed for a row.
        std::vector<uint32_t> idx(ids);
        std::stable_sort(idx.begin(), idx.end(), [un](uint32_t p, uint32_t q) {
            if (un[p].expert != un[q].expert) return un[p].expert < un[q].expert;
            return un[p].row0 < un[q].row0;
        });
        // First the runs of row-adjacent units of one expert, then each run cut into ceil(rows/256)
        // segments of (nearly) equal numbers of 32-row tiles: workgroups that share an expert's weight
        // tiles then advance through K at the same pace and meet in L2, which a 256/256/256/128 cut
        // does not give them.
        struct Run { uint32_t row0, rows; uint16_t expert; };
        std::vector<Run> runs;
        for (uint32_t i : idx) {
            const moe_unit &u = un[i];
            if (!runs.empty() && runs.back().expert == (uint16_t)u.expert && runs.back().row0 + runs.back().rows == (uint32_t)u.row0)
                runs.back().rows += (uint32_t)u.rows;
            else
                runs.push_back(Run{(uint32_t)u.row0, (uint32_t)u.rows, (uint16_t)u.expert});
        }
        std::vector<qmoe::Seg> segs;
        for (const Run &r : runs) {
            const uint32_t nseg = (r.rows + 255) / 256, tiles = (r.rows + 31) / 32;
            const uint32_t base = tiles / nseg, extra = tiles % nseg;
            uint32_t row = r.row0, left = r.rows;
            for (uint32_t j = 0; j < nseg; ++j) {
                const uint32_t want = (base + (j < extra ? 1 : 0)) * 32;
                const uint32_t take = want < left ? want : left;
                segs.push_back(qmoe::Seg{row, (uint16_t)take, r.expert});
                row += take;
                left -= take;
            }
        }
        if (segs.size() > (size_t)qmoe::kMaxSegs && contiguous) {
            // too many segments for the kernel arguments: the launch reads the device unit list
            if (ranges)
                for (uint32_t i : ids) ranges->push_back(qmoe::Seg{(uint32_t)un[i].row0, (uint16_t)un[i].rows, (uint16_t)un[i].expert});
            a.u0 = ids.front(); a.nu = (uint32_t)ids.size();
            a.max_rows = 0;
            for (uint32_t i : ids) a.max_rows = std::max(a.max_rows, (int)un[i].rows);
            a.segs = nullptr; a.nseg = 0;
            e = qmoe::launch_experts(a, stream);
        } else {
            if (ranges) ranges->insert(ranges->end(), segs.begin(), segs.end());
            for (size_t s0 = 0; s0 < segs.size() && e == hipSuccess; s0 += qmoe::kMaxSegs) {
                const size_t cnt = std::min(segs.size() - s0, (size_t)qmoe::kMaxSegs);
                a.segs = segs.data() + s0; a.nseg = (int)cnt;
                a.u0 = 0; a.nu = 0;
                a.max_rows = 0;
                for (size_t i = 0; i < cnt; ++i) a.max_rows = std::max(a.max_rows, (int)segs[s0 + i].rows);
                e = qmoe::launch_experts(a, stream);
            }
        }
    } else {
        // fp32 kernels walk ranges of the device unit list: one launch per run of consecutive ids
        if (ranges)
            for (uint32_t i : ids) ranges->push_back(qmoe::Seg{(uint32_t)un[i].row0, (uint16_t)un[i].rows, (uint16_t)un[i].expert});
        for (size_t i = 0; i < ids.size() && e == hipSuccess;) {
            size_t j = i + 1;
            while (j < ids.size() && ids[j] == ids[j - 1] + 1) ++j;
            a.u0 = ids[i]; a.nu = (uint32_t)(j - i);
            a.max_rows = 0;
            for (size_t q = i; q < j; ++q) a.max_rows = std::max(a.max_rows, (int)un[ids[q]].rows);
            a.segs = nullptr; a.nseg = 0;
            e = qmoe::launch_experts(a, stream);
            i = j;
        }
    }
    if (e != hipSuccess) return hip_fail(e, who);
    return MOE_OK;
}

// Books units as executed and moves the cursor to the first unit that has not run.
static void book_units(moe_ctx *ctx, const std::vector<uint32_t> &ids) {
    for (uint32_t i : ids) {
        ctx->executed[i] = 1;
        ctx->n_done += 1;
        ctx->n_ls_done += ctx->units[i].cls == 0;
        ctx->unmarked.push_back(i);
        if (ctx->lay.has_partial) ctx->unreduced.push_back(i);
    }
    while (ctx->next_unit < ctx->n_units && ctx->executed[ctx->next_unit]) ++ctx->next_unit;
}

static int32_t run_unit_list(moe_ctx *ctx, const void *x, const moe_weights *w, const std::vector<uint32_t> &ids,
                             hipStream_t stream, const char *who) {
    const int32_t rc = launch_unit_list(ctx, x, w, ids, nullptr, nullptr, stream, who);
    if (rc == MOE_OK) book_units(ctx, ids);
    return rc;
}

static int32_t check_run_args(moe_ctx *ctx, const void *x, const moe_weights *w, const char *who) {
    if (!ctx) return fail(MOE_E_ARG, "%s: null context", who);
    if (ctx->state != ST_PERMUTED) return fail(MOE_E_STATE, "%s: call moe_permute first", who);
    if (ctx->pending) return fail(MOE_E_STATE, "%s: an enqueued launch sequence is pending; call moe_expert_collect first", who);
    if (!w || (ctx->N > 0 && !x)) return fail(MOE_E_ARG, "%s: null x or weights", who);
    if (x != ctx->x || w->W1 != ctx->w.W1 || w->W3 != ctx->w.W3 || w->W2 != ctx->w.W2 || w->layout != ctx->w.layout ||
        w->S1 != ctx->w.S1 || w->S3 != ctx->w.S3 || w->S2 != ctx->w.S2)
        return fail(MOE_E_ARG, "%s: x and weights must be the tensors given to moe_route", who);
    return MOE_OK;
}

int32_t moe_expert_run(moe_ctx *ctx, const void *x, const moe_weights *w, uint32_t max_units, moe_cursor *cursor,
                       void *stream) {
    if (ctx && !cursor) return fail(MOE_E_ARG, "moe_expert_run: null cursor");
    int32_t rc = check_run_args(ctx, x, w, "moe_expert_run");
    if (rc != MOE_OK) return rc;
    if (cursor->n_units != ctx->n_units || cursor->next_unit != ctx->next_unit)
        return fail(MOE_E_ARG, "moe_expert_run: cursor {%u,%u} is not this context's {%u,%u}", cursor->next_unit,
                    cursor->n_units, ctx->next_unit, ctx->n_units);
    std::vector<uint32_t> ids;
    for (uint32_t u = ctx->next_unit; u < ctx->n_units && ids.size() < (size_t)max_units; ++u)
        if (!ctx->executed[u]) ids.push_back(u);
    rc = run_unit_list(ctx, x, w, ids, (hipStream_t)stream, "moe_expert_run: launch");
    if (rc != MOE_OK) return rc;
    cursor->next_unit = ctx->next_unit;
    return ctx->n_done == ctx->n_units ? MOE_DONE : MOE_OK;
}

int32_t moe_expert_run_units(moe_ctx *ctx, const void *x, const moe_weights *w, const uint32_t *unit_ids, uint32_t n,
                             moe_cursor *cursor, void *stream) {
    int32_t rc = check_run_args(ctx, x, w, "moe_expert_run_units");
    if (rc != MOE_OK) return rc;
    if (n > 0 && !unit_ids) return fail(MOE_E_ARG, "moe_expert_run_units: null unit_ids");
    std::vector<uint32_t> ids(unit_ids, unit_ids + n);
    std::vector<uint8_t> seen(ctx->n_units, 0);
    for (uint32_t u : ids) {
        if (u >= ctx->n_units) return fail(MOE_E_ARG, "moe_expert_run_units: unit %u out of range (%u units)", u, ctx->n_units);
        if (ctx->executed[u]) return fail(MOE_E_ARG, "moe_expert_run_units: unit %u has already been executed", u);
        if (seen[u]) return fail(MOE_E_ARG, "moe_expert_run_units: unit %u listed twice", u);
        seen[u] = 1;
    }
    rc = run_unit_list(ctx, x, w, ids, (hipStream_t)stream, "moe_expert_run_units: launch");
    if (rc != MOE_OK) return rc;
    if (cursor) { cursor->next_unit = ctx->next_unit; cursor->n_units = ctx->n_units; }
    return ctx->n_done == ctx->n_units ? MOE_DONE : MOE_OK;
}

int32_t moe_expert_enqueue(moe_ctx *ctx, const void *x, const moe_weights *w, uint32_t units_per_launch, void *stream) {
    int32_t rc = check_run_args(ctx, x, w, "moe_expert_enqueue");
    if (rc != MOE_OK) return rc;
    if (units_per_launch == 0) return fail(MOE_E_ARG, "moe_expert_enqueue: units_per_launch must be at least 1");
    hipStream_t s = (hipStream_t)stream;
    std::vector<std::vector<uint32_t>> groups;
    for (uint32_t u = ctx->next_unit; u < ctx->n_units; ++u) {
        if (ctx->executed[u]) continue;
        if (groups.empty() || groups.back().size() >= units_per_launch) groups.emplace_back();
        groups.back().push_back(u);
    }
    if (groups.empty()) return MOE_DONE;
    const int E = ctx->cfg.E;
    // No kernel of an earlier sequence is left (it was collected): clear the range flags the report
    // kernel will set, so that a sequence cut short by an error reports nothing, and the stop word.
    memset(ctx->pinned + 2 * E + 4, 0, (size_t)ctx->lay.max_units * sizeof(int32_t));
    __atomic_store_n(ctx->pinned + 2 * E + 2, 0, __ATOMIC_SEQ_CST);
    const int32_t *stop_dev = ctx->pinned_dev + 2 * E + 2;
    int32_t *go = at<int32_t>(ctx, ctx->lay.go);
    ctx->plan.clear();
    ctx->plan_ranges.clear();
    ctx->pending = true;     // from here on the stream holds launches that read this context's state
    // the progress counters of the row ranges start at zero (a fill kernel: the call may be captured)
    hipError_t e = qmoe::launch_clear_words(at<int32_t>(ctx, ctx->lay.prog), 2 * (long)ctx->N * ctx->cfg.k, s);
    if (e != hipSuccess) return hip_fail(e, "moe_expert_enqueue: clearing the counters");
    for (size_t g = 0; g < groups.size(); ++g) {
        e = qmoe::launch_gate(stop_dev, go, (int)g, s);
        if (e != hipSuccess) return hip_fail(e, "moe_expert_enqueue: gate");
        rc = launch_unit_list(ctx, x, w, groups[g], go + g, &ctx->plan_ranges, s, "moe_expert_enqueue: launch");
        if (rc != MOE_OK) return rc;
        ctx->plan.insert(ctx->plan.end(), groups[g].begin(), groups[g].end());
    }
    if (ctx->plan_ranges.size() > ctx->lay.max_units)
        return fail(MOE_E_HIP, "moe_expert_enqueue: %zu row ranges exceed the bound %u", ctx->plan_ranges.size(), ctx->lay.max_units);
    // behind the last launch: which row ranges are complete, written to host memory
    e = qmoe::launch_report(ctx->plan_ranges.data(), (int)ctx->plan_ranges.size(),
                            at<int32_t>(ctx, ctx->lay.prog) + (size_t)ctx->N * ctx->cfg.k,
                            ctx->pinned_dev + 2 * E + 4, ctx->cfg.dtype, ctx->cfg.H, ctx->lay.ksplit, s);
    if (e != hipSuccess) return hip_fail(e, "moe_expert_enqueue: report");
    return MOE_OK;
}

int32_t moe_expert_stop(moe_ctx *ctx) {
    if (!ctx) return fail(MOE_E_ARG, "moe_expert_stop: null context");
    if (!ctx->pinned) return fail(MOE_E_STATE, "moe_expert_stop: nothing has been routed on this context");
    __atomic_store_n(ctx->pinned + 2 * ctx->cfg.E + 2, 1, __ATOMIC_SEQ_CST);
    return MOE_OK;
}

int32_t moe_expert_collect(moe_ctx *ctx, moe_cursor *cursor, void *stream) {
    if (!ctx) return fail(MOE_E_ARG, "moe_expert_collect: null context");
    if (!cursor) return fail(MOE_E_ARG, "moe_expert_collect: null cursor");
    if (ctx->state != ST_PERMUTED) return fail(MOE_E_STATE, "moe_expert_collect: call moe_permute first");
    if (ctx->pending) {
        hipError_t e = hipStreamSynchronize((hipStream_t)stream);
        if (e != hipSuccess) return hip_fail(e, "moe_expert_collect: waiting for the stream");
        std::atomic_thread_fence(std::memory_order_acquire);
        // A unit has run when every row range that overlaps it is complete.  Ranges are disjoint, so a
        // table over the sorted rows of the sequence decides it.
        const volatile int32_t *ok = ctx->pinned + 2 * ctx->cfg.E + 4;
        std::vector<uint8_t> row_ok((size_t)ctx->N * ctx->cfg.k, 0);
        for (size_t i = 0; i < ctx->plan_ranges.size(); ++i) {
            const int32_t v = ok[i];
            if (v != 0 && v != 1) return fail(MOE_E_HIP, "moe_expert_collect: the device reports %d for row range %zu", v, i);
            if (v) std::fill(row_ok.begin() + ctx->plan_ranges[i].row0, row_ok.begin() + ctx->plan_ranges[i].row0 + ctx->plan_ranges[i].rows, 1);
        }
        std::vector<uint32_t> ran;
        for (uint32_t u : ctx->plan) {
            const moe_unit &un = ctx->units[u];
            bool all = true;
            for (int32_t r = un.row0; r < un.row0 + un.rows && all; ++r) all = row_ok[(size_t)r] != 0;
            if (all) ran.push_back(u);
        }
        book_units(ctx, ran);
        ctx->plan.clear();
        ctx->plan_ranges.clear();
        ctx->pending = false;
        __atomic_store_n(ctx->pinned + 2 * ctx->cfg.E + 2, 0, __ATOMIC_SEQ_CST);
    }
    cursor->next_unit = ctx->next_unit;
    cursor->n_units = ctx->n_units;
    return ctx->n_done == ctx->n_units ? MOE_DONE : MOE_OK;
}

// Where the combine reads the expert outputs: `out`, or, on a context with a K-split down projection,
// the partial planes, which it adds as it reads them.
static void fill_out_source(moe_ctx *ctx, qmoe::CombineArgs &a) {
    if (ctx->lay.has_partial) {
        a.out = at<float>(ctx, ctx->lay.partial);
        a.ksplit = ctx->lay.ksplit;
        a.plane = (long)ctx->cfg.max_tokens * ctx->cfg.k * ctx->cfg.H;
    } else {
        a.out = at<float>(ctx, ctx->lay.out);
        a.ksplit = 1;
        a.plane = 0;
    }
}

int32_t moe_combine(moe_ctx *ctx, void *y, int32_t class_mask, void *stream) {
    if (!ctx) return fail(MOE_E_ARG, "moe_combine: null context");
    if (ctx->state != ST_PERMUTED) return fail(MOE_E_STATE, "moe_combine: call moe_permute first");
    if (ctx->pending) return fail(MOE_E_STATE, "moe_combine: an enqueued launch sequence is pending; call moe_expert_collect first");
    const bool y_f32 = (class_mask & MOE_Y_F32) != 0;
    class_mask &= ~MOE_Y_F32;
    if (class_mask < 1 || class_mask > 3) return fail(MOE_E_ARG, "moe_combine: class_mask must be 1, 2 or 3 (optionally | MOE_Y_F32)");
    if (ctx->N > 0 && !y) return fail(MOE_E_ARG, "moe_combine: null y");
    const uint32_t ls_left = ctx->n_ls_units - ctx->n_ls_done;
    const uint32_t be_left = (ctx->n_units - ctx->n_ls_units) - (ctx->n_done - ctx->n_ls_done);
    if ((class_mask & MOE_CLASS_LS) && ls_left)
        return fail(MOE_E_INCOMPLETE, "moe_combine: LS tokens still have %u unexecuted units", ls_left);
    if ((class_mask & MOE_CLASS_BE) && be_left)
        return fail(MOE_E_INCOMPLETE, "moe_combine: BE tokens still have %u unexecuted units", be_left);
    if (ctx->N == 0) return MOE_OK;
    qmoe::CombineArgs a{};
    fill_out_source(ctx, a);
    a.topk_w = at<float>(ctx, ctx->lay.topk_w);
    a.inv = at<int32_t>(ctx, ctx->lay.inv);
    a.cls = at<uint8_t>(ctx, ctx->lay.cls);
    a.y = y;
    a.N = ctx->N; a.H = ctx->cfg.H; a.k = ctx->cfg.k; a.dtype = y_f32 ? MOE_F32 : ctx->cfg.dtype; a.class_mask = class_mask;
    hipError_t e = qmoe::launch_combine(a, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "moe_combine: launch");
    return MOE_OK;
}

int32_t moe_combine_complete(moe_ctx *ctx, void *y, uint8_t *complete, void *stream) {
    if (!ctx) return fail(MOE_E_ARG, "moe_combine_complete: null context");
    if (ctx->state != ST_PERMUTED) return fail(MOE_E_STATE, "moe_combine_complete: call moe_permute first");
    if (ctx->pending) return fail(MOE_E_STATE, "moe_combine_complete: an enqueued launch sequence is pending; call moe_expert_collect first");
    if (ctx->N > 0 && !y) return fail(MOE_E_ARG, "moe_combine_complete: null y");
    if (ctx->N == 0) return MOE_OK;
    hipStream_t s = (hipStream_t)stream;
    uint8_t *done = at<uint8_t>(ctx, ctx->lay.done);
    // Bring the device's per-row completion flags up to date with what has been executed since
    // the last call (they are not maintained on the moe_expert_run path, which does not need them).
    hipError_t e = hipSuccess;
    if (!ctx->done_valid) {
        e = qmoe::launch_clear_done(done, (long)ctx->N * ctx->cfg.k, s);
        if (e != hipSuccess) return hip_fail(e, "moe_combine_complete: clearing the flags");
        ctx->done_valid = true;
    }
    if (!ctx->unmarked.empty()) {
        std::vector<qmoe::Seg> segs;
        segs.reserve(ctx->unmarked.size());
        for (uint32_t u : ctx->unmarked)
            segs.push_back(qmoe::Seg{(uint32_t)ctx->units[u].row0, (uint16_t)ctx->units[u].rows, (uint16_t)ctx->units[u].expert});
        e = qmoe::launch_mark_done(segs.data(), (int)segs.size(), done, s);
        if (e != hipSuccess) return hip_fail(e, "moe_combine_complete: setting the flags");
        ctx->unmarked.clear();
    }
    qmoe::CombineArgs a{};
    fill_out_source(ctx, a);
    a.topk_w = at<float>(ctx, ctx->lay.topk_w);
    a.inv = at<int32_t>(ctx, ctx->lay.inv);
    a.cls = at<uint8_t>(ctx, ctx->lay.cls);
    a.done = done;
    a.complete = complete;
    a.y = y;
    a.N = ctx->N; a.H = ctx->cfg.H; a.k = ctx->cfg.k; a.dtype = ctx->cfg.dtype; a.class_mask = MOE_CLASS_ALL;
    e = qmoe::launch_combine(a, s);
    if (e != hipSuccess) return hip_fail(e, "moe_combine_complete: launch");
    return MOE_OK;
}

int32_t moe_get(moe_ctx *ctx, int32_t what, const void **dev_ptr, size_t *bytes) {
    if (!ctx || !dev_ptr || !bytes) return fail(MOE_E_ARG, "moe_get: null argument");
    if (ctx->state == ST_CREATED) return fail(MOE_E_STATE, "moe_get: nothing routed yet");
    const size_t N = (size_t)ctx->N, A = N * (size_t)ctx->cfg.k, E = (size_t)ctx->cfg.E;
    const size_t es = ctx->cfg.dtype == MOE_BF16 ? 2 : 4;
    size_t off = 0, sz = 0;
    const bool need_perm = what >= MOE_GET_COUNTS;
    if (need_perm && ctx->state != ST_PERMUTED) return fail(MOE_E_STATE, "moe_get: call moe_permute first");
    switch (what) {
        case MOE_GET_LOGITS: off = ctx->lay.logits; sz = N * E * 4; break;
        case MOE_GET_TOPK_IDX: off = ctx->lay.topk_idx; sz = A * 4; break;
        case MOE_GET_TOPK_W: off = ctx->lay.topk_w; sz = A * 4; break;
        case MOE_GET_COUNTS: off = ctx->lay.cnt; sz = 2 * E * 4; break;
        case MOE_GET_OFFSETS: off = ctx->lay.off; sz = (2 * E + 1) * 4; break;
        case MOE_GET_PERM: off = ctx->lay.perm; sz = A * 4; break;
        case MOE_GET_INV: off = ctx->lay.inv; sz = A * 4; break;
        case MOE_GET_EXPERT_OUT:
            off = ctx->lay.out; sz = A * (size_t)ctx->cfg.H * 4;
            if (ctx->pending) return fail(MOE_E_STATE, "moe_get: an enqueued launch sequence is pending; call moe_expert_collect first");
            if (!ctx->unreduced.empty()) {
                // K-split context: the down projection left partial planes, which moe_combine adds on
                // the fly; materialise the rows executed since the last request, behind the launches
                // that produced them
                std::vector<qmoe::Seg> segs;
                segs.reserve(ctx->unreduced.size());
                for (uint32_t u : ctx->unreduced)
                    segs.push_back(qmoe::Seg{(uint32_t)ctx->units[u].row0, (uint16_t)ctx->units[u].rows, (uint16_t)ctx->units[u].expert});
                hipError_t e = qmoe::launch_reduce_planes(segs.data(), (int)segs.size(), at<float>(ctx, ctx->lay.partial),
                                                          at<float>(ctx, ctx->lay.out), ctx->cfg.H, ctx->lay.ksplit,
                                                          (long)ctx->cfg.max_tokens * ctx->cfg.k * ctx->cfg.H, ctx->last_stream);
                if (e != hipSuccess) return hip_fail(e, "moe_get: adding the partial planes");
                ctx->unreduced.clear();
            }
            break;
        case MOE_GET_ACT: off = ctx->lay.act; sz = A * (size_t)ctx->cfg.F * es; break;
        case MOE_GET_UNITS: off = ctx->lay.units; sz = (size_t)ctx->n_units * sizeof(moe_unit); break;
        default: return fail(MOE_E_ARG, "moe_get: unknown item %d", what);
    }
    *dev_ptr = ctx->ws + off;
    *bytes = sz;
    return MOE_OK;
}

int32_t moe_profile(moe_ctx *ctx, int32_t kinds) {
    if (!ctx) return fail(MOE_E_ARG, "moe_profile: null context");
    if (kinds < 0 || kinds > MOE_PROF_ALL) return fail(MOE_E_ARG, "moe_profile: kinds must be a mask of MOE_PROF_* bits (0..%d)", MOE_PROF_ALL);
    ctx->prof_on = kinds != 0;
    ctx->prof.kinds = kinds;
    return MOE_OK;
}

int32_t moe_profile_read(moe_ctx *ctx, float *ms, uint32_t *launches) {
    if (!ctx || !ms || !launches) return fail(MOE_E_ARG, "moe_profile_read: null argument");
    for (int i = 0; i < MOE_PROF_KINDS; ++i) { ms[i] = 0.f; launches[i] = 0; }
    for (auto &sp : ctx->prof.spans) {
        hipError_t e = hipEventSynchronize(sp.b);
        float t = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&t, sp.a, sp.b);
        if (e != hipSuccess) return hip_fail(e, "moe_profile_read");
        ms[sp.kind] += t;
        launches[sp.kind] += 1;
        ctx->prof.pool.push_back(sp.a);
        ctx->prof.pool.push_back(sp.b);
    }
    ctx->prof.spans.clear();
    return MOE_OK;
}

int32_t moe_units(moe_ctx *ctx, moe_unit *out, uint32_t cap, uint32_t *n_units) {
    if (!ctx || !n_units || (cap && !out)) return fail(MOE_E_ARG, "moe_units: null argument");
    if (ctx->state != ST_PERMUTED) return fail(MOE_E_STATE, "moe_units: call moe_permute first");
    const uint32_t n = ctx->n_units < cap ? ctx->n_units : cap;
    if (n) memcpy(out, ctx->units.data(), (size_t)n * sizeof(moe_unit));
    *n_units = ctx->n_units;
    return MOE_OK;
}

}  // extern "C"
