// Host side of libqmoe: context object, workspace carving, call-order state machine, the
// work-unit list and the cursor.  Every arithmetic step runs in the kernels of the other
// translation units; nothing here computes layer values.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <algorithm>
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
    if (c->down_ksplit != 0 && c->down_ksplit != 1 && c->down_ksplit != 4) { *why = "down_ksplit must be 0, 1 or 4"; return false; }
    if (c->down_ksplit == 4 && (c->dtype != MOE_BF16 || c->F % 256)) { *why = "down_ksplit 4 needs bf16 and F a multiple of 256"; return false; }
    if ((int64_t)c->max_tokens * c->k >= (int64_t)1 << 31) { *why = "max_tokens*k must be below 2^31"; return false; }
    if (c->dtype == MOE_BF16 && ((int64_t)c->max_tokens * c->H * 2 >= (int64_t)1 << 32 ||
                                 (int64_t)c->max_tokens * c->k * c->F * 2 >= (int64_t)1 << 32)) {
        *why = "bf16: x (max_tokens*H) and the activation (max_tokens*k*F) must each stay below 4 GiB";
        return false;
    }
    return true;
}

// Offsets of the workspace regions, computed the same way for sizing and for carving.
struct Layout {
    size_t logits, topk_idx, topk_w, cnt, off, n_units, perm, inv, rank, blockoff, cls, units, wgt, act, out, partial, total;
    bool has_partial;
    uint32_t max_units;
};

int down_ksplit(const moe_config &c) {
    if (c.dtype != MOE_BF16 || c.F % 256) return 1;
    if (c.down_ksplit) return c.down_ksplit;
    return (int64_t)c.max_tokens * c.k <= (int64_t)256 * c.E ? 4 : 1;
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
    L.units = take((size_t)L.max_units * sizeof(moe_unit));
    L.wgt = take(((E + 15) / 16 * 16) * (size_t)c.H * 2);
    L.act = take(A * (size_t)c.F * es);
    L.out = take(A * (size_t)c.H * 4);
    // K-split down projection (bf16, F a multiple of 256): four partial planes shaped like `out`
    L.has_partial = down_ksplit(c) == 4;
    L.partial = L.has_partial ? take(4 * A * (size_t)c.H * 4) : 0;
    L.total = p ? p : kAlign;
    return L;
}

enum State { ST_CREATED = 0, ST_ROUTED = 1, ST_PERMUTED = 2 };

}  // namespace

struct moe_ctx {
    moe_config cfg;
    Layout lay;
    char *ws;
    int state;
    int32_t N;
    uint32_t next_unit, n_units, n_ls_units;
    std::vector<moe_unit> units;
    std::vector<int32_t> cnt;
    int32_t *pinned;  // 2E counts + 1 unit count, pinned host memory (allocated at first route)
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
    if (src->layout != MOE_W_ROWMAJOR) return fail(MOE_E_ARG, "moe_pack_weights: source must be row-major");
    if (src->W1 == dst->W1 || src->W3 == dst->W3 || src->W2 == dst->W2 || src->Wg == dst->Wg)
        return fail(MOE_E_ARG, "moe_pack_weights: cannot pack in place");
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = qmoe::launch_pack(src->W1, const_cast<void *>(dst->W1), cfg->E, cfg->F, cfg->H, s);
    if (e == hipSuccess) e = qmoe::launch_pack(src->W3, const_cast<void *>(dst->W3), cfg->E, cfg->F, cfg->H, s);
    if (e == hipSuccess) e = qmoe::launch_pack(src->W2, const_cast<void *>(dst->W2), cfg->E, cfg->H, cfg->F, s);
    if (e == hipSuccess) e = qmoe::launch_pack_gate(src->Wg, const_cast<void *>(dst->Wg), cfg->H, cfg->E, s);
    if (e != hipSuccess) return hip_fail(e, "moe_pack_weights: launch");
    dst->layout = MOE_W_PACKED;
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
    c->next_unit = c->n_units = c->n_ls_units = 0;
    c->pinned = nullptr;
    c->prof_on = false;
    c->x = nullptr;
    c->w = moe_weights{};
    *out = c;
    return MOE_OK;
}

int32_t moe_destroy(moe_ctx *ctx) {
    if (!ctx) return fail(MOE_E_ARG, "moe_destroy: null context");
    if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    for (auto &sp : ctx->prof.spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
    for (auto e : ctx->prof.pool) (void)hipEventDestroy(e);
    delete ctx;
    return MOE_OK;
}

int32_t moe_route(moe_ctx *ctx, const void *x, int32_t n_tokens, const moe_weights *w, const float *logit_bias,
                  void *stream) {
    if (!ctx) return fail(MOE_E_ARG, "moe_route: null context");
    if (n_tokens < 0 || n_tokens > ctx->cfg.max_tokens)
        return fail(MOE_E_ARG, "moe_route: n_tokens %d outside 0..%d", n_tokens, ctx->cfg.max_tokens);
    if (!w || !w->Wg || !w->W1 || !w->W3 || !w->W2) return fail(MOE_E_ARG, "moe_route: null weight pointer");
    if (w->layout != MOE_W_ROWMAJOR && w->layout != MOE_W_PACKED) return fail(MOE_E_ARG, "moe_route: unknown weight layout %d", w->layout);
    if (w->layout == MOE_W_PACKED && ctx->cfg.dtype != MOE_BF16) return fail(MOE_E_ARG, "moe_route: packed weights are bf16 only");
    if (n_tokens > 0 && !x) return fail(MOE_E_ARG, "moe_route: null x");
    if (!ctx->pinned) {
        hipError_t e = hipHostMalloc((void **)&ctx->pinned, (2 * (size_t)ctx->cfg.E + 1) * sizeof(int32_t), hipHostMallocDefault);
        if (e != hipSuccess) { ctx->pinned = nullptr; return hip_fail(e, "moe_route: hipHostMalloc"); }
    }
    if (n_tokens > 0) {
        qmoe::RouteArgs a{};
        a.x = x; a.Wg = w->Wg; a.bias = logit_bias;
        a.WgT = at<void>(ctx, ctx->lay.wgt);
        a.logits = at<float>(ctx, ctx->lay.logits);
        a.topk_idx = at<int32_t>(ctx, ctx->lay.topk_idx);
        a.topk_w = at<float>(ctx, ctx->lay.topk_w);
        a.N = n_tokens; a.H = ctx->cfg.H; a.E = ctx->cfg.E; a.k = ctx->cfg.k; a.dtype = ctx->cfg.dtype;
        a.packed = w->layout == MOE_W_PACKED;
        hipError_t e = qmoe::launch_route(a, (hipStream_t)stream);
        if (e != hipSuccess) return hip_fail(e, "moe_route: launch");
    }
    ctx->N = n_tokens;
    ctx->x = x;
    ctx->w = *w;
    ctx->state = ST_ROUTED;
    ctx->next_unit = ctx->n_units = ctx->n_ls_units = 0;
    ctx->units.clear();
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
        hipError_t e = qmoe::launch_permute(a, s);
        if (e != hipSuccess) return hip_fail(e, "moe_permute: launch");
        e = hipMemcpyAsync(ctx->pinned, a.cnt, (2 * (size_t)E + 1) * sizeof(int32_t), hipMemcpyDeviceToHost, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) return hip_fail(e, "moe_permute: reading the counts back");
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
    ctx->state = ST_PERMUTED;
    cursor->next_unit = 0;
    cursor->n_units = n;
    return MOE_OK;
}

int32_t moe_expert_run(moe_ctx *ctx, const void *x, const moe_weights *w, uint32_t max_units, moe_cursor *cursor,
                       void *stream) {
    if (!ctx) return fail(MOE_E_ARG, "moe_expert_run: null context");
    if (!cursor) return fail(MOE_E_ARG, "moe_expert_run: null cursor");
    if (ctx->state != ST_PERMUTED) return fail(MOE_E_STATE, "moe_expert_run: call moe_permute first");
    if (cursor->n_units != ctx->n_units || cursor->next_unit != ctx->next_unit)
        return fail(MOE_E_ARG, "moe_expert_run: cursor {%u,%u} is not this context's {%u,%u}", cursor->next_unit,
                    cursor->n_units, ctx->next_unit, ctx->n_units);
    if (!w || (ctx->N > 0 && !x)) return fail(MOE_E_ARG, "moe_expert_run: null x or weights");
    if (x != ctx->x || w->W1 != ctx->w.W1 || w->W3 != ctx->w.W3 || w->W2 != ctx->w.W2 || w->layout != ctx->w.layout)
        return fail(MOE_E_ARG, "moe_expert_run: x and weights must be the tensors given to moe_route");
    const uint32_t u0 = ctx->next_unit;
    const uint32_t left = ctx->n_units - u0;
    const uint32_t nu = max_units < left ? max_units : left;
    if (nu > 0) {
        qmoe::ExpertArgs a{};
        a.x = x; a.W1 = w->W1; a.W3 = w->W3; a.W2 = w->W2;
        a.perm = at<int32_t>(ctx, ctx->lay.perm);
        a.units = at<moe_unit>(ctx, ctx->lay.units);
        a.act = at<void>(ctx, ctx->lay.act);
        a.out = at<float>(ctx, ctx->lay.out);
        a.H = ctx->cfg.H; a.F = ctx->cfg.F; a.k = ctx->cfg.k; a.dtype = ctx->cfg.dtype;
        a.u0 = u0; a.nu = nu;
        a.prof = ctx->prof_on ? &ctx->prof : nullptr;
        a.packed = w->layout == MOE_W_PACKED;
        a.ksplit = ctx->lay.has_partial ? 4 : 1;
        a.partial = ctx->lay.has_partial ? at<float>(ctx, ctx->lay.partial) : nullptr;
        a.plane = (long)ctx->cfg.max_tokens * ctx->cfg.k * ctx->cfg.H;
        // Row segments of this launch: units sorted by (expert, row), row-adjacent units of one
        // expert (its LS part and the start of its BE part, or consecutive chunks) merged while they
        // fit 256 rows, so that one pass over the expert's weights serves them all.  Which rows
        // share a workgroup never changes what is computed for a row.
        std::vector<qmoe::Seg> segs;
        a.max_rows = 0;
        if (ctx->cfg.dtype == MOE_BF16) {
            std::vector<uint32_t> idx(nu);
            for (uint32_t i = 0; i < nu; ++i) idx[i] = u0 + i;
            const moe_unit *un = ctx->units.data();
            std::stable_sort(idx.begin(), idx.end(), [un](uint32_t x, uint32_t y) {
                if (un[x].expert != un[y].expert) return un[x].expert < un[y].expert;
                return un[x].row0 < un[y].row0;
            });
            for (uint32_t i : idx) {
                const moe_unit &u = un[i];
                if (!segs.empty()) {
                    qmoe::Seg &b = segs.back();
                    if (b.expert == (uint16_t)u.expert && b.row0 + b.rows == (uint32_t)u.row0 && b.rows + u.rows <= 256) {
                        b.rows = (uint16_t)(b.rows + u.rows);
                        continue;
                    }
                }
                segs.push_back(qmoe::Seg{(uint32_t)u.row0, (uint16_t)u.rows, (uint16_t)u.expert});
            }
            if (segs.size() > (size_t)qmoe::kMaxSegs) segs.clear();
        }
        if (!segs.empty()) {
            for (const qmoe::Seg &g : segs) if (g.rows > a.max_rows) a.max_rows = g.rows;
            a.segs = segs.data();
            a.nseg = (int)segs.size();
        } else {
            for (uint32_t u = u0; u < u0 + nu; ++u) if (ctx->units[u].rows > a.max_rows) a.max_rows = ctx->units[u].rows;
            a.segs = nullptr;
            a.nseg = 0;
        }
        hipError_t e = qmoe::launch_experts(a, (hipStream_t)stream);
        if (e != hipSuccess) return hip_fail(e, "moe_expert_run: launch");
    }
    ctx->next_unit = u0 + nu;
    cursor->next_unit = ctx->next_unit;
    return ctx->next_unit == ctx->n_units ? MOE_DONE : MOE_OK;
}

int32_t moe_combine(moe_ctx *ctx, void *y, int32_t class_mask, void *stream) {
    if (!ctx) return fail(MOE_E_ARG, "moe_combine: null context");
    if (ctx->state != ST_PERMUTED) return fail(MOE_E_STATE, "moe_combine: call moe_permute first");
    if (class_mask < 1 || class_mask > 3) return fail(MOE_E_ARG, "moe_combine: class_mask must be 1, 2 or 3");
    if (ctx->N > 0 && !y) return fail(MOE_E_ARG, "moe_combine: null y");
    if ((class_mask & MOE_CLASS_LS) && ctx->next_unit < ctx->n_ls_units)
        return fail(MOE_E_INCOMPLETE, "moe_combine: LS tokens still have %u unexecuted units", ctx->n_ls_units - ctx->next_unit);
    if ((class_mask & MOE_CLASS_BE) && ctx->next_unit < ctx->n_units)
        return fail(MOE_E_INCOMPLETE, "moe_combine: BE tokens still have %u unexecuted units", ctx->n_units - ctx->next_unit);
    if (ctx->N == 0) return MOE_OK;
    qmoe::CombineArgs a{};
    a.out = at<float>(ctx, ctx->lay.out);
    a.topk_w = at<float>(ctx, ctx->lay.topk_w);
    a.inv = at<int32_t>(ctx, ctx->lay.inv);
    a.cls = at<uint8_t>(ctx, ctx->lay.cls);
    a.y = y;
    a.N = ctx->N; a.H = ctx->cfg.H; a.k = ctx->cfg.k; a.dtype = ctx->cfg.dtype; a.class_mask = class_mask;
    hipError_t e = qmoe::launch_combine(a, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "moe_combine: launch");
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
        case MOE_GET_EXPERT_OUT: off = ctx->lay.out; sz = A * (size_t)ctx->cfg.H * 4; break;
        case MOE_GET_ACT: off = ctx->lay.act; sz = A * (size_t)ctx->cfg.F * es; break;
        case MOE_GET_UNITS: off = ctx->lay.units; sz = (size_t)ctx->n_units * sizeof(moe_unit); break;
        default: return fail(MOE_E_ARG, "moe_get: unknown item %d", what);
    }
    *dev_ptr = ctx->ws + off;
    *bytes = sz;
    return MOE_OK;
}

int32_t moe_profile(moe_ctx *ctx, int32_t enable) {
    if (!ctx) return fail(MOE_E_ARG, "moe_profile: null context");
    ctx->prof_on = enable != 0;
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
