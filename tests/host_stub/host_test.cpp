// Host-logic test driver, built with -fsanitize=address,undefined against the recording stubs: the
// context state machine, the unit planner, the segment builder of moe_expert_run, policy-chosen unit
// order, the bookkeeping of an enqueued sequence (including: no other call, moe_destroy included,
// while it is pending) and the scheduler's queues under a random trace.  Exits 0 when every check holds.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <set>
#include <vector>

#include "qmoe.h"
#include "qsched.h"
#include "stub_hooks.h"

static int g_fail = 0;
#define CHECK(c) do { if (!(c)) { printf("FAILED %s:%d: %s   [%s]\n", __FILE__, __LINE__, #c, moe_last_error()); ++g_fail; } } while (0)

struct Ctx {
    moe_config cfg;
    std::vector<char> ws;
    void *base;
    moe_ctx *h = nullptr;
    moe_weights w{};
    char x[64];
    Ctx(int E, int k, int H, int F, int dtype, int C, int max_tokens, int ks = 0) {
        cfg = moe_config{E, k, H, F, dtype, C, max_tokens, ks};
        const size_t n = moe_workspace_bytes(&cfg);
        ws.resize(n + 512);
        base = (void *)(((uintptr_t)ws.data() + 255) / 256 * 256);
        CHECK(n > 0);
        CHECK(moe_create(&cfg, base, n, &h) == MOE_OK);
        static char wbuf[4][64];
        w.Wg = wbuf[0]; w.W1 = wbuf[1]; w.W3 = wbuf[2]; w.W2 = wbuf[3]; w.layout = MOE_W_ROWMAJOR;
    }
    ~Ctx() { if (h) CHECK(moe_destroy(h) == MOE_OK); }
};

// Routes and permutes a batch whose queue lengths are cnt [E][2]; returns the cursor.
static moe_cursor start(Ctx &c, const std::vector<int32_t> &cnt) {
    int tot = 0;
    for (int32_t v : cnt) tot += v;
    CHECK(tot % c.cfg.k == 0 && tot / c.cfg.k <= c.cfg.max_tokens);
    stub_set_counts(cnt.data(), (int)cnt.size());
    static uint8_t prio[1 << 16];
    moe_cursor cur{7, 7};
    CHECK(moe_route(c.h, c.x, tot / c.cfg.k, &c.w, nullptr, nullptr) == MOE_OK);
    CHECK(moe_permute(c.h, prio, &cur, nullptr) == MOE_OK);
    return cur;
}

static std::vector<moe_unit> units_of(Ctx &c) {
    uint32_t n = 0;
    CHECK(moe_units(c.h, nullptr, 0, &n) == MOE_OK);
    std::vector<moe_unit> u(n ? n : 1);
    CHECK(moe_units(c.h, u.data(), n, &n) == MOE_OK);
    u.resize(n);
    return u;
}

// Rows covered by the launches recorded since the last reset (bf16: row ranges in the arguments).
static std::multiset<uint32_t> launched_rows(const std::vector<moe_unit> &units) {
    std::multiset<uint32_t> rows;
    for (int i = 0; i < stub_n_launches(); ++i) {
        const StubLaunch *L = stub_launch(i);
        if (L->nseg > 0) {
            for (int s = 0; s < L->nseg; ++s) {
                CHECK(L->rows[s] >= 1 && L->rows[s] <= 256 && (int)L->rows[s] <= L->max_rows);
                for (uint32_t r = 0; r < L->rows[s]; ++r) rows.insert(L->row0[s] + r);
            }
        } else {
            for (uint32_t u = L->u0; u < L->u0 + L->nu; ++u)
                for (int r = 0; r < units[u].rows; ++r) rows.insert((uint32_t)(units[u].row0 + r));
        }
    }
    return rows;
}

static void test_plan_and_cursor(int dtype) {
    Ctx c(6, 2, 128, 256, dtype, 100, 4096);
    const std::vector<int32_t> cnt = {30, 500, 0, 0, 257, 1, 0, 64, 100, 100, 0, 948};
    moe_cursor cur = start(c, cnt);
    std::vector<moe_unit> units = units_of(c);
    std::vector<moe_unit> plan(64);
    uint32_t n = 0;
    CHECK(moe_plan_units(cnt.data(), 6, 100, plan.data(), 64, &n) == MOE_OK);
    CHECK(n == units.size() && cur.n_units == n && cur.next_unit == 0);
    CHECK(memcmp(plan.data(), units.data(), n * sizeof(moe_unit)) == 0);
    // every LS unit comes before every BE unit; rows tile [0, A) exactly once
    std::multiset<uint32_t> all;
    bool seen_be = false;
    for (const moe_unit &u : units) {
        CHECK(u.rows >= 1 && u.rows <= 100);
        if (u.cls) seen_be = true; else CHECK(!seen_be);
        for (int r = 0; r < u.rows; ++r) all.insert((uint32_t)(u.row0 + r));
    }
    CHECK(all.size() == 2000 && *all.begin() == 0 && *all.rbegin() == 1999 && std::set<uint32_t>(all.begin(), all.end()).size() == 2000);
    // combine before any work: both classes incomplete
    char y[8];
    CHECK(moe_combine(c.h, y, MOE_CLASS_LS, nullptr) == MOE_E_INCOMPLETE);
    CHECK(moe_combine(c.h, y, 0, nullptr) == MOE_E_ARG && moe_combine(c.h, y, 8, nullptr) == MOE_E_ARG);
    // run in pieces of 1, 2, 3, ... units; each call launches exactly the rows of its units
    uint32_t done = 0, step = 1;
    std::multiset<uint32_t> total;
    while (true) {
        stub_reset_launches();
        const uint32_t before = cur.next_unit;
        const int32_t rc = moe_expert_run(c.h, c.x, &c.w, step, &cur, nullptr);
        CHECK(rc == MOE_OK || rc == MOE_DONE);
        std::multiset<uint32_t> want;
        for (uint32_t u = before; u < cur.next_unit; ++u)
            for (int r = 0; r < units[u].rows; ++r) want.insert((uint32_t)(units[u].row0 + r));
        CHECK(cur.next_unit == std::min<uint32_t>(before + step, n));
        CHECK(launched_rows(units) == want);
        total.insert(want.begin(), want.end());
        done = cur.next_unit;
        // a stale cursor is refused and runs nothing
        moe_cursor stale{before, n};
        if (before != cur.next_unit) {
            stub_reset_launches();
            CHECK(moe_expert_run(c.h, c.x, &c.w, 1, &stale, nullptr) == MOE_E_ARG && stub_n_launches() == 0);
        }
        uint32_t n_ls = 0;
        for (const moe_unit &u : units) n_ls += u.cls == 0;
        CHECK((moe_combine(c.h, y, MOE_CLASS_LS, nullptr) == MOE_OK) == (done >= n_ls));
        CHECK((moe_combine(c.h, y, MOE_CLASS_BE | MOE_Y_F32, nullptr) == MOE_OK) == (done == n));
        if (rc == MOE_DONE) break;
        ++step;
    }
    CHECK(total == all && done == n);
    // wrong tensors, wrong order of calls
    char other[8];
    CHECK(moe_expert_run(c.h, other, &c.w, 1, &cur, nullptr) == MOE_E_ARG);
    CHECK(moe_permute(c.h, (const uint8_t *)other, &cur, nullptr) == MOE_E_STATE);
}

static void test_segments_share_weights_evenly() {
    // one expert with 896 rows in a single call: 4 row ranges of 7 tiles (224 rows), not 256/256/256/128
    Ctx c(2, 1, 128, 128, MOE_BF16, 256, 2048);
    moe_cursor cur = start(c, {0, 896, 40, 60});
    stub_reset_launches();
    CHECK(moe_expert_run(c.h, c.x, &c.w, UINT32_MAX, &cur, nullptr) == MOE_DONE);
    CHECK(stub_n_launches() == 1);
    const StubLaunch *L = stub_launch(0);
    CHECK(L->nseg == 5);
    for (int s = 0; s < 4 && s < L->nseg; ++s) CHECK(L->rows[s] == 224 && L->expert[s] == 0 && L->row0[s] == (uint32_t)(224 * s));
    // expert 1: its LS rows (40) and BE rows (60) are adjacent and share one range
    CHECK(L->nseg == 5 && L->rows[4] == 100 && L->row0[4] == 896 && L->expert[4] == 1);
}

static void test_policy_order_and_errors() {
    Ctx c(4, 2, 64, 64, MOE_F32, 16, 512);
    moe_cursor cur = start(c, {20, 30, 0, 50, 16, 16, 5, 3});
    std::vector<moe_unit> units = units_of(c);
    const uint32_t n = (uint32_t)units.size();
    uint32_t bad[] = {n}, twice[] = {1, 1}, pick[] = {n - 1, 0, 2};
    stub_reset_launches();
    CHECK(moe_expert_run_units(c.h, c.x, &c.w, bad, 1, &cur, nullptr) == MOE_E_ARG);
    CHECK(moe_expert_run_units(c.h, c.x, &c.w, twice, 2, &cur, nullptr) == MOE_E_ARG);
    CHECK(stub_n_launches() == 0);
    CHECK(moe_expert_run_units(c.h, c.x, &c.w, pick, 3, &cur, nullptr) == MOE_OK);
    CHECK(cur.next_unit == 1 && cur.n_units == n);
    CHECK(moe_expert_run_units(c.h, c.x, &c.w, pick, 1, &cur, nullptr) == MOE_E_ARG);     // already executed
    // the cursor call skips what the policy ran
    stub_reset_launches();
    CHECK(moe_expert_run(c.h, c.x, &c.w, UINT32_MAX, &cur, nullptr) == MOE_DONE);
    std::multiset<uint32_t> want;
    for (uint32_t u = 0; u < n; ++u)
        if (u != n - 1 && u != 0 && u != 2)
            for (int r = 0; r < units[u].rows; ++r) want.insert((uint32_t)(units[u].row0 + r));
    CHECK(launched_rows(units) == want);
}

static void test_enqueued_sequence_bookkeeping(int dtype) {
    Ctx c(3, 2, 128, 256, dtype, 64, 1024, dtype == MOE_BF16 ? 2 : 0);
    moe_cursor cur = start(c, {10, 300, 0, 200, 64, 26});
    std::vector<moe_unit> units = units_of(c);
    const uint32_t n = (uint32_t)units.size();
    stub_reset_launches();
    stub_complete_first(3);                          // the device will report only the first 3 row ranges complete
    CHECK(moe_expert_enqueue(c.h, c.x, &c.w, 4, nullptr) == MOE_OK);
    for (int i = 0; i < stub_n_launches(); ++i) CHECK(stub_launch(i)->gated);
    // pending: every other call is refused, destroying the context included (its kernels use the pinned buffer)
    char y[8];
    const void *p; size_t nb;
    CHECK(moe_destroy(c.h) == MOE_E_STATE);
    CHECK(moe_route(c.h, c.x, 1, &c.w, nullptr, nullptr) == MOE_E_STATE);
    CHECK(moe_expert_run(c.h, c.x, &c.w, 1, &cur, nullptr) == MOE_E_STATE);
    CHECK(moe_expert_enqueue(c.h, c.x, &c.w, 4, nullptr) == MOE_E_STATE);
    CHECK(moe_combine(c.h, y, MOE_CLASS_ALL, nullptr) == MOE_E_STATE);
    CHECK(moe_combine_complete(c.h, y, nullptr, nullptr) == MOE_E_STATE);
    CHECK(moe_get(c.h, MOE_GET_EXPERT_OUT, &p, &nb) == MOE_E_STATE);
    CHECK(moe_expert_stop(c.h) == MOE_OK);
    // collect: exactly the units whose rows all lie in the complete ranges are booked
    std::multiset<uint32_t> launched = launched_rows(units);
    CHECK(launched.size() == 600);
    CHECK(moe_expert_collect(c.h, &cur, nullptr) == MOE_OK);
    uint32_t booked_rows = 0;
    {   // recompute from the recorded ranges: the first 3 ranges in launch order
        std::vector<uint8_t> ok(600, 0);
        int seen = 0;
        for (int i = 0; i < stub_n_launches() && seen < 3; ++i) {
            const StubLaunch *L = stub_launch(i);
            if (L->nseg > 0) {
                for (int s = 0; s < L->nseg && seen < 3; ++s, ++seen)
                    for (uint32_t r = 0; r < L->rows[s]; ++r) ok[L->row0[s] + r] = 1;
            } else {
                for (uint32_t u = L->u0; u < L->u0 + L->nu && seen < 3; ++u, ++seen)
                    for (int r = 0; r < units[u].rows; ++r) ok[(size_t)(units[u].row0 + r)] = 1;
            }
        }
        uint32_t first_not = n;
        for (uint32_t u = 0; u < n; ++u) {
            bool all = true;
            for (int r = 0; r < units[u].rows; ++r) all = all && ok[(size_t)(units[u].row0 + r)];
            if (all) booked_rows += (uint32_t)units[u].rows;
            else if (first_not == n) first_not = u;
        }
        CHECK(cur.next_unit == first_not);
        CHECK(booked_rows > 0 && booked_rows < 600);
    }
    // resume: the rest runs, each unit once
    stub_reset_launches();
    stub_complete_first(-1);
    CHECK(moe_expert_enqueue(c.h, c.x, &c.w, UINT32_MAX, nullptr) == MOE_OK);
    CHECK(launched_rows(units).size() == 600 - booked_rows);
    CHECK(moe_expert_collect(c.h, &cur, nullptr) == MOE_DONE && cur.next_unit == n);
    CHECK(moe_expert_enqueue(c.h, c.x, &c.w, 2, nullptr) == MOE_DONE);
    CHECK(moe_combine(c.h, y, MOE_CLASS_ALL, nullptr) == MOE_OK);
    CHECK(moe_get(c.h, MOE_GET_EXPERT_OUT, &p, &nb) == MOE_OK && nb == (size_t)600 * 128 * 4);
    // an empty batch
    moe_cursor e = start(c, {0, 0, 0, 0, 0, 0});
    CHECK(e.n_units == 0 && moe_expert_run(c.h, c.x, &c.w, 5, &e, nullptr) == MOE_DONE);
}

static void test_config_and_workspace_errors() {
    moe_config bad = {0, 1, 64, 64, MOE_BF16, 16, 8, 0};
    CHECK(moe_workspace_bytes(&bad) == 0);
    moe_config ok = {4, 2, 64, 64, MOE_BF16, 16, 8, 0};
    const size_t n = moe_workspace_bytes(&ok);
    std::vector<char> ws(n + 512);
    void *base = (void *)(((uintptr_t)ws.data() + 255) / 256 * 256);
    moe_ctx *h = nullptr;
    CHECK(moe_create(&ok, (char *)base + 8, n, &h) == MOE_E_WORKSPACE && h == nullptr);
    CHECK(moe_create(&ok, base, n - 1, &h) == MOE_E_WORKSPACE);
    CHECK(moe_create(&ok, base, n, &h) == MOE_OK);
    moe_cursor cur;
    CHECK(moe_permute(h, nullptr, &cur, nullptr) == MOE_E_STATE);
    CHECK(moe_expert_stop(h) == MOE_E_STATE);
    CHECK(moe_destroy(h) == MOE_OK);
    CHECK(moe_destroy(nullptr) == MOE_E_ARG);
}

static void test_scheduler_random_trace() {
    std::mt19937 rng(12345);
    sched *s = sched_create(4);
    CHECK(s != nullptr);
    std::set<uint64_t> running, queued;
    uint64_t next_id = 1;
    uint64_t jobs[4];
    for (int it = 0; it < 20000; ++it) {
        const int op = (int)(rng() % 3);
        if (op == 0) {
            CHECK(sched_submit(s, next_id, (int)(rng() % 2)) == SCHED_OK);
            CHECK(sched_submit(s, next_id, 0) == SCHED_E_JOB);
            queued.insert(next_id++);
        } else if (op == 1) {
            sched_batch b;
            const int32_t rc = sched_next_batch(s, jobs, 4, &b);
            CHECK(rc == SCHED_OK || rc == SCHED_NONE);
            if (rc == SCHED_OK) {
                CHECK(b.n >= 1 && b.n <= 4 && b.n_ls <= b.n);
                for (uint32_t i = 0; i < b.n; ++i) { CHECK(queued.erase(jobs[i]) == 1); running.insert(jobs[i]); }
            } else {
                CHECK(queued.empty());
            }
        } else if (!running.empty()) {
            const uint64_t id = *running.begin();
            running.erase(running.begin());
            const int fin = (int)(rng() % 3 == 0);
            CHECK(sched_token(s, id, fin) == SCHED_OK);
            CHECK(sched_token(s, id, 0) == SCHED_E_JOB);
            if (!fin) queued.insert(id);
        }
        CHECK(sched_running(s) == running.size());
        CHECK(sched_queue_len(s, 0) + sched_queue_len(s, 1) + sched_queue_len(s, 2) + sched_queue_len(s, 3) == queued.size());
    }
    sched_destroy(s);
}

int main() {
    test_config_and_workspace_errors();
    test_plan_and_cursor(MOE_BF16);
    test_plan_and_cursor(MOE_F32);
    test_segments_share_weights_evenly();
    test_policy_order_and_errors();
    test_enqueued_sequence_bookkeeping(MOE_BF16);
    test_enqueued_sequence_bookkeeping(MOE_F32);
    test_scheduler_random_trace();
    printf(g_fail ? "%d checks failed\n" : "all host-logic checks passed\n", g_fail);
    return g_fail ? 1 : 0;
}
