/* The CPU oracle (oracle/moe_oracle.c) walked through one small layer, both dtypes, under
 * AddressSanitizer and UndefinedBehaviorSanitizer: every buffer is a heap allocation of exactly the
 * documented size, so any access beyond it aborts the run.  Also checks the integer invariants on the
 * way (counts sum to N*k, perm is a bijection with inverse inv, units tile the rows).  Exits 0 if all hold. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void oracle_gate_logits(const void *, const void *, const float *, int, int, int, int, double *);
void oracle_softmax(const double *, int, int, double *);
void oracle_topk(const double *, const double *, int, int, int, int32_t *, double *);
void oracle_topk_margin(const double *, int, int, int, double *);
void oracle_queues(const int32_t *, const uint8_t *, int, int, int, int32_t *, int32_t *, int32_t *, int32_t *);
int oracle_units(const int32_t *, int, int, int32_t *, int);
void oracle_expert_rows(const void *, const void *, const void *, const void *, int, int, int, int, const int32_t *, int,
                        double *, double *);
void oracle_combine(const double *, const uint8_t *, const int32_t *, const double *, int, int, const int32_t *, int, double *,
                    uint8_t *);

static int fails = 0;
#define CHECK(c) do { if (!(c)) { printf("FAILED line %d: %s\n", __LINE__, #c); ++fails; } } while (0)

static uint32_t rng = 12345;
static float frand(void) { rng = rng * 1664525u + 1013904223u; return (float)((rng >> 8) & 0xffff) / 32768.0f - 1.0f; }

static void *tensor(size_t n, int dtype, float scale) {          /* fp32, or bf16 bit patterns (truncated) */
    if (dtype == 0) { float *p = malloc(n * 4); for (size_t i = 0; i < n; ++i) p[i] = scale * frand(); return p; }
    uint16_t *p = malloc(n * 2);
    for (size_t i = 0; i < n; ++i) { float v = scale * frand(); uint32_t b; memcpy(&b, &v, 4); p[i] = (uint16_t)(b >> 16); }
    return p;
}

static void run(int dtype, int N, int H, int F, int E, int k, int C) {
    const int A = N * k;
    void *X = tensor((size_t)N * H, dtype, 1.0f), *Wg = tensor((size_t)H * E, dtype, 0.05f);
    void *W1 = tensor((size_t)E * F * H, dtype, 0.05f), *W3 = tensor((size_t)E * F * H, dtype, 0.05f);
    void *W2 = tensor((size_t)E * H * F, dtype, 0.05f);
    float *bias = malloc(sizeof(float) * E);
    for (int e = 0; e < E; ++e) bias[e] = 0.1f * (float)e;
    uint8_t *prio = malloc(N);
    for (int n = 0; n < N; ++n) prio[n] = (uint8_t)(n % 3 == 0);
    double *L = malloc(sizeof(double) * N * E), *P = malloc(sizeof(double) * N * E), *wt = malloc(sizeof(double) * A);
    double *margin = malloc(sizeof(double) * N);
    int32_t *idx = malloc(4 * A), *cnt = malloc(4 * 2 * E), *off = malloc(4 * (2 * E + 1)), *perm = malloc(4 * A), *inv = malloc(4 * A);
    oracle_gate_logits(X, Wg, bias, dtype, N, H, E, L);
    oracle_softmax(L, N, E, P);
    oracle_topk(L, P, N, E, k, idx, wt);
    oracle_topk_margin(L, N, E, k, margin);
    oracle_queues(idx, prio, N, E, k, cnt, off, perm, inv);
    int tot = 0;
    for (int i = 0; i < 2 * E; ++i) tot += cnt[i];
    CHECK(tot == A && off[2 * E] == A);
    for (int r = 0; r < A; ++r) CHECK(perm[r] >= 0 && perm[r] < A && inv[perm[r]] == r);
    for (int n = 0; n < N; ++n) { double s = 0; for (int j = 0; j < k; ++j) s += wt[n * k + j]; CHECK(s > 1 - 1e-12 && s < 1 + 1e-12); }
    const int nu = oracle_units(cnt, E, C, NULL, 0);
    int32_t *units = malloc(sizeof(int32_t) * 4 * (nu ? nu : 1));
    CHECK(oracle_units(cnt, E, C, units, nu) == nu);
    double *O = malloc(sizeof(double) * (size_t)A * H), *act = malloc(sizeof(double) * (size_t)C * F);
    uint8_t *done = calloc(A, 1);
    int rows = 0;
    for (int u = 0; u < nu; ++u) {
        const int e = units[4 * u], r0 = units[4 * u + 2], nr = units[4 * u + 3];
        CHECK(nr >= 1 && nr <= C && r0 >= 0 && r0 + nr <= A);
        int32_t *tok = malloc(4 * nr);
        for (int r = 0; r < nr; ++r) { tok[r] = perm[r0 + r] / k; CHECK(idx[perm[r0 + r]] == e); }
        oracle_expert_rows(X, W1, W3, W2, dtype, H, F, e, tok, nr, O + (size_t)r0 * H, (u & 1) ? act : NULL);
        memset(done + r0, 1, nr);
        rows += nr;
        free(tok);
    }
    CHECK(rows == A);
    int32_t *toks = malloc(4 * N);
    for (int n = 0; n < N; ++n) toks[n] = n;
    double *y = malloc(sizeof(double) * (size_t)N * H);
    uint8_t *comp = malloc(N);
    oracle_combine(O, done, inv, wt, k, H, toks, N, y, comp);
    for (int n = 0; n < N; ++n) CHECK(comp[n] == 1);
    for (size_t i = 0; i < (size_t)N * H; ++i) CHECK(y[i] == y[i]);
    free(X); free(Wg); free(W1); free(W3); free(W2); free(bias); free(prio); free(L); free(P); free(wt); free(margin);
    free(idx); free(cnt); free(off); free(perm); free(inv); free(units); free(O); free(act); free(done); free(toks); free(y); free(comp);
}

int main(void) {
    run(0, 37, 20, 28, 5, 2, 4);
    run(1, 64, 24, 40, 7, 3, 16);
    run(1, 1, 8, 8, 2, 2, 1);
    printf(fails ? "%d checks failed\n" : "oracle ran clean under the sanitizers\n", fails);
    return fails ? 1 : 0;
}
