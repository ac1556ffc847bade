/*
 * CPU oracle of one priority-ordered, preemptible Mixture-of-Experts layer.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64.  Shares no code with the GPU library and is
 * never on the product path: only the test-suite, the smoke check and the benchmark's
 * `cpu_baseline` leg call it.
 *
 * What it follows.  The paper (QLLM, arXiv 2503.09304) prints no equation for the layer; it
 * re-organises the MoE block of a Hugging-Face Mixtral-style model (Introduction, contribution
 * "Novel MoE Layer Design"; Evaluation, "Models and Dataset") into per-expert FIFO queues
 * (Sec. 3.3 "queues per expert") that run latency-sensitive (LS) work before best-effort (BE)
 * work (Abstract; Sec. 3.2, Algorithm 1) and can stop at expert granularity without losing
 * finished work (Introduction, "Fine-Grained Expert-Level Preemption").  The arithmetic below is
 * therefore the plain definition of that block:
 *
 *   1. router logits   L[n,e] = sum_h X[n,h] * Wg[h,e] + bias[e]             (Sec. 2.1 router)
 *   2. probabilities   P[n,:] = softmax(L[n,:]) over all E experts
 *   3. top-k           experts ordered by (L descending, index ascending), first k;
 *                      wt[n,j] = P[n,idx[n,j]] / sum_{i<k} P[n,idx[n,i]]
 *   4. queues          for e, for pr in (LS, BE), for n ascending: if token n has priority pr
 *                      and picked e in slot j, append assignment n*k+j   (Sec. 3.3: per-expert
 *                      FIFO; Sec. 3.2: LS first)
 *   5. expert          FFN_e(x) = W2[e] * ( silu(W1[e] x) (.) (W3[e] x) ),  silu(z) = z/(1+exp(-z))
 *   6. combine         y[n,:] = sum_{j<k} wt[n,j] * FFN_{idx[n,j]}(X[n,:]); only tokens whose k
 *                      assignments are all finished produce a row (Sec. 3.1 "Top-k expert
 *                      selection": only complete tokens feed the next layer)
 *   7. work units      phase LS then phase BE; inside a phase experts ascending; inside an
 *                      expert's sub-queue consecutive chunks of C rows, the last one short
 *
 * Storage types: inputs come as fp32 values or as bf16 bit patterns (dtype 0 / 1) and are
 * widened exactly to fp64; nothing is rounded afterwards.
 *
 * Pins (tests/test_oracle_*.py): logits and the dense-run-every-expert-then-mask layer against
 * numpy.matmul; queues against numpy.lexsort/bincount; top-k against exhaustive subset search;
 * silu closed forms; identical-experts => y = FFN(x); k=1, k=E; unit list tiling invariants;
 * any split of the unit list into calls reproduces the uninterrupted result.
 * Nothing here is pinned by a value printed in the paper: it prints none for this path.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static inline double load_elem(const void *base, int dtype, size_t i)
{
    if (dtype == ORACLE_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return (double)((const float *)base)[i];
}

static void load_row(const void *base, int dtype, size_t first, int n, double *dst)
{
    for (int i = 0; i < n; ++i) dst[i] = load_elem(base, dtype, first + (size_t)i);
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* silu(z) = z / (1 + exp(-z)) */
double oracle_silu(double z) { return z / (1.0 + exp(-z)); }

/* Step 1.  X [N,H], Wg [H,E] row-major, bias [E] fp32 or NULL  ->  L [N,E] fp64. */
void oracle_gate_logits(const void *X, const void *Wg, const float *bias, int dtype,
                        int N, int H, int E, double *L)
{
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int h = 0; h < H; ++h)
                acc += load_elem(X, dtype, (size_t)n * H + h) * load_elem(Wg, dtype, (size_t)h * E + e);
            L[(size_t)n * E + e] = acc + (bias ? (double)bias[e] : 0.0);
        }
    }
}

/* Step 2.  Row-wise softmax with the row maximum subtracted. */
void oracle_softmax(const double *L, int N, int E, double *P)
{
    for (int n = 0; n < N; ++n) {
        const double *l = L + (size_t)n * E;
        double mx = l[0], s = 0.0;
        for (int e = 1; e < E; ++e) if (l[e] > mx) mx = l[e];
        for (int e = 0; e < E; ++e) { P[(size_t)n * E + e] = exp(l[e] - mx); s += P[(size_t)n * E + e]; }
        for (int e = 0; e < E; ++e) P[(size_t)n * E + e] /= s;
    }
}

/* Step 3.  Selection on the logits: slot j holds the j-th expert in the order
 * (logit descending, expert index ascending); weights are the selected probabilities
 * divided by their sum. */
void oracle_topk(const double *L, const double *P, int N, int E, int k, int32_t *idx, double *wt)
{
    uint8_t *taken = (uint8_t *)malloc((size_t)E);
    for (int n = 0; n < N; ++n) {
        const double *l = L + (size_t)n * E;
        memset(taken, 0, (size_t)E);
        double s = 0.0;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || l[e] > l[best]) best = e;   /* strict '>' keeps the lowest index on ties */
            }
            taken[best] = 1;
            idx[(size_t)n * k + j] = best;
            s += P[(size_t)n * E + best];
        }
        for (int j = 0; j < k; ++j) wt[(size_t)n * k + j] = P[(size_t)n * E + idx[(size_t)n * k + j]] / s;
    }
    free(taken);
}

/* Smallest gap between consecutive logits among the k+1 largest of each row (the distance of the
 * selection and of the slot order from a tie).  margin[n] = +inf when k == E and E == 1. */
void oracle_topk_margin(const double *L, int N, int E, int k, double *margin)
{
    double *v = (double *)malloc(sizeof(double) * (size_t)E);
    for (int n = 0; n < N; ++n) {
        memcpy(v, L + (size_t)n * E, sizeof(double) * (size_t)E);
        int top = k + 1 < E ? k + 1 : E;
        for (int j = 0; j < top; ++j) {          /* partial selection sort, descending */
            int b = j;
            for (int e = j + 1; e < E; ++e) if (v[e] > v[b]) b = e;
            double t = v[j]; v[j] = v[b]; v[b] = t;
        }
        double m = INFINITY;
        for (int j = 0; j + 1 < top; ++j) if (v[j] - v[j + 1] < m) m = v[j] - v[j + 1];
        margin[n] = m;
    }
    free(v);
}

/* Step 4.  The per-expert FIFO queues written out as the definition: no sort routine.
 * cnt [E][2] (column 0 = LS, 1 = BE), off [2E+1] running total in bucket order
 * e0-LS, e0-BE, e1-LS, ..., perm [N*k] sorted position -> assignment id n*k+j,
 * inv [N*k] assignment id -> sorted position.  prio[n] != 0 means LS. */
void oracle_queues(const int32_t *idx, const uint8_t *prio, int N, int E, int k,
                   int32_t *cnt, int32_t *off, int32_t *perm, int32_t *inv)
{
    int32_t pos = 0;
    off[0] = 0;
    for (int e = 0; e < E; ++e) {
        for (int cls = 0; cls < 2; ++cls) {            /* 0: LS queue part, 1: BE queue part */
            int32_t c = 0;
            for (int n = 0; n < N; ++n) {
                int is_ls = prio[n] != 0;
                if ((cls == 0) != is_ls) continue;
                for (int j = 0; j < k; ++j) {
                    if (idx[(size_t)n * k + j] == e) {
                        perm[pos] = (int32_t)(n * k + j);
                        inv[(size_t)n * k + j] = pos;
                        ++pos; ++c;
                    }
                }
            }
            cnt[e * 2 + cls] = c;
            off[e * 2 + cls + 1] = pos;
        }
    }
}

/* Step 7.  units[u] = {expert, cls (0 = LS, 1 = BE), first sorted row, rows}.  Returns the
 * number of units (also when it exceeds cap; only the first cap are written). */
int oracle_units(const int32_t *cnt, int E, int C, int32_t *units, int cap)
{
    int nu = 0;
    for (int cls = 0; cls < 2; ++cls) {
        int32_t base = 0;
        for (int e = 0; e < E; ++e) {
            int32_t seg0 = base + (cls == 1 ? cnt[e * 2 + 0] : 0);
            int32_t len = cnt[e * 2 + cls];
            for (int32_t r = 0; r < len; r += C) {
                if (nu < cap) {
                    units[nu * 4 + 0] = e;
                    units[nu * 4 + 1] = cls;
                    units[nu * 4 + 2] = seg0 + r;
                    units[nu * 4 + 3] = (len - r < C) ? (len - r) : C;
                }
                ++nu;
            }
            base += cnt[e * 2 + 0] + cnt[e * 2 + 1];
        }
    }
    return nu;
}

/* Step 5 for a list of tokens through one expert.
 * X [N,H]; W1, W3 [E,F,H]; W2 [E,H,F]; tokens[nrows] = token index of each row;
 * out [nrows,H] fp64 = FFN_e(X[tokens[r],:]).   act, if not NULL, receives
 * silu(W1 x) (.) (W3 x) as [nrows,F]. */
void oracle_expert_rows(const void *X, const void *W1, const void *W3, const void *W2, int dtype,
                        int H, int F, int e, const int32_t *tokens, int nrows,
                        double *out, double *act)
{
    if (nrows <= 0) return;
    double *xs = (double *)malloc(sizeof(double) * (size_t)nrows * H);
    double *m = act ? act : (double *)malloc(sizeof(double) * (size_t)nrows * F);
    for (int r = 0; r < nrows; ++r) load_row(X, dtype, (size_t)tokens[r] * H, H, xs + (size_t)r * H);

#pragma omp parallel
    {
        double *w1 = (double *)malloc(sizeof(double) * (size_t)H);
        double *w3 = (double *)malloc(sizeof(double) * (size_t)H);
#pragma omp for schedule(static)
        for (int f = 0; f < F; ++f) {
            load_row(W1, dtype, ((size_t)e * F + f) * H, H, w1);
            load_row(W3, dtype, ((size_t)e * F + f) * H, H, w3);
            for (int r = 0; r < nrows; ++r) {
                const double *x = xs + (size_t)r * H;
                double g = 0.0, u = 0.0;
#pragma omp simd reduction(+ : g, u)
                for (int h = 0; h < H; ++h) { g += w1[h] * x[h]; u += w3[h] * x[h]; }
                m[(size_t)r * F + f] = oracle_silu(g) * u;
            }
        }
        free(w1); free(w3);

        double *w2 = (double *)malloc(sizeof(double) * (size_t)F);
#pragma omp for schedule(static)
        for (int h = 0; h < H; ++h) {
            load_row(W2, dtype, ((size_t)e * H + h) * F, F, w2);
            for (int r = 0; r < nrows; ++r) {
                const double *mr = m + (size_t)r * F;
                double o = 0.0;
#pragma omp simd reduction(+ : o)
                for (int f = 0; f < F; ++f) o += w2[f] * mr[f];
                out[(size_t)r * H + h] = o;
            }
        }
        free(w2);
    }
    free(xs);
    if (!act) free(m);
}

/* Step 6 for the tokens listed.  O [A,H] fp64 indexed by SORTED position; done [A] marks the
 * sorted positions whose unit has run.  y [ntok,H]; complete[ntok] = 1 where all k assignments
 * of the token were finished (only those rows of y are written, the others are left alone). */
void oracle_combine(const double *O, const uint8_t *done, const int32_t *inv, const double *wt,
                    int k, int H, const int32_t *tokens, int ntok, double *y, uint8_t *complete)
{
    for (int t = 0; t < ntok; ++t) {
        int n = tokens[t];
        int ok = 1;
        for (int j = 0; j < k; ++j) if (!done[inv[(size_t)n * k + j]]) ok = 0;
        complete[t] = (uint8_t)ok;
        if (!ok) continue;
        for (int h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int j = 0; j < k; ++j)
                acc += wt[(size_t)n * k + j] * O[(size_t)inv[(size_t)n * k + j] * H + h];
            y[(size_t)t * H + h] = acc;
        }
    }
}
