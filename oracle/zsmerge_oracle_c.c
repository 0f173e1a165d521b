/* CPU oracle for the ZSMerge budgeted KV-cache step, plain C.  TEST INFRASTRUCTURE ONLY.
 *
 * A second, independent statement of what oracle/zsmerge_oracle.py computes, fast enough for
 * the full-size workloads: the same definitions written as loops, fp64 arithmetic, one OpenMP
 * thread per unit, no blocking, no reordering beyond "one unit after the other".  It shares no
 * code with the HIP path and the product never links or loads it; only the tests, the smoke
 * check and the benchmark's CPU-baseline leg do.
 *
 * Per (layer, sequence, KV head) unit:
 *   - compensated attention of one query per query head over the retained slots and the
 *     incoming token                                               (Eq. 4, Sec. 3.5)
 *   - decayed contribution scores                                  (Eq. 3, Sec. 3.3)
 *   - the online update: the token joins the proximity set, that set's oldest member is
 *     demoted to the context set, the context token of lowest score is evicted and absorbed by
 *     the residual set                                             (Alg. 1)
 *   - absorption: an unused residual slot is opened, otherwise the slot whose key has the
 *     largest dot product with the evicted key takes it into its running mean
 *                                                                  (Eq. 5, Eq. 6, Sec. 3.4)
 *   - one-shot prefill compression from the last W prompt queries  (Sec. 3.2; appendix
 *     "Implementation Details")
 *
 * Stored state is rounded to its storage type at every store, as in the Python oracle: token
 * slots hold input rows (already representable in the cache's element type), residual rows and
 * scores are fp32 values carried in doubles, counts and positions are integers.
 *
 * Readings of the paper fixed here (the same as in the Python oracle): a step attends over
 * the cache and the incoming token itself; the score update uses the compensated
 * probabilities; the eviction looks at the scores after this step's update; ties go to the
 * lowest (score, position) for eviction, to the earliest position for the prefill selection
 * and to the lowest index for Eq. 5; grouped queries have their own softmax each and pool
 * their probabilities by the plain mean; an unused residual slot takes no part in the softmax.
 *
 * The sets of Alg. 1 are not kept as lists here (the Python oracle does that, literally): a token
 * enters the proximity set when it arrives and positions only grow, so the proximity set is the
 * B_p most recent tokens and the context set the other retained ones; the state is the per-slot
 * arrays alone and the sets are read off the positions at every step.  That the two statements
 * agree step by step is itself tested (tests/test_oracle_c.py).
 *
 * Parity pins: tests/test_oracle_pins.py runs every pin against this file as well as against
 * the Python oracle, and tests/test_oracle_c.py compares the two on random workloads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t n_units, d, G, B_r, cap; /* cap: slot stride of the per-slot arrays, >= B_r + B_p + B_c of every unit */
    int32_t pad_;
    double lam, alpha, scale;
    /* state, unit-major, owned by the caller */
    double *K, *V;       /* [n][cap][d]   slots [0, B_r) residual, [B_r, B) token slots */
    int64_t *pos, *w;    /* [n][cap]      position (-1: empty), fusion count (0: empty) */
    double *s;           /* [n][cap]      scores, fp32 values */
    int64_t *n_seen;     /* [n]           T: tokens seen so far */
    const int32_t *B_p, *B_c; /* [n] */
} zso_batch;

static double store32(double x) { return (double)(float)x; }

static double dot(const double *a, const double *b, int d) {
    double p = 0.0;
    for (int i = 0; i < d; ++i) p += a[i] * b[i];
    return p;
}

/* Alg. 1, residual branch: open a residual slot while one is unused (they are opened in index
 * order), otherwise Eq. 5 (largest raw dot product, lowest index on ties), then Eq. 6. */
static int absorb(const zso_batch *b, int u, const double *k, const double *v, int64_t pos, double s) {
    const int d = b->d;
    double *K = b->K + (size_t)u * b->cap * d, *V = b->V + (size_t)u * b->cap * d;
    int64_t *w = b->w + (size_t)u * b->cap, *ps = b->pos + (size_t)u * b->cap;
    double *sc = b->s + (size_t)u * b->cap;
    if (b->B_r == 0) return -1;
    for (int r = 0; r < b->B_r; ++r) {      /* the lowest unused residual slot, if there is one */
        if (w[r] != 0) continue;
        for (int i = 0; i < d; ++i) { K[(size_t)r * d + i] = store32(k[i]); V[(size_t)r * d + i] = store32(v[i]); }
        w[r] = 1; ps[r] = pos; sc[r] = s;
        return r;
    }
    int best = 0;
    double bd = dot(K, k, d);
    for (int r = 1; r < b->B_r; ++r) {
        const double p = dot(K + (size_t)r * d, k, d);
        if (p > bd) { bd = p; best = r; }
    }
    const double wr = (double)w[best];
    for (int i = 0; i < d; ++i) {
        K[(size_t)best * d + i] = store32((wr * K[(size_t)best * d + i] + k[i]) / (wr + 1.0));
        V[(size_t)best * d + i] = store32((wr * V[(size_t)best * d + i] + v[i]) / (wr + 1.0));
    }
    w[best] += 1;
    return best;
}

typedef struct { int64_t pos; int32_t slot; } placed;

static int by_position(const void *x, const void *y) {
    const placed *a = (const placed *)x, *b = (const placed *)y;
    return a->pos < b->pos ? -1 : (a->pos > b->pos ? 1 : 0);
}

/* One pass of Alg. 1's loop body for unit u.  a_dbg [G][cap + 1] (probabilities by slot, the
 * incoming token at index cap), cand_dbg [cap + 1] (count, then the context-set candidates of the
 * eviction) and cand_s_dbg, cand_pos_dbg [cap] (their scores and positions as the choice saw them)
 * may be NULL. */
static int decode_unit(const zso_batch *b, int u, const double *q, const double *k_new, const double *v_new,
                       double *out, int32_t *write_slot, int32_t *evicted_pos, int32_t *merged_slot,
                       double *a_dbg, int32_t *cand_dbg, double *cand_s_dbg, int64_t *cand_pos_dbg) {
    const int d = b->d, G = b->G, cap = b->cap;
    const int B_p = b->B_p[u], B_c = b->B_c[u], B = b->B_r + B_p + B_c;
    double *K = b->K + (size_t)u * cap * d, *V = b->V + (size_t)u * cap * d;
    int64_t *w = b->w + (size_t)u * cap, *ps = b->pos + (size_t)u * cap;
    double *sc = b->s + (size_t)u * cap;
    const int64_t T = b->n_seen[u];
    if (B > cap || B_p < 1) return -1;

    double *z = (double *)malloc(sizeof(double) * (size_t)(B + 1));
    double *abar = (double *)calloc((size_t)(B + 1), sizeof(double));
    if (!z || !abar) { free(z); free(abar); return -2; }
    if (a_dbg) memset(a_dbg, 0, sizeof(double) * (size_t)G * (cap + 1));

    /* Eq. 4 over the occupied slots and the incoming token (index B here); w = 1 adds log 1 = 0 */
    for (int g = 0; g < G; ++g) {
        const double *qg = q + (size_t)g * d;
        double m = -INFINITY;
        for (int j = 0; j < B; ++j) {
            if (w[j] <= 0) continue;
            z[j] = dot(qg, K + (size_t)j * d, d) * b->scale + b->alpha * log((double)w[j]);
            if (z[j] > m) m = z[j];
        }
        z[B] = dot(qg, k_new, d) * b->scale;
        if (z[B] > m) m = z[B];
        double L = 0.0;
        for (int j = 0; j <= B; ++j) {
            if (j < B && w[j] <= 0) continue;
            z[j] = exp(z[j] - m);
            L += z[j];
        }
        double *og = out + (size_t)g * d;
        for (int i = 0; i < d; ++i) og[i] = 0.0;
        for (int j = 0; j <= B; ++j) {
            if (j < B && w[j] <= 0) continue;
            const double a = z[j] / L;
            const double *vj = j < B ? V + (size_t)j * d : v_new;
            for (int i = 0; i < d; ++i) og[i] += a * vj[i];
            abar[j] += a;
            if (a_dbg) a_dbg[(size_t)g * (cap + 1) + (j < B ? j : cap)] = a;
        }
    }
    /* Eq. 3 on the pooled probabilities; a new token starts from s = 0 */
    for (int j = 0; j < B; ++j)
        if (w[j] > 0) sc[j] = store32(b->lam * sc[j] + abar[j] / (double)G);
    const double s_new = store32(abar[B] / (double)G);
    free(z); free(abar);

    /* Alg. 1: the token joins the proximity set; with it the set holds the new token and the
     * B_p - 1 most recent retained ones, every other retained token belongs to the context set,
     * and the context set, if it now has more than B_c members, loses the one of lowest
     * (score, position). */
    int freed = -1, ev = -1, merged = -1;
    if (cand_dbg) cand_dbg[0] = 0;
    int n_tok = 0;
    placed *tok = (placed *)malloc(sizeof(placed) * (size_t)(B > 0 ? B : 1));
    if (!tok) return -2;
    for (int j = b->B_r; j < B; ++j)
        if (w[j] > 0) { tok[n_tok].pos = ps[j]; tok[n_tok].slot = j; ++n_tok; }
    const int n_ctx = n_tok - (B_p - 1);          /* members of the context set after the demotion */
    if (n_ctx > B_c) {
        qsort(tok, (size_t)n_tok, sizeof(placed), by_position);   /* oldest first: the context set is tok[0 .. n_ctx) */
        int ci = 0;
        for (int x = 1; x < n_ctx; ++x) {
            const int j = tok[x].slot, c = tok[ci].slot;
            if (sc[j] < sc[c] || (sc[j] == sc[c] && ps[j] < ps[c])) ci = x;
        }
        if (cand_dbg) {
            cand_dbg[0] = n_ctx;
            for (int x = 0; x < n_ctx; ++x) {
                cand_dbg[1 + x] = tok[x].slot;
                if (cand_s_dbg) cand_s_dbg[x] = sc[tok[x].slot];
                if (cand_pos_dbg) cand_pos_dbg[x] = ps[tok[x].slot];
            }
        }
        const int c_hat = tok[ci].slot;
        ev = (int)ps[c_hat];
        double *kcopy = (double *)malloc(sizeof(double) * 2 * (size_t)d);
        if (!kcopy) { free(tok); return -2; }
        memcpy(kcopy, K + (size_t)c_hat * d, sizeof(double) * d);
        memcpy(kcopy + d, V + (size_t)c_hat * d, sizeof(double) * d);
        merged = absorb(b, u, kcopy, kcopy + d, ps[c_hat], sc[c_hat]);
        free(kcopy);
        freed = c_hat;
    }
    free(tok);
    if (freed < 0) {
        for (int j = b->B_r; j < B; ++j)
            if (w[j] == 0) { freed = j; break; }
        if (freed < 0) return -3;
    }
    memcpy(K + (size_t)freed * d, k_new, sizeof(double) * d);
    memcpy(V + (size_t)freed * d, v_new, sizeof(double) * d);
    ps[freed] = T; w[freed] = 1; sc[freed] = s_new;
    b->n_seen[u] = T + 1;
    *write_slot = freed; *evicted_pos = ev; *merged_slot = merged;
    return 0;
}

/* q [n][G][d], k_new, v_new [n][d], out [n][G][d]; write_slot, evicted_pos, merged_slot [n];
 * a_dbg [n][G][cap+1], cand_dbg [n][cap+1], cand_s_dbg, cand_pos_dbg [n][cap]: each may be NULL.
 * Returns 0, or an error of one of the units. */
int zso_decode_step(const zso_batch *b, const double *q, const double *k_new, const double *v_new, double *out,
                    int32_t *write_slot, int32_t *evicted_pos, int32_t *merged_slot, double *a_dbg,
                    int32_t *cand_dbg, double *cand_s_dbg, int64_t *cand_pos_dbg) {
    int err = 0;
    const int d = b->d, G = b->G;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < b->n_units; ++u) {
        const int e = decode_unit(b, u, q + (size_t)u * G * d, k_new + (size_t)u * d, v_new + (size_t)u * d,
                                  out + (size_t)u * G * d, write_slot + u, evicted_pos + u, merged_slot + u,
                                  a_dbg ? a_dbg + (size_t)u * G * (b->cap + 1) : NULL,
                                  cand_dbg ? cand_dbg + (size_t)u * (b->cap + 1) : NULL,
                                  cand_s_dbg ? cand_s_dbg + (size_t)u * b->cap : NULL,
                                  cand_pos_dbg ? cand_pos_dbg + (size_t)u * b->cap : NULL);
        if (e) {
#pragma omp critical
            err = e;
        }
    }
    return err;
}

/* Scores of the T prompt tokens after the prompt: Eq. 3 taken step by step over the last W
 * query steps, grouped queries pooled by their mean; query row i' is the query at position
 * i = T - W + i' and attends to positions t <= i (Eq. 1).  Qw [G][W][d], K [T][d], s_out [T]
 * (fp32 values). */
int zso_prompt_scores(int G, int W, int T, int d, const double *Qw, const double *K, double lam, double scale,
                      double *s_out) {
    double *z = (double *)malloc(sizeof(double) * (size_t)T);
    double *a = (double *)malloc(sizeof(double) * (size_t)T);
    if (!z || !a) { free(z); free(a); return -2; }
    for (int t = 0; t < T; ++t) s_out[t] = 0.0;
    for (int ip = 0; ip < W; ++ip) {
        const int i = T - W + ip;
        for (int t = 0; t <= i; ++t) a[t] = 0.0;
        for (int g = 0; g < G; ++g) {
            const double *qg = Qw + ((size_t)g * W + ip) * d;
            double m = -INFINITY, L = 0.0;
            for (int t = 0; t <= i; ++t) {
                z[t] = dot(qg, K + (size_t)t * d, d) * scale;
                if (z[t] > m) m = z[t];
            }
            for (int t = 0; t <= i; ++t) { z[t] = exp(z[t] - m); L += z[t]; }
            for (int t = 0; t <= i; ++t) a[t] += z[t] / L;
        }
        for (int t = 0; t <= i; ++t) s_out[t] = lam * s_out[t] + a[t] / (double)G;
    }
    for (int t = 0; t < T; ++t) s_out[t] = store32(s_out[t]);
    free(z); free(a);
    return 0;
}

typedef struct { double s; int32_t t; } scored;

static int by_score_then_position(const void *x, const void *y) {
    const scored *a = (const scored *)x, *b = (const scored *)y;
    if (a->s != b->s) return a->s > b->s ? -1 : 1;      /* higher score first */
    return a->t < b->t ? -1 : (a->t > b->t ? 1 : 0);    /* among equal scores the earlier position */
}

static void put_token(const zso_batch *b, int u, int j, const double *k, const double *v, int64_t pos, double s) {
    const int d = b->d;
    memcpy(b->K + ((size_t)u * b->cap + j) * d, k, sizeof(double) * d);
    memcpy(b->V + ((size_t)u * b->cap + j) * d, v, sizeof(double) * d);
    b->pos[(size_t)u * b->cap + j] = pos;
    b->w[(size_t)u * b->cap + j] = 1;
    b->s[(size_t)u * b->cap + j] = s;
}

/* One-shot compression of unit u's T-token prompt into its empty cache: keep the latest B_p
 * tokens and the B_c of highest score among the others, absorb the rest in position order. */
static int prefill_unit(const zso_batch *b, int u, int W, int T, const double *Qw, const double *K, const double *V,
                        double *s) {
    const int d = b->d, cap = b->cap;
    const int B_p = b->B_p[u], B_c = b->B_c[u], n_tok = B_p + B_c;
    if (b->B_r + n_tok > cap || W > T || b->n_seen[u] != 0) return -1;
    for (int j = 0; j < cap; ++j)
        if (b->w[(size_t)u * cap + j] != 0) return -1;          /* the cache must be empty */
    int e = zso_prompt_scores(b->G, W, T, d, Qw, K, b->lam, b->scale, s);
    if (e) return e;
    char *kept = (char *)calloc((size_t)T, 1);
    if (!kept) return -2;
    int n_ctx, n_prox;
    if (T <= n_tok) {
        n_prox = T < B_p ? T : B_p;
        n_ctx = T - n_prox;
        for (int t = 0; t < T; ++t) kept[t] = 1;
    } else {
        n_prox = B_p;
        n_ctx = B_c;
        const int nh = T - B_p;
        scored *h = (scored *)malloc(sizeof(scored) * (size_t)(nh > 0 ? nh : 1));
        if (!h) { free(kept); return -2; }
        for (int t = 0; t < nh; ++t) { h[t].s = s[t]; h[t].t = t; }
        qsort(h, (size_t)nh, sizeof(scored), by_score_then_position);
        for (int x = 0; x < B_c; ++x) kept[h[x].t] = 1;
        for (int t = T - B_p; t < T; ++t) kept[t] = 1;
        free(h);
    }
    /* context tokens by position, then the proximity tokens, from the first token slot on */
    int j = b->B_r, c = 0;
    for (int t = 0; t < T - n_prox; ++t)
        if (kept[t]) { put_token(b, u, j++, K + (size_t)t * d, V + (size_t)t * d, t, s[t]); ++c; }
    if (c != n_ctx) { free(kept); return -4; }
    for (int t = T - n_prox; t < T; ++t) put_token(b, u, j++, K + (size_t)t * d, V + (size_t)t * d, t, s[t]);
    for (int t = 0; t < T; ++t)
        if (!kept[t]) absorb(b, u, K + (size_t)t * d, V + (size_t)t * d, t, s[t]);
    b->n_seen[u] = T;
    free(kept);
    return 0;
}

/* Qw [n][G][W][d]; K, V [n][T_max][d]; T [n] (each >= W); s_out [n][T_max] (prompt scores, fp32
 * values; entries past a unit's T are left alone). */
int zso_prefill_compress(const zso_batch *b, int W, int T_max, const int32_t *T, const double *Qw, const double *K,
                         const double *V, double *s_out) {
    int err = 0;
    const int d = b->d;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < b->n_units; ++u) {
        const int e = prefill_unit(b, u, W, T[u], Qw + (size_t)u * b->G * W * d, K + (size_t)u * T_max * d,
                                   V + (size_t)u * T_max * d, s_out + (size_t)u * T_max);
        if (e) {
#pragma omp critical
            err = e;
        }
    }
    return err;
}

/* Eq. 1 for one query over all T keys: out [d], a [T]. */
int zso_full_attention_row(int T, int d, const double *q, const double *K, const double *V, double scale, double *out,
                           double *a) {
    double m = -INFINITY, L = 0.0;
    for (int t = 0; t < T; ++t) {
        a[t] = dot(K + (size_t)t * d, q, d) * scale;
        if (a[t] > m) m = a[t];
    }
    for (int t = 0; t < T; ++t) { a[t] = exp(a[t] - m); L += a[t]; }
    for (int i = 0; i < d; ++i) out[i] = 0.0;
    for (int t = 0; t < T; ++t) {
        a[t] /= L;
        for (int i = 0; i < d; ++i) out[i] += a[t] * V[(size_t)t * d + i];
    }
    return 0;
}

int zso_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
