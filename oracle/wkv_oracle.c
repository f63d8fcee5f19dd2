/*
 * TEST INFRASTRUCTURE ONLY -- CPU oracle for the WeightedKV decode step.
 *
 * A plain, slow, fp64 implementation of what the paper's method computes per
 * (sequence, head) unit and per generated token: append the new key/value to
 * the cache, attend, accumulate attention-score sums and counts, and, once the
 * cache exceeds its budget, drop the key of the token with the lowest average
 * score and fold its value into the right-hand neighbour by the convex
 * combination weighted with the two average scores (Algorithm 1; Sections
 * III-A and IV of the paper).  WeightedKV is a heuristic, so the oracle is the
 * algorithm's own steps in the paper's order: ordered arrays, literal removal
 * of index j, explicit count list n.  No blocking, no fusion, no intrinsics.
 *
 * Pins: every function below is checked in tests/test_oracle_pins.py against something
 * other than itself (numbers the paper prints, library softmax attention, closed forms,
 * invariants, a separately written token-table simulator; the eviction-rule variants at every
 * step against an uncompressed library-attention run restricted to the survivors).  Parity
 * unpinned: only what no implementation-free fact covers -- how close the compressed cache
 * stays to full attention (the paper's evidence is perplexity on data that is not
 * available).  The zero-denominator branch of the merge is a reading of a case the paper
 * leaves undefined; the tests check that it does what the reading says, nothing more.  The bulk prefill
 * (orc_prefill) is a reading, not the paper's procedure; it is pinned to causal library
 * attention, to the streaming path where the two must coincide (P <= m + 1), to the list
 * simulator, and to the sorted-score consequence of its fixed scores.
 *
 * It shares no code with the HIP library and nothing on the product path may
 * link or call it; only tests, the smoke check and the benchmark's
 * cpu_baseline leg use it.
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - softmax scale 1/sqrt(d): Section III-A drops it, Section III-B carries it;
 *   - the output o_t uses the m+1 slots before compression (in Algorithm 1 the
 *     attention weights are obtained before the capacity test);
 *   - the arg-min of Algorithm 1 excludes the newest slot only; `recent` = R >= 1
 *     generalises that to the R newest tokens (R = 1 is the algorithm as printed; Section V-A keeps a
 *     recent region).  `n_sink` initial tokens can be protected too (Section
 *     V-A keeps 4); 0 is Algorithm 1;
 *   - arg-min ties go to the oldest token (lowest index);
 *   - the removal step of Algorithm 1 deletes K[j], a[j], n[j] only: the survivor keeps its own key,
 *     score sum and count;
 *   - a zero denominator in the merge (both averages underflowed) merges 1/2, 1/2;
 *   - the paper names no number format: `storage` says to which format the
 *     merged value row is rounded when it is written back (what an in-place
 *     fp16/bf16/fp32 cache does); -1 keeps fp64.
 *   - score_mode / merge_mode select the variants the paper discusses around
 *     the method: merge_mode 1 is the "Eviction" ablation of Section V-B (same
 *     selection, value dropped); score_mode 1 ranks by the cumulative score a
 *     (the H2O rule of Section II), score_mode 2 by the current step's
 *     attention weight (the TOVA rule of Section II); both are eviction rules
 *     and are accepted with merge_mode 1 only.  Mode 0/0 is WeightedKV.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int L;              /* live slots */
    int64_t t;          /* tokens seen */
    double *K, *V;      /* [m+1][d], logical (oldest first) order */
    double *a;          /* [m+1] score sums     */
    int64_t *n;         /* [m+1] counts         */
    int32_t *pos;       /* [m+1] original token index of the retained key */
    int32_t *nmerged;   /* [m+1] raw values folded into the slot */
    double *s, *p;      /* [m+1] scratch: logits, probabilities */
} unit_t;

typedef struct orc {
    int units, d, m, R, storage, n_sink, score_mode, merge_mode;
    unit_t *u;
} orc_t;

/* ---- rounding to a binary floating-point format, nearest-even ------------ */
/* prec = significand bits including the hidden one, emin = exponent of the
 * smallest normal, emax = exponent of the largest finite binade.            */
static double round_format(double x, int prec, int emin, int emax)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);            /* |x| = f * 2^e, f in [0.5, 1)  => leading bit at e-1 */
    int lead = e - 1;
    if (lead < emin) lead = emin;  /* subnormal range: fixed spacing */
    double ulp = ldexp(1.0, lead - (prec - 1));
    double r = nearbyint(x / ulp) * ulp;   /* default rounding mode: ties to even */
    double maxfinite = ldexp(2.0 - ldexp(1.0, -(prec - 1)), emax);
    if (fabs(r) > maxfinite) r = copysign(INFINITY, x);
    return r;
}

double orc_round_storage(double x, int storage)
{
    switch (storage) {
    case 0: return round_format(x, 24, -126, 127);   /* fp32 */
    case 1: return round_format(x, 11, -14, 15);     /* fp16 */
    case 2: return round_format(x, 8, -126, 127);    /* bf16 */
    default: return x;
    }
}

/* ---- the pieces of one step ---------------------------------------------- */

/* A = softmax(q^T K / sqrt(d)) over L rows, o = A^T V.  (Section III-A, with
 * the 1/sqrt(d) of Section III-B.)  s and p are caller scratch of length L. */
void orc_attend(int L, int d, const double *q, const double *K, const double *V,
                double *s, double *p, double *o)
{
    double sq = sqrt((double)d);
    double mx = -INFINITY;
    for (int i = 0; i < L; ++i) {
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += q[c] * K[(size_t)i * d + c];
        s[i] = acc / sq;
        if (s[i] > mx) mx = s[i];
    }
    double S = 0.0;
    for (int i = 0; i < L; ++i) { p[i] = exp(s[i] - mx); S += p[i]; }
    for (int i = 0; i < L; ++i) p[i] /= S;
    for (int c = 0; c < d; ++c) o[c] = 0.0;
    for (int i = 0; i < L; ++i)
        for (int c = 0; c < d; ++c) o[c] += p[i] * V[(size_t)i * d + c];
}

/* arg-min of score over the candidate index range [lo, hi), ties to the lowest
 * index.  (The selection step of Algorithm 1 has lo = 0, hi = m.)  Also reports the second
 * smallest candidate score (+inf when there is a single candidate). */
int orc_select(const double *score, int lo, int hi, double *runner_up)
{
    int j = lo;
    double second = INFINITY;
    for (int i = lo + 1; i < hi; ++i) {
        if (score[i] < score[j]) { second = score[j]; j = i; }
        else if (score[i] < second) second = score[i];
    }
    if (runner_up) *runner_up = second;
    return j;
}

/* (w_j V_j + w_r V_r) / (w_j + w_r), rounded to the storage format.
 * (The merge step of Algorithm 1; worked example in Section IV: 0.1, 0.5 -> 1/6, 5/6.) */
void orc_merge_pair(double wj, double wr, const double *Vj, const double *Vr,
                    int d, int storage, double *dst)
{
    double den = wj + wr;
    for (int c = 0; c < d; ++c) {
        double x = (den > 0.0) ? (wj * Vj[c] + wr * Vr[c]) / den
                               : 0.5 * Vj[c] + 0.5 * Vr[c];
        dst[c] = orc_round_storage(x, storage);
    }
}

static void remove_index(unit_t *u, int d, int j)
{
    int tail = u->L - 1 - j;
    memmove(u->K + (size_t)j * d, u->K + (size_t)(j + 1) * d, sizeof(double) * (size_t)tail * d);
    memmove(u->V + (size_t)j * d, u->V + (size_t)(j + 1) * d, sizeof(double) * (size_t)tail * d);
    memmove(u->a + j, u->a + j + 1, sizeof(double) * tail);
    memmove(u->n + j, u->n + j + 1, sizeof(int64_t) * tail);
    memmove(u->pos + j, u->pos + j + 1, sizeof(int32_t) * tail);
    memmove(u->nmerged + j, u->nmerged + j + 1, sizeof(int32_t) * tail);
    u->L -= 1;
}

/* One token for one unit.  forced_pos >= 0 overrides the arg-min with the
 * candidate whose retained key is that original token (used only to classify
 * a disagreement as a near-tie); returns -1 if that token is not a candidate. */
static int unit_step(const orc_t *o, unit_t *u, const float *q, const float *k, const float *v,
                     double *out, int32_t *ev_slot, int32_t *ev_pos,
                     double *ev_score, double *runner_up, int32_t forced_pos, double *forced_score)
{
    int d = o->d;
    double qd[d];
    /* K_t = [K_{t-1}, k_t], V_t = [V_{t-1}, v_t]   (Section III-A) */
    int L = u->L;
    for (int c = 0; c < d; ++c) {
        qd[c] = (double)q[c];
        u->K[(size_t)L * d + c] = (double)k[c];
        u->V[(size_t)L * d + c] = (double)v[c];
    }
    u->a[L] = 0.0; u->n[L] = 0; u->pos[L] = (int32_t)u->t; u->nmerged[L] = 1;
    L = ++u->L;
    double obuf[d];
    orc_attend(L, d, qd, u->K, u->V, u->s, u->p, obuf);
    if (out) memcpy(out, obuf, sizeof(double) * d);
    /* a = [a, 0] + A_t,  n = [n, 0] + 1   (Algorithm 1, score bookkeeping) */
    for (int i = 0; i < L; ++i) { u->a[i] += u->p[i]; u->n[i] += 1; }

    *ev_slot = -1; *ev_pos = -1;
    if (ev_score) *ev_score = NAN;
    if (runner_up) *runner_up = NAN;
    if (forced_score) *forced_score = NAN;
    int rc = 0;
    if (L > o->m) {                                     /* cache exceeds m */
        double *score = u->s;                           /* logits no longer needed */
        for (int i = 0; i < L; ++i) {
            double abar = u->a[i] / (double)u->n[i];    /* average score */
            score[i] = (o->score_mode == 0) ? abar : (o->score_mode == 1) ? u->a[i] : u->p[i];
        }
        double second;
        int j = orc_select(score, o->n_sink, L - o->R, &second);   /* least important candidate */
        if (ev_score) *ev_score = score[j];
        if (runner_up) *runner_up = second;
        if (forced_pos >= 0 && forced_pos != u->pos[j]) {
            int f = -1;
            for (int i = o->n_sink; i < L - o->R; ++i) if (u->pos[i] == forced_pos) f = i;
            if (f < 0) rc = -1;
            else { if (forced_score) *forced_score = score[f]; j = f; }
        }
        if (o->merge_mode == 0) {                       /* convex merge into the right neighbour */
            orc_merge_pair(score[j], score[j + 1], u->V + (size_t)j * d, u->V + (size_t)(j + 1) * d,
                           d, o->storage, u->V + (size_t)(j + 1) * d);
            u->nmerged[j + 1] += u->nmerged[j];
        }
        *ev_slot = j; *ev_pos = u->pos[j];
        remove_index(u, d, j);                          /* drop K[j], a[j], n[j] */
    }
    u->t += 1;
    return rc;
}

/* ---- handle ---------------------------------------------------------------- */
orc_t *orc_create(int units, int d, int m, int R, int storage, int n_sink, int score_mode, int merge_mode)
{
    if (units <= 0 || d <= 0 || m <= 0 || R < 1 || n_sink < 0 || n_sink + R > m) return NULL;
    if (score_mode < 0 || score_mode > 2 || merge_mode < 0 || merge_mode > 1) return NULL;
    if (score_mode != 0 && merge_mode != 1) return NULL;   /* the two baselines only evict */
    orc_t *o = calloc(1, sizeof(*o));
    if (!o) return NULL;
    o->units = units; o->d = d; o->m = m; o->R = R; o->storage = storage;
    o->n_sink = n_sink; o->score_mode = score_mode; o->merge_mode = merge_mode;
    o->u = calloc((size_t)units, sizeof(unit_t));
    size_t cap = (size_t)m + 1;
    for (int i = 0; i < units; ++i) {
        unit_t *u = &o->u[i];
        u->K = calloc(cap * d, sizeof(double));
        u->V = calloc(cap * d, sizeof(double));
        u->a = calloc(cap, sizeof(double));
        u->n = calloc(cap, sizeof(int64_t));
        u->pos = calloc(cap, sizeof(int32_t));
        u->nmerged = calloc(cap, sizeof(int32_t));
        u->s = calloc(cap, sizeof(double));
        u->p = calloc(cap, sizeof(double));
    }
    return o;
}

void orc_destroy(orc_t *o)
{
    if (!o) return;
    for (int i = 0; i < o->units; ++i) {
        unit_t *u = &o->u[i];
        free(u->K); free(u->V); free(u->a); free(u->n); free(u->pos); free(u->nmerged);
        free(u->s); free(u->p);
    }
    free(o->u); free(o);
}

/* Run nsteps tokens.  q,k,v: [nsteps][units][d] floats holding the exact values
 * of the storage format.  Every output pointer may be NULL.  out: [nsteps][units][d];
 * the int/double logs: [nsteps][units].  forced_pos: NULL, or [nsteps][units]
 * with -1 meaning "no override".  Returns 0, or -(1+step) of the first step in
 * which a forced token was not a legal candidate.  threads <= 0: OpenMP default. */
int orc_run(orc_t *o, int nsteps, const float *q, const float *k, const float *v,
            double *out, int32_t *ev_slot, int32_t *ev_pos, double *ev_score, double *runner_up,
            const int32_t *forced_pos, double *forced_score, int threads)
{
    int d = o->d, U = o->units, bad = 0;
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
    for (int iu = 0; iu < U; ++iu) {
        for (int s = 0; s < nsteps; ++s) {
            size_t row = (size_t)s * U + iu;
            int32_t sl, ps;
            int rc = unit_step(o, &o->u[iu], q + row * d, k + row * d, v + row * d,
                               out ? out + row * d : NULL, &sl, &ps,
                               ev_score ? ev_score + row : NULL,
                               runner_up ? runner_up + row : NULL,
                               forced_pos ? forced_pos[row] : -1,
                               forced_score ? forced_score + row : NULL);
            if (ev_slot) ev_slot[row] = sl;
            if (ev_pos) ev_pos[row] = ps;
            if (rc) {
#ifdef _OPENMP
#pragma omp critical
#endif
                { if (!bad || -(1 + s) > bad) bad = -(1 + s); }
            }
        }
    }
    return bad;
}

/* ---- bulk prefill -----------------------------------------------------------
 * The paper streams from an empty cache (Algorithm 1) and says nothing about a prompt that is
 * given at once.  Reading taken here: the P prompt tokens attend causally to each other over
 * the UNcompressed prompt (row t is softmax attention of q_t over tokens 0..t, Section III-A);
 * the score list is what Algorithm 1's bookkeeping accumulates over those rows, a_i = sum_t
 * A_t[i], n_i = P - i (rows that attended token i); then, while more than m entries remain,
 * the selection and merge of Algorithm 1 are repeated with those scores (no new attention
 * between two merges; the survivor keeps its own a and n, so every abar is fixed).  None of
 * the intermediate rows of this compression is ever held in the cache, so the merges are
 * carried out in fp64 and a row is rounded to the storage format once, when it enters the
 * cache (the paper names no number format).  This is
 * NOT the same function as feeding the prompt token by token, where every token beyond the
 * m-th attends to an already compressed cache; the two coincide for P <= m + 1.
 *
 * Only on an empty cache.  q,k,v: [P][units][d]; out: [P][units][d] or NULL.  ev_pos,
 * ev_score, runner_up: [max(P-m,0)][units] or NULL -- the tokens removed, in order.
 * The last-step scoring rule has no meaning for a prompt (which step?): returns -2.
 * Returns 0, -1 if the cache is not empty. */
int orc_prefill(orc_t *o, int P, const float *q, const float *k, const float *v, double *out,
                int32_t *ev_pos, double *ev_score, double *runner_up, int threads)
{
    int d = o->d, U = o->units, m = o->m;
    if (o->score_mode == 2) return -2;
    for (int iu = 0; iu < U; ++iu) if (o->u[iu].t != 0) return -1;
    if (P <= 0) return 0;
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
#endif
    for (int iu = 0; iu < U; ++iu) {
        unit_t *u = &o->u[iu];
        double *K = malloc(sizeof(double) * (size_t)P * d), *V = malloc(sizeof(double) * (size_t)P * d);
        double *a = calloc((size_t)P, sizeof(double)), *s = malloc(sizeof(double) * P), *p = malloc(sizeof(double) * P);
        double *score = malloc(sizeof(double) * P);
        int64_t *n = malloc(sizeof(int64_t) * P);
        int32_t *idx = malloc(sizeof(int32_t) * P), *nm = malloc(sizeof(int32_t) * P);
        double qd[d], obuf[d];
        for (int t = 0; t < P; ++t)
            for (int c = 0; c < d; ++c) {
                K[(size_t)t * d + c] = (double)k[((size_t)t * U + iu) * d + c];
                V[(size_t)t * d + c] = (double)v[((size_t)t * U + iu) * d + c];
            }
        /* rows of the prompt: A_t over tokens 0..t, o_t = A_t^T V, a += A_t   (Section III-A, Algorithm 1) */
        for (int t = 0; t < P; ++t) {
            for (int c = 0; c < d; ++c) qd[c] = (double)q[((size_t)t * U + iu) * d + c];
            orc_attend(t + 1, d, qd, K, V, s, p, obuf);
            if (out) memcpy(out + ((size_t)t * U + iu) * d, obuf, sizeof(double) * d);
            for (int i = 0; i <= t; ++i) a[i] += p[i];
        }
        int L = P;
        for (int i = 0; i < P; ++i) { n[i] = P - i; idx[i] = i; nm[i] = 1; }
        /* P - m times: least important candidate folds into its right neighbour and is removed.
         * idx[] lists the remaining tokens oldest first; a, n, nm are kept aligned with it; the
         * rows of K and V stay where they are (row idx[i]), V rows are rewritten in place. */
        for (int e = 0; L > m; ++e) {
            for (int i = 0; i < L; ++i)
                score[i] = (o->score_mode == 0) ? a[i] / (double)n[i] : a[i];
            double second;
            int j = orc_select(score, o->n_sink, L - o->R, &second);
            if (ev_pos) ev_pos[(size_t)e * U + iu] = idx[j];
            if (ev_score) ev_score[(size_t)e * U + iu] = score[j];
            if (runner_up) runner_up[(size_t)e * U + iu] = second;
            if (o->merge_mode == 0) {
                double *Vj = V + (size_t)idx[j] * d, *Vr = V + (size_t)idx[j + 1] * d;
                orc_merge_pair(score[j], score[j + 1], Vj, Vr, d, -1, Vr);     /* fp64, not rounded yet */
                nm[j + 1] += nm[j];
            }
            int tail = L - 1 - j;
            memmove(idx + j, idx + j + 1, sizeof(int32_t) * tail);
            memmove(a + j, a + j + 1, sizeof(double) * tail);
            memmove(n + j, n + j + 1, sizeof(int64_t) * tail);
            memmove(nm + j, nm + j + 1, sizeof(int32_t) * tail);
            L -= 1;
        }
        for (int i = 0; i < L; ++i) {
            memcpy(u->K + (size_t)i * d, K + (size_t)idx[i] * d, sizeof(double) * d);
            for (int c = 0; c < d; ++c)                                         /* the row enters the cache */
                u->V[(size_t)i * d + c] = orc_round_storage(V[(size_t)idx[i] * d + c], o->storage);
            u->a[i] = a[i]; u->n[i] = n[i]; u->pos[i] = idx[i]; u->nmerged[i] = nm[i];
        }
        u->L = L; u->t = P;
        free(K); free(V); free(a); free(s); free(p); free(score); free(n); free(idx); free(nm);
    }
    return 0;
}

int orc_len(const orc_t *o, int unit) { return o->u[unit].L; }
int64_t orc_tokens(const orc_t *o, int unit) { return o->u[unit].t; }
int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Copy one unit's state out, logical order.  Any pointer may be NULL. */
void orc_state(const orc_t *o, int unit, double *K, double *V, double *a, int64_t *n,
               int32_t *pos, int32_t *nmerged)
{
    const unit_t *u = &o->u[unit];
    size_t L = (size_t)u->L;
    if (K) memcpy(K, u->K, sizeof(double) * L * o->d);
    if (V) memcpy(V, u->V, sizeof(double) * L * o->d);
    if (a) memcpy(a, u->a, sizeof(double) * L);
    if (n) memcpy(n, u->n, sizeof(int64_t) * L);
    if (pos) memcpy(pos, u->pos, sizeof(int32_t) * L);
    if (nmerged) memcpy(nmerged, u->nmerged, sizeof(int32_t) * L);
}
