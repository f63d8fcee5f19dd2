/*
 * Runs the CPU oracle (oracle/wkv_oracle.c, compiled into this program with
 * -fsanitize=address,undefined) over cases read from a file, and writes what it computed to
 * another file; tests/test_oracle_sanitized.py prepares the cases and compares the results with
 * those of the regular build.  Any invalid memory access, leak or undefined operation in the
 * oracle makes the sanitizers abort this program with a report.
 *
 * Case file (native endianness), repeated until end of file:
 *   int32 kind (0 = stream, 1 = prompt), units, d, m, R, storage, n_sink, score_mode, merge_mode, n, forced
 *   float32 q[n][units][d], k[...], v[...]
 *   if forced: int32 forced_pos[n][units]
 * Result file, per case: int32 rc; float64 out[n][units][d]; int32 evict_pos[rows][units]
 *   (rows = n for a stream, max(n - m, 0) for a prompt); then per unit: int32 L, float64 V[L][d],
 *   float64 a[L], int32 pos[L].
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

typedef struct orc orc_t;
orc_t *orc_create(int units, int d, int m, int R, int storage, int n_sink, int score_mode, int merge_mode);
void orc_destroy(orc_t *o);
int orc_run(orc_t *o, int nsteps, const float *q, const float *k, const float *v, double *out, int32_t *ev_slot,
            int32_t *ev_pos, double *ev_score, double *runner_up, const int32_t *forced_pos, double *forced_score,
            int threads);
int orc_prefill(orc_t *o, int P, const float *q, const float *k, const float *v, double *out, int32_t *ev_pos,
                double *ev_score, double *runner_up, int threads);
int orc_len(const orc_t *o, int unit);
void orc_state(const orc_t *o, int unit, double *K, double *V, double *a, int64_t *n, int32_t *pos, int32_t *nmerged);

static void *xmalloc(size_t n) { void *p = malloc(n ? n : 1); if (!p) { perror("malloc"); exit(3); } return p; }
static void rd(void *p, size_t n, FILE *f) { if (fread(p, 1, n, f) != n) { fprintf(stderr, "short read\n"); exit(3); } }

int main(int argc, char **argv)
{
    if (argc != 3) { fprintf(stderr, "usage: %s cases results\n", argv[0]); return 2; }
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) { perror("fopen"); return 2; }
    int32_t h[11];
    int cases = 0;
    while (fread(h, sizeof h, 1, in) == 1) {
        int kind = h[0], units = h[1], d = h[2], m = h[3], R = h[4], n = h[9], forced = h[10];
        size_t rows = (size_t)n * units, elems = rows * d;
        float *q = xmalloc(elems * 4), *k = xmalloc(elems * 4), *v = xmalloc(elems * 4);
        rd(q, elems * 4, in); rd(k, elems * 4, in); rd(v, elems * 4, in);
        int32_t *fp = NULL;
        if (forced) { fp = xmalloc(rows * 4); rd(fp, rows * 4, in); }
        orc_t *o = orc_create(units, d, m, R, h[5], h[6], h[7], h[8]);
        if (!o) { fprintf(stderr, "case %d: invalid configuration\n", cases); return 3; }
        double *res = xmalloc(elems * 8), *sc = xmalloc(rows * 8), *ru = xmalloc(rows * 8), *fs = xmalloc(rows * 8);
        int32_t *es = xmalloc(rows * 4), *ep = xmalloc(rows * 4);
        size_t ev_rows = kind == 0 ? (size_t)n : (size_t)(n > m ? n - m : 0);
        int32_t rc = kind == 0 ? orc_run(o, n, q, k, v, res, es, ep, sc, ru, fp, fp ? fs : NULL, 2)
                               : orc_prefill(o, n, q, k, v, res, ep, sc, ru, 2);
        fwrite(&rc, 4, 1, out);
        fwrite(res, 8, elems, out);
        fwrite(ep, 4, ev_rows * units, out);
        for (int u = 0; u < units; ++u) {
            int32_t L = orc_len(o, u);
            double *V = xmalloc((size_t)L * d * 8), *a = xmalloc((size_t)L * 8);
            int32_t *pos = xmalloc((size_t)L * 4);
            orc_state(o, u, NULL, V, a, NULL, pos, NULL);
            fwrite(&L, 4, 1, out); fwrite(V, 8, (size_t)L * d, out); fwrite(a, 8, L, out); fwrite(pos, 4, L, out);
            free(V); free(a); free(pos);
        }
        orc_destroy(o);
        free(q); free(k); free(v); free(fp); free(res); free(sc); free(ru); free(fs); free(es); free(ep);
        ++cases;
    }
    fclose(in); fclose(out);
    printf("%d cases\n", cases);
    return 0;
}
