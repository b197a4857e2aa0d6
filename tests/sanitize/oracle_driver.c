/* Runs the CPU oracle on a workload file under the sanitizers (built together with
 * oracle/distsim_oracle.c by tests/test_sanitizers.py; CPU only).  File layout, all little endian:
 *   int64 header[16]: L V N g alpha0 alpha1 beta0 beta1 bucket blocking C pool_len n_sched words_len has_chunks timeline
 *   int32 variant_tp[V]; int64 fc, bc, fa, ba, act, grad, a2a [V*L] each
 *   int32 dp, tp, pp, m [C] each; uint8 schedule[C]; int32 chunks[C]; int64 part_off[C]; uint8 pool[pool_len]
 *   int64 sched_off[n_sched+1]; int32 words[words_len]
 * Prints one line per output array: name and a 64-bit FNV-1a hash of its bytes. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_simulate(int32_t, int32_t, const int32_t *, const int64_t *, const int64_t *, const int64_t *, const int64_t *,
                    const int64_t *, const int64_t *, const int64_t *, int32_t, int32_t, const int64_t *, const int64_t *,
                    int64_t, int32_t, int64_t, const int32_t *, const int32_t *, const int32_t *, const int32_t *,
                    const uint8_t *, const int32_t *, const int64_t *, const uint8_t *, int64_t, int64_t, const int64_t *,
                    const int32_t *, int64_t, int32_t *, int64_t *, int64_t *, int64_t *, int64_t *, int64_t *, double *,
                    int64_t *, int64_t *, int64_t *, int32_t);
int oracle_stage_table(int32_t, int32_t, const int32_t *, const int64_t *, const int64_t *, const int64_t *, const int64_t *,
                       const int64_t *, const int64_t *, const int64_t *, int32_t, int32_t, const int64_t *, const int64_t *,
                       int64_t, const int32_t *, const int32_t *, const int32_t *, const uint8_t *, const int64_t *,
                       const uint8_t *, const int32_t *, const int64_t *, int64_t *, int32_t *, int32_t *);
int oracle_search(const int64_t *, const int64_t *, int64_t, int32_t, int64_t *);

static void *rd(FILE *f, size_t n, size_t sz) {
    /* exact-size buffers, so that any read past an array's end is seen */
    void *p = malloc(n * sz ? n * sz : 1);
    if (n && fread(p, sz, n, f) != n) { fprintf(stderr, "short file\n"); exit(3); }
    return p;
}
static void hash(const char *name, const void *p, size_t bytes) {
    uint64_t h = 1469598103934665603ull;
    for (size_t i = 0; i < bytes; i++) { h ^= ((const unsigned char *)p)[i]; h *= 1099511628211ull; }
    printf("%s %016llx\n", name, (unsigned long long)h);
}

int main(int argc, char **argv) {
    if (argc < 2) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int64_t *H = rd(f, 16, 8);
    const int64_t L = H[0], V = H[1], C = H[10], pool_len = H[11], ns = H[12], wl = H[13];
    int32_t *vt = rd(f, V, 4);
    int64_t *col[7];
    for (int i = 0; i < 7; i++) col[i] = rd(f, V * L, 8);
    int32_t *dp = rd(f, C, 4), *tp = rd(f, C, 4), *pp = rd(f, C, 4), *m = rd(f, C, 4);
    uint8_t *sc = rd(f, C, 1);
    int32_t *ch = rd(f, C, 4);
    int64_t *po = rd(f, C, 8);
    uint8_t *pool = rd(f, pool_len, 1);
    int64_t *so = rd(f, ns + 1, 8);
    int32_t *words = rd(f, wl, 4);
    fclose(f);
    int64_t S = 0;
    for (int64_t c = 0; c < C; c++) S += pp[c] > 0 ? pp[c] : 0;
    int32_t *status = malloc((C ? C : 1) * 4);
    int64_t *batch = malloc((C ? C : 1) * 8), *nev = malloc((C ? C : 1) * 8), *soff = malloc((C + 1) * 8);
    int64_t *comp = calloc(S ? S : 1, 8), *comm = calloc(S ? S : 1, 8);
    double *util = calloc(S ? S : 1, 8);
    int64_t *tls = NULL, *tle = NULL, *tar = NULL;
    size_t tl_n = 0;
    if (H[15] && C == 1) {                               /* timeline of the single candidate: [2][rows][m] */
        int64_t rows = pp[0];
        if (sc[0] == 3 && H[14]) rows = (int64_t)pp[0] * ch[0];
        if (sc[0] == 4 && H[14] && ch[0] >= 0 && ch[0] < ns && so[ch[0]] + 5 <= wl) rows = words[so[ch[0]] + 1];
        if (rows < 1) rows = 1;
        tl_n = (size_t)(2 * rows * m[0]);
        tls = malloc(tl_n * 8); tle = malloc(tl_n * 8); tar = malloc((size_t)(2 * (pp[0] > 0 ? pp[0] : 1)) * 8);
        for (size_t i = 0; i < tl_n; i++) { tls[i] = -1; tle[i] = -1; }
    }
    const int64_t alpha[2] = { H[4], H[5] }, beta[2] = { H[6], H[7] };
    int rc = oracle_simulate((int32_t)L, (int32_t)V, vt, col[0], col[1], col[2], col[3], col[4], col[5], col[6],
                             (int32_t)H[2], (int32_t)H[3], alpha, beta, H[8], (int32_t)H[9], C, dp, tp, pp, m, sc,
                             H[14] ? ch : NULL, po, pool, pool_len, ns, ns ? so : NULL, ns ? words : NULL, wl,
                             status, batch, nev, soff, comp, comm, util, tls, tle, tar, 2);
    if (rc) return 4;
    hash("status", status, C * 4); hash("batch_ns", batch, C * 8); hash("num_events", nev, C * 8);
    hash("stage_off", soff, (C + 1) * 8); hash("comp_busy_ns", comp, soff[C] * 8); hash("comm_busy_ns", comm, soff[C] * 8);
    hash("util", util, soff[C] * 8);
    if (tls) { hash("start", tls, tl_n * 8); hash("end", tle, tl_n * 8); hash("ar_window", tar, (size_t)(2 * pp[0]) * 8); }
    const int64_t n = soff[C];
    int64_t *tab = malloc((n ? 8 * n : 1) * 8);
    int32_t *lo = malloc((n ? n : 1) * 4), *hi = malloc((n ? n : 1) * 4);
    rc = oracle_stage_table((int32_t)L, (int32_t)V, vt, col[0], col[1], col[2], col[3], col[4], col[5], col[6],
                            (int32_t)H[2], (int32_t)H[3], alpha, beta, C, dp, tp, pp, sc, po, pool, status, soff, tab, lo, hi);
    if (rc) return 5;
    hash("tab", tab, n * 64); hash("layer_lo", lo, n * 4); hash("layer_hi", hi, n * 4);
    int64_t best[2];
    int64_t *wgt = malloc((C ? C : 1) * 8);
    for (int64_t c = 0; c < C; c++) wgt[c] = (int64_t)dp[c] * m[c];
    oracle_search(batch, NULL, C, 0, best); hash("best0", best, 16);
    oracle_search(batch, wgt, C, 1, best); hash("best1", best, 16);
    free(H); free(vt); for (int i = 0; i < 7; i++) free(col[i]);
    free(dp); free(tp); free(pp); free(m); free(sc); free(ch); free(po); free(pool); free(so); free(words);
    free(status); free(batch); free(nev); free(soff); free(comp); free(comm); free(util); free(tls); free(tle); free(tar);
    free(tab); free(lo); free(hi); free(wgt);
    return 0;
}
