/* Runs every function of the C oracle (oracle/moc_oracle.c, compiled into this program with
 * -fsanitize=address,undefined by tests/test_host_sanitizers.py) on a small ragged layout, in the
 * whole-sequence mode and in the query / chunk subset modes, so that an out-of-bounds index or
 * undefined arithmetic in the oracle is reported. Prints "ok" and a checksum. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

typedef long long i64;
void moc_oracle_chunk_map(int N, int C, const int *off, int *chunk_of);
void moc_oracle_chunk_kind(int C, const int *off, int T, const int *spans, int *kind);
void moc_oracle_pool(int N, int d, int C, const int *off, const double *k, double *kbar);
void moc_oracle_route(int N, int d, int C, const int *off, const int *kind, const int *win, int causal, int topk,
                      const double *q, const double *kbar, int nq, const int *qidx, int *sel, double *scores_out,
                      i64 *n_eligible);
void moc_oracle_attn_fwd(int N, int d, int C, const int *off, const int *kind, const int *win, int topk,
                         const int *sel, const double *q, const double *k, const double *v, double scale, int nq,
                         const int *qidx, double *o, double *lse, i64 *n_pairs);
void moc_oracle_attn_bwd_dq(int N, int d, int C, const int *off, const int *kind, const int *win, int topk,
                            const int *sel, const double *q, const double *k, const double *v, double scale, int nq,
                            const int *qidx, const double *o, const double *lse, const double *d_o, double *dq);
void moc_oracle_attn_bwd_dkdv(int N, int d, int C, const int *off, const int *kind, const int *win, int topk,
                              const int *sel, const double *q, const double *k, const double *v, double scale,
                              const double *o, const double *lse, const double *d_o, int nchunks, const int *chunks,
                              double *dk, double *dv);

static double lcg(unsigned *s) { *s = *s * 1664525u + 1013904223u; return ((*s >> 8) / 16777216.0) * 2.0 - 1.0; }

int main(void)
{
    enum { C = 9, D = 8, K = 3 };
    const int off[C + 1] = {0, 5, 6, 13, 20, 21, 30, 37, 44, 50};
    const int win[C] = {0, 1, 1, 2, 3, 4, 4, 4, 5};
    const int spans[4] = {0, 5, 20, 21};
    const int N = off[C];
    int kind[C], *cof = malloc(sizeof(int) * N);
    moc_oracle_chunk_kind(C, off, 2, spans, kind);
    moc_oracle_chunk_map(N, C, off, cof);
    unsigned s = 12345u;
    double *q = malloc(sizeof(double) * N * D), *k = malloc(sizeof(double) * N * D), *v = malloc(sizeof(double) * N * D),
           *dO = malloc(sizeof(double) * N * D);
    for (int i = 0; i < N * D; ++i) { q[i] = lcg(&s); k[i] = lcg(&s); v[i] = lcg(&s); dO[i] = lcg(&s); }
    double *kbar = malloc(sizeof(double) * C * D);
    moc_oracle_pool(N, D, C, off, k, kbar);
    double sum = 0.0;
    for (int causal = 0; causal < 2; ++causal) {
        int *sel = malloc(sizeof(int) * N * K);
        double *scores = malloc(sizeof(double) * N * C);
        i64 ne = 0, np = 0;
        moc_oracle_route(N, D, C, off, kind, win, causal, K, q, kbar, N, NULL, sel, scores, &ne);
        double *o = malloc(sizeof(double) * N * D), *lse = malloc(sizeof(double) * N), *dq = malloc(sizeof(double) * N * D);
        double *dk = calloc(N * D, sizeof(double)), *dv = calloc(N * D, sizeof(double));
        moc_oracle_attn_fwd(N, D, C, off, kind, win, K, sel, q, k, v, 0.35, N, NULL, o, lse, &np);
        moc_oracle_attn_bwd_dq(N, D, C, off, kind, win, K, sel, q, k, v, 0.35, N, NULL, o, lse, dO, dq);
        moc_oracle_attn_bwd_dkdv(N, D, C, off, kind, win, K, sel, q, k, v, 0.35, o, lse, dO, C, NULL, dk, dv);
        /* subset modes: a few queries, a few chunks, topk = 0 */
        const int qidx[5] = {0, 7, 20, 33, N - 1}, chunks[3] = {0, 4, 8};
        int sel_s[5 * K];
        double o_s[5 * D], lse_s[5], dq_s[5 * D], dO_s[5 * D];
        for (int a = 0; a < 5; ++a)
            for (int x = 0; x < D; ++x) dO_s[a * D + x] = dO[qidx[a] * D + x];
        moc_oracle_route(N, D, C, off, kind, win, causal, K, q, kbar, 5, qidx, sel_s, NULL, NULL);
        moc_oracle_attn_fwd(N, D, C, off, kind, win, K, sel_s, q, k, v, 0.35, 5, qidx, o_s, lse_s, NULL);
        moc_oracle_attn_bwd_dq(N, D, C, off, kind, win, K, sel_s, q, k, v, 0.35, 5, qidx, o_s, lse_s, dO_s, dq_s);
        double *dk2 = calloc(N * D, sizeof(double)), *dv2 = calloc(N * D, sizeof(double));
        moc_oracle_attn_bwd_dkdv(N, D, C, off, kind, win, K, sel, q, k, v, 0.35, o, lse, dO, 3, chunks, dk2, dv2);
        for (int a = 0; a < 5; ++a)
            for (int x = 0; x < D; ++x)
                if (o_s[a * D + x] != o[qidx[a] * D + x] || dq_s[a * D + x] != dq[qidx[a] * D + x]) { puts("subset mismatch"); return 1; }
        for (int a = 0; a < 3; ++a)
            for (int t = off[chunks[a]]; t < off[chunks[a] + 1]; ++t)
                for (int x = 0; x < D; ++x)
                    if (dk2[t * D + x] != dk[t * D + x] || dv2[t * D + x] != dv[t * D + x]) { puts("chunk subset mismatch"); return 1; }
        int none[1] = {0};
        moc_oracle_route(N, D, C, off, kind, win, causal, 0, q, kbar, N, NULL, none, NULL, &ne);
        moc_oracle_attn_fwd(N, D, C, off, kind, win, 0, none, q, k, v, 0.35, N, NULL, o, lse, &np);
        for (int i = 0; i < N * D; ++i) sum += o[i] + dq[i] + dk[i] + dv[i];
        if (!isfinite(sum)) { puts("non-finite"); return 1; }
        free(sel); free(scores); free(o); free(lse); free(dq); free(dk); free(dv); free(dk2); free(dv2);
    }
    free(cof); free(q); free(k); free(v); free(dO); free(kbar);
    printf("ok %.6f\n", sum);
    return 0;
}
