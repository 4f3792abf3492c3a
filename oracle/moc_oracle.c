/*
 * CPU oracle for the Mixture-of-Contexts (MoC) attention layer.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH. Only the test-suite, the
 * smoke check and the benchmark's cpu-baseline leg may call it. It shares no
 * code, header, table or helper with the HIP library.
 *
 * It is the algorithm itself, written out step by step in the paper's order
 * (Sec. 3.1 Eq. 1-3; Sec. 3.2 forced links and causal routing mask; Sec. 3.3
 * pre-routing mask and on-the-fly mean pooling), one (batch, head) slice per
 * call, everything in double precision, no tiling, no fusion, no reordering.
 *
 * Notation: N tokens, d head dim, C chunks, off[C+1] chunk offsets,
 * c(i) chunk of token i, kind[j] (1 = caption/text chunk, 0 = video),
 * win[j] local-window id, k = topk.
 *
 * Readings of passages where the paper is silent or loose:
 *  - routing score is the raw inner product q . mean(K_chunk) (Eq. 3 has no
 *    1/sqrt(d)); attention logits carry 1/sqrt(d) (Eq. 1, 2);
 *  - mandatory chunks M(i) = all text chunks + chunks with the window id of
 *    the query's chunk; they are removed from the candidate set BEFORE top-k,
 *    so k counts routed chunks only (Sec. 3.3 pre-routing mask; App. ablation:
 *    fan-out k+1);
 *  - the causal mask acts on routing only: candidates are chunks with index
 *    j < c(i), later and own chunks being removed before top-k (Sec. 3.2);
 *    mandatory links are exempt;
 *  - fewer than k candidates: take them all, pad the selection with -1;
 *  - ties: the lower chunk index wins;
 *  - backward: the selection is a constant (top-k is not differentiable,
 *    Sec. 3.1); gradients flow only through attention on the chosen tokens.
 *
 *  - a selection row is read as a set: an entry that repeats another one or
 *    names a mandatory chunk adds nothing (M(i) and R(i) are joined, Sec. 3.1).
 *
 * Parity pins live in tests/test_oracle_*.py (brute force with an explicit
 * N x N mask, reductions to dense / causal attention, invariants, central
 * finite differences, closed-form pair counts, subset modes against the
 * whole-sequence rows).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

typedef long long i64;

/* ---- O1: token -> chunk map and chunk kinds (Sec. 3.3, boundary tables) ---- */

void moc_oracle_chunk_map(int N, int C, const int *off, int *chunk_of)
{
    for (int i = 0; i < N; ++i) {
        int found = -1;
        for (int j = 0; j < C; ++j)
            if (off[j] <= i && i < off[j + 1]) { found = j; break; }
        chunk_of[i] = found;
    }
}

/* a chunk is text iff it lies wholly inside one caption span */
void moc_oracle_chunk_kind(int C, const int *off, int T, const int *spans, int *kind)
{
    for (int j = 0; j < C; ++j) {
        kind[j] = 0;
        for (int s = 0; s < T; ++s)
            if (spans[2 * s] <= off[j] && off[j + 1] <= spans[2 * s + 1]) kind[j] = 1;
    }
}

static int chunk_of_token(int i, int C, const int *off)
{
    for (int j = 0; j < C; ++j)
        if (off[j] <= i && i < off[j + 1]) return j;
    return -1;
}

/* ---- O2: descriptor phi = arithmetic mean of the chunk's keys (Sec. 3.1) ---- */

void moc_oracle_pool(int N, int d, int C, const int *off, const double *k, double *kbar)
{
    (void)N;
    for (int j = 0; j < C; ++j) {
        int m = off[j + 1] - off[j];
        for (int x = 0; x < d; ++x) {
            double s = 0.0;
            for (int t = off[j]; t < off[j + 1]; ++t) s += k[(size_t)t * d + x];
            kbar[(size_t)j * d + x] = s / (double)m;
        }
    }
}

/* ---- O3: mandatory set, candidate set, top-k (Eq. 3; Sec. 3.2; Sec. 3.3) ---- */

static int is_mandatory(int j, int cq, const int *kind, const int *win)
{
    return kind[j] == 1 || win[j] == win[cq];
}

typedef struct { double s; int j; } cand_t;

static int cand_cmp(const void *a, const void *b)
{
    const cand_t *x = (const cand_t *)a, *y = (const cand_t *)b;
    if (x->s > y->s) return -1;          /* larger score first            */
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j); /* equal scores: lower index first */
}

/*
 * For each listed query (qidx == NULL: queries 0..nq-1) write sel[n*topk ..]:
 * the routed chunks in score-descending order, -1 padded.
 * scores_out (optional, [nq*C]): s_ij for candidates, NaN elsewhere.
 * n_eligible (optional): sum over listed queries of the candidate count.
 */
void moc_oracle_route(int N, int d, int C, const int *off, const int *kind, const int *win,
                      int causal, int topk, const double *q, const double *kbar,
                      int nq, const int *qidx, int *sel, double *scores_out, i64 *n_eligible)
{
    (void)N;
    i64 total = 0;
#pragma omp parallel for schedule(dynamic, 16) reduction(+ : total)
    for (int n = 0; n < nq; ++n) {
        int i = qidx ? qidx[n] : n;
        int cq = chunk_of_token(i, C, off);
        cand_t *cand = (cand_t *)malloc(sizeof(cand_t) * (size_t)(C > 0 ? C : 1));
        int ne = 0;
        for (int j = 0; j < C; ++j) {
            int eligible = !is_mandatory(j, cq, kind, win) && (!causal || j < cq);
            if (scores_out) scores_out[(size_t)n * C + j] = NAN;
            if (!eligible) continue;
            double s = 0.0;
            for (int x = 0; x < d; ++x) s += q[(size_t)i * d + x] * kbar[(size_t)j * d + x];
            cand[ne].s = s;
            cand[ne].j = j;
            ++ne;
            if (scores_out) scores_out[(size_t)n * C + j] = s;
        }
        qsort(cand, (size_t)ne, sizeof(cand_t), cand_cmp);
        for (int r = 0; r < topk; ++r) sel[(size_t)n * topk + r] = (r < ne) ? cand[r].j : -1;
        total += ne;
        free(cand);
    }
    if (n_eligible) *n_eligible = total;
}

/* does query i (in chunk cq, with routed set selrow[topk]) attend chunk j ? */
static int attends(int j, int cq, const int *kind, const int *win, const int *selrow, int topk)
{
    if (is_mandatory(j, cq, kind, win)) return 1;
    for (int r = 0; r < topk; ++r)
        if (selrow[r] == j) return 1;
    return 0;
}

/* ---- O4: routed attention, Eq. 2, over Omega(i) = tokens of M(i) + R(i) ---- */

/*
 * sel is indexed like the query list: row n belongs to query qidx[n]
 * (qidx == NULL: n). o [nq*d], lse [nq]. n_pairs (optional) = sum |Omega(i)|.
 */
void moc_oracle_attn_fwd(int N, int d, int C, const int *off, const int *kind, const int *win,
                         int topk, const int *sel, const double *q, const double *k,
                         const double *v, double scale, int nq, const int *qidx,
                         double *o, double *lse, i64 *n_pairs)
{
    i64 total = 0;
#pragma omp parallel for schedule(dynamic, 8) reduction(+ : total)
    for (int n = 0; n < nq; ++n) {
        int i = qidx ? qidx[n] : n;
        int cq = chunk_of_token(i, C, off);
        const int *selrow = sel + (size_t)n * topk;
        double *logit = (double *)malloc(sizeof(double) * (size_t)N);
        int *tok = (int *)malloc(sizeof(int) * (size_t)N);
        int cnt = 0;
        for (int j = 0; j < C; ++j) {
            if (!attends(j, cq, kind, win, selrow, topk)) continue;
            for (int t = off[j]; t < off[j + 1]; ++t) {
                double s = 0.0;
                for (int x = 0; x < d; ++x) s += q[(size_t)i * d + x] * k[(size_t)t * d + x];
                logit[cnt] = s * scale;
                tok[cnt] = t;
                ++cnt;
            }
        }
        double m = -INFINITY;
        for (int a = 0; a < cnt; ++a) if (logit[a] > m) m = logit[a];
        double z = 0.0;
        for (int a = 0; a < cnt; ++a) z += exp(logit[a] - m);
        double L = m + log(z);
        for (int x = 0; x < d; ++x) o[(size_t)n * d + x] = 0.0;
        for (int a = 0; a < cnt; ++a) {
            double p = exp(logit[a] - L);
            for (int x = 0; x < d; ++x) o[(size_t)n * d + x] += p * v[(size_t)tok[a] * d + x];
        }
        lse[n] = L;
        total += cnt;
        free(logit);
        free(tok);
    }
    if (n_pairs) *n_pairs = total;
}

/* ---- O5: backward with Omega frozen ---------------------------------------- */

/*
 * dQ for listed queries. o, lse, d_o, sel, dq are indexed like the query list.
 *   delta_i = dO_i . o_i ; P_it = exp(l_it - lse_i) ;
 *   dS_it = P_it (dO_i . v_t - delta_i) ; dQ_i = scale * sum_t dS_it k_t
 */
void moc_oracle_attn_bwd_dq(int N, int d, int C, const int *off, const int *kind, const int *win,
                            int topk, const int *sel, const double *q, const double *k,
                            const double *v, double scale, int nq, const int *qidx,
                            const double *o, const double *lse, const double *d_o, double *dq)
{
    (void)N;
#pragma omp parallel for schedule(dynamic, 8)
    for (int n = 0; n < nq; ++n) {
        int i = qidx ? qidx[n] : n;
        int cq = chunk_of_token(i, C, off);
        const int *selrow = sel + (size_t)n * topk;
        double delta = 0.0;
        for (int x = 0; x < d; ++x) delta += d_o[(size_t)n * d + x] * o[(size_t)n * d + x];
        for (int x = 0; x < d; ++x) dq[(size_t)n * d + x] = 0.0;
        for (int j = 0; j < C; ++j) {
            if (!attends(j, cq, kind, win, selrow, topk)) continue;
            for (int t = off[j]; t < off[j + 1]; ++t) {
                double s = 0.0, dp = 0.0;
                for (int x = 0; x < d; ++x) {
                    s += q[(size_t)i * d + x] * k[(size_t)t * d + x];
                    dp += d_o[(size_t)n * d + x] * v[(size_t)t * d + x];
                }
                double p = exp(s * scale - lse[n]);
                double ds = p * (dp - delta);
                for (int x = 0; x < d; ++x) dq[(size_t)n * d + x] += scale * ds * k[(size_t)t * d + x];
            }
        }
    }
}

/*
 * dK, dV for the tokens of the listed chunks (chunks == NULL: all C chunks).
 * Here sel [N*topk], o [N*d], lse [N], d_o [N*d] cover ALL N queries in token
 * order (rows of queries that attend none of the listed chunks are not read
 * beyond delta). dk, dv are [N*d]; only rows of listed chunks are written.
 *   dV_t = sum_i P_it dO_i ; dK_t = scale * sum_i dS_it q_i
 */
void moc_oracle_attn_bwd_dkdv(int N, int d, int C, const int *off, const int *kind, const int *win,
                              int topk, const int *sel, const double *q, const double *k,
                              const double *v, double scale, const double *o, const double *lse,
                              const double *d_o, int nchunks, const int *chunks,
                              double *dk, double *dv)
{
    int *cof = (int *)malloc(sizeof(int) * (size_t)N);
    double *delta = (double *)malloc(sizeof(double) * (size_t)N);
    moc_oracle_chunk_map(N, C, off, cof);
    for (int i = 0; i < N; ++i) {
        double s = 0.0;
        for (int x = 0; x < d; ++x) s += d_o[(size_t)i * d + x] * o[(size_t)i * d + x];
        delta[i] = s;
    }
    /* flat list of the key tokens to produce */
    int ntok = 0;
    for (int a = 0; a < nchunks; ++a) {
        int j = chunks ? chunks[a] : a;
        ntok += off[j + 1] - off[j];
    }
    int *tl = (int *)malloc(sizeof(int) * (size_t)(ntok > 0 ? ntok : 1));
    ntok = 0;
    for (int a = 0; a < nchunks; ++a) {
        int j = chunks ? chunks[a] : a;
        for (int t = off[j]; t < off[j + 1]; ++t) tl[ntok++] = t;
    }
#pragma omp parallel for schedule(dynamic, 4)
    for (int a = 0; a < ntok; ++a) {
        int t = tl[a];
        int j = cof[t];
        double *dkt = dk + (size_t)t * d, *dvt = dv + (size_t)t * d;
        for (int x = 0; x < d; ++x) { dkt[x] = 0.0; dvt[x] = 0.0; }
        for (int i = 0; i < N; ++i) {
            if (!attends(j, cof[i], kind, win, sel + (size_t)i * topk, topk)) continue;
            double s = 0.0, dp = 0.0;
            for (int x = 0; x < d; ++x) {
                s += q[(size_t)i * d + x] * k[(size_t)t * d + x];
                dp += d_o[(size_t)i * d + x] * v[(size_t)t * d + x];
            }
            double p = exp(s * scale - lse[i]);
            double ds = p * (dp - delta[i]);
            for (int x = 0; x < d; ++x) {
                dvt[x] += p * d_o[(size_t)i * d + x];
                dkt[x] += scale * ds * q[(size_t)i * d + x];
            }
        }
    }
    free(tl);
    free(delta);
    free(cof);
}
