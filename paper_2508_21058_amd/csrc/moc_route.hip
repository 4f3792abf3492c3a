// Stages (b2)+(c): routing scores and per-query top-k (Eq. 3; Sec. 3.2 causal
// routing mask; Sec. 3.3 pre-routing mask that removes forced links from the
// candidates).
//
// One lane per query. The query row lives in registers (fp32); pooled keys are
// wave-uniform and arrive through scalar loads; scores are accumulated in fp32
// and never written to memory. Each lane keeps its top-k as a register-resident
// list sorted by (score desc, index asc); chunks are visited in ascending index
// order and a candidate must beat the list strictly, so ties keep the lower
// index. Causality bounds the chunk loop per wave.
#include "moc_device.h"
#include "moc_internal.h"

namespace moc {

template <int D, typename T, int KMAX>
__global__ __launch_bounds__(256) void route_kernel(const T *__restrict__ q, const float *__restrict__ kbar,
                                                    const int32_t *__restrict__ chunk_of,
                                                    const int32_t *__restrict__ kind,
                                                    const int32_t *__restrict__ win,
                                                    const int32_t *__restrict__ wfirst,
                                                    const int32_t *__restrict__ wlast, int N, int C, int topk,
                                                    int causal, int32_t *__restrict__ sel) {
    const int bh = blockIdx.y;
    const int i = blockIdx.x * 256 + threadIdx.x;
    const bool valid = i < N;
    const int ic = valid ? i : N - 1;
    const int cq = chunk_of[ic];
    const int w = win[cq];
    const int wf = wfirst[w], wl = wlast[w];
    const int limit = causal ? cq : C;           // candidates have index < limit
    // queries of a wave are consecutive, so the last lane has the largest limit
    const int jmax = __shfl(limit, 63, 64);

    float qf[D];
    {
        const T *qp = q + ((size_t)bh * N + ic) * D;
#pragma unroll
        for (int x = 0; x < D; x += 8) Io<T>::load8f(qp + x, qf + x);
    }

    // right-aligned list: positions [KMAX-topk, KMAX) hold the current best in
    // descending order; the others hold +inf and are never displaced
    float val[KMAX];
    int idx[KMAX];
    const int base = KMAX - topk;
#pragma unroll
    for (int p = 0; p < KMAX; ++p) {
        val[p] = (p >= base) ? -INFINITY : INFINITY;
        idx[p] = -1;
    }

    const float *kb_bh = kbar + (size_t)bh * C * D;
    for (int j0 = 0; j0 < jmax; j0 += 4) {
        float s[4] = {0.f, 0.f, 0.f, 0.f};
        const float *kb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) kb[u] = kb_bh + (size_t)min(j0 + u, C - 1) * D;
#pragma unroll
        for (int x = 0; x < D; ++x) {
#pragma unroll
            for (int u = 0; u < 4; ++u) s[u] = fmaf(qf[x], kb[u][x], s[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = j0 + u;
            if (j >= jmax) break;                 // uniform
            if (kind[j]) continue;                // uniform: text is a forced link
            const bool elig = (j < limit) && (j < wf || j > wl);
            if (elig && s[u] > val[KMAX - 1]) {
                float x = s[u];
                int xi = j;
#pragma unroll
                for (int p = 0; p < KMAX; ++p) {
                    const bool sw = x > val[p];
                    const float tv = val[p];
                    const int ti = idx[p];
                    val[p] = sw ? x : tv;
                    idx[p] = sw ? xi : ti;
                    x = sw ? tv : x;
                    xi = sw ? ti : xi;
                }
            }
        }
    }
    if (valid) {
        int32_t *out = sel + ((size_t)bh * N + i) * topk;
#pragma unroll
        for (int p = 0; p < KMAX; ++p)
            if (p >= base) out[p - base] = idx[p];
    }
}

hipError_t launch_route(const moc_meta *m, int BH, int d, int dtype, const void *q, const float *kbar, int topk,
                        int causal, int32_t *sel, hipStream_t st) {
    dim3 grid((m->N + 255) / 256, BH), block(256);
    MOC_PROF("route_topk", st);
#define MOC_ROUTE(DD, TT, KK)                                                                              \
    route_kernel<DD, TT, KK><<<grid, block, 0, st>>>(static_cast<const TT *>(q), kbar, m->d_chunk_of, m->d_kind, \
                                                     m->d_win, m->d_wfirst, m->d_wlast, m->N, m->C, topk,  \
                                                     causal != 0, sel)
#define MOC_ROUTE_K(DD, TT)                      \
    do {                                         \
        if (topk <= 8) MOC_ROUTE(DD, TT, 8);     \
        else if (topk <= 16) MOC_ROUTE(DD, TT, 16); \
        else MOC_ROUTE(DD, TT, 32);              \
    } while (0)
    if (dtype == MOC_BF16) { if (d == 128) MOC_ROUTE_K(128, bf16_t); else MOC_ROUTE_K(64, bf16_t); }
    else { if (d == 128) MOC_ROUTE_K(128, float); else MOC_ROUTE_K(64, float); }
#undef MOC_ROUTE_K
#undef MOC_ROUTE
    return hipGetLastError();
}

}  // namespace moc
