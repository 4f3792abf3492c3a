// Routing regularisers applied to the routed set of every (head, query) row
// (Sec. 3.2, "Context Drop-off" and "Context Drop-in"): a random number of the
// routed chunks is removed, a Poisson number of further candidates is added.
//
// One lane per row. Random words come from Philox4x32-10 (Salmon et al., SC'11)
// with counter (query, head, block, 0) and the 64-bit seed as key; draw t of a
// row is word t mod 4 of block t / 4: draw 0 sets the drop probability, draw 1
// the Poisson count, the next draws pick what to remove and then what to add.
// Both picks are uniform without replacement by rank: floor(draw * n / 2^32)
// among the n entries still alive (routed order), respectively among the n
// candidates not routed and not yet added (ascending chunk index). The rank of
// a candidate is found without enumerating candidates: a prefix count of
// non-text chunks gives the rank of any chunk among the query's candidates, the
// ranks already excluded are kept sorted per lane in LDS, and a binary search
// over the prefix counts turns the final rank back into a chunk index.
#include "moc_internal.h"
#include "moc_device.h"

namespace moc {

struct PerturbArgs {
    int32_t *sel;                          // [BH][N][width], the first topk columns hold the routed chunks
    const int32_t *chunk_of, *win, *wfirst, *wlast;
    const int32_t *ntb;                    // [C+1] number of non-text chunks with index < j
    int N, C, topk, max_in, causal;
    float p_max;
    uint32_t key0, key1;
    uint64_t thr[MOC_MAX_TOPK];            // floor(CDF(j) * 2^32) of the Poisson law, j < max_in
};

struct Philox {
    uint32_t c0, c1, k0, k1;               // counter words 0, 1 and the key
    uint32_t w[4];
    int t = 0;
    __device__ void block(uint32_t blk) {
        uint32_t x0 = c0, x1 = c1, x2 = blk, x3 = 0, a = k0, b = k1;
#pragma unroll
        for (int r = 0; r < 10; ++r) {
            const uint32_t h0 = __umulhi(0xD2511F53u, x0), l0 = 0xD2511F53u * x0;
            const uint32_t h1 = __umulhi(0xCD9E8D57u, x2), l1 = 0xCD9E8D57u * x2;
            x0 = h1 ^ x1 ^ a; x1 = l1; x2 = h0 ^ x3 ^ b; x3 = l0;
            a += 0x9E3779B9u; b += 0xBB67AE85u;
        }
        w[0] = x0; w[1] = x1; w[2] = x2; w[3] = x3;
    }
    __device__ uint32_t next() {
        const int word = t & 3;
        if (word == 0) block((uint32_t)(t >> 2));
        ++t;
        return word == 0 ? w[0] : word == 1 ? w[1] : word == 2 ? w[2] : w[3];
    }
};

constexpr int kPerturbThreads = 128;

__global__ __launch_bounds__(kPerturbThreads) void perturb_kernel(PerturbArgs a) {
    // per lane: the routed chunks (topk slots), then the sorted excluded ranks (topk + max_in slots);
    // sized at launch so that small rows leave room for many workgroups per CU
    extern __shared__ int32_t lds[];
    int32_t (*ent)[kPerturbThreads] = reinterpret_cast<int32_t (*)[kPerturbThreads]>(lds);
    int32_t (*ex)[kPerturbThreads] = ent + a.topk;
    const int tid = threadIdx.x;
    const int i = blockIdx.x * kPerturbThreads + tid;
    if (i >= a.N) return;
    const int bh = blockIdx.y;
    const int width = a.topk + a.max_in;
    int32_t *row = a.sel + ((size_t)bh * a.N + i) * width;

    const int cq = a.chunk_of[i];
    const int w = a.win[cq];
    const int limit = a.causal ? cq : a.C;
    const int wf = min(a.wfirst[w], limit), wl1 = min(a.wlast[w] + 1, limit);   // own window inside [0, limit)
    const int nt_wf = a.ntb[wf];
    const int win_nt = a.ntb[wl1] - nt_wf;                                      // its non-text chunks
    const int n_elig = a.ntb[limit] - win_nt;

    int nv = 0;
    for (int r = 0; r < a.topk; ++r) {
        const int c = row[r];
        if (c >= 0) ent[nv++][tid] = c;
    }

    Philox g;
    g.c0 = (uint32_t)i; g.c1 = (uint32_t)bh; g.k0 = a.key0; g.k1 = a.key1;
    const uint32_t r_drop = g.next(), r_in = g.next();

    // ---- drop-off: floor(p k) of the routed chunks, p = u p_max, single precision
    const float u = (float)(r_drop >> 8) * 0x1p-24f;
    const float pk = (u * a.p_max) * (float)a.topk;
    const int nd = min((int)floorf(pk), nv);
    uint32_t alive = nv >= 32 ? 0xffffffffu : ((1u << nv) - 1u);
    for (int s = 0; s < nd; ++s) {
        const int t = (int)__umulhi(g.next(), (uint32_t)(nv - s));
        uint32_t b = alive;
        for (int x = 0; x < t; ++x) b &= b - 1;            // skip t alive entries
        alive &= ~(b & (0u - b));                          // clear the lowest remaining one
    }

    // ---- drop-in: m ~ Poisson by inversion, truncated, capped by what is available
    int m = 0;
    for (int j = 0; j < a.max_in; ++j) m += (uint64_t)r_in >= a.thr[j] ? 1 : 0;
    m = min(m, n_elig - nv);
    int out = 0;
    if (m > 0) {
        // ranks (among the query's candidates) of the routed chunks, sorted ascending
        for (int r = 0; r < nv; ++r) {
            const int c = ent[r][tid];
            const int rk = a.ntb[c] - (c >= wl1 ? win_nt : 0);
            int p = r;
            while (p > 0 && ex[p - 1][tid] > rk) { ex[p][tid] = ex[p - 1][tid]; --p; }
            ex[p][tid] = rk;
        }
    }
    // survivors first, in routed order
    for (int r = 0; r < nv; ++r)
        if ((alive >> r) & 1u) row[out++] = ent[r][tid];
    int nex = nv;
    for (int s = 0; s < m; ++s) {
        int t = (int)__umulhi(g.next(), (uint32_t)(n_elig - nv - s));
        int p = 0;
        while (p < nex && ex[p][tid] <= t) { ++t; ++p; }   // step over excluded ranks
        for (int x = nex; x > p; --x) ex[x][tid] = ex[x - 1][tid];
        ex[p][tid] = t;
        ++nex;
        const int nt_rank = t < nt_wf ? t : t + win_nt;    // rank among all non-text chunks
        int lo = 0, hi = a.C;                              // largest j with ntb[j] <= nt_rank
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (a.ntb[mid] <= nt_rank) lo = mid; else hi = mid;
        }
        row[out++] = lo;
    }
    for (; out < width; ++out) row[out] = -1;
}

hipError_t launch_perturb(const moc_meta *m, int BH, int topk, int max_in, int causal, float p_max,
                          const uint64_t *thr, uint64_t seed, int32_t *sel, hipStream_t st) {
    PerturbArgs a{};
    a.sel = sel;
    a.chunk_of = m->d_chunk_of; a.win = m->d_win; a.wfirst = m->d_wfirst; a.wlast = m->d_wlast; a.ntb = m->d_ntb;
    a.N = m->N; a.C = m->C; a.topk = topk; a.max_in = max_in; a.causal = causal != 0;
    a.p_max = p_max;
    a.key0 = (uint32_t)seed; a.key1 = (uint32_t)(seed >> 32);
    for (int j = 0; j < max_in; ++j) a.thr[j] = thr[j];
    dim3 grid((m->N + kPerturbThreads - 1) / kPerturbThreads, BH);
    MOC_PROF("route_perturb", st);
    const size_t lds_bytes = (size_t)(2 * topk + max_in) * kPerturbThreads * sizeof(int32_t);   // <= 48 KB
    perturb_kernel<<<grid, kPerturbThreads, lds_bytes, st>>>(a);
    return hipGetLastError();
}

}  // namespace moc
