// Stages (b2)+(c): routing scores and per-query top-k (Eq. 3; Sec. 3.2 causal
// routing mask; Sec. 3.3 pre-routing mask that removes forced links from the
// candidates).
//
// Scores on matrix cores at fp32 accuracy: the fp32 pooled keys arrive split
// into three bf16 planes (hi + mid + lo == value); a bf16 query is exact, an
// fp32 query is split the same way, and all partial products of order <= 2 are
// accumulated in fp32, so a score differs from the exact inner product only by
// accumulation rounding. S^T[chunk][query] tiles of 32 chunks x 32 queries put
// one query in each lane (two half-waves share a query and own 16 chunks of a
// tile each); the [N, C] score matrix never exists in memory.
//
// Per-lane top-k without a sort and without paying wave divergence per score:
//   filter  scores >= tau, the lane's k-th best so far (-inf-like until k scores
//           have been seen), are appended to a per-lane queue in LDS: after the
//           first tiles only a few per tile pass;
//   drain   when a queue would overflow (and at the end) it is inserted into a
//           register-resident sorted list with strict comparisons, in chunk
//           order, so ties keep the lower index; tau rises to the new k-th best;
//   merge   the two half-waves exchange their lists.
// One pass over the chunks; any data (ties, few tiles) stays exact.
#include "moc_attn_common.h"
#include "moc_pool_unit.h"

namespace moc {

struct RouteArgs {
    const void *q;
    const bf16_t *split;          // [BH][3][Cpad][D]
    const int32_t *chunk_of, *win, *wfirst, *wlast;
    const uint32_t *textmask;
    int32_t *sel;
    int N, C, Cpad, topk, causal;
    int stride;                   // int32 words between consecutive rows of sel (>= topk)
};

constexpr int kQCap = 15;         // queue entries per lane (plus one spill row: 2 x 16 KB of LDS for 256 lanes)

// sorted insert (descending), strict: an equal score stays behind the entries already there.
// Position p takes the median of (val[p-1], val[p], x): the shifted neighbour if x passed it, x if it
// lands here, else what it held; the index follows with one comparison per position.
template <int KMAX>
__device__ __forceinline__ void topk_insert(float (&val)[KMAX], int (&idx)[KMAX], float x, int xi) {
    bool above = false;                 // x > val[p-1]
    float pv = INFINITY;                // val[p-1] before this insert
    int pi = -1;
#pragma unroll
    for (int p = 0; p < KMAX; ++p) {
        const bool here = x > val[p];
        const float tv = val[p];
        const int ti = idx[p];
        val[p] = __builtin_amdgcn_fmed3f(pv, tv, x);
        idx[p] = above ? pi : (here ? xi : ti);
        above = here; pv = tv; pi = ti;
    }
}

// sorted insert ordering by (score desc, index asc)
template <int KMAX>
__device__ __forceinline__ void topk_insert_tie(float (&val)[KMAX], int (&idx)[KMAX], float x, int xi) {
#pragma unroll
    for (int p = 0; p < KMAX; ++p) {
        const bool sw = (x > val[p]) || (x == val[p] && (unsigned)xi < (unsigned)idx[p]);
        const float tv = val[p];
        const int ti = idx[p];
        val[p] = sw ? x : tv;
        idx[p] = sw ? xi : ti;
        x = sw ? tv : x;
        xi = sw ? ti : xi;
    }
}

// Four waves x 32 queries per workgroup, two workgroups per CU, two staged tiles of pooled keys (one
// in use, one in flight). The pass is bound by the selection's vector instructions, not by the
// latency of the tile copies: eight waves with three stages (one workgroup per CU) measured 13 %
// slower, because a barrier per tile then couples twice as many waves whose queue drains fall on
// different tiles.
constexpr int kRouteThreads = 256;
constexpr int kRouteStages = 2;

template <int D, typename T, int KMAX>
__device__ __forceinline__ void route_body(const RouteArgs &a, char *smem, u32x2 (*queue)[kRouteThreads]) {
    constexpr int KS = D / 16;
    constexpr int NQ = sizeof(T) == 2 ? 1 : 3;       // query planes
    constexpr int PB = 32 * D * 2;                   // bytes of one plane tile (32 chunks)
    constexpr int TB = 3 * PB;                       // bytes of one staged tile
    constexpr int NWV = kRouteThreads / 64;
    constexpr int QPW = kRouteThreads / 2;           // queries per workgroup

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int bh = blockIdx.y, N = a.N, C = a.C;
    const int q0 = blockIdx.x * QPW;
    const int i = q0 + wave * 32 + l32;
    const bool valid = i < N;
    const int ic = valid ? i : N - 1;
    const int cq = a.chunk_of[ic];
    const int w = a.win[cq];
    const int wf = a.wfirst[w], wl = a.wlast[w];
    const int limit = a.causal ? cq : C;                               // candidates have index < limit
    // queries ascend with the lane, so do chunk, window and limit
    const int lim_wg = __builtin_amdgcn_readfirstlane(a.causal ? a.chunk_of[min(q0 + QPW - 1, N - 1)] : C);  // uniform: largest limit in the workgroup
    const int ntiles = (lim_wg + 31) >> 5;
    const int lim_lo = __shfl(limit, 0, 64);                            // smallest limit in the wave
    const int wf_lo = __shfl(wf, 0, 64), wl_hi = __shfl(wl, 31, 64);    // chunks that may be forced links in the wave
    const int topk = a.topk;
    int32_t *out = a.sel + ((size_t)bh * N + ic) * a.stride;
    if (ntiles == 0) {                                                  // no candidates at all
        if (valid && half == 0)
            for (int r = 0; r < topk; ++r) out[r] = -1;
        return;
    }

    // query operand planes (B operand: lane -> query column)
    bf16x8 qf[NQ][KS];
    {
        const T *qp = static_cast<const T *>(a.q) + ((size_t)bh * N + ic) * D;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if constexpr (NQ == 1) {
                qf[0][s] = Io<T>::load8(qp + s * 16 + half * 8);
            } else {
                float f[8];
                Io<T>::load8f(qp + s * 16 + half * 8, f);
                float hi[8], mid[8], lo[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bf16_t h = (bf16_t)f[e];
                    const float r1 = f[e] - (float)h;
                    const bf16_t m = (bf16_t)r1;
                    hi[e] = (float)h; mid[e] = (float)m; lo[e] = r1 - (float)m;
                }
                u32x4 ph, pm, pl;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    ph[e] = pack_bf16(hi[2 * e], hi[2 * e + 1]);
                    pm[e] = pack_bf16(mid[2 * e], mid[2 * e + 1]);
                    pl[e] = pack_bf16(lo[2 * e], lo[2 * e + 1]);
                }
                qf[0][s] = __builtin_bit_cast(bf16x8, ph);
                qf[NQ > 1 ? 1 : 0][s] = __builtin_bit_cast(bf16x8, pm);
                qf[NQ > 2 ? 2 : 0][s] = __builtin_bit_cast(bf16x8, pl);
            }
        }
    }
    // The query fragments are consumed here, before the first tile copy is issued: the waits the
    // compiler needs for their loads then sit in front of the loop, not inside it, where they would
    // also wait for the tile copies in flight.
#pragma unroll
    for (int qa = 0; qa < NQ; ++qa)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            u32x4 w = __builtin_bit_cast(u32x4, qf[qa][s]);
            asm volatile("" : "+v"(w));
            qf[qa][s] = __builtin_bit_cast(bf16x8, w);
        }
    LaneOffs<D> lo;
    lo.init(lane);

    // Copies of one staged tile (3 planes x 32 rows), spread over the eight waves: a wave instruction
    // moves 1 KB (512 / D rows). Every wave issues the same number of copies per tile so that one
    // vmcnt bound fits all (with D = 64 the last four waves repeat a copy of the first four).
    constexpr int RPI = 512 / D, NI = 32 / RPI, TOT = 3 * NI, PW = (TOT + NWV - 1) / NWV;
    const int uwave = __builtin_amdgcn_readfirstlane(wave);
    const int rlo = lane / (D / 8), cgp = lane % (D / 8);
    const bf16_t *sp = a.split + (size_t)bh * 3 * a.Cpad * D;
    auto issue = [&](int t, int buf) {
        const uint32_t at = lds_address(smem + buf * TB);
#pragma unroll
        for (int p = 0; p < PW; ++p) {
            const int n = (uwave + NWV * p) % TOT;
            const int plane = n / NI, sub = n % NI;
            const int row = sub * RPI + rlo;
            const int cg = cgp ^ SwTile<D>::sw(row);
            const bf16_t *src = sp + ((size_t)plane * a.Cpad + (size_t)t * 32) * D;
            async_copy16_at(src, (uint32_t)(row * D + cg * 8) * 2u, at + plane * PB + sub * 1024);
        }
    };
    // tile t + 1 has landed once at most the copies of the tiles after it are still in flight
    constexpr int DIST = kRouteStages - 1;           // tiles issued ahead of the one in use
    auto landed = [&](int t_next) {
        if (DIST > 1 && t_next + DIST - 1 < ntiles) wait_vmcnt<(DIST - 1) * PW>(); else wait_vmcnt<0>();
    };

    // scores of tile t for this lane: 16 chunks, ineligible ones set to -inf
    auto scores = [&](auto cur, int t) -> f32x16 {
        constexpr int CUR = decltype(cur)::value;
        lo.pin();
        f32x16 acc = zero16();
#pragma unroll
        for (int qa = 0; qa < NQ; ++qa)
#pragma unroll
            for (int kp = 0; kp < 3; ++kp) {
                if (qa + kp > 2) continue;
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    bf16x8 kf;
                    if (kp == 0) kf = lo.template frag<CUR * TB>(smem, s);
                    else if (kp == 1) kf = lo.template frag<CUR * TB + PB>(smem, s);
                    else kf = lo.template frag<CUR * TB + 2 * PB>(smem, s);
                    acc = mfma32(kf, qf[qa][s], acc);
                }
            }
        const int j0 = t * 32;
        const uint32_t tm = uniform_load_u32(a.textmask, t);
        // fast path: the whole tile is a candidate for every query of the wave
        const bool clean = tm == 0 && j0 + 32 <= lim_lo && (j0 + 32 <= wf_lo || j0 > wl_hi);
        if (!clean) {
            // One 32-bit word per lane, bit b = chunk j0 + b is a candidate of this lane's query:
            // below the causal limit, outside the own window [wf, wl], not text. The lane then
            // tests its 16 bits, (r >> 2) * 8 + half * 4 + (r & 3), at compile-time positions.
            auto below = [](int n) { return n >= 32 ? 0xffffffffu : (n <= 0 ? 0u : ((1u << n) - 1u)); };
            const uint32_t okm = below(limit - j0) & (below(wf - j0) | ~below(wl - j0 + 1)) & ~tm;
            const uint32_t mine = okm >> (half * 4);
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (!((mine >> ((r >> 2) * 8 + (r & 3))) & 1u)) acc[r] = -INFINITY;
        }
        return acc;
    };

    // ---------------- collect scores >= tau (the k-th best so far), keep an exact sorted list
    const int base = KMAX - topk;
    float tau = -3.0e38f;      // never let -inf (an ineligible chunk) pass the filter
    float val[KMAX];
    int idx[KMAX];
#pragma unroll
    for (int p = 0; p < KMAX; ++p) { val[p] = (p >= base) ? -INFINITY : INFINITY; idx[p] = -1; }
    int cnt = 0;
    auto drain = [&]() {
        int mx = cnt;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) mx = max(mx, __shfl_xor(mx, o, 64));
        for (int e = 0; e < mx; ++e) {
            const bool has = e < cnt;
            const u32x2 ent = queue[e][tid];
            const uint32_t bits = ent[0];
            const float x = has ? __builtin_bit_cast(float, bits) : -INFINITY;
            const int xi = has ? (int)ent[1] : -1;
            topk_insert<KMAX>(val, idx, x, xi);
        }
        cnt = 0;
        tau = fmaxf(tau, val[KMAX - 1]);     // once the list is full its tail bounds the k-th best
        // The other half-wave holds the other 16 chunks of every tile for the same query: the k-th best
        // of either half is a lower bound of the k-th best of both, so the larger of the two bounds
        // serves both halves and about half as many scores reach the queues.
        tau = fmaxf(tau, xhalf(tau));
        // With full lists (topk == KMAX) the two sorted lists give more: the k-th best of their union is
        // the largest of min(mine[p], other[k - 2 - p]) over p (take p + 1 scores from one list and the
        // rest from the other) and of the two tails above. Both halves see the same terms.
        if (base == 0) {
#pragma unroll
            for (int p = 0; p + 1 < KMAX; ++p) tau = fmaxf(tau, fminf(val[p], xhalf(val[KMAX - 2 - p])));
        }
    };
    auto scan = [&](auto cur, int t) {
        constexpr int CUR = decltype(cur)::value;
        const bool more = t + 1 < ntiles;
        if (t + DIST < ntiles) issue(t + DIST, (CUR + DIST) % kRouteStages);
        const f32x16 sc = scores(cur, t);
        // Branch-free append: every score is written at the lane's cursor and the cursor moves only if
        // the score passes, so a later score overwrites a rejected one. Entries past the capacity go
        // to a spill row; if any lane spilled, the appends of that half tile are taken back, the queues
        // drained (which also raises the bounds) and the half appended again: 8 scores always fit then.
        const int jb = t * 32 + half * 4;
        auto append = [&](auto first) {
            constexpr int R0 = decltype(first)::value;
#pragma unroll
            for (int r = R0; r < R0 + 8; ++r) {
                const int slot = min(cnt, kQCap);
                const float x = sc[r];      // (a bit cast straight from the vector element picks element 0)
                const u32x2 ent = {__builtin_bit_cast(uint32_t, x), (uint32_t)(jb + (r >> 2) * 8 + (r & 3))};
                queue[slot][tid] = ent;
                cnt += sc[r] >= tau ? 1 : 0;
            }
        };
        auto append_checked = [&](auto first) {
            const int before = cnt;
            append(first);
            if (__any(cnt > kQCap)) {
                cnt = before;
                drain();
                append(first);
            }
        };
        append_checked(IC<0>{});
        append_checked(IC<8>{});
        if (more) { landed(t + 1); __syncthreads(); }
        return more;
    };
#pragma unroll
    for (int u = 0; u < DIST; ++u)
        if (u < ntiles) issue(u, u);
    landed(0);
    __syncthreads();
    for (int t = 0;;) {
        if (!scan(IC<0>{}, t++)) break;
        if (!scan(IC<1 % kRouteStages>{}, t++)) break;
        if (kRouteStages > 2 && !scan(IC<2 % kRouteStages>{}, t++)) break;
    }
    drain();

    // ---------------- merge the two half-waves (score desc, index asc)
    {
        float ov[KMAX];
        int oi[KMAX];
#pragma unroll
        for (int p = 0; p < KMAX; ++p) { ov[p] = xhalf(val[p]); oi[p] = __shfl_xor(idx[p], 32, 64); }
#pragma unroll
        for (int p = 0; p < KMAX; ++p)
            if (p >= base) topk_insert_tie<KMAX>(val, idx, ov[p], oi[p]);
    }
    if (valid && half == 0) {
#pragma unroll
        for (int p = 0; p < KMAX; ++p)
            if (p >= base) out[p - base] = idx[p];
    }
}

template <int D, typename T, int KMAX>
__global__ __launch_bounds__(kRouteThreads, kRouteThreads == 256 ? 2 : 1) void route_kernel(RouteArgs a) {
    __shared__ __attribute__((aligned(1024))) char smem[kRouteStages * 3 * 32 * D * 2];
    __shared__ u32x2 queue[kQCap + 1][kRouteThreads];    // (score bits, chunk) pairs; row kQCap takes what does not fit
    route_body<D, T, KMAX>(a, smem, queue);
}

// ---------------------------------------------------------------------------------------------
// Pooling, scoring and top-k in ONE launch (the fusion the paper lists as future work, Sec. 5).
// Every query needs the mean key of every earlier chunk, so the scoring part of every workgroup
// depends on the whole pooling pass: the first kFusePoolWgs workgroups of the launch (they are
// dispatched first and never wait before they pool) share the chunks among themselves, count the
// chunks they have finished in a device word, and every workgroup waits for that count before it
// scores. The wait is bounded (kFuseSpinLimit sleeps of a few hundred cycles): if it runs out, a
// flag is raised, the workgroup scores whatever the planes hold, and every wave still exits.
// The words live in a static device array (zero when the module loads); the last workgroup of a
// launch clears them again, so launches must not overlap on one GPU.
constexpr int kFusePoolWgs = 256;
constexpr long long kFuseSpinLimit = 20000000;
static __device__ unsigned int g_fuse_sync[4];       // [0] chunks pooled, [1] workgroups finished, [2] a wait ran out

struct FuseArgs {
    const void *k;
    const int32_t *off;
    float *kbar;
    bf16_t *split;
    unsigned int units;      // Cpad * BH (chunk, head) pairs to pool
};

template <int D, typename T, int KMAX>
__global__ __launch_bounds__(kRouteThreads, 2) void route_fused_kernel(RouteArgs a, FuseArgs f) {
    static_assert(kRouteThreads == 256, "the pooling unit is written for 256 threads");
    __shared__ __attribute__((aligned(1024))) char smem[kRouteStages * 3 * 32 * D * 2];
    __shared__ u32x2 queue[kQCap + 1][kRouteThreads];
    static_assert(PoolShape<D, T>::kRedFloats * 4 <= kRouteStages * 3 * 32 * D * 2, "pooling scratch fits the tile buffers");
    const unsigned int wg = blockIdx.y * gridDim.x + blockIdx.x, nwg = gridDim.x * gridDim.y;
    const unsigned int npool = min(nwg, (unsigned int)kFusePoolWgs);
    if (wg < npool) {
        unsigned int done = 0;
        for (unsigned int u = wg; u < f.units; u += npool) {
            pool_unit<D, T>(static_cast<const T *>(f.k), f.off, a.N, a.C, a.Cpad, f.kbar, f.split, (int)(u % a.Cpad),
                            (int)(u / a.Cpad), reinterpret_cast<float *>(smem));
            ++done;
        }
        __syncthreads();                                       // every thread's stores are issued
        if (threadIdx.x == 0)
            __hip_atomic_fetch_add(&g_fuse_sync[0], done, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (threadIdx.x == 0) {
        long long spins = 0;
        while (__hip_atomic_load(&g_fuse_sync[0], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < f.units) {
            if (++spins > kFuseSpinLimit) { g_fuse_sync[2] = 1u; break; }
            __builtin_amdgcn_s_sleep(8);
        }
    }
    __syncthreads();
    route_body<D, T, KMAX>(a, smem, queue);
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int fin = __hip_atomic_fetch_add(&g_fuse_sync[1], 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        if (fin == nwg - 1) {                                  // the last one out: every workgroup is past its wait
            __hip_atomic_store(&g_fuse_sync[0], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&g_fuse_sync[1], 0u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

hipError_t launch_route_fused(const moc_meta *m, int BH, int d, const void *q, const void *k, float *kbar,
                              void *kb_split, int Cpad, int topk, int causal, int32_t *sel, hipStream_t st) {
    RouteArgs a{};
    a.q = q;
    a.split = static_cast<const bf16_t *>(kb_split);
    a.chunk_of = m->d_chunk_of; a.win = m->d_win; a.wfirst = m->d_wfirst; a.wlast = m->d_wlast;
    a.textmask = m->d_textmask;
    a.sel = sel;
    a.N = m->N; a.C = m->C; a.Cpad = Cpad; a.topk = topk; a.causal = causal != 0;
    a.stride = topk;
    FuseArgs f{k, m->d_off, kbar, static_cast<bf16_t *>(kb_split), (unsigned int)Cpad * (unsigned int)BH};
    dim3 grid((m->N + kRouteThreads / 2 - 1) / (kRouteThreads / 2), BH), block(kRouteThreads);
    MOC_PROF("route_fused", st);
#define MOC_FUSED(DD, KK) route_fused_kernel<DD, bf16_t, KK><<<grid, block, 0, st>>>(a, f)
#define MOC_FUSED_K(DD)                         \
    do {                                        \
        if (topk <= 8) MOC_FUSED(DD, 8);        \
        else if (topk <= 16) MOC_FUSED(DD, 16); \
        else MOC_FUSED(DD, 32);                 \
    } while (0)
    if (d == 128) MOC_FUSED_K(128); else MOC_FUSED_K(64);
#undef MOC_FUSED_K
#undef MOC_FUSED
    return hipGetLastError();
}

// blocking: has any wait of a fused launch run out since the module was loaded? (also clears the flag)
hipError_t fused_wait_flag(int *timed_out) {
    unsigned int w[4] = {};
    hipError_t e = hipMemcpyFromSymbol(w, HIP_SYMBOL(g_fuse_sync), sizeof(w), 0, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return e;
    *timed_out = w[2] != 0;
    if (w[2]) {
        const unsigned int zero = 0;
        e = hipMemcpyToSymbol(HIP_SYMBOL(g_fuse_sync), &zero, sizeof(zero), 2 * sizeof(unsigned int), hipMemcpyHostToDevice);
    }
    return e;
}

hipError_t launch_route(const moc_meta *m, int BH, int d, int dtype, const void *q, const void *kb_split, int Cpad,
                        int topk, int causal, int32_t *sel, int sel_stride, hipStream_t st) {
    RouteArgs a{};
    a.q = q;
    a.split = static_cast<const bf16_t *>(kb_split);
    a.chunk_of = m->d_chunk_of; a.win = m->d_win; a.wfirst = m->d_wfirst; a.wlast = m->d_wlast;
    a.textmask = m->d_textmask;
    a.sel = sel;
    a.N = m->N; a.C = m->C; a.Cpad = Cpad; a.topk = topk; a.causal = causal != 0;
    a.stride = sel_stride;
    dim3 grid((m->N + kRouteThreads / 2 - 1) / (kRouteThreads / 2), BH), block(kRouteThreads);
    MOC_PROF("route_topk", st);
#define MOC_ROUTE(DD, TT, KK) route_kernel<DD, TT, KK><<<grid, block, 0, st>>>(a)
#define MOC_ROUTE_K(DD, TT)                         \
    do {                                            \
        if (topk <= 8) MOC_ROUTE(DD, TT, 8);        \
        else if (topk <= 16) MOC_ROUTE(DD, TT, 16); \
        else MOC_ROUTE(DD, TT, 32);                 \
    } while (0)
    if (dtype == MOC_BF16) { if (d == 128) MOC_ROUTE_K(128, bf16_t); else MOC_ROUTE_K(64, bf16_t); }
    else { if (d == 128) MOC_ROUTE_K(128, float); else MOC_ROUTE_K(64, float); }
#undef MOC_ROUTE_K
#undef MOC_ROUTE
    return hipGetLastError();
}

}  // namespace moc
