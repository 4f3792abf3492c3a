// Stage (d) forward: routed softmax attention (Eq. 2) on bf16 matrix cores.
//
// Work is split into two kinds of dense items, both "a tile of <= 128 query
// rows against contiguous key ranges":
//   forced-link items  queries of one window tile x (all text spans + the window)
//   routed items       queries gathered through a chunk's inverse list x that chunk
// Every item produces a normalised partial output and its log-sum-exp in the
// slot of the (query, link) pair; a merge kernel combines the <= topk+1 partials
// of a query (the usual split-softmax identity), so no item ever waits on another.
//
// Per workgroup: 4 waves x 32 query rows. K and V tiles (64 keys) are staged
// row-major in swizzled LDS tiles; V is read back through the transposing LDS
// load. S^T = K Q^T and O^T = V^T P^T are computed so that each lane owns one
// query column: softmax statistics are per-lane scalars and the S^T accumulator
// feeds the second product without any shuffle.
#include "moc_attn_common.h"

namespace moc {

// One tile (BN = 64 keys) of the online-softmax recurrence for this wave's 32
// queries; the K tile sits at byte offset KOFF of the workgroup's LDS, the V
// tile at VOFF. Rows >= valid of a ragged tile hold copies of the last valid key
// and are masked to -inf. LDS reads are pinned a few fragments ahead of the
// matrix instructions that consume them.
// LEAN stages the K fragments of one 32-key block at a time (half the registers).
template <int D, int KOFF, int VOFF, bool LEAN = false>
__device__ __forceinline__ void fwd_tile(const char *smem, LaneOffs<D> &lo, const bf16x8 *qf, f32x16 *oacc,
                                         float &m_run, float &l_run, float c, int valid, int lane) {
    constexpr int KS = D / 16, DB = D / 32;
    const int half = lane >> 5;
    lo.pin();
    f32x16 sacc[2];
    if (LEAN) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            bf16x8 kf[KS];
#pragma unroll
            for (int s = 0; s < KS; ++s)
                kf[s] = kb == 0 ? lo.template frag<KOFF>(smem, s) : lo.template frag<KOFF + 32 * D * 2>(smem, s);
            sacc[kb] = mfma32(kf[0], qf[0], zero16());
#pragma unroll
            for (int s = 1; s < KS; ++s) sacc[kb] = mfma32(kf[s], qf[s], sacc[kb]);
            __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
            for (int u = 0; u < KS - 4; ++u) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
        }
    } else {
        bf16x8 kf[2 * KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) kf[s] = lo.template frag<KOFF>(smem, s);
#pragma unroll
        for (int s = 0; s < KS; ++s) kf[KS + s] = lo.template frag<KOFF + 32 * D * 2>(smem, s);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            sacc[kb] = mfma32(kf[kb * KS], qf[0], zero16());
#pragma unroll
            for (int s = 1; s < KS; ++s) sacc[kb] = mfma32(kf[kb * KS + s], qf[s], sacc[kb]);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int u = 0; u < 2 * KS - 4; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
    if (valid < 64) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int key = kb * 32 + (i >> 2) * 8 + half * 4 + (i & 3);
                if (key >= valid) sacc[kb][i] = -INFINITY;
            }
    }
    // online softmax over this lane's 32 keys, then across the two halves
    float mx = sacc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kb][i]);
    // Lazy rescaling: the running maximum is only a reference point (any value cancels in the
    // final normalisation), so it is moved, and the accumulators rescaled, only when some query's
    // maximum has grown by more than 2^8; until then the probabilities may exceed 1 by that factor.
    const float m_new = fmaxf(m_run, xhalf_max(mx));
    if (__any((m_new - m_run) * c > 8.f)) {
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
        l_run *= alpha;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[b][i] *= alpha;
        m_run = m_new;
    }
    const float mc = m_run * c;
    float ls = 0.f;
    // O^T[feature][query] += V^T P^T, 16 keys at a time; V is read transposed
    // straight from its row-major tile
#define MOC_PV_STEP(KSTEP)                                                                         \
    {                                                                                              \
        bf16x8 vf[DB];                                                                             \
        _Pragma("unroll") for (int b = 0; b < DB; ++b)                                             \
            vf[b] = lo.template tfrag<VOFF + (KSTEP) * 16 * D * 2>(smem, b);                       \
        f32x16 &sa = sacc[(KSTEP) >> 1];                                                           \
        _Pragma("unroll") for (int i = 8 * ((KSTEP) & 1); i < 8 * ((KSTEP) & 1) + 8; ++i) {        \
            const float p = __builtin_amdgcn_exp2f(fmaf(sa[i], c, -mc));                           \
            sa[i] = p;                                                                             \
            ls += p;                                                                               \
        }                                                                                          \
        const bf16x8 pf = acc_to_frag(sa, (KSTEP) & 1);                                            \
        _Pragma("unroll") for (int b = 0; b < DB; ++b) oacc[b] = mfma32(vf[b], pf, oacc[b]);       \
    }
    MOC_PV_STEP(0) MOC_PV_STEP(1) MOC_PV_STEP(2) MOC_PV_STEP(3)
#undef MOC_PV_STEP
    l_run += ls;
    // 2*DB transposing reads per 16-key step; keep one step of reads in flight
    __builtin_amdgcn_sched_group_barrier(0x100, 4 * DB, 0);
#pragma unroll
    for (int u = 0; u < 2 * DB; ++u) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
    }
    __builtin_amdgcn_sched_group_barrier(0x008, 2 * DB, 0);
}

// Epilogue of the forced-link items when the routed items of the same pass have
// already run: instead of storing its partial and leaving the combination to a
// merge kernel, the wave combines right here (the split-softmax identity
// o = sum_s exp(lse_s - lse) o_s over the forced-link slot and the used routed
// slots). One lane per query turns the <= topk+1 partial log-sum-exps into
// weights; the forced-link part, already weighted, is transposed through the
// wave's LDS patch as in store_rows_bf16; then every lane owns 8 features of a
// row, adds the weighted routed partials (16-byte loads, a batch in flight) and
// stores the final row. The forced-link partial never goes to memory.
// `smem` must be free (barrier before); needs 4 * (32 * (D + 4) + 64) * 2 + 4 * 32 * 34 * 4 bytes.
template <int D>
__device__ __forceinline__ void merge_store_rows(char *smem, int wave, int lane, const f32x16 *acc, float m_run,
                                                 float l_tot, bool row_valid, int qi, size_t bhN, const FwdArgs &a) {
    constexpr int DB = D / 32, RS = D + 4, WS = 34;    // WS: floats per row of the weight table (32 weights, lse)
    const int half = lane >> 5, l32 = lane & 31;
    const int topk = a.topk, slots = topk + 1;
    bf16_t *patch = reinterpret_cast<bf16_t *>(smem) + wave * (32 * RS + 64);
    int32_t *rowidx = reinterpret_cast<int32_t *>(patch + 32 * RS);
    float *wts = reinterpret_cast<float *>(smem + 4 * (32 * RS + 64) * 2) + wave * 32 * WS;
    float wf = 0.f;
    if (half == 0) {
        const size_t row = bhN + qi;
        const float lf = m_run * a.scale + __logf(l_tot);
        const float *pl = a.plse + row * slots;
        const uint32_t used = topk > 0 ? a.vmask[row] : 0u;     // the routed slots that count
        float mx = lf;
        for (int s = 0; s < topk; ++s)
            if ((used >> s) & 1u) mx = fmaxf(mx, pl[s]);
        float z = __expf(lf - mx);
        for (int s = 0; s < topk; ++s)
            if ((used >> s) & 1u) z += __expf(pl[s] - mx);
        const float tot = mx + __logf(z);
        for (int s = 0; s < topk; ++s) wts[l32 * WS + s] = ((used >> s) & 1u) ? __expf(pl[s] - tot) : 0.f;
        wts[l32 * WS + 32] = tot;
        wf = __expf(lf - tot);
        rowidx[l32] = row_valid ? qi : -1;
    }
    wf = xhalf_sum(wf);                                // the other half-wave holds the same query
    const float scale = wf / l_tot;
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g)
            Io<bf16_t>::store4(patch + l32 * RS + b * 32 + g * 8 + half * 4, acc[b][4 * g] * scale,
                               acc[b][4 * g + 1] * scale, acc[b][4 * g + 2] * scale, acc[b][4 * g + 3] * scale);
    __builtin_amdgcn_wave_barrier();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    constexpr int LPR = D / 8, RPI = 64 / LPR;          // lanes per row, rows per instruction
    const int cg = lane % LPR, r0 = lane / LPR;
    const bf16_t *qsafe = static_cast<const bf16_t *>(a.q);      // finite values for the loads of unused slots
    for (int it = 0; it < 32 / RPI; ++it) {
        const int r = it * RPI + r0;
        const int dr = rowidx[r];
        if (dr < 0) continue;
        const size_t row = bhN + dr;
        float o8[8];
        {
            const u32x2 lo2 = *reinterpret_cast<const u32x2 *>(patch + r * RS + cg * 8);
            const u32x2 hi2 = *reinterpret_cast<const u32x2 *>(patch + r * RS + cg * 8 + 4);
            o8[0] = bf16_lo(lo2[0]); o8[1] = bf16_hi(lo2[0]); o8[2] = bf16_lo(lo2[1]); o8[3] = bf16_hi(lo2[1]);
            o8[4] = bf16_lo(hi2[0]); o8[5] = bf16_hi(hi2[0]); o8[6] = bf16_lo(hi2[1]); o8[7] = bf16_hi(hi2[1]);
        }
        const bf16_t *pbase = a.po + row * slots * D + cg * 8;
        for (int s0 = 0; s0 < topk; s0 += 8) {
            float w[8], f[8][8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int s = s0 + u;
                w[u] = s < topk ? wts[r * WS + s] : 0.f;
                const bf16_t *src = w[u] != 0.f ? pbase + (size_t)s * D : qsafe + row * D + cg * 8;
                Io<bf16_t>::load8f(src, f[u]);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) o8[e] = fmaf(w[u], f[u][e], o8[e]);
        }
        Io<bf16_t>::store8(static_cast<bf16_t *>(a.o_out) + row * D + cg * 8, o8);
        if (cg == 0) a.lse_out[row] = wts[r * WS + 32];
    }
}

template <int D, typename T, int MODE>
__global__ __launch_bounds__(256, 2) void attn_fwd_kernel(FwdArgs a) {
    constexpr int BN = 64;
    constexpr int KS = D / 16;   // feature steps of the QK product
    constexpr int DB = D / 32;   // 32-feature blocks of the output
    constexpr int TB = BN * D * 2;   // bytes per tile
    // LDS: K buffers at 0 and TB, V buffers at 2 TB and 3 TB
    __shared__ __attribute__((aligned(1024))) char smem[4 * TB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int N = a.N;

    int logical;
    if (!xcd_remap((long long)a.items_per_head * a.BH, logical)) return;
    const int bh = logical / a.items_per_head;
    ItemDesc it;
    if (!decode_item<MODE>(a, bh, logical - bh * a.items_per_head, it)) return;

    // ---- this lane's query row
    const int r = wave * 32 + l32;
    const bool row_valid = r < it.q_count;
    const bool wave_active = wave * 32 < it.q_count;
    const int rc = row_valid ? r : it.q_count - 1;
    int qi, slot;
    if (MODE == MODE_ANCHOR) { qi = it.q_start + rc; slot = a.topk; }
    else { const int e = it.entries[rc]; qi = e >> 5; slot = e & 31; }

    const T *qbase = static_cast<const T *>(a.q) + (size_t)bh * N * D;
    const T *kbase = static_cast<const T *>(a.k) + (size_t)bh * N * D;
    const T *vbase = static_cast<const T *>(a.v) + (size_t)bh * N * D;

    bf16x8 qf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = Io<T>::load8(qbase + (size_t)qi * D + s * 16 + half * 8);

    f32x16 oacc[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b) oacc[b] = zero16();
    float m_run = -INFINITY, l_run = 0.f;
    const float c = a.scale_log2;
    LaneOffs<D> lo;
    lo.init(lane);

    // Double-buffered pipeline, one barrier per tile: while tile t is consumed
    // from one LDS buffer, tile t+1 streams from global memory into the other.
    // The loop is unrolled by two so every access has a constant buffer offset.
    TileLoader<D, T, BN> kld(tid), vld(tid);
    TileIter<BN> ti(it);
    int valid = ti.valid();
    bool more;
    auto issue = [&](int buf) {
        const size_t st = (size_t)ti.start() * D;
        kld.issue_rows(kbase + st, ti.valid(), reinterpret_cast<bf16_t *>(smem + buf * TB));
        vld.issue_rows(vbase + st, ti.valid(), reinterpret_cast<bf16_t *>(smem + (2 + buf) * TB));
    };
    auto commit = [&](int buf) {
        kld.commit(reinterpret_cast<bf16_t *>(smem + buf * TB));
        vld.commit(reinterpret_cast<bf16_t *>(smem + (2 + buf) * TB));
    };
    auto stage = [&](auto cur) {
        constexpr int CUR = decltype(cur)::value;
        const int cur_valid = valid;
        more = ti.next();
        if (more) { valid = ti.valid(); issue(CUR ^ 1); }
        if (wave_active)
            fwd_tile<D, CUR * TB, (2 + CUR) * TB>(smem, lo, qf, oacc, m_run, l_run, c, cur_valid, lane);
        if (more) { commit(CUR ^ 1); __syncthreads(); }
        return more;       // false: that was the last tile
    };
    issue(0);
    commit(0);
    __syncthreads();
    while (true) {
        if (!stage(IC<0>{})) break;
        if (!stage(IC<1>{})) break;
    }

    __syncthreads();      // every wave is done with the tile buffers: reuse them for the output transpose
    const float l_tot = xhalf_sum(l_run);
    const float inv = 1.f / l_tot;
    if constexpr (MODE == MODE_ANCHOR && sizeof(T) == 2) {
        if (a.o_out) {      // the routed items are done: combine here, no forced-link partial, no merge kernel
            merge_store_rows<D>(smem, wave, lane, oacc, m_run, l_tot, row_valid, qi, (size_t)bh * N, a);
            return;
        }
    }
    const size_t prow = ((size_t)bh * N + qi) * a.slots + slot;
    store_rows_bf16<D>(smem, wave, lane, oacc, inv, row_valid ? (int)prow : -1, a.po);
    if (row_valid && half == 0) a.plse[prow] = m_run * a.scale + __logf(l_tot);
}

// Routed items, chunk-stationary (bf16 storage, chunks of at most kChunkRows
// keys): the K and V rows of a chunk stay in LDS while the chunk's inverse list
// streams past. A workgroup takes kGroupTiles consecutive routed items (128
// list entries each, usually of one or two chunks); per chunk it loads K / V
// once, then its eight waves work through the 32-query blocks on their own:
// query fragments straight from global memory into registers, the
// online-softmax recurrence over the resident key tiles, the normalised partial
// output and its log-sum-exp into the slot of the (query, link) pair. Inside a
// chunk there is no barrier and no shared staging, so one wave's memory and
// LDS latencies are covered by the other wave of its SIMD.

template <int D>
__global__ __launch_bounds__(512, 1) void attn_fwd_chunk_kernel(FwdArgs a) {
    typedef bf16_t T;
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int RB = D * 2;                     // bytes per row
    constexpr int KBYTES = kChunkRows * RB;       // K region; the last 64-key tile may run 32 rows into the V region
    constexpr int VBYTES = (kChunkRows + 32) * RB;   // (those keys are masked), so the V region is a full tile longer
    constexpr int RPI = 1024 / RB;                // rows per copy instruction
    __shared__ __attribute__((aligned(1024))) char smem[KBYTES + VBYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int N = a.N, C = a.C;
    const int groups_per_head = (a.items_per_head + kGroupTiles - 1) / kGroupTiles;
    int logical;
    if (!xcd_remap((long long)groups_per_head * a.BH, logical)) return;
    const int bh = logical / groups_per_head;
    const int32_t *toff = a.tile_off + (size_t)bh * (C + 1);
    const int32_t *loff = a.list_off + (size_t)bh * (C + 1);
    int t0 = (logical - bh * groups_per_head) * kGroupTiles;
    const int t1 = min(t0 + kGroupTiles, toff[C]);
    if (t0 >= t1) return;
    int j;
    {
        int lo = 0, hi = C;   // largest j with toff[j] <= t0
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (toff[mid] <= t0) lo = mid; else hi = mid;
        }
        j = lo;
    }
    const char *qbase = static_cast<const char *>(a.q) + (size_t)bh * N * RB;
    const char *kbase = static_cast<const char *>(a.k) + (size_t)bh * N * RB;
    const char *vbase = static_cast<const char *>(a.v) + (size_t)bh * N * RB;
    const float c = a.scale_log2;
    LaneOffs<D> lo;
    lo.init(lane);
    const int rlo = lane / (D / 8), cgp = lane % (D / 8);

    while (t0 < t1) {
        while (toff[j + 1] <= t0) ++j;            // chunk of tile t0 (chunks without routed queries have no tiles)
        const int te = min(t1, toff[j + 1]);      // this chunk's tiles in the group: [t0, te)
        const int key0 = a.off[j], len = a.off[j + 1] - key0;
        const int ntile = (len + 63) >> 6;
        // ---- K / V of the chunk -> LDS (rows past the end repeat the last row: finite, and masked as keys)
        {
            const int nk = (min(ntile * 64, kChunkRows) + RPI - 1) / RPI, nv = ntile * 64 / RPI;
            for (int i = wave; i < nk + nv; i += 8) {
                const bool isk = i < nk;
                const int ii = isk ? i : i - nk;
                const int row = ii * RPI + rlo;
                const uint32_t off = (uint32_t)(min(row, len - 1) * RB + ((cgp ^ SwTile<D>::sw(row)) << 4));
                async_copy16((isk ? kbase : vbase) + (size_t)key0 * RB, off, smem + (isk ? 0 : KBYTES) + ii * 1024);
            }
            wait_vmcnt<0>();
            __syncthreads();
        }
        // ---- the chunk's list entries covered by tiles [t0, te)
        const int cnt = loff[j + 1] - loff[j];
        const int q_first = (t0 - toff[j]) * kBM;
        const int nq = min(cnt, (te - toff[j]) * kBM) - q_first;
        const int32_t *entries = a.qlist + (size_t)bh * N * a.topk + loff[j] + q_first;
        // software pipeline over the wave's blocks: the list entry of the next block is loaded
        // before the first key tile of the current one, its query fragments after it
        auto entry_of = [&](int blk) { return entries[min(blk * 32 + l32, nq - 1)]; };
        auto load_q = [&](int e, bf16x8 *qf) {
#pragma unroll
            for (int s = 0; s < KS; ++s)
                qf[s] = Io<T>::load8(reinterpret_cast<const T *>(qbase + (size_t)(e >> 5) * RB) + s * 16 + half * 8);
        };
        int blk = wave;
        int e_cur = 0;
        bf16x8 qf[KS];
        if (blk * 32 < nq) { e_cur = entry_of(blk); load_q(e_cur, qf); }
        while (blk * 32 < nq) {
            const bool more = (blk + 8) * 32 < nq;
            int e_nxt = e_cur;
            if (more) e_nxt = entry_of(blk + 8);
            f32x16 oacc[DB];
#pragma unroll
            for (int b = 0; b < DB; ++b) oacc[b] = zero16();
            float m_run = -INFINITY, l_run = 0.f;
            fwd_tile<D, 0, KBYTES, true>(smem, lo, qf, oacc, m_run, l_run, c, min(64, len), lane);
            bf16x8 qn[KS];
            if (more) load_q(e_nxt, qn);
            for (int t = 1; t < ntile; ++t)
                fwd_tile<D, 0, KBYTES, true>(smem + t * 64 * RB, lo, qf, oacc, m_run, l_run, c, min(64, len - t * 64), lane);
            const float l_tot = xhalf_sum(l_run);
            const float inv = 1.f / l_tot;
            const size_t prow = ((size_t)bh * N + (e_cur >> 5)) * a.slots + (e_cur & 31);
            // The two half-waves hold adjacent 4-feature pieces of the same query: exchange them so
            // that the lower half stores features [16 u, 16 u + 8) and the upper half [16 u + 8, 16 u + 16)
            // of a 32-feature block as one 16-byte word each.
            if (blk * 32 + l32 < nq) {
                T *dst = a.po + prow * D + half * 8;
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int g = 2 * u;
                        const uint32_t x0 = pack_bf16(oacc[b][4 * g] * inv, oacc[b][4 * g + 1] * inv);
                        const uint32_t x1 = pack_bf16(oacc[b][4 * g + 2] * inv, oacc[b][4 * g + 3] * inv);
                        const uint32_t y0 = pack_bf16(oacc[b][4 * g + 4] * inv, oacc[b][4 * g + 5] * inv);
                        const uint32_t y1 = pack_bf16(oacc[b][4 * g + 6] * inv, oacc[b][4 * g + 7] * inv);
                        const auto r0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
                        const auto r1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
                        const u32x4 w = {r0[0], r1[0], r0[1], r1[1]};
                        *reinterpret_cast<u32x4 *>(dst + b * 32 + u * 16) = w;
                    }
                if (half == 0) a.plse[prow] = m_run * a.scale + __logf(l_tot);
            }
            blk += 8;
            e_cur = e_nxt;
#pragma unroll
            for (int s = 0; s < KS; ++s) qf[s] = qn[s];
        }
        t0 = te;
        if (t0 < t1) __syncthreads();             // every wave is done with this chunk's K / V
    }
}

// o = sum_s exp(lse_s - lse) o_s over the forced-link slot and the used routed slots
template <int D, typename T>
__global__ __launch_bounds__(256) void fwd_merge_kernel(const bf16_t *__restrict__ po,
                                                        const float *__restrict__ plse,
                                                        const uint32_t *__restrict__ vmask, int N, int topk,
                                                        T *__restrict__ o, float *__restrict__ lse) {
    constexpr int TPQ = D / 8, QPW = 256 / TPQ;
    const int bh = blockIdx.y;
    const int i = blockIdx.x * QPW + threadIdx.x / TPQ;
    const int c8 = threadIdx.x % TPQ;
    if (i >= N) return;
    const int slots = topk + 1;
    const size_t row = (size_t)bh * N + i;
    const float *pl = plse + row * slots;
    const uint32_t used = topk > 0 ? vmask[row] : 0u;       // the routed slots that count
    float mx = pl[topk];
    for (int s = 0; s < topk; ++s)
        if ((used >> s) & 1u) mx = fmaxf(mx, pl[s]);
    float z = __expf(pl[topk] - mx);
    for (int s = 0; s < topk; ++s)
        if ((used >> s) & 1u) z += __expf(pl[s] - mx);
    const float tot = mx + __logf(z);
    // unused slots read the forced-link slot again with weight 0, so all loads
    // are unconditional and several are in flight
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    const bf16_t *pbase = po + row * slots * D + c8 * 8;
    for (int s0 = 0; s0 < slots; s0 += 4) {
        float w[4], f[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = s0 + u;
            const bool ok = s == topk || (s < topk && ((used >> s) & 1u));
            const int src = ok ? s : topk;
            w[u] = ok ? __expf(pl[src] - tot) : 0.f;
            Io<bf16_t>::load8f(pbase + (size_t)src * D, f[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(w[u], f[u][e], acc[e]);
    }
    Io<T>::store8(o + row * D + c8 * 8, acc);
    if (c8 == 0) lse[row] = tot;
}

template <int D, typename T>
static hipError_t fwd_dispatch(const moc_meta *m, int BH, FwdArgs &a, void *o, float *lse, hipStream_t st) {
    a.BH = BH;
    if (a.topk > 0) {
        a.items_per_head = (m->N * a.topk + kBM - 1) / kBM + m->C;   // upper bound; surplus items exit at once
        MOC_PROF("attn_fwd_routed", st);
        if constexpr (sizeof(T) == 2) {
            if (m->max_chunk_len <= kChunkRows) {
                const int groups = (a.items_per_head + kGroupTiles - 1) / kGroupTiles;
                attn_fwd_chunk_kernel<D><<<dim3(xcd_grid((long long)groups * BH)), dim3(512), 0, st>>>(a);
            } else {
                attn_fwd_kernel<D, T, MODE_ROUTED><<<dim3(xcd_grid((long long)a.items_per_head * BH)), dim3(256), 0, st>>>(a);
            }
        } else {
            attn_fwd_kernel<D, T, MODE_ROUTED><<<dim3(xcd_grid((long long)a.items_per_head * BH)), dim3(256), 0, st>>>(a);
        }
    }
    // bf16 storage: the forced-link items run after the routed ones and merge in their epilogue
    // (needs the LDS of the tile buffers to hold the transposition patches and the weight table)
    const bool fuse = sizeof(T) == 2 && 4 * (32 * (D + 4) + 64) * 2 + 4 * 32 * 34 * 4 <= 4 * 64 * D * 2;
    { MOC_PROF("attn_fwd_forced", st);
    a.items_per_head = m->n_atiles;
    a.o_out = fuse ? o : nullptr; a.lse_out = lse;
    attn_fwd_kernel<D, T, MODE_ANCHOR><<<dim3(xcd_grid((long long)a.items_per_head * BH)), dim3(256), 0, st>>>(a); }
    if (fuse) return hipGetLastError();
    MOC_PROF("fwd_merge", st);
    constexpr int QPW = 256 / (D / 8);
    fwd_merge_kernel<D, T><<<dim3((m->N + QPW - 1) / QPW, BH), dim3(256), 0, st>>>(
        a.po, a.plse, a.vmask, m->N, a.topk, static_cast<T *>(o), lse);
    return hipGetLastError();
}

hipError_t launch_attn_fwd(const moc_meta *m, int BH, int d, int dtype, const void *q, const void *k, const void *v,
                           int topk, float scale, void *o, float *lse, char *ws, const AttnWs &L, hipStream_t st) {
    FwdArgs a{};
    a.q = q; a.k = k; a.v = v;
    a.po = reinterpret_cast<bf16_t *>(ws + L.po);
    a.plse = reinterpret_cast<float *>(ws + L.plse);
    a.N = m->N; a.C = m->C; a.topk = topk; a.slots = topk + 1;
    a.scale = scale; a.scale_log2 = scale * kLog2e;
    a.atiles = m->d_atiles; a.arange_off = m->d_arange_off; a.aranges = m->d_aranges;
    a.off = m->d_off;
    a.list_off = reinterpret_cast<const int32_t *>(ws + L.list_off);
    a.tile_off = reinterpret_cast<const int32_t *>(ws + L.tile_off);
    a.qlist = reinterpret_cast<const int32_t *>(ws + L.qlist);
    a.vmask = reinterpret_cast<const uint32_t *>(ws + L.vmask);
    if (dtype == MOC_BF16) return d == 128 ? fwd_dispatch<128, bf16_t>(m, BH, a, o, lse, st)
                                           : fwd_dispatch<64, bf16_t>(m, BH, a, o, lse, st);
    return d == 128 ? fwd_dispatch<128, float>(m, BH, a, o, lse, st)
                    : fwd_dispatch<64, float>(m, BH, a, o, lse, st);
}

}  // namespace moc
