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
template <int D, int KOFF, int VOFF>
__device__ __forceinline__ void fwd_tile(const char *smem, LaneOffs<D> &lo, const bf16x8 *qf, f32x16 *oacc,
                                         float &m_run, float &l_run, float c, int valid, int lane) {
    constexpr int KS = D / 16, DB = D / 32;
    const int half = lane >> 5;
    lo.pin();
    f32x16 sacc[2];
    {
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
    const float m_new = fmaxf(m_run, xhalf_max(mx));
    if (__any(m_new > m_run)) {
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
    const size_t prow = ((size_t)bh * N + qi) * a.slots + slot;
    store_rows_bf16<D>(smem, wave, lane, oacc, inv, row_valid ? (int)prow : -1, a.po);
    if (row_valid && half == 0) a.plse[prow] = m_run * a.scale + __logf(l_tot);
}

// o = sum_s exp(lse_s - lse) o_s over the forced-link slot and the used routed slots
template <int D, typename T>
__global__ __launch_bounds__(256) void fwd_merge_kernel(const bf16_t *__restrict__ po,
                                                        const float *__restrict__ plse,
                                                        const int32_t *__restrict__ sel, int N, int C, int topk,
                                                        T *__restrict__ o, float *__restrict__ lse) {
    constexpr int TPQ = D / 8, QPW = 256 / TPQ;
    const int bh = blockIdx.y;
    const int i = blockIdx.x * QPW + threadIdx.x / TPQ;
    const int c8 = threadIdx.x % TPQ;
    if (i >= N) return;
    const int slots = topk + 1;
    const size_t row = (size_t)bh * N + i;
    const float *pl = plse + row * slots;
    const int32_t *sr = sel + row * topk;
    float mx = pl[topk];
    for (int s = 0; s < topk; ++s) {
        const int j = sr[s];
        if (j >= 0 && j < C) mx = fmaxf(mx, pl[s]);
    }
    float z = __expf(pl[topk] - mx);
    for (int s = 0; s < topk; ++s) {
        const int j = sr[s];
        if (j >= 0 && j < C) z += __expf(pl[s] - mx);
    }
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
            bool ok = s == topk;
            if (s < topk) { const int j = sr[s]; ok = j >= 0 && j < C; }
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
static hipError_t fwd_dispatch(const moc_meta *m, int BH, FwdArgs &a, const int32_t *sel, void *o, float *lse,
                               hipStream_t st) {
    a.BH = BH;
    if (a.topk > 0) {
        a.items_per_head = (m->N * a.topk + kBM - 1) / kBM + m->C;   // upper bound; surplus items exit at once
        MOC_PROF("attn_fwd_routed", st);
        attn_fwd_kernel<D, T, MODE_ROUTED><<<dim3(xcd_grid((long long)a.items_per_head * BH)), dim3(256), 0, st>>>(a);
    }
    { MOC_PROF("attn_fwd_forced", st);
    a.items_per_head = m->n_atiles;
    attn_fwd_kernel<D, T, MODE_ANCHOR><<<dim3(xcd_grid((long long)a.items_per_head * BH)), dim3(256), 0, st>>>(a); }
    MOC_PROF("fwd_merge", st);
    constexpr int QPW = 256 / (D / 8);
    fwd_merge_kernel<D, T><<<dim3((m->N + QPW - 1) / QPW, BH), dim3(256), 0, st>>>(
        a.po, a.plse, sel, m->N, m->C, a.topk, static_cast<T *>(o), lse);
    return hipGetLastError();
}

hipError_t launch_attn_fwd(const moc_meta *m, int BH, int d, int dtype, const void *q, const void *k, const void *v,
                           const int32_t *sel, int topk, float scale, void *o, float *lse, char *ws, const AttnWs &L,
                           hipStream_t st) {
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
    if (dtype == MOC_BF16) return d == 128 ? fwd_dispatch<128, bf16_t>(m, BH, a, sel, o, lse, st)
                                           : fwd_dispatch<64, bf16_t>(m, BH, a, sel, o, lse, st);
    return d == 128 ? fwd_dispatch<128, float>(m, BH, a, sel, o, lse, st)
                    : fwd_dispatch<64, float>(m, BH, a, sel, o, lse, st);
}

}  // namespace moc
