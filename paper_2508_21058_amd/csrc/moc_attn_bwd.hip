// Stage (d) backward with the routed set fixed (Sec. 3.1: top-k is not
// differentiable; the gradient reaches q, k, v only through attention on the
// selected tokens).
//
//   delta_i = dO_i . o_i
//   P_it = exp(scale * q_i.k_t - lse_i),  dS_it = P_it (dO_i.v_t - delta_i)
//   dV_t = sum_i P_it dO_i,  dK_t = scale sum_i dS_it q_i,  dQ_i = scale sum_t dS_it k_t
//
// Two passes over the same dense items as the forward, neither uses atomics:
//   dQ pass    query-stationary (forced-link items and routed items, exactly the
//              forward's work list); each item writes its partial dQ to the slot
//              of its (query, link) pair, a merge kernel adds the slots.
//   dK/dV pass key-stationary: a workgroup owns <= 128 keys of one chunk and
//              walks every query that attends them - the chunk's window
//              (contiguous) and the chunk's inverse routing list (gathered) -
//              so dK and dV of video tokens are written once, final. Text keys
//              are attended by all N queries; their items split the queries
//              into segments, write fp32 partials, and a reduce kernel sums them.
#include "moc_attn_common.h"

namespace moc {

// ------------------------------------------------------------------ delta
template <int D, typename T>
__global__ __launch_bounds__(256) void delta_kernel(const T *__restrict__ o, const T *__restrict__ d_o, size_t rows,
                                                    const float *__restrict__ lse, float *__restrict__ delta,
                                                    float *__restrict__ lse2) {
    constexpr int TPQ = D / 8, QPW = 256 / TPQ;
    const size_t row = (size_t)blockIdx.x * QPW + threadIdx.x / TPQ;
    const int c8 = threadIdx.x % TPQ;
    float s = 0.f;
    if (row < rows) {
        float a[8], b[8];
        Io<T>::load8f(o + row * D + c8 * 8, a);
        Io<T>::load8f(d_o + row * D + c8 * 8, b);
#pragma unroll
        for (int e = 0; e < 8; ++e) s = fmaf(a[e], b[e], s);
    }
#pragma unroll
    for (int w = TPQ / 2; w >= 1; w >>= 1) s += __shfl_xor(s, w, 64);
    if (row < rows && c8 == 0) { delta[row] = s; lse2[row] = lse[row] * kLog2e; }
}

// ------------------------------------------------------------------ dQ pass
// 32 keys (rows ROW0 .. ROW0+31 of the staged 64-key tiles at byte offsets KOFF
// and VOFF) against this wave's 32 queries: S^T and dP^T from row reads of K
// and V, dS^T, then dQ^T[feature][query] += K^T dS^T with K read transposed
// from the same tile.
template <int D, int KOFF, int VOFF, int ROW0>
__device__ __forceinline__ void dq_half_tile(const char *smem, LaneOffs<D> &lo, const bf16x8 *qf, const bf16x8 *dof,
                                             f32x16 *dqacc, float c, float lse2, float dl, int valid, int lane) {
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int RB = ROW0 * D * 2;
    const int half = lane >> 5;
    lo.pin();
    f32x16 sacc, dpacc;
    {
        bf16x8 kf[KS], vf[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) kf[s] = lo.template frag<KOFF + RB>(smem, s);
#pragma unroll
        for (int s = 0; s < KS; ++s) vf[s] = lo.template frag<VOFF + RB>(smem, s);
        sacc = mfma32(kf[0], qf[0], zero16());
#pragma unroll
        for (int s = 1; s < KS; ++s) sacc = mfma32(kf[s], qf[s], sacc);
        dpacc = mfma32(vf[0], dof[0], zero16());
#pragma unroll
        for (int s = 1; s < KS; ++s) dpacc = mfma32(vf[s], dof[s], dpacc);
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int u = 0; u < 2 * KS - 4; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int key = ROW0 + (i >> 2) * 8 + half * 4 + (i & 3);
        float p = __builtin_amdgcn_exp2f(fmaf(sacc[i], c, -lse2));
        if (key >= valid) p = 0.f;
        sacc[i] = p * (dpacc[i] - dl);
    }
    {
        bf16x8 ktf[DB];
#pragma unroll
        for (int b = 0; b < DB; ++b) ktf[b] = lo.template tfrag<KOFF + RB>(smem, b);
        const bf16x8 dsf = acc_to_frag(sacc, 0);
#pragma unroll
        for (int b = 0; b < DB; ++b) dqacc[b] = mfma32(ktf[b], dsf, dqacc[b]);
    }
    {
        bf16x8 ktf[DB];
#pragma unroll
        for (int b = 0; b < DB; ++b) ktf[b] = lo.template tfrag<KOFF + RB + 16 * D * 2>(smem, b);
        const bf16x8 dsf = acc_to_frag(sacc, 1);
#pragma unroll
        for (int b = 0; b < DB; ++b) dqacc[b] = mfma32(ktf[b], dsf, dqacc[b]);
    }
}

template <int D, typename T, int MODE>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(FwdArgs a) {
    constexpr int BN = 64;
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int TB = BN * D * 2;
    __shared__ __attribute__((aligned(1024))) char smem[4 * TB];   // K0 K1 V0 V1

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int N = a.N;

    int logical;
    if (!xcd_remap((long long)a.items_per_head * a.BH, logical)) return;
    const int bh = logical / a.items_per_head;
    ItemDesc it;
    if (!decode_item<MODE>(a, bh, logical - bh * a.items_per_head, it)) return;

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
    const T *dobase = static_cast<const T *>(a.d_o) + (size_t)bh * N * D;

    bf16x8 qf[KS], dof[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        qf[s] = Io<T>::load8(qbase + (size_t)qi * D + s * 16 + half * 8);
        dof[s] = Io<T>::load8(dobase + (size_t)qi * D + s * 16 + half * 8);
    }
    const float c = a.scale_log2;
    const float lse2 = a.lse[(size_t)bh * N + qi] * kLog2e;
    const float dl = a.delta[(size_t)bh * N + qi];

    f32x16 dqacc[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b) dqacc[b] = zero16();
    LaneOffs<D> lo;
    lo.init(lane);

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
        if (wave_active) {
            dq_half_tile<D, CUR * TB, (2 + CUR) * TB, 0>(smem, lo, qf, dof, dqacc, c, lse2, dl, cur_valid, lane);
            if (cur_valid > 32)
                dq_half_tile<D, CUR * TB, (2 + CUR) * TB, 32>(smem, lo, qf, dof, dqacc, c, lse2, dl, cur_valid, lane);
        }
        if (more) { commit(CUR ^ 1); __syncthreads(); }
        return more;
    };
    issue(0);
    commit(0);
    __syncthreads();
    while (true) {
        if (!stage(IC<0>{})) break;
        if (!stage(IC<1>{})) break;
    }

    __syncthreads();      // tile buffers are free: reuse them for the output transpose
    const size_t prow = ((size_t)bh * N + qi) * a.slots + slot;
    store_rows_bf16<D>(smem, wave, lane, dqacc, a.scale, row_valid ? (int)prow : -1, a.po);
}

template <int D, typename T>
__global__ __launch_bounds__(256) void dq_merge_kernel(const bf16_t *__restrict__ part,
                                                       const int32_t *__restrict__ sel, int N, int C, int topk,
                                                       T *__restrict__ dq) {
    constexpr int TPQ = D / 8, QPW = 256 / TPQ;
    const int bh = blockIdx.y;
    const int i = blockIdx.x * QPW + threadIdx.x / TPQ;
    const int c8 = threadIdx.x % TPQ;
    if (i >= N) return;
    const int slots = topk + 1;
    const size_t row = (size_t)bh * N + i;
    const int32_t *sr = sel + row * topk;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    const bf16_t *pbase = part + row * slots * D + c8 * 8;
    for (int s0 = 0; s0 < slots; s0 += 4) {
        float w[4], f[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = s0 + u;
            bool ok = s == topk;
            if (s < topk) { const int j = sr[s]; ok = j >= 0 && j < C; }
            w[u] = ok ? 1.f : 0.f;
            Io<bf16_t>::load8f(pbase + (size_t)(ok ? s : topk) * D, f[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(w[u], f[u][e], acc[e]);
    }
    Io<T>::store8(dq + row * D + c8 * 8, acc);
}

// ------------------------------------------------------------------ dK/dV pass
struct KvArgs {
    const void *q, *k, *v, *d_o;
    const float *lse, *delta, *lse2;   // lse2 = lse * log2(e)
    const float *glse, *gdelta;        // lse2 / delta gathered in the order of the inverse lists
    void *dk, *dv;
    float *tpart_k, *tpart_v;
    const KvItem *items;
    const int32_t *list_off, *qlist;
    int N, C, topk, n_partials, n_items, BH;
    float scale, scale_log2;
};

// One block of 32 queries (rows ROW0.. of the staged 64-query Q and dO tiles at
// byte offsets QOFF / DOOFF) against this wave's 32 keys:
//   S = Q K^T, dP = dO V^T (row reads of Q, dO; K, V fragments in registers)
//   P, dS (lane owns a key column, registers run over query rows)
//   dV^T += dO^T P, dK^T += Q^T dS (Q, dO read transposed from the same tiles)
template <int D, int QOFF, int DOOFF, int ROW0>
__device__ __forceinline__ void dkdv_block(const char *smem, LaneOffs<D> &lo, const float *lse_s, const float *delta_s,
                                           const bf16x8 *kf, const bf16x8 *vf, f32x16 *dkacc, f32x16 *dvacc,
                                           float c, int nv, int lane) {
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int RB = ROW0 * D * 2;
    const int half = lane >> 5;
    lo.pin();
    f32x16 sacc, dpacc;
    {
        bf16x8 qa[KS], da[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) qa[s] = lo.template frag<QOFF + RB>(smem, s);
#pragma unroll
        for (int s = 0; s < KS; ++s) da[s] = lo.template frag<DOOFF + RB>(smem, s);
        sacc = mfma32(qa[0], kf[0], zero16());
#pragma unroll
        for (int s = 1; s < KS; ++s) sacc = mfma32(qa[s], kf[s], sacc);
        dpacc = mfma32(da[0], vf[0], zero16());
#pragma unroll
        for (int s = 1; s < KS; ++s) dpacc = mfma32(da[s], vf[s], dpacc);
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int u = 0; u < 2 * KS - 4; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int row = ROW0 + g * 8 + half * 4;
        const f32x4 l4 = *reinterpret_cast<const f32x4 *>(lse_s + row);
        const f32x4 d4 = *reinterpret_cast<const f32x4 *>(delta_s + row);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 4 * g + e;
            float p = __builtin_amdgcn_exp2f(fmaf(sacc[i], c, -l4[e]));
            if (row + e >= nv) p = 0.f;
            sacc[i] = p;
            dpacc[i] = p * (dpacc[i] - d4[e]);
        }
    }
#define MOC_KV_STEP(KSTEP)                                                                                   \
    {                                                                                                        \
        bf16x8 dot[DB], qt[DB];                                                                              \
        _Pragma("unroll") for (int b = 0; b < DB; ++b)                                                       \
            dot[b] = lo.template tfrag<DOOFF + RB + (KSTEP) * 16 * D * 2>(smem, b);                          \
        _Pragma("unroll") for (int b = 0; b < DB; ++b)                                                       \
            qt[b] = lo.template tfrag<QOFF + RB + (KSTEP) * 16 * D * 2>(smem, b);                            \
        const bf16x8 pf = acc_to_frag(sacc, KSTEP);                                                          \
        const bf16x8 dsf = acc_to_frag(dpacc, KSTEP);                                                        \
        _Pragma("unroll") for (int b = 0; b < DB; ++b) dvacc[b] = mfma32(dot[b], pf, dvacc[b]);              \
        _Pragma("unroll") for (int b = 0; b < DB; ++b) dkacc[b] = mfma32(qt[b], dsf, dkacc[b]);              \
    }
    MOC_KV_STEP(0) MOC_KV_STEP(1)
#undef MOC_KV_STEP
}

// Register-staged, double-buffered variant: used for fp32 storage (which must be
// converted on the way into LDS).
template <int D, typename T>
__global__ __launch_bounds__(256, 1) void attn_bwd_dkdv_kernel(KvArgs a) {
    constexpr int BQ = 64;
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int TB = BQ * D * 2;
    // LDS: Q buffers at 0 and TB, dO buffers at 2 TB and 3 TB
    __shared__ __attribute__((aligned(1024))) char smem[4 * TB];
    __shared__ __attribute__((aligned(16))) float lse_s[2][BQ], delta_s[2][BQ];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int N = a.N;
    int logical;
    if (!xcd_remap((long long)a.n_items * a.BH, logical)) return;
    const int bh = logical / a.n_items;
    const KvItem item = a.items[logical - bh * a.n_items];

    const T *qbase = static_cast<const T *>(a.q) + (size_t)bh * N * D;
    const T *kbase = static_cast<const T *>(a.k) + (size_t)bh * N * D;
    const T *vbase = static_cast<const T *>(a.v) + (size_t)bh * N * D;
    const T *dobase = static_cast<const T *>(a.d_o) + (size_t)bh * N * D;
    const float *lse = a.lse + (size_t)bh * N;
    const float *delta = a.delta + (size_t)bh * N;

    // this wave's 32 keys (B operands stay in registers for the whole item)
    // A tile of <= 32 keys (the ragged tail of a chunk) would leave three waves
    // idle: instead all four waves take the same keys, split the query blocks
    // among themselves and add their accumulators at the end.
    const bool split = item.key_len <= 32;
    const int kblk = split ? 0 : wave;
    const int nk = min(32, item.key_len - kblk * 32);
    const bool wave_active = nk > 0;
    const int key = wave_active ? item.key_start + kblk * 32 + min(l32, nk - 1) : item.key_start;
    bf16x8 kf[KS], vf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        kf[s] = Io<T>::load8(kbase + (size_t)key * D + s * 16 + half * 8);
        vf[s] = Io<T>::load8(vbase + (size_t)key * D + s * 16 + half * 8);
    }
    f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b) { dkacc[b] = zero16(); dvacc[b] = zero16(); }
    LaneOffs<D> lo;
    lo.init(lane);

    // query sources: a contiguous range, then (video chunks) the chunk's routed list
    const int nA = (item.q_len + BQ - 1) / BQ;
    int cntB = 0;
    const int32_t *entries = nullptr;
    if (item.chunk >= 0 && a.topk > 0) {
        const int32_t *loff = a.list_off + (size_t)bh * (a.C + 1);
        cntB = loff[item.chunk + 1] - loff[item.chunk];
        entries = a.qlist + (size_t)bh * N * a.topk + loff[item.chunk];
    }
    const int ntiles = nA + (cntB + BQ - 1) / BQ;
    if (ntiles == 0) return;

    TileLoader<D, T, BQ> qld(tid), dold(tid);
    float lreg = 0.f, dreg = 0.f;
    auto tile_valid = [&](int t) { return t < nA ? min(BQ, item.q_len - t * BQ) : min(BQ, cntB - (t - nA) * BQ); };
    auto issue = [&](int t, int buf) {
        const int nv = tile_valid(t);
        bf16_t *qdst = reinterpret_cast<bf16_t *>(smem + buf * TB);
        bf16_t *dodst = reinterpret_cast<bf16_t *>(smem + (2 + buf) * TB);
        if (t < nA) {
            const int q0 = item.q_start + t * BQ;
            qld.issue_rows(qbase + (size_t)q0 * D, nv, qdst);
            dold.issue_rows(dobase + (size_t)q0 * D, nv, dodst);
            if (tid < BQ) { const int i = q0 + min(tid, nv - 1); lreg = lse[i] * kLog2e; dreg = delta[i]; }
        } else {
            const int32_t *en = entries + (t - nA) * BQ;
            auto fn = [=](int r) { return en[min(r, nv - 1)] >> 5; };
            qld.issue(qbase, fn, qdst);
            dold.issue(dobase, fn, dodst);
            if (tid < BQ) { const int i = fn(tid); lreg = lse[i] * kLog2e; dreg = delta[i]; }
        }
    };
    auto commit = [&](int buf) {
        qld.commit(reinterpret_cast<bf16_t *>(smem + buf * TB));
        dold.commit(reinterpret_cast<bf16_t *>(smem + (2 + buf) * TB));
        if (tid < BQ) { lse_s[buf][tid] = lreg; delta_s[buf][tid] = dreg; }
    };
    const float c = a.scale_log2;
    int t = 0;
    auto stage = [&](auto cur) {
        constexpr int CUR = decltype(cur)::value;
        const int nv = tile_valid(t);
        const bool more = t + 1 < ntiles;
        if (more) issue(t + 1, CUR ^ 1);
        // split mode: wave w takes query block (w & 1) of the steps with parity (w >> 1)
        const bool do0 = wave_active && (!split || (CUR == (wave >> 1) && (wave & 1) == 0));
        const bool do1 = wave_active && nv > 32 && (!split || (CUR == (wave >> 1) && (wave & 1) == 1));
        if (do0)
            dkdv_block<D, CUR * TB, (2 + CUR) * TB, 0>(smem, lo, lse_s[CUR], delta_s[CUR], kf, vf, dkacc, dvacc, c, nv, lane);
        if (do1)
            dkdv_block<D, CUR * TB, (2 + CUR) * TB, 32>(smem, lo, lse_s[CUR], delta_s[CUR], kf, vf, dkacc, dvacc, c, nv, lane);
        if (more) { commit(CUR ^ 1); __syncthreads(); }
        ++t;
        return more;
    };
    issue(0, 0);
    commit(0);
    __syncthreads();
    while (true) {
        if (!stage(IC<0>{})) break;
        if (!stage(IC<1>{})) break;
    }

    if (split) {
        // the four waves hold partial sums for the same keys in the same register
        // layout: exchange them through LDS (16 KB per wave and tensor), wave 0 adds
        float *xch = reinterpret_cast<float *>(smem);
        static_assert(4 * DB * 16 * 64 * 4 <= 4 * TB, "exchange buffer must fit the tile buffers");
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            f32x16 *acc = pass == 0 ? dkacc : dvacc;
            __syncthreads();
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) xch[((wave * DB + b) * 16 + i) * 64 + lane] = acc[b][i];
            __syncthreads();
            if (wave == 0) {
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float v = 0.f;
#pragma unroll
                        for (int w = 0; w < 4; ++w) v += xch[((w * DB + b) * 16 + i) * 64 + lane];
                        acc[b][i] = v;
                    }
            }
        }
        if (wave != 0) return;
    }
    if (!wave_active || l32 >= nk) return;
    const float sc = a.scale;
    if (item.partial < 0) {
        T *dk = static_cast<T *>(a.dk) + ((size_t)bh * N + key) * D;
        T *dv = static_cast<T *>(a.dv) + ((size_t)bh * N + key) * D;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int x = b * 32 + g * 8 + half * 4;
                Io<T>::store4(dk + x, dkacc[b][4 * g] * sc, dkacc[b][4 * g + 1] * sc, dkacc[b][4 * g + 2] * sc,
                              dkacc[b][4 * g + 3] * sc);
                Io<T>::store4(dv + x, dvacc[b][4 * g], dvacc[b][4 * g + 1], dvacc[b][4 * g + 2], dvacc[b][4 * g + 3]);
            }
    } else {
        const size_t prow = ((size_t)bh * a.n_partials + item.partial) * kKeyTile + kblk * 32 + l32;
        float *pk = a.tpart_k + prow * D, *pv = a.tpart_v + prow * D;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int x = b * 32 + g * 8 + half * 4;
                Io<float>::store4(pk + x, dkacc[b][4 * g] * sc, dkacc[b][4 * g + 1] * sc, dkacc[b][4 * g + 2] * sc,
                                  dkacc[b][4 * g + 3] * sc);
                Io<float>::store4(pv + x, dvacc[b][4 * g], dvacc[b][4 * g + 1], dvacc[b][4 * g + 2], dvacc[b][4 * g + 3]);
            }
    }
}

// lse2 and delta of the queries of every inverse list, in list order, so the
// key-stationary pass reads them as contiguous vectors
__global__ __launch_bounds__(256) void gather_stats_kernel(const int32_t *__restrict__ qlist,
                                                           const int32_t *__restrict__ list_off, int N, int NK, int C,
                                                           const float *__restrict__ lse2,
                                                           const float *__restrict__ delta, float *__restrict__ glse,
                                                           float *__restrict__ gdelta) {
    const int bh = blockIdx.y;
    const int pos = blockIdx.x * 256 + threadIdx.x;
    if (pos >= list_off[(size_t)bh * (C + 1) + C]) return;
    const int i = qlist[(size_t)bh * NK + pos] >> 5;
    glse[(size_t)bh * NK + pos] = lse2[(size_t)bh * N + i];
    gdelta[(size_t)bh * NK + pos] = delta[(size_t)bh * N + i];
}

// s_waitcnt that only bounds the number of outstanding vector-memory operations
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// bf16 storage: the query stream of an item is mostly a gather of rows scattered
// over the sequence, so one tile of look-ahead does not cover the memory
// latency. This variant keeps NS - 1 tiles of asynchronous global->LDS loads in
// flight: before tile t is consumed the wave waits only until its own loads of
// tile t have landed (vmcnt bound, no drain), then one barrier publishes the tile
// and frees the buffer of tile t-1 for the loads of tile t+NS-1. Everything the
// loop loads, per-query lse and delta included, goes through the async path, so
// no register-destination load forces an early wait.
template <int D>
__global__ __launch_bounds__(256, 1) void attn_bwd_dkdv_pipe_kernel(KvArgs a) {
    typedef bf16_t T;
    constexpr int BQ = 64, NS = 4;
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int TB = BQ * D * 2;                 // bytes of one Q (or dO) tile
    constexpr int SB = 2 * TB;                     // bytes of one stage: Q tile, dO tile
    constexpr int LPT = 2 * (BQ * D * 2 / 1024 / 4) + 2;   // async loads per wave and tile
    __shared__ __attribute__((aligned(1024))) char smem[NS * SB];
    __shared__ __attribute__((aligned(256))) float lse_s[NS][BQ], delta_s[NS][BQ];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int N = a.N;
    int logical;
    if (!xcd_remap((long long)a.n_items * a.BH, logical)) return;
    const int bh = logical / a.n_items;
    const KvItem item = a.items[logical - bh * a.n_items];

    const T *qbase = static_cast<const T *>(a.q) + (size_t)bh * N * D;
    const T *kbase = static_cast<const T *>(a.k) + (size_t)bh * N * D;
    const T *vbase = static_cast<const T *>(a.v) + (size_t)bh * N * D;
    const T *dobase = static_cast<const T *>(a.d_o) + (size_t)bh * N * D;
    const float *lse2 = a.lse2 + (size_t)bh * N;
    const float *delta = a.delta + (size_t)bh * N;

    const bool split = item.key_len <= 32;         // see the register-staged variant
    const int kblk = split ? 0 : wave;
    const int nk = min(32, item.key_len - kblk * 32);
    const bool wave_active = nk > 0;
    const int key = wave_active ? item.key_start + kblk * 32 + min(l32, nk - 1) : item.key_start;
    bf16x8 kf[KS], vf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        kf[s] = Io<T>::load8(kbase + (size_t)key * D + s * 16 + half * 8);
        vf[s] = Io<T>::load8(vbase + (size_t)key * D + s * 16 + half * 8);
    }
    f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
    for (int b = 0; b < DB; ++b) { dkacc[b] = zero16(); dvacc[b] = zero16(); }
    LaneOffs<D> lo;
    lo.init(lane);

    const int nA = (item.q_len + BQ - 1) / BQ;
    // all of these are plain values (never reassigned), so nothing of the loop state lives in memory
    const bool routed = item.chunk >= 0 && a.topk > 0;
    const int32_t *loff = a.list_off + (size_t)bh * (a.C + 1);
    const int lbeg = routed ? loff[item.chunk] : 0;
    const int cntB = routed ? loff[item.chunk + 1] - lbeg : 0;
    const size_t lpos = (size_t)bh * N * a.topk + lbeg;
    const int32_t *const entries = a.qlist + lpos;
    const float *const glse = a.glse + lpos;
    const float *const gdelta = a.gdelta + lpos;
    const int ntiles = nA + (cntB + BQ - 1) / BQ;
    if (ntiles == 0) return;

    TileLoader<D, T, BQ> ld(tid);
    auto tile_valid = [&](int t) { return t < nA ? min(BQ, item.q_len - t * BQ) : min(BQ, cntB - (t - nA) * BQ); };
    // every wave issues exactly LPT async loads per tile
    auto issue = [&](int t, int st) {
        const int nv = tile_valid(t);
        bf16_t *qdst = reinterpret_cast<bf16_t *>(smem + st * SB);
        bf16_t *dodst = reinterpret_cast<bf16_t *>(smem + st * SB + TB);
        const int r16 = min(wave * 16 + (lane & 15), nv - 1);    // this wave's 16 rows of the lse / delta vectors
        const bool contig = t < nA;
        const int q0 = item.q_start + t * BQ, g0 = (t - nA) * BQ;
        if (contig) {
            ld.issue_rows(qbase + (size_t)q0 * D, nv, qdst);
            ld.issue_rows(dobase + (size_t)q0 * D, nv, dodst);
        } else {
            const auto lr = ld.list_rows(entries + g0, nv);
            ld.issue_list(qbase, lr, qdst);
            ld.issue_list(dobase, lr, dodst);
        }
        const float *lp = (contig ? lse2 + q0 : glse + g0) + r16;
        const float *dp = (contig ? delta + q0 : gdelta + g0) + r16;
        if (lane < 16) {
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)lp,
                                             (__attribute__((address_space(3))) void *)(&lse_s[st][wave * 16]), 4, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)dp,
                                             (__attribute__((address_space(3))) void *)(&delta_s[st][wave * 16]), 4, 0, 0);
        }
    };

    const float c = a.scale_log2;
    wait_vmcnt<0>();     // K / V fragments are in registers before the asynchronous stream starts
#pragma unroll
    for (int p = 0; p < NS - 1; ++p)
        if (p < ntiles) issue(p, p);
    for (int t = 0; t < ntiles; ++t) {
        const int st = t % NS;
        // tile t complete for this wave: at most the loads of the younger tiles may be outstanding
        const int younger = min(NS - 2, ntiles - 1 - t);
        if (younger >= 2) wait_vmcnt<2 * LPT>();
        else if (younger == 1) wait_vmcnt<LPT>();
        else wait_vmcnt<0>();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (t + NS - 1 < ntiles) issue(t + NS - 1, (t + NS - 1) % NS);
        const int nv = tile_valid(t);
        LaneOffs<D> lc = lo;
#pragma unroll
        for (int s = 0; s < KS; ++s) lc.row[s] += st * SB;
#pragma unroll
        for (int u = 0; u < 2 * DB; ++u) lc.tr[u] += st * SB;
        const bool mine = !split || (t & 1) == (wave >> 1);
        const bool do0 = wave_active && mine && (!split || (wave & 1) == 0);
        const bool do1 = wave_active && mine && nv > 32 && (!split || (wave & 1) == 1);
        if (do0) dkdv_block<D, 0, TB, 0>(smem, lc, lse_s[st], delta_s[st], kf, vf, dkacc, dvacc, c, nv, lane);
        if (do1) dkdv_block<D, 0, TB, 32>(smem, lc, lse_s[st], delta_s[st], kf, vf, dkacc, dvacc, c, nv, lane);
    }

    if (split) {
        float *xch = reinterpret_cast<float *>(smem);
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            f32x16 *acc = pass == 0 ? dkacc : dvacc;
            __syncthreads();
#pragma unroll
            for (int b = 0; b < DB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) xch[((wave * DB + b) * 16 + i) * 64 + lane] = acc[b][i];
            __syncthreads();
            if (wave == 0) {
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float v = 0.f;
#pragma unroll
                        for (int w = 0; w < 4; ++w) v += xch[((w * DB + b) * 16 + i) * 64 + lane];
                        acc[b][i] = v;
                    }
            }
        }
        if (wave != 0) return;
    }
    if (!wave_active || l32 >= nk) return;
    const float sc = a.scale;
    if (item.partial < 0) {
        T *dk = static_cast<T *>(a.dk) + ((size_t)bh * N + key) * D;
        T *dv = static_cast<T *>(a.dv) + ((size_t)bh * N + key) * D;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int x = b * 32 + g * 8 + half * 4;
                Io<T>::store4(dk + x, dkacc[b][4 * g] * sc, dkacc[b][4 * g + 1] * sc, dkacc[b][4 * g + 2] * sc,
                              dkacc[b][4 * g + 3] * sc);
                Io<T>::store4(dv + x, dvacc[b][4 * g], dvacc[b][4 * g + 1], dvacc[b][4 * g + 2], dvacc[b][4 * g + 3]);
            }
    } else {
        const size_t prow = ((size_t)bh * a.n_partials + item.partial) * kKeyTile + kblk * 32 + l32;
        float *pk = a.tpart_k + prow * D, *pv = a.tpart_v + prow * D;
#pragma unroll
        for (int b = 0; b < DB; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int x = b * 32 + g * 8 + half * 4;
                Io<float>::store4(pk + x, dkacc[b][4 * g] * sc, dkacc[b][4 * g + 1] * sc, dkacc[b][4 * g + 2] * sc,
                                  dkacc[b][4 * g + 3] * sc);
                Io<float>::store4(pv + x, dvacc[b][4 * g], dvacc[b][4 * g + 1], dvacc[b][4 * g + 2], dvacc[b][4 * g + 3]);
            }
    }
}

// sums the per-segment partials of a text key tile in a fixed order
template <int D, typename T>
__global__ __launch_bounds__(256) void text_reduce_kernel(const float *__restrict__ tpart_k,
                                                          const float *__restrict__ tpart_v,
                                                          const TextTile *__restrict__ tiles, int n_partials, int N,
                                                          T *__restrict__ dk, T *__restrict__ dv) {
    const TextTile tt = tiles[blockIdx.x];
    const int bh = blockIdx.y;
    constexpr int V4 = D / 4;                       // float4 groups per row
    for (int u = threadIdx.x; u < tt.key_len * V4; u += 256) {
        const int kr = u / V4, x = (u % V4) * 4;
        f32x4 sk = {0.f, 0.f, 0.f, 0.f}, sv = {0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < tt.n_partials; ++p) {
            const size_t prow = ((size_t)bh * n_partials + tt.first_partial + p) * kKeyTile + kr;
            sk += *reinterpret_cast<const f32x4 *>(tpart_k + prow * D + x);
            sv += *reinterpret_cast<const f32x4 *>(tpart_v + prow * D + x);
        }
        const size_t row = (size_t)bh * N + tt.key_start + kr;
        Io<T>::store4(dk + row * D + x, sk[0], sk[1], sk[2], sk[3]);
        Io<T>::store4(dv + row * D + x, sv[0], sv[1], sv[2], sv[3]);
    }
}

template <int D, typename T>
static hipError_t bwd_dispatch(const moc_meta *m, int BH, FwdArgs &a, KvArgs &kv, const void *o, const int32_t *sel,
                               void *dq, hipStream_t st) {
    constexpr int QPW = 256 / (D / 8);
    const size_t rows = (size_t)BH * m->N;
    { MOC_PROF("delta", st);
    delta_kernel<D, T><<<dim3((unsigned)((rows + QPW - 1) / QPW)), dim3(256), 0, st>>>(
        static_cast<const T *>(o), static_cast<const T *>(a.d_o), rows, a.lse, const_cast<float *>(a.delta),
        const_cast<float *>(kv.lse2)); }
    { MOC_PROF("attn_bwd_dkdv", st);
    if constexpr (sizeof(T) == 2) {
        if (a.topk > 0) {
            const int NK = m->N * a.topk;
            gather_stats_kernel<<<dim3((NK + 255) / 256, BH), dim3(256), 0, st>>>(
                kv.qlist, kv.list_off, m->N, NK, m->C, kv.lse2, kv.delta, const_cast<float *>(kv.glse),
                const_cast<float *>(kv.gdelta));
        }
        attn_bwd_dkdv_pipe_kernel<D><<<dim3(xcd_grid((long long)m->n_kvitems * BH)), dim3(256), 0, st>>>(kv);
    } else
        attn_bwd_dkdv_kernel<D, T><<<dim3(xcd_grid((long long)m->n_kvitems * BH)), dim3(256), 0, st>>>(kv); }
    if (m->n_text_tiles > 0) { MOC_PROF("text_reduce", st);
        text_reduce_kernel<D, T><<<dim3(m->n_text_tiles, BH), dim3(256), 0, st>>>(
            kv.tpart_k, kv.tpart_v, m->d_text_tiles, m->n_partials, m->N, static_cast<T *>(kv.dk),
            static_cast<T *>(kv.dv)); }
    a.BH = BH;
    if (a.topk > 0) {
        a.items_per_head = (m->N * a.topk + kBM - 1) / kBM + m->C;
        MOC_PROF("attn_bwd_dq_routed", st);
        attn_bwd_dq_kernel<D, T, MODE_ROUTED><<<dim3(xcd_grid((long long)a.items_per_head * BH)), dim3(256), 0, st>>>(a);
    }
    { MOC_PROF("attn_bwd_dq_forced", st);
    a.items_per_head = m->n_atiles;
    attn_bwd_dq_kernel<D, T, MODE_ANCHOR><<<dim3(xcd_grid((long long)a.items_per_head * BH)), dim3(256), 0, st>>>(a); }
    MOC_PROF("dq_merge", st);
    dq_merge_kernel<D, T><<<dim3((m->N + QPW - 1) / QPW, BH), dim3(256), 0, st>>>(a.po, sel, m->N, m->C, a.topk,
                                                                                static_cast<T *>(dq));
    return hipGetLastError();
}

hipError_t launch_attn_bwd(const moc_meta *m, int BH, int d, int dtype, const void *q, const void *k, const void *v,
                           const void *o, const float *lse, const void *d_o, const int32_t *sel, int topk, float scale,
                           void *dq, void *dk, void *dv, char *ws, const AttnWs &L, hipStream_t st) {
    FwdArgs a{};
    a.q = q; a.k = k; a.v = v; a.d_o = d_o;
    a.po = reinterpret_cast<bf16_t *>(ws + L.po);
    a.plse = nullptr;
    a.N = m->N; a.C = m->C; a.topk = topk; a.slots = topk + 1;
    a.scale = scale; a.scale_log2 = scale * kLog2e;
    a.atiles = m->d_atiles; a.arange_off = m->d_arange_off; a.aranges = m->d_aranges;
    a.off = m->d_off;
    a.list_off = reinterpret_cast<const int32_t *>(ws + L.list_off);
    a.tile_off = reinterpret_cast<const int32_t *>(ws + L.tile_off);
    a.qlist = reinterpret_cast<const int32_t *>(ws + L.qlist);
    a.lse = lse;
    a.delta = reinterpret_cast<const float *>(ws + L.delta);
    KvArgs kv{};
    kv.q = q; kv.k = k; kv.v = v; kv.d_o = d_o;
    kv.lse = lse; kv.delta = a.delta;
    kv.lse2 = reinterpret_cast<const float *>(ws + L.lse2);
    kv.glse = reinterpret_cast<const float *>(ws + L.glse);
    kv.gdelta = reinterpret_cast<const float *>(ws + L.gdelta);
    kv.dk = dk; kv.dv = dv;
    kv.tpart_k = reinterpret_cast<float *>(ws + L.tpart_k);
    kv.tpart_v = reinterpret_cast<float *>(ws + L.tpart_v);
    kv.items = m->d_kvitems;
    kv.list_off = a.list_off; kv.qlist = a.qlist;
    kv.N = m->N; kv.C = m->C; kv.topk = topk; kv.n_partials = m->n_partials; kv.n_items = m->n_kvitems; kv.BH = BH;
    kv.scale = scale; kv.scale_log2 = a.scale_log2;
    if (dtype == MOC_BF16) return d == 128 ? bwd_dispatch<128, bf16_t>(m, BH, a, kv, o, sel, dq, st)
                                           : bwd_dispatch<64, bf16_t>(m, BH, a, kv, o, sel, dq, st);
    return d == 128 ? bwd_dispatch<128, float>(m, BH, a, kv, o, sel, dq, st)
                    : bwd_dispatch<64, float>(m, BH, a, kv, o, sel, dq, st);
}

}  // namespace moc
