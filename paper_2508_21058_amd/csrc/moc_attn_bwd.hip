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
                                                    float *__restrict__ stats2) {
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
    // stats2 holds per query the pair (lse * log2(e), delta) the key-stationary pass works with
    if (row < rows && c8 == 0) {
        delta[row] = s;
        stats2[2 * row] = lse[row] * kLog2e;
        stats2[2 * row + 1] = s;
    }
    // one pair past the end holds lse2 = +inf: the padding rows of ragged query tiles
    if (blockIdx.x == 0 && threadIdx.x == 0) { stats2[2 * rows] = INFINITY; stats2[2 * rows + 1] = 0.f; }
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
    if (valid >= ROW0 + 32) {      // all 32 keys exist (wave-uniform): no masking in the common case
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const float p = __builtin_amdgcn_exp2f(fmaf(sacc[i], c, -lse2));
            sacc[i] = p * (dpacc[i] - dl);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int key = ROW0 + (i >> 2) * 8 + half * 4 + (i & 3);
            float p = __builtin_amdgcn_exp2f(fmaf(sacc[i], c, -lse2));
            if (key >= valid) p = 0.f;
            sacc[i] = p * (dpacc[i] - dl);
        }
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

// Epilogue of the forced-link dQ items when the routed items of the same pass
// have already run: dQ of a query is the sum of its forced-link part and of the
// partials in its used routed slots, so the wave adds them right here instead
// of storing its own partial for a merge kernel. The forced-link part is
// transposed through the wave's LDS patch (as in store_rows_bf16); then every
// lane owns 8 features of a row, adds the routed partials (16-byte loads, a
// batch in flight) and stores the final row.
// `smem` must be free (barrier before); needs 4 * (32 * (D + 4) + 128) * 2 bytes.
template <int D>
__device__ __forceinline__ void sum_store_rows(char *smem, int wave, int lane, const f32x16 *acc, float scale,
                                               bool row_valid, int qi, size_t bhN, const FwdArgs &a) {
    constexpr int DB = D / 32, RS = D + 4;
    const int half = lane >> 5, l32 = lane & 31;
    const int topk = a.topk, slots = topk + 1;
    bf16_t *patch = reinterpret_cast<bf16_t *>(smem) + wave * (32 * RS + 128);
    int32_t *rowidx = reinterpret_cast<int32_t *>(patch + 32 * RS);
    uint32_t *used = reinterpret_cast<uint32_t *>(rowidx + 32);
    if (half == 0) {
        used[l32] = topk > 0 ? a.vmask[bhN + qi] : 0u;     // the routed slots that count
        rowidx[l32] = row_valid ? qi : -1;
    }
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
        const uint32_t mask = used[r];
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
                const bool ok = s < topk && ((mask >> s) & 1u);
                w[u] = ok ? 1.f : 0.f;
                Io<bf16_t>::load8f(ok ? pbase + (size_t)s * D : qsafe + row * D + cg * 8, f[u]);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) o8[e] = fmaf(w[u], f[u][e], o8[e]);
        }
        Io<bf16_t>::store8(static_cast<bf16_t *>(a.o_out) + row * D + cg * 8, o8);
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
    if constexpr (MODE == MODE_ANCHOR && sizeof(T) == 2) {
        if (a.o_out) {      // the routed items are done: sum here, no forced-link partial, no merge kernel
            sum_store_rows<D>(smem, wave, lane, dqacc, a.scale, row_valid, qi, (size_t)bh * N, a);
            return;
        }
    }
    const size_t prow = ((size_t)bh * N + qi) * a.slots + slot;
    store_rows_bf16<D>(smem, wave, lane, dqacc, a.scale, row_valid ? (int)prow : -1, a.po);
}

// Routed dQ items, chunk-stationary (bf16 storage, chunks of at most kChunkRows keys): as in the
// forward, K and V of one chunk stay in LDS (K is read both as a row operand for S and transposed
// for dQ from the same swizzled tile) and the eight waves stream the chunk's inverse list through
// them independently, 32 list entries at a time: no barrier and no staging inside a chunk, K / V
// fetched once per group of query tiles instead of once per query tile. Each (query, link) pair
// writes its partial dQ to its slot; the forced-link items add the slots afterwards.
template <int D>
__global__ __launch_bounds__(512, 1) void attn_bwd_dq_chunk_kernel(FwdArgs a) {
    typedef bf16_t T;
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int RB = D * 2;                     // bytes per row
    constexpr int KBYTES = kChunkRows * RB;
    constexpr int VBYTES = (kChunkRows + 32) * RB;
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
    const char *dobase = static_cast<const char *>(a.d_o) + (size_t)bh * N * RB;
    const char *kbase = static_cast<const char *>(a.k) + (size_t)bh * N * RB;
    const char *vbase = static_cast<const char *>(a.v) + (size_t)bh * N * RB;
    const float c = a.scale_log2;
    LaneOffs<D> lo;
    lo.init(lane);
    const int rlo = lane / (D / 8), cgp = lane % (D / 8);

    while (t0 < t1) {
        while (toff[j + 1] <= t0) ++j;            // chunk of tile t0
        const int te = min(t1, toff[j + 1]);      // this chunk's tiles in the group: [t0, te)
        const int key0 = a.off[j], len = a.off[j + 1] - key0;
        const int nhalf = (len + 31) >> 5;        // 32-key half tiles
        // ---- K / V of the chunk -> LDS (rows past the end repeat the last row: finite, masked as keys)
        {
            const int nk = (min(nhalf * 32, kChunkRows) + RPI - 1) / RPI;
            for (int i = wave; i < 2 * nk; i += 8) {
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
        const size_t lbase = (size_t)bh * N * a.topk + loff[j] + q_first;
        const int32_t *entries = a.qlist + lbase;
        const float2 *stats = reinterpret_cast<const float2 *>(a.gstats2) + lbase;
        // software pipeline over the wave's blocks: the list entry and the statistics of the next
        // block are fetched before the key tiles of the current one; its Q and dO fragments are
        // fetched into the registers of the current ones once the last key tile is done, so their
        // latency runs under the stores of the current block's partial dQ
        auto load_qdo = [&](int ent, bf16x8 *qf, bf16x8 *dof) {
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                qf[s] = Io<T>::load8(reinterpret_cast<const T *>(qbase + (size_t)(ent >> 5) * RB) + s * 16 + half * 8);
                dof[s] = Io<T>::load8(reinterpret_cast<const T *>(dobase + (size_t)(ent >> 5) * RB) + s * 16 + half * 8);
            }
        };
        bf16x8 qf[KS], dof[KS];
        int e = 0;
        float2 st2 = make_float2(0.f, 0.f);
        if (wave * 32 < nq) {
            const int pos = min(wave * 32 + l32, nq - 1);
            e = entries[pos];
            st2 = stats[pos];                                 // (lse * log2 e, delta)
            load_qdo(e, qf, dof);
        }
        for (int blk = wave; blk * 32 < nq; blk += 8) {
            const bool more = (blk + 8) * 32 < nq;
            int e_next = e;
            float2 st_next = st2;
            if (more) {
                const int pn = min((blk + 8) * 32 + l32, nq - 1);
                e_next = entries[pn];
                st_next = stats[pn];
            }
            f32x16 dqacc[DB];
#pragma unroll
            for (int b = 0; b < DB; ++b) dqacc[b] = zero16();
            for (int h = 0; h < nhalf; h += 2) {
                const char *tile = smem + h * 32 * RB;
                const int valid = len - h * 32;
                dq_half_tile<D, 0, KBYTES, 0>(tile, lo, qf, dof, dqacc, c, st2.x, st2.y, valid, lane);
                if (valid > 32) dq_half_tile<D, 0, KBYTES, 32>(tile, lo, qf, dof, dqacc, c, st2.x, st2.y, valid, lane);
            }
            const int e_cur = e;
            if (more) load_qdo(e_next, qf, dof);
            e = e_next;
            st2 = st_next;
            // 16-byte stores: the two half-waves hold adjacent 4-feature pieces of the same query and
            // exchange them (lower half: features [16 u, 16 u + 8), upper half: [16 u + 8, 16 u + 16))
            if (blk * 32 + l32 < nq) {
                const size_t prow = ((size_t)bh * N + (e_cur >> 5)) * a.slots + (e_cur & 31);
                T *dst = a.po + prow * D + half * 8;
                const float sc = a.scale;
#pragma unroll
                for (int b = 0; b < DB; ++b)
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int g = 2 * u;
                        const uint32_t x0 = pack_bf16(dqacc[b][4 * g] * sc, dqacc[b][4 * g + 1] * sc);
                        const uint32_t x1 = pack_bf16(dqacc[b][4 * g + 2] * sc, dqacc[b][4 * g + 3] * sc);
                        const uint32_t y0 = pack_bf16(dqacc[b][4 * g + 4] * sc, dqacc[b][4 * g + 5] * sc);
                        const uint32_t y1 = pack_bf16(dqacc[b][4 * g + 6] * sc, dqacc[b][4 * g + 7] * sc);
                        const auto r0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
                        const auto r1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
                        const u32x4 w = {r0[0], r1[0], r0[1], r1[1]};
                        *reinterpret_cast<u32x4 *>(dst + b * 32 + u * 16) = w;
                    }
            }
        }
        t0 = te;
        if (t0 < t1) __syncthreads();             // every wave is done with this chunk's K / V
    }
}

template <int D, typename T>
__global__ __launch_bounds__(256) void dq_merge_kernel(const bf16_t *__restrict__ part,
                                                       const uint32_t *__restrict__ vmask, int N, int topk,
                                                       T *__restrict__ dq) {
    constexpr int TPQ = D / 8, QPW = 256 / TPQ;
    const int bh = blockIdx.y;
    const int i = blockIdx.x * QPW + threadIdx.x / TPQ;
    const int c8 = threadIdx.x % TPQ;
    if (i >= N) return;
    const int slots = topk + 1;
    const size_t row = (size_t)bh * N + i;
    const uint32_t used = topk > 0 ? vmask[row] : 0u;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    const bf16_t *pbase = part + row * slots * D + c8 * 8;
    for (int s0 = 0; s0 < slots; s0 += 4) {
        float w[4], f[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int s = s0 + u;
            const bool ok = s == topk || (s < topk && ((used >> s) & 1u));
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
    const float *lse, *delta;
    const float *stats2;               // per query (lse * log2(e), delta); one extra pair (+inf, 0) at the end
    const float *gstats2;              // the same pairs gathered in the order of the inverse lists
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
        // the dO fragments reuse the registers of the Q fragments as those are consumed
        bf16x8 fr[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) fr[s] = lo.template frag<QOFF + RB>(smem, s);
        sacc = zero16();
        dpacc = zero16();
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            sacc = mfma32(fr[s], kf[s], sacc);
            fr[s] = lo.template frag<DOOFF + RB>(smem, s);
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) dpacc = mfma32(fr[s], vf[s], dpacc);
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int u = 0; u < KS - 4; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int u = 0; u < KS; ++u) {
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

// (lse2, delta) of the queries of every inverse list, in list order, so the
// key-stationary pass reads them as contiguous vectors
__global__ __launch_bounds__(256) void gather_stats_kernel(const int32_t *__restrict__ qlist,
                                                           const int32_t *__restrict__ list_off, int N, int NK, int C,
                                                           const float2 *__restrict__ stats2,
                                                           float2 *__restrict__ gstats2) {
    const int bh = blockIdx.y;
    const int pos = blockIdx.x * 256 + threadIdx.x;
    if (pos >= list_off[(size_t)bh * (C + 1) + C]) return;
    const int i = qlist[(size_t)bh * NK + pos] >> 5;
    gstats2[(size_t)bh * NK + pos] = stats2[(size_t)bh * N + i];
}

// The two halves of the 8-wave key-stationary kernel, for one tile of 32 queries
// and one block of 32 keys.
//   score (waves 0-3): S = Q K^T and delta - dP = delta - dO V^T on the matrix
//     cores (the V fragments are held negated and the accumulator starts at
//     delta, read from LDS straight into the accumulator registers), then
//     P = exp2(c S - lse2) and -dS = P (delta - dP); both leave through LDS as
//     bf16 operand fragments (the register image acc_to_frag produces, one
//     16-byte word per lane and 16-query step). Rows past the end of a ragged
//     tile carry lse2 = +inf, so their P and dS come out as exact zeros.
//   grad (waves 4-7): dV^T += dO^T P and -dK^T += Q^T (-dS) with the transposed
//     tile reads; a fragment word is read by the lane number that wrote it.
//     The sign of dK is put right in the final scaling.
// score is split into its matrix half and its vector half so that the caller
// can run the matrix half of the next tile under the vector half of this one.
// Per-stage statistics in LDS: for each group of 8 queries, 8 x lse2 then 8 x delta.
template <int D, int QOFF, int DOOFF>
__device__ __forceinline__ void score_mfma(const char *smem, const LaneOffs<D> &lo, const float *stats, const bf16x8 *kf,
                                           const bf16x8 *nvf, f32x16 &sacc, f32x16 &dpacc, int lane) {
    constexpr int KS = D / 16;
    const int half = lane >> 5;
    bf16x8 qa[KS], da[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) qa[s] = lo.template frag<QOFF>(smem, s);
#pragma unroll
    for (int s = 0; s < KS; ++s) da[s] = lo.template frag<DOOFF>(smem, s);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const f32x4 d4 = *reinterpret_cast<const f32x4 *>(stats + g * 16 + 8 + half * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) dpacc[4 * g + e] = d4[e];
    }
    sacc = mfma32(qa[0], kf[0], zero16());
    dpacc = mfma32(da[0], nvf[0], dpacc);
#pragma unroll
    for (int s = 1; s < KS; ++s) {
        sacc = mfma32(qa[s], kf[s], sacc);
        dpacc = mfma32(da[s], nvf[s], dpacc);
    }
}
__device__ __forceinline__ void score_valu(const float *stats, f32x16 &sacc, f32x16 &dpacc, char *pds, float c,
                                           int lane) {
    const int half = lane >> 5;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const f32x4 l4 = *reinterpret_cast<const f32x4 *>(stats + g * 16 + half * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 4 * g + e;
            const float p = __builtin_amdgcn_exp2f(fmaf(sacc[i], c, -l4[e]));
            sacc[i] = p;
            dpacc[i] *= p;
        }
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        *reinterpret_cast<bf16x8 *>(pds + ks * 1024) = acc_to_frag(sacc, ks);
        *reinterpret_cast<bf16x8 *>(pds + (2 + ks) * 1024) = acc_to_frag(dpacc, ks);
    }
}

// Steady state of a score wave. Everything a step needs from LDS is read at the
// end of the step before (ScoreIn: the Q / dO fragments of the tile whose matrix
// half comes next, the lse2 of the tile whose vector half comes next; delta goes
// straight into the accumulator that matrix half will add to), so after the
// barrier the matrix instructions start at once. score_step writes the matrix
// half of the next tile (s_nxt, dp_nxt) out between the vector half of the
// current one (s_cur, dp_cur); the order below is the order of issue:
// scheduling barriers keep the compiler from regrouping it into a matrix phase
// and a vector phase, which would leave the matrix pipe idle meanwhile.
template <int D> struct ScoreIn {
    bf16x8 qa[D / 16], da[D / 16];
    f32x4 l4[4];
};
template <int D, int QOFF, int DOOFF>
__device__ __forceinline__ void score_load(const char *smem, const LaneOffs<D> &lo_m, const float *stats_m,
                                           const float *stats_v, ScoreIn<D> &in, f32x16 &dp_init, int lane) {
    const int half = lane >> 5;
#pragma unroll
    for (int g = 0; g < 4; ++g) in.l4[g] = *reinterpret_cast<const f32x4 *>(stats_v + g * 16 + half * 4);
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
        in.qa[s] = lo_m.template frag<QOFF>(smem, s);
        in.da[s] = lo_m.template frag<DOOFF>(smem, s);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const f32x4 d4 = *reinterpret_cast<const f32x4 *>(stats_m + g * 16 + 8 + half * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) dp_init[4 * g + e] = d4[e];
    }
}
// One steady-state step. The fragments a contraction step has consumed are refilled from the
// next tile (at the offsets lo_m) right behind it; the rest of the next step's operands (last
// fragments, lse2 from stats_v, delta from stats_m into dp_cur, which is free once its P / dS
// are emitted) follow the last P / dS write. On return at most kScoreTail LDS reads are
// younger than that write: wait_lgkm<kScoreTail>() before the barrier that publishes P / dS.
constexpr int kScoreTail = 10;
template <int D, int QOFF, int DOOFF>
__device__ __forceinline__ void score_step(const char *smem, const LaneOffs<D> &lo_m, const float *stats_m,
                                           const float *stats_v, ScoreIn<D> &in, const bf16x8 *kf, const bf16x8 *nvf,
                                           f32x16 &s_nxt, f32x16 &dp_nxt, f32x16 &s_cur, f32x16 &dp_cur, char *pds,
                                           float c, int lane) {
    constexpr int KS = D / 16, EPS = 16 / KS;      // vector elements per contraction step
    const int half = lane >> 5;
    auto vec = [&](int i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s_cur[i], c, -in.l4[i >> 2][i & 3]));
        s_cur[i] = p;
        dp_cur[i] *= p;
    };
    auto emit = [&](int ks) {      // fragments of 16 queries, complete once elements [8 ks, 8 ks + 8) are done
        *reinterpret_cast<bf16x8 *>(pds + ks * 1024) = acc_to_frag(s_cur, ks);
        *reinterpret_cast<bf16x8 *>(pds + (2 + ks) * 1024) = acc_to_frag(dp_cur, ks);
    };
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        s_nxt = mfma32(in.qa[s], kf[s], s == 0 ? zero16() : s_nxt);
        dp_nxt = mfma32(in.da[s], nvf[s], dp_nxt);
#pragma unroll
        for (int i = s * EPS; i < (s + 1) * EPS; ++i) vec(i);
        if ((s + 1) * EPS == 8) emit(0);
        __builtin_amdgcn_sched_barrier(0);
        if (s >= 1) {
            in.qa[s - 1] = lo_m.template frag<QOFF>(smem, s - 1);
            in.da[s - 1] = lo_m.template frag<DOOFF>(smem, s - 1);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    emit(1);
    __builtin_amdgcn_sched_barrier(0);
    in.qa[KS - 1] = lo_m.template frag<QOFF>(smem, KS - 1);
    in.da[KS - 1] = lo_m.template frag<DOOFF>(smem, KS - 1);
#pragma unroll
    for (int g = 0; g < 4; ++g) in.l4[g] = *reinterpret_cast<const f32x4 *>(stats_v + g * 16 + half * 4);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const f32x4 d4 = *reinterpret_cast<const f32x4 *>(stats_m + g * 16 + 8 + half * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) dp_cur[4 * g + e] = d4[e];
    }
    __builtin_amdgcn_sched_barrier(0);
}

// bf16 storage. Eight waves per workgroup, two per SIMD, in two roles: waves
// 0-3 turn a query tile into P and dS for key blocks 0-3 (they hold the K and
// V fragments and do all the exponentials), waves 4-7 hold the dK / dV
// accumulators (one block of 32 features each, for all key blocks), consume P
// and dS one step later, and issue all the global->LDS copies. The matrix work is split evenly, no
// contraction is done twice, each role fits the 256-register budget of two
// resident waves, and on every SIMD the exponentials and LDS waits of one role
// run under the matrix instructions of the other. A wave issues at most one
// instruction every four cycles, so the loop is written for a low instruction
// count per matrix instruction: inside a score wave the matrix instructions of
// tile t+1 sit between the vector instructions of tile t, and the copy
// addressing is kept to a few scalar and vector operations per tile.
//
// Step t (t = -1 .. ntiles+1), one workgroup barrier per step:
//   score waves: matrix half on tile t+1, vector half on tile t -> P/dS buffer t&1
//   grad waves : read Q^T / dO^T of tile t-1 and P/dS buffer (t-1)&1 into registers, multiply what
//                they read the step before (tile t-2)
// so tiles t-1 .. t+1 are resident and the stage of tile t-2 is free.
// The query stream of an item is mostly a gather of rows scattered over the
// sequence, so one tile of look-ahead does not cover the memory latency: the
// remaining NS - 3 stages are asynchronous copies in flight. Before the barrier
// of step t a grad wave waits only until its own copies of tile t+1 have landed
// (vmcnt bound, no drain). Everything the loop loads, per-query lse and delta
// included, goes through the async path, so no register-destination load
// forces an early wait; the list words that name the gathered rows are scalar
// loads issued one step before the copies that use them.
template <int D>
__global__ __launch_bounds__(512, 1) void attn_bwd_dkdv_pipe_kernel(KvArgs a) {
    typedef bf16_t T;
    constexpr int BQ = 32, NS = 7;
    constexpr int kWide = 3;                       // query tiles per step of a single-key-block item
    static_assert(2 * kWide <= NS && kWide <= 4, "two alternating sets of stages, one P / dS slot per score wave");
    constexpr int KS = D / 16, DB = D / 32;
    constexpr int TB = BQ * D * 2;                 // bytes of one Q (or dO) tile
    constexpr int SB = 2 * TB;                     // bytes of one stage: Q tile, dO tile
    constexpr int RPI = 512 / D;                   // tile rows per copy instruction (a wave moves 1 KB)
    constexpr int NI = BQ / RPI;                   // copy instructions per tile and tensor
    constexpr int PI = NI / 4;                     // ... per grad wave
    constexpr int LPT = 2 * PI + 2;                // copies per grad wave and tile: list words, Q, dO, lse/delta
    static_assert(NI % 4 == 0, "tile rows must divide evenly among the four grad waves");
    __shared__ __attribute__((aligned(1024))) char smem[NS * SB];
    // [tile parity][key block][P step 0, P step 1, dS step 0, dS step 1][lane] 16-byte fragment words
    __shared__ __attribute__((aligned(1024))) char pds_s[2 * 4 * 4 * 1024];
    __shared__ __attribute__((aligned(256))) float stats_s[NS][2 * BQ];
    // list words ((query << 5) | slot) of the gathered tiles about to be copied: [tile & 7][grad wave][8]
    __shared__ __attribute__((aligned(128))) int32_t ent_s[8][BQ];
    static_assert(PI * RPI == 8, "a grad wave copies 8 rows per tensor and tile");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const bool grad_role = wave >= 4;
    const int w4 = wave & 3;
    const int N = a.N;
    int logical;
    if (!xcd_remap((long long)a.n_items * a.BH, logical)) return;
    const int bh = logical / a.n_items;
    const KvItem item = a.items[logical - bh * a.n_items];

    // A tile of <= 32 keys (the ragged tail of a chunk) would leave three score waves
    // idle: instead the four take the same keys and the query tiles round-robin, each
    // writing its P / dS into its own key-block slot (the grad waves share every tile anyway).
    const bool split = item.key_len <= 32;
    const int kblk = split ? 0 : w4;
    const int nk = min(32, item.key_len - kblk * 32);
    const bool wave_active = nk > 0;
    const int key = wave_active ? item.key_start + kblk * 32 + min(l32, nk - 1) : item.key_start;

    const int nA = (item.q_len + BQ - 1) / BQ;
    // all of these are plain values (never reassigned), so nothing of the loop state lives in memory
    const bool routed = item.chunk >= 0 && a.topk > 0;
    const int32_t *loff = a.list_off + (size_t)bh * (a.C + 1);
    const int lbeg = routed ? loff[item.chunk] : 0;
    const int cntB = routed ? loff[item.chunk + 1] - lbeg : 0;
    const int ntiles = nA + (cntB + BQ - 1) / BQ;
    if (ntiles == 0) return;

    auto step_barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    auto next_stage = [&](int st) { return st == NS - 1 ? 0 : st + 1; };
    LaneOffs<D> lo;
    lo.init(lane);
    char *const pds = pds_s + w4 * 4096 + lane * 16;
    // split mode: the four waves of a role take the tiles round-robin
    auto mine = [&](int t) { return wave_active && (!split || (t & 3) == w4); };
    const bool fused = wave_active && !split;

    if (!grad_role) {
        // ------------------------------------------------------------ score waves
        const T *kbase = static_cast<const T *>(a.k) + (size_t)bh * N * D;
        const T *vbase = static_cast<const T *>(a.v) + (size_t)bh * N * D;
        bf16x8 kf[KS], nvf[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            kf[s] = Io<T>::load8(kbase + (size_t)key * D + s * 16 + half * 8);
            u32x4 v = __builtin_bit_cast(u32x4, Io<T>::load8(vbase + (size_t)key * D + s * 16 + half * 8));
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] ^= 0x80008000u;      // -V
            nvf[s] = __builtin_bit_cast(bf16x8, v);
        }
        const float c = a.scale_log2;
        // Row-operand offsets of a stage (stages are too far apart for an instruction offset). The
        // swizzle is an XOR of the 16-byte group index, and the groups of contraction step s are 2s
        // and 2s+1, so the eight offsets of a lane differ from the first one by XOR with 32 s: one
        // register is kept, the rest is rebuilt where needed (the empty asm keeps the rebuilt values
        // from being hoisted into eight long-lived registers).
        int row0 = lo.row[0];
        auto at_stage = [&](int st) {
            asm volatile("" : "+v"(row0));
            LaneOffs<D> lc;
            const int b = row0 + st * SB;
#pragma unroll
            for (int s = 0; s < KS; ++s) lc.row[s] = b ^ (32 * s);
            return lc;
        };
        if (fused) {
            // two accumulator sets take turns: while one goes through the vector half, the
            // matrix half of the next tile fills the other (no copies: the loop body is two steps).
            // At the top of step t (t even) set A holds S / delta - dP of tile t, `in` the
            // fragments of tile t+1 and the lse2 of tile t, and dpB starts at the delta of tile t+1.
            f32x16 sA, dpA, sB, dpB;
            ScoreIn<D> in;
            auto load_in = [&](int st_m, int st_v, f32x16 &dp_init) {
                score_load<D, 0, TB>(smem, at_stage(st_m), stats_s[st_m], stats_s[st_v], in, dp_init, lane);
                wait_lgkm0();   // P / dS are in LDS before the next barrier publishes them; the reads are done too
            };
            step_barrier();                                           // step -1: tiles 0 and 1 have landed
            score_mfma<D, 0, TB>(smem, at_stage(0), stats_s[0], kf, nvf, sA, dpA, lane);
            load_in(ntiles > 1 ? 1 : 0, 0, dpB);
            // one step; next_m / next_v: stages of the tiles whose matrix / vector half comes in the step after
            auto step = [&](f32x16 &s_nxt, f32x16 &dp_nxt, f32x16 &s_cur, f32x16 &dp_cur, int next_m, int next_v,
                            int buf) {
                score_step<D, 0, TB>(smem, at_stage(next_m), stats_s[next_m], stats_s[next_v], in, kf, nvf, s_nxt,
                                     dp_nxt, s_cur, dp_cur, pds + (buf << 14), c, lane);
                wait_lgkm<kScoreTail>();    // P / dS are in LDS before the next barrier publishes them
            };
            int st = 0, t = 0;      // st = stage of tile t
            for (; t + 2 < ntiles; t += 2) {
                const int st1 = next_stage(st), st2 = next_stage(st1), st3 = next_stage(st2);
                step_barrier();                                       // step t: tile t+2 has landed
                step(sB, dpB, sA, dpA, st2, st1, 0);
                step_barrier();                                       // step t + 1
                step(sA, dpA, sB, dpB, t + 3 < ntiles ? st3 : st2, st2, 1);
                st = st2;
            }
            if (t + 1 < ntiles) {                                     // two tiles left
                const int st1 = next_stage(st);
                step_barrier();
                step(sB, dpB, sA, dpA, st1, st1, 0);                  // (the refills are not used)
                wait_lgkm0();
                step_barrier();
                score_valu(stats_s[st1], sB, dpB, pds + (1 << 14), c, lane);
            } else {                                                  // one tile left
                step_barrier();
                score_valu(stats_s[st], sA, dpA, pds, c, lane);
            }
            wait_lgkm0();
            step_barrier();                                           // step ntiles
            step_barrier();                                           // step ntiles + 1 (the gradient waves' last)
        } else if (split) {
            // a single key block: kWide query tiles per step, one per score wave (see the grad waves)
            for (int k = 0; k * kWide < ntiles; ++k) {
                step_barrier();                                       // the tiles of step k have landed
                if (w4 < kWide && k * kWide + w4 < ntiles) {
                    const int st = (k & 1) * kWide + w4;
                    f32x16 sacc, dpacc;
                    score_mfma<D, 0, TB>(smem, at_stage(st), stats_s[st], kf, nvf, sacc, dpacc, lane);
                    score_valu(stats_s[st], sacc, dpacc, pds + ((k & 1) << 14), c, lane);
                    wait_lgkm0();
                }
                step_barrier();                                       // P / dS of step k are in LDS
            }
        } else {
            int st = NS - 1;     // stage of tile t
            for (int t = -1; t <= ntiles + 1; ++t) {
                step_barrier();
                if (t >= 0 && t < ntiles && mine(t)) {
                    f32x16 sacc, dpacc;
                    score_mfma<D, 0, TB>(smem, at_stage(st), stats_s[st], kf, nvf, sacc, dpacc, lane);
                    score_valu(stats_s[st], sacc, dpacc, pds + ((t & 1) << 14), c, lane);
                    wait_lgkm0();
                }
                st = next_stage(st);
            }
        }
    } else {
        // ------------------------------------------------------------ grad waves
        // Issue priority above the score wave of the same SIMD: the copies of a step go out at once and the
        // gradient products fill the matrix pipe while the score wave is in its vector half (measured: 3 %
        // of the kernel; raising the score waves instead changes nothing).
        __builtin_amdgcn_s_setprio(1);
        const char *qbase = static_cast<const char *>(a.q) + (size_t)bh * N * D * 2;
        const char *dobase = static_cast<const char *>(a.d_o) + (size_t)bh * N * D * 2;
        const float *const inf_slot = a.stats2 + (size_t)a.BH * N * 2;   // the pair (+inf, 0)
        const size_t lpos = (size_t)bh * N * a.topk + lbeg;
        const int32_t *const entries = a.qlist + lpos;

        // ---- copy addressing. This wave's copy p of a tensor covers tile rows (w4 + 4p) * RPI + [0, RPI).
        // Per tile ("group") a wave issues, in this order: the list words of the tile four groups
        // ahead (into a small LDS ring; a dummy copy when that tile is not a gathered one), PI copies
        // of Q, PI of dO, one of lse2 / delta: LPT in all, always, so that a vmcnt bound counts groups.
        // By the time a gathered tile's copies are issued its list words have landed: they are older
        // than the three groups that may still be in flight.
        const int rlo = lane / (D / 8), cgp = lane % (D / 8);
        uint32_t vcol[PI], voff[PI];
        auto trow = [&](int p) { return (w4 + 4 * p) * RPI + rlo; };
#pragma unroll
        for (int p = 0; p < PI; ++p) {
            vcol[p] = (uint32_t)((cgp ^ SwTile<D>::sw(trow(p))) * 16);
            voff[p] = (uint32_t)(trow(p) * D * 2) + vcol[p];
        }
        // lanes 0-7 copy lse2, lanes 8-15 delta, of the wave's 8 queries of a tile (pairs in memory)
        const uint32_t soff = (uint32_t)(((w4 * 8 + (lane & 7)) * 2 + ((lane >> 3) & 1)) * 4);
        const float *stc = a.stats2 + ((size_t)bh * N + item.q_start) * 2;    // next contiguous tile
        const float *stg = a.gstats2 + lpos * 2;                              // next gathered tile
        const uint32_t smem_at = lds_address(smem), stats_at = lds_address(stats_s), ent_at = lds_address(ent_s);
        const uint32_t ent_rd = ent_at + w4 * 32 + rlo * 4;
        auto tile_valid = [&](int t) { return t < nA ? min(BQ, item.q_len - t * BQ) : min(BQ, cntB - (t - nA) * BQ); };
        auto issue_words = [&](int v) {       // list words of tile v -> ring slot v & 7
            const uint32_t dst = ent_at + (v & 7) * 128 + w4 * 32;
            if (lane < 8) {
                if (v >= nA && v < ntiles) {
                    const int nvv = min(BQ, cntB - (v - nA) * BQ);
                    const int eidx = (w4 + 4 * ((lane & 7) / RPI)) * RPI + (lane & 7) % RPI;
                    async_copy4_at(entries + (v - nA) * BQ, (uint32_t)(min(eidx, nvv - 1) * 4), dst);
                } else {
                    async_copy4_at(inf_slot, 0u, dst);
                }
            }
        };
        int ist = 0;                          // stage of the next tile to be issued (tiles go out in order)
        const char *qp = qbase + (size_t)item.q_start * (D * 2), *dop = dobase + (size_t)item.q_start * (D * 2);
        auto issue_group = [&](int u) {
            issue_words(u + 4);
            const uint32_t qat = smem_at + ist * SB + w4 * 1024, sat = stats_at + ist * (2 * BQ * 4) + w4 * 64;
            ist = next_stage(ist);
            const int nv = tile_valid(u);
            // (plain selects: a pointer picked and advanced inside the branches ends up in scratch memory)
            const bool contig = u < nA;
            const float *const st2 = contig ? stc : stg;
            stc += contig ? BQ * 2 : 0;
            stg += contig ? 0 : BQ * 2;
            if (contig) {
                if (nv == BQ) {
#pragma unroll
                    for (int p = 0; p < PI; ++p) {
                        async_copy16_at(qp, voff[p], qat + p * 4096);
                        async_copy16_at(dop, voff[p], qat + TB + p * 4096);
                    }
                } else {
#pragma unroll
                    for (int p = 0; p < PI; ++p) {
                        const uint32_t off = (uint32_t)(min(trow(p), nv - 1) * D * 2) + vcol[p];
                        async_copy16_at(qp, off, qat + p * 4096);
                        async_copy16_at(dop, off, qat + TB + p * 4096);
                    }
                }
                qp += BQ * D * 2;
                dop += BQ * D * 2;
            } else {
#pragma unroll
                for (int p = 0; p < PI; ++p) {
                    const int e = *reinterpret_cast<const __attribute__((address_space(3))) int *>(
                        (uintptr_t)(ent_rd + (u & 7) * 128 + p * RPI * 4));
                    const size_t off = ((size_t)(uint32_t)(e >> 5) * (D * 2)) | vcol[p];
                    async_copy16_at(qbase + off, qat + p * 4096);
                    async_copy16_at(dobase + off, qat + TB + p * 4096);
                }
            }
            if (lane < 16) {
                if (nv == BQ) {
                    async_copy4_at(st2, soff, sat);
                } else {
                    // ragged tile: rows past the end take lse2 = +inf and the delta of the last row
                    const int srow = w4 * 8 + (lane & 7);
                    const float *sp = st2 + min(srow, nv - 1) * 2 + ((lane >> 3) & 1);
                    if (lane < 8 && srow >= nv) sp = inf_slot;
                    async_copy4_at(sp, sat);
                }
            }
        };
        // own copies of tile u landed: at most the copies of the younger tiles may be outstanding
        auto wait_tile = [&](int u) {
            const int younger = min(NS - 5, ntiles - 1 - u);
            static_assert(NS - 5 >= 1 && NS - 5 <= 4 && 4 * LPT < 64, "cases below");
            if (younger >= 4) wait_vmcnt<(NS - 5 >= 4 ? 4 : 0) * LPT>();
            else if (younger == 3) wait_vmcnt<(NS - 5 >= 3 ? 3 : 0) * LPT>();
            else if (younger == 2) wait_vmcnt<(NS - 5 >= 2 ? 2 : 0) * LPT>();
            else if (younger == 1) wait_vmcnt<LPT>();
            else wait_vmcnt<0>();
        };
        // the barrier of step t publishes tile t+2 (the score waves read it at the end of step t)
        auto step_wait = [&](int t) {
            if (t < ntiles) wait_tile(min(t + 2, ntiles - 1));
            step_barrier();
        };
        auto step_issue = [&](int t) {
            if (t + NS - 2 < ntiles) issue_group(t + NS - 2);
        };
        // the list words of the first four tiles go ahead of everything (needed only if one of them is gathered)
        if (nA < 4) {
#pragma unroll
            for (int v = 0; v < 4; ++v) issue_words(v);
            wait_vmcnt<0>();
        }
        if (!split) {
#pragma unroll
            for (int p = 0; p <= NS - 4; ++p)
                if (p < ntiles) issue_group(p);
        }

        // ---- matrix work. A grad wave owns one block of 32 features (rows of dK^T / dV^T) for
        // KPW key blocks: the transposed Q / dO fragments it reads from a tile are then shared by
        // all its key blocks (a wave that owned a key block would read the whole tile, four times
        // the transposed reads, and those run at half the rate of the plain 16-byte reads that
        // fetch P and dS instead). With a single key block (split mode) the four waves still
        // share every tile, one feature block each.
        constexpr int DBW = DB < 4 ? DB : 4;       // feature blocks across the waves
        constexpr int KPW = DBW;                   // key blocks per wave (4 waves cover DBW x (4 / DBW) x KPW blocks)
        const int db = w4 % DBW, kg = w4 / DBW;
        const int nkb = split ? 1 : (item.key_len + 31) / 32;                  // key blocks of the item
        const int nmine = max(0, min(KPW, nkb - kg * KPW));                    // ... of this wave
        f32x16 dk[KPW], dv[KPW];
#pragma unroll
        for (int j = 0; j < KPW; ++j) dk[j] = zero16(), dv[j] = zero16();
        // lane offsets of the transposed reads of feature block db (see LaneOffs::init), 16-query step 0
        int tr0, tr1;
        {
            const int i = lane & 15, bq = (lane >> 4) & 1;
            const int x = 32 * db + 16 * bq + 4 * (i & 3), r0 = 4 * half + (i >> 2);
            tr0 = (SwTile<D>::off(r0, x >> 3) + (x & 7)) * 2;
            tr1 = (SwTile<D>::off(r0 + 8, x >> 3) + (x & 7)) * 2;
        }
        struct TFrags { bf16x8 qt[2], dot[2]; };   // Q^T and dO^T of the wave's features, both 16-query steps
        auto tload = [&](int st) {
            asm volatile("" : "+v"(tr0), "+v"(tr1));     // keep the stage base out of loop-invariant copies
            typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
            typedef short s16x8 __attribute__((ext_vector_type(8)));
            const char *base = smem + st * SB;
            TFrags f;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int w = 0; w < 2; ++w) {
                    const char *pt = base + w * TB + ks * 16 * D * 2;
                    const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(pt + tr0));
                    const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(pt + tr1));
                    const s16x8 r = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
                    (w == 0 ? f.qt[ks] : f.dot[ks]) = __builtin_bit_cast(bf16x8, r);
                }
            return f;
        };
        const char *const pds_rd = pds_s + lane * 16;
        // P / dS fragments of tile u, key block slot kb0 + j: P step 0, P step 1, dS step 0, dS step 1
        auto pload = [&](int u, int j, bf16x8 *P) {
            const int kb0 = split ? (u & 3) : kg * KPW;
            const char *pp = pds_rd + ((u & 1) << 14) + (kb0 + j) * 4096;
#pragma unroll
            for (int i = 0; i < 4; ++i) P[i] = *reinterpret_cast<const bf16x8 *>(pp + i * 1024);
        };
        auto gmfma = [&](const TFrags &f, const bf16x8 *P, int j) {
            dv[j] = mfma32(f.dot[0], P[0], dv[j]);
            dk[j] = mfma32(f.qt[0], P[2], dk[j]);
            dv[j] = mfma32(f.dot[1], P[1], dv[j]);
            dk[j] = mfma32(f.qt[1], P[3], dk[j]);
        };
        if (split) {
            // A tile of <= 32 keys (the ragged tail of a chunk) is one key block: per step each of
            // kWide score waves takes a query tile of its own and the grad waves multiply all of
            // them, so a step still carries a full load of matrix work. Two sets of kWide stages
            // alternate; two barriers per step (tiles landed, P / dS written), no deeper pipeline.
            ist = 0;
#pragma unroll
            for (int i = 0; i < kWide; ++i)
                if (i < ntiles) issue_group(i);
            for (int k = 0; k * kWide < ntiles; ++k) {
                wait_vmcnt<0>();
                step_barrier();                                       // the tiles of step k have landed
                ist = ((k + 1) & 1) * kWide;
#pragma unroll
                for (int i = 0; i < kWide; ++i)
                    if ((k + 1) * kWide + i < ntiles) issue_group((k + 1) * kWide + i);
                TFrags f[kWide];
#pragma unroll
                for (int i = 0; i < kWide; ++i) f[i] = tload((k & 1) * kWide + min(i, ntiles - 1 - k * kWide));
                step_barrier();                                       // P / dS of step k are in LDS
                if (nmine > 0) {
#pragma unroll
                    for (int i = 0; i < kWide; ++i)
                        if (k * kWide + i < ntiles) {
                            const char *pp = pds_rd + ((k & 1) << 14) + i * 4096;
                            bf16x8 P[4];
#pragma unroll
                            for (int x = 0; x < 4; ++x) P[x] = *reinterpret_cast<const bf16x8 *>(pp + x * 1024);
                            gmfma(f[i], P, 0);
                        }
                }
            }
        } else {
        step_wait(-1);
        step_issue(-1);
        step_wait(0);
        step_issue(0);
        if (nmine == KPW) {
            // Two steps behind the score waves: everything a step multiplies was read into registers
            // during the step before (the P / dS of tile t-2 were published by the barrier of step
            // t-1), so the matrix instructions start right after the barrier, and the reads for the
            // next step are issued behind them, key block by key block, into the registers they free.
            // The reads must be over before the next barrier: the score waves then rewrite that buffer.
            step_wait(1);
            step_issue(1);
            bf16x8 P[KPW][4];
#pragma unroll
            for (int j = 0; j < KPW; ++j) pload(0, j, P[j]);
            TFrags f = tload(0);
            int st = 0;      // stage of the tile held in f (tile t - 2 at the top of step t)
            wait_lgkm0();
            for (int t = 2; t <= ntiles + 1; ++t) {
                step_wait(t);
                const int stn = t - 1 < ntiles ? next_stage(st) : st;     // past the end: any resident tile, unused
                step_issue(t);       // first: measured best (better than between or behind the matrix instructions)
#pragma unroll
                for (int j = 0; j < KPW; ++j) {
                    gmfma(f, P[j], j);
                    __builtin_amdgcn_sched_barrier(0);
                    pload(t - 1, j, P[j]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                f = tload(stn);
                st = stn;
                __builtin_amdgcn_sched_barrier(0);
                wait_lgkm<8>();      // the P / dS reads are over (the 8 transposed tile reads behind them need not be)
            }
        } else {
            // one step behind, reading as it goes (partly filled or tail tiles)
            TFrags f = tload(0);
            int st = 0;      // stage of tile t - 1
            for (int t = 1; t <= ntiles + 1; ++t) {
                step_wait(t);
                step_issue(t);
                if (t <= ntiles) {
#pragma unroll
                    for (int j = 0; j < KPW; ++j)
                        if (j < nmine) {
                            bf16x8 P[4];
                            pload(t - 1, j, P);
                            gmfma(f, P, j);
                        }
                    st = t < ntiles ? next_stage(st) : st;
                    f = tload(st);
                    wait_lgkm0();
                }
            }
        }
        }

        // ---- results: lane = key, registers = the wave's 32 features; the accumulator holds -dK
        const float dks = -a.scale;
#pragma unroll
        for (int j = 0; j < KPW; ++j) {
            if (j >= nmine) break;
            const int kb = split ? 0 : kg * KPW + j;
            if (kb * 32 + l32 >= item.key_len) continue;
            if (item.partial < 0) {
                const size_t row = (size_t)bh * N + item.key_start + kb * 32 + l32;
                T *dkp = static_cast<T *>(a.dk) + row * D + db * 32, *dvp = static_cast<T *>(a.dv) + row * D + db * 32;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int x = g * 8 + half * 4;
                    Io<T>::store4(dkp + x, dk[j][4 * g] * dks, dk[j][4 * g + 1] * dks, dk[j][4 * g + 2] * dks,
                                  dk[j][4 * g + 3] * dks);
                    Io<T>::store4(dvp + x, dv[j][4 * g], dv[j][4 * g + 1], dv[j][4 * g + 2], dv[j][4 * g + 3]);
                }
            } else {
                const size_t prow = ((size_t)bh * a.n_partials + item.partial) * kKeyTile + kb * 32 + l32;
                float *dkp = a.tpart_k + prow * D + db * 32, *dvp = a.tpart_v + prow * D + db * 32;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int x = g * 8 + half * 4;
                    Io<float>::store4(dkp + x, dk[j][4 * g] * dks, dk[j][4 * g + 1] * dks, dk[j][4 * g + 2] * dks,
                                      dk[j][4 * g + 3] * dks);
                    Io<float>::store4(dvp + x, dv[j][4 * g], dv[j][4 * g + 1], dv[j][4 * g + 2], dv[j][4 * g + 3]);
                }
            }
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
static hipError_t bwd_dispatch(const moc_meta *m, int BH, FwdArgs &a, KvArgs &kv, const void *o, void *dq,
                               hipStream_t st) {
    constexpr int QPW = 256 / (D / 8);
    const size_t rows = (size_t)BH * m->N;
    { MOC_PROF("delta", st);
    delta_kernel<D, T><<<dim3((unsigned)((rows + QPW - 1) / QPW)), dim3(256), 0, st>>>(
        static_cast<const T *>(o), static_cast<const T *>(a.d_o), rows, a.lse, const_cast<float *>(a.delta),
        const_cast<float *>(kv.stats2)); }
    { MOC_PROF("attn_bwd_dkdv", st);
    if constexpr (sizeof(T) == 2) {
        if (a.topk > 0) {
            const int NK = m->N * a.topk;
            gather_stats_kernel<<<dim3((NK + 255) / 256, BH), dim3(256), 0, st>>>(
                kv.qlist, kv.list_off, m->N, NK, m->C, reinterpret_cast<const float2 *>(kv.stats2),
                reinterpret_cast<float2 *>(const_cast<float *>(kv.gstats2)));
        }
        attn_bwd_dkdv_pipe_kernel<D><<<dim3(xcd_grid((long long)m->n_kvitems * BH)), dim3(512), 0, st>>>(kv);
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
        bool chunk_path = false;
        if constexpr (sizeof(T) == 2) {
            if (m->max_chunk_len <= kChunkRows) {
                chunk_path = true;
                const int groups = (a.items_per_head + kGroupTiles - 1) / kGroupTiles;
                attn_bwd_dq_chunk_kernel<D><<<dim3(xcd_grid((long long)groups * BH)), dim3(512), 0, st>>>(a);
            }
        }
        if (!chunk_path)
            attn_bwd_dq_kernel<D, T, MODE_ROUTED><<<dim3(xcd_grid((long long)a.items_per_head * BH)), dim3(256), 0, st>>>(a);
    }
    { MOC_PROF("attn_bwd_dq_forced", st);
    a.items_per_head = m->n_atiles;
    // bf16 storage: the forced-link items run after the routed ones and add the routed partials themselves
    a.o_out = sizeof(T) == 2 ? dq : nullptr;
    attn_bwd_dq_kernel<D, T, MODE_ANCHOR><<<dim3(xcd_grid((long long)a.items_per_head * BH)), dim3(256), 0, st>>>(a); }
    if (sizeof(T) == 2) return hipGetLastError();
    MOC_PROF("dq_merge", st);
    dq_merge_kernel<D, T><<<dim3((m->N + QPW - 1) / QPW, BH), dim3(256), 0, st>>>(a.po, a.vmask, m->N, a.topk,
                                                                                static_cast<T *>(dq));
    return hipGetLastError();
}

hipError_t launch_attn_bwd(const moc_meta *m, int BH, int d, int dtype, const void *q, const void *k, const void *v,
                           const void *o, const float *lse, const void *d_o, int topk, float scale, void *dq, void *dk,
                           void *dv, char *ws, const AttnWs &L, hipStream_t st) {
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
    a.vmask = reinterpret_cast<const uint32_t *>(ws + L.vmask);
    a.lse = lse;
    a.delta = reinterpret_cast<const float *>(ws + L.delta);
    a.gstats2 = reinterpret_cast<const float *>(ws + L.gstats2);
    KvArgs kv{};
    kv.q = q; kv.k = k; kv.v = v; kv.d_o = d_o;
    kv.lse = lse; kv.delta = a.delta;
    kv.stats2 = reinterpret_cast<const float *>(ws + L.stats2);
    kv.gstats2 = reinterpret_cast<const float *>(ws + L.gstats2);
    kv.dk = dk; kv.dv = dv;
    kv.tpart_k = reinterpret_cast<float *>(ws + L.tpart_k);
    kv.tpart_v = reinterpret_cast<float *>(ws + L.tpart_v);
    kv.items = m->d_kvitems;
    kv.list_off = a.list_off; kv.qlist = a.qlist;
    kv.N = m->N; kv.C = m->C; kv.topk = topk; kv.n_partials = m->n_partials; kv.n_items = m->n_kvitems; kv.BH = BH;
    kv.scale = scale; kv.scale_log2 = a.scale_log2;
    if (dtype == MOC_BF16) return d == 128 ? bwd_dispatch<128, bf16_t>(m, BH, a, kv, o, dq, st)
                                           : bwd_dispatch<64, bf16_t>(m, BH, a, kv, o, dq, st);
    return d == 128 ? bwd_dispatch<128, float>(m, BH, a, kv, o, dq, st)
                    : bwd_dispatch<64, float>(m, BH, a, kv, o, dq, st);
}

}  // namespace moc
