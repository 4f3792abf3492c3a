// Work-item decoding and global->LDS staging shared by the attention passes.
#pragma once
#include "moc_device.h"
#include "moc_internal.h"

namespace moc {

// compile-time integer tag (selects an LDS buffer in the unrolled pipelines)
template <int V> struct IC { static constexpr int value = V; };

constexpr int MODE_ANCHOR = 0;  // forced links: window query tile x (text spans + window)
constexpr int MODE_ROUTED = 1;  // routed links: gathered queries of a chunk x that chunk

// Arguments of the query-stationary passes (forward, and dQ of the backward).
struct FwdArgs {
    const void *q, *k, *v;
    bf16_t *po;        // [BH, N, slots, D] partial outputs (forward) / partial dQ (backward)
    float *plse;       // [BH, N, slots]   partial log-sum-exp (forward only)
    int N, C, topk, slots;
    int BH, items_per_head;   // work list of the launch: items_per_head entries per (batch, head)
    float scale, scale_log2;
    const AnchorTile *atiles;
    const int32_t *arange_off;
    const KeyRange *aranges;
    const int32_t *off, *list_off, *tile_off, *qlist;
    // backward only
    const void *d_o;
    const float *lse, *delta;
    const float *gstats2;   // [BH, N*topk] pairs (lse * log2 e, delta) in inverse-list order
    // forced-link forward items with the merge fused into their epilogue
    const uint32_t *vmask;  // [BH, N] bit r: routed slot r of the query counts (set by the list builder)
    void *o_out;            // [BH, N, D] final output
    float *lse_out;         // [BH, N] final log-sum-exp
};

// Chunk-stationary routed items (forward and dQ pass): a workgroup keeps the keys and values of one
// chunk in LDS and serves a group of that chunk's query tiles from them.
constexpr int kChunkRows = 288;       // resident keys (K region; the V region holds 32 rows more)
constexpr int kGroupTiles = 16;       // query tiles (of kBM list entries) per workgroup

// The GPU has 8 XCDs with private L2 caches and hands consecutive workgroups to
// them round-robin. Work lists are ordered so that neighbours share K/V (or
// Q/dO), hence XCD x takes the contiguous slice [x*per, (x+1)*per) of the list.
// Launch ceil(total/8)*8 workgroups on a 1-D grid; returns false for padding.
constexpr int kXcds = 8;
__host__ __device__ inline int xcd_grid(long long total) { return (int)((total + kXcds - 1) / kXcds) * kXcds; }
__device__ __forceinline__ bool xcd_remap(long long total, int &logical) {
    const int L = blockIdx.x;
    const int per = (int)((total + kXcds - 1) / kXcds);
    logical = (L % kXcds) * per + L / kXcds;
    return logical < total;
}

struct ItemDesc {
    int q_start, q_count;
    const int32_t *entries;   // gathered rows ((query << 5) | slot) or nullptr
    int nranges;
    const KeyRange *ranges;   // nullptr: use `single`
    KeyRange single;
    __device__ __forceinline__ KeyRange range(int r) const { return ranges ? ranges[r] : single; }
};

template <int MODE>
__device__ __forceinline__ bool decode_item(const FwdArgs &a, int bh, int t, ItemDesc &it) {
    if (MODE == MODE_ANCHOR) {
        const AnchorTile at = a.atiles[t];
        it.q_start = at.q_start;
        it.q_count = at.q_count;
        it.entries = nullptr;
        const int r0 = a.arange_off[at.win];
        it.nranges = a.arange_off[at.win + 1] - r0;
        it.ranges = a.aranges + r0;
        it.single = KeyRange{0, 0};
        return true;
    } else {
        const int C = a.C;
        const int32_t *toff = a.tile_off + (size_t)bh * (C + 1);
        if (t >= toff[C]) return false;
        int lo = 0, hi = C;   // largest j with toff[j] <= t
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (toff[mid] <= t) lo = mid; else hi = mid;
        }
        const int j = lo;
        const int32_t *loff = a.list_off + (size_t)bh * (C + 1);
        const int tl = t - toff[j];
        const int cnt = loff[j + 1] - loff[j];
        it.q_start = 0;
        it.q_count = min(kBM, cnt - tl * kBM);
        it.entries = a.qlist + (size_t)bh * a.N * a.topk + loff[j] + tl * kBM;
        it.nranges = 1;
        it.ranges = nullptr;
        it.single = KeyRange{a.off[j], a.off[j + 1] - a.off[j]};
        return true;
    }
}

// Walks the key ranges of an item in tiles of BN keys; the last tile of every
// range may be ragged (valid() < BN).
template <int BN> struct TileIter {
    const ItemDesc &it;
    int r, pos;
    KeyRange cur;
    __device__ __forceinline__ explicit TileIter(const ItemDesc &d) : it(d), r(0), pos(0), cur(d.range(0)) {}
    __device__ __forceinline__ int start() const { return cur.start + pos; }
    __device__ __forceinline__ int valid() const { return min(BN, cur.len - pos); }
    __device__ __forceinline__ bool next() {
        pos += BN;
        if (pos >= cur.len) {
            ++r;
            pos = 0;
            if (r >= it.nranges) return false;
            cur = it.range(r);
        }
        return true;
    }
};

// Stages ROWS source rows of D features into a swizzled LDS tile (SwTile<D>),
// 16 bytes per lane and pass, through registers (conversion to bf16 on the way)
// so the global loads of the next tile overlap the math on the current one.
// rowfn(r) gives the global row of tile row r (clamped by the caller).
template <int D, typename T, int ROWS> struct RowStager {
    static constexpr int CG = D / 8, RPP = 256 / CG, P = (ROWS + RPP - 1) / RPP;
    int cg, rr;
    bf16x8 reg[P];
    __device__ __forceinline__ explicit RowStager(int tid) : cg(tid % CG), rr(tid / CG) {}
    template <typename F> __device__ __forceinline__ void load_fn(const T *base, F rowfn) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int row = rr + p * RPP;
            if (ROWS % RPP == 0 || row < ROWS) reg[p] = Io<T>::load8(base + (size_t)rowfn(row) * D + cg * 8);
        }
    }
    __device__ __forceinline__ void load(const T *base, int start, int valid) {
        load_fn(base, [=](int r) { return start + min(r, valid - 1); });
    }
    __device__ __forceinline__ void store_sw(bf16_t *lds) const {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int row = rr + p * RPP;
            if (ROWS % RPP == 0 || row < ROWS)
                *reinterpret_cast<u32x4 *>(lds + SwTile<D>::off(row, cg)) = __builtin_bit_cast(u32x4, reg[p]);
        }
    }
};

// Epilogue of the query-stationary passes. A transposed accumulator holds, per
// lane, 4-feature pieces of ONE row; storing those directly scatters 8-byte
// writes over 32 rows per instruction and the L2 writes partial lines back
// several times. Instead every wave transposes its 32 x D tile through its own
// 32 x (D + 4) bf16 patch of LDS and stores whole 16-byte groups, 16 lanes per
// 256-byte row. `dst_row` is this lane's destination row index (in rows of D
// bf16) or -1 if its row is not to be written; `scale` multiplies the values.
// All waves of the workgroup must have finished reading `smem` (barrier before).
template <int D>
__device__ __forceinline__ void store_rows_bf16(char *smem, int wave, int lane, const f32x16 *acc, float scale,
                                                int dst_row, bf16_t *out) {
    constexpr int DB = D / 32, RS = D + 4;             // padded row: consecutive rows shift by 2 banks
    const int half = lane >> 5, l32 = lane & 31;
    bf16_t *patch = reinterpret_cast<bf16_t *>(smem) + wave * (32 * RS + 64);
    int32_t *rowidx = reinterpret_cast<int32_t *>(patch + 32 * RS);
#pragma unroll
    for (int b = 0; b < DB; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g)
            Io<bf16_t>::store4(patch + l32 * RS + b * 32 + g * 8 + half * 4, acc[b][4 * g] * scale,
                               acc[b][4 * g + 1] * scale, acc[b][4 * g + 2] * scale, acc[b][4 * g + 3] * scale);
    if (half == 0) rowidx[l32] = dst_row;
    __builtin_amdgcn_wave_barrier();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    constexpr int LPR = D / 8, RPI = 64 / LPR;          // lanes per row, rows per instruction
    const int cg = lane % LPR, r0 = lane / LPR;
#pragma unroll
    for (int it = 0; it < 32 / RPI; ++it) {
        const int r = it * RPI + r0;
        const int dr = rowidx[r];
        const u32x2 lo2 = *reinterpret_cast<const u32x2 *>(patch + r * RS + cg * 8);
        const u32x2 hi2 = *reinterpret_cast<const u32x2 *>(patch + r * RS + cg * 8 + 4);
        if (dr >= 0) {
            u32x4 v = {lo2[0], lo2[1], hi2[0], hi2[1]};
            *reinterpret_cast<u32x4 *>(out + (size_t)dr * D + cg * 8) = v;
        }
    }
}

// Moves ROWS source rows of D features into a swizzled LDS tile (SwTile<D>).
//   issue(base, rowfn, lds)  starts the transfer of a tile into `lds`
//   commit(lds)              finishes it (before the barrier that publishes `lds`)
// bf16 storage: asynchronous global->LDS loads (global_load_lds_dwordx4): no
// staging registers, no LDS store instructions. One wave instruction fills 1 KB
// of LDS, lane l writing bytes [16 l, 16 l + 16), so each lane fetches the
// global element that belongs at its swizzled LDS position.
// fp32 storage needs a conversion, so it goes through registers.
template <int D, typename T, int ROWS> struct TileLoader;

template <int D, int ROWS> struct TileLoader<D, bf16_t, ROWS> {
    static constexpr int NW = 4;                        // waves of the workgroup that share the loads
    static constexpr int RPI = 512 / D;                 // rows per wave instruction
    static constexpr int NI = ROWS / RPI;               // wave instructions per tile
    static constexpr int P = (NI + NW - 1) / NW;        // per wave
    static_assert(NI % NW == 0, "tile rows must divide evenly among the waves");
    int wave, rlo, cgp;
    __device__ __forceinline__ int slot(int p) const { return wave + NW * p; }
    __device__ __forceinline__ explicit TileLoader(int tid)
        : wave(__builtin_amdgcn_readfirstlane(tid >> 6)), rlo((tid & 63) / (D / 8)), cgp((tid & 63) % (D / 8)) {}
    // arbitrary (gathered) rows: rowfn(r) is the global row of tile row r
    template <typename F> __device__ __forceinline__ void issue(const bf16_t *base, F rowfn, bf16_t *lds) const {
        const uint32_t at = lds_address(lds);      // one pointer conversion per tile, not one per copy
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int n = slot(p);
            const int row = n * RPI + rlo;
            const int cg = cgp ^ SwTile<D>::sw(row);
            async_copy16_at(base + (size_t)rowfn(row) * D + cg * 8, at + n * 1024);
        }
    }
    // contiguous rows [0, valid) of a tile whose first row is at `tile` (a
    // wave-uniform pointer): scalar base + one 32-bit lane offset per load
    __device__ __forceinline__ void issue_rows(const bf16_t *tile, int valid, bf16_t *lds) const {
        const uint32_t at = lds_address(lds);
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int n = slot(p);
            const int row = n * RPI + rlo;
            const int cg = cgp ^ SwTile<D>::sw(row);
            const uint32_t off = (uint32_t)(min(row, valid - 1) * D + cg * 8) * 2u;
            async_copy16_at(tile, off, at + n * 1024);
        }
    }
    // the tile is complete once this wave's copies have landed (and the workgroup has met at a barrier)
    __device__ __forceinline__ void commit(bf16_t *) const { wait_vmcnt<0>(); }
};

template <int D, int ROWS> struct TileLoader<D, float, ROWS> {
    RowStager<D, float, ROWS> st;
    __device__ __forceinline__ explicit TileLoader(int tid) : st(tid) {}
    template <typename F> __device__ __forceinline__ void issue(const float *base, F rowfn, bf16_t *) {
        st.load_fn(base, rowfn);
    }
    __device__ __forceinline__ void issue_rows(const float *tile, int valid, bf16_t *) {
        st.load_fn(tile, [=](int r) { return min(r, valid - 1); });
    }
    __device__ __forceinline__ void commit(bf16_t *lds) const { st.store_sw(lds); }
};

}  // namespace moc
