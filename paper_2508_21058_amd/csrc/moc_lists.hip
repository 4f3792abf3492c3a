// Inverse routing lists: for every (head, chunk) the queries that routed to it.
//
// Routing is per query (Eq. 3), so under incoherent selections a tile of
// neighbouring queries touches far more chunks than k. The attention passes
// therefore visit routed work chunk-major: the rows gathered through these
// lists form dense query tiles against one chunk's keys - the packing the
// paper obtains from a variable-length attention call (Sec. 3.3).
//
// A stable counting sort on the device, no host synchronisation, no global
// atomics, so every list is in ascending query order and the same input gives
// the same lists (and the same summation order in dK / dV) on every call:
//   count  one wave per block of kRowsPerBlk queries: which entries of a
//          row count at all (see entry_ok), an LDS histogram over the chunks,
//          written out whole as row `block` of a [blocks][C] table;
//   scan   down the blocks of every chunk (a block's first position inside the
//          chunk's list), then across the chunks (list offsets, tile offsets);
//   fill   one wave per block walks its queries in order; the lanes hold the
//          entries of ONE query, whose chunks are distinct, and take their
//          positions from LDS counters. LDS operations of a wave complete in
//          program order, so the positions do not depend on scheduling.
// An entry packs query and slot as (i << 5) | r (r < MOC_MAX_TOPK = 32).
//
// Which entries of a selection row count (Sec. 3.3 pre-routing mask): forced
// links are attended anyway, so an entry naming a caption chunk or a chunk of
// the query's own window is dropped, as is the second mention of a chunk in a
// row and anything outside [0, C). The union M(i) + R(i) is a set. Bit r of
// vmask[query] says whether slot r counts; the attention epilogues read the
// same word, so a dropped slot is never merged.
#include "moc_device.h"
#include "moc_internal.h"

namespace moc {

// Both passes below walk a block of kRowsPerBlk queries 64 / topk queries at a time: lane L holds
// entry L of the step's rows (query L / topk, slot L % topk), read with one coalesced load.

// One wave per block. An entry counts if it names a video chunk (rw >= 0) outside the query's own
// window that no earlier slot of the row names (the row-mates sit in the neighbouring lanes).
__global__ __launch_bounds__(64) void list_count_kernel(const int32_t *__restrict__ sel, int N, int topk, int C,
                                                        const int32_t *__restrict__ chunk_of,
                                                        const int32_t *__restrict__ win,
                                                        const int32_t *__restrict__ rw, int NB,
                                                        uint32_t *__restrict__ vmask, int32_t *__restrict__ cnt_blk) {
    extern __shared__ int32_t hist[];    // [C]
    const int bh = blockIdx.y, blk = blockIdx.x, lane = threadIdx.x;
    const int i0 = blk * kRowsPerBlk, nrow = min(kRowsPerBlk, N - i0);
    for (int b = lane; b < C; b += 64) hist[b] = 0;
    __syncthreads();
    const int rpb = 64 / topk;                     // queries per step (topk <= 32: at least two)
    const int mu = lane / topk, r = lane - mu * topk;
    const bool lane_on = mu < rpb;
    const int32_t *src = sel + ((size_t)bh * N + i0) * topk;
    uint32_t *vm = vmask + (size_t)bh * N + i0;
    const uint32_t rowbits = topk >= 32 ? 0xffffffffu : ((1u << topk) - 1u);
    for (int u0 = 0; u0 < nrow; u0 += rpb) {
        const int u = u0 + mu;
        const bool in = lane_on && u < nrow;
        const int j = in ? src[(size_t)u * topk + r] : -1;
        const int wq = in ? win[chunk_of[i0 + u]] : -1;
        bool ok = j >= 0 && j < C;
        const int w = ok ? rw[j] : -1;
        ok = ok && w >= 0 && w != wq;
        for (int p = 0; p + 1 < topk; ++p) {
            const int other = __shfl(j, mu * topk + p, 64);
            if (p < r && other == j) ok = false;
        }
        if (ok) atomicAdd(&hist[j], 1);
        const unsigned long long bal = __ballot(ok);
        if (in && r == 0) vm[u] = (uint32_t)(bal >> (mu * topk)) & rowbits;
    }
    __syncthreads();
    int32_t *out = cnt_blk + ((size_t)bh * NB + blk) * C;
    for (int b = lane; b < C; b += 64) out[b] = hist[b];
}

// Down the blocks in two levels (the table is [block][chunk], so neighbouring threads read
// neighbouring words): the blocks are cut into kScanGroups groups; pass 1 sums every chunk's
// entries per group, pass 2 turns the group's entries into the number of entries of that chunk
// in all earlier blocks and leaves the chunk's total behind.
constexpr int kScanGroups = 32;
__global__ __launch_bounds__(256) void list_group_sum_kernel(const int32_t *__restrict__ cnt_blk, int NB, int C,
                                                             int32_t *__restrict__ gsum) {
    const int bh = blockIdx.z, g = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= C) return;
    const int per = (NB + kScanGroups - 1) / kScanGroups;
    const int b0 = g * per, b1 = min(NB, b0 + per);
    const int32_t *col = cnt_blk + (size_t)bh * NB * C + j;
    int sum = 0;
    for (int b = b0; b < b1; ++b) sum += col[(size_t)b * C];
    gsum[((size_t)bh * kScanGroups + g) * C + j] = sum;
}
__global__ __launch_bounds__(256) void list_block_scan_kernel(int32_t *__restrict__ cnt_blk, int NB, int C,
                                                              const int32_t *__restrict__ gsum,
                                                              int32_t *__restrict__ cnt) {
    const int bh = blockIdx.z, g = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= C) return;
    const int per = (NB + kScanGroups - 1) / kScanGroups;
    const int b0 = g * per, b1 = min(NB, b0 + per);
    const int32_t *gs = gsum + (size_t)bh * kScanGroups * C + j;
    int run = 0;
    for (int u = 0; u < g; ++u) run += gs[(size_t)u * C];
    int32_t *col = cnt_blk + (size_t)bh * NB * C + j;
    for (int b = b0; b < b1; ++b) {
        const int c = col[(size_t)b * C];
        col[(size_t)b * C] = run;
        run += c;
    }
    if (g == kScanGroups - 1) cnt[(size_t)bh * C + j] = run;
}

// per head: list_off = exclusive scan of cnt, tile_off = exclusive scan of ceil(cnt / kBM)
__global__ __launch_bounds__(256) void list_scan_kernel(const int32_t *__restrict__ cnt, int C,
                                                        int32_t *__restrict__ list_off,
                                                        int32_t *__restrict__ tile_off) {
    __shared__ int32_t sa[256], sb[256];
    const int bh = blockIdx.x;
    const int32_t *c = cnt + (size_t)bh * C;
    int32_t *lo = list_off + (size_t)bh * (C + 1);
    int32_t *to = tile_off + (size_t)bh * (C + 1);
    const int seg = (C + 255) / 256;
    const int b0 = threadIdx.x * seg, b1 = min(C, b0 + seg);
    int a = 0, b = 0;
    for (int j = b0; j < b1; ++j) { a += c[j]; b += (c[j] + kBM - 1) / kBM; }
    sa[threadIdx.x] = a;
    sb[threadIdx.x] = b;
    __syncthreads();
    if (threadIdx.x == 0) {
        int ra = 0, rb = 0;
        for (int t = 0; t < 256; ++t) {
            const int xa = sa[t], xb = sb[t];
            sa[t] = ra; sb[t] = rb;
            ra += xa; rb += xb;
        }
        lo[C] = ra;
        to[C] = rb;
    }
    __syncthreads();
    a = sa[threadIdx.x];
    b = sb[threadIdx.x];
    for (int j = b0; j < b1; ++j) {
        lo[j] = a;
        to[j] = b;
        a += c[j];
        b += (c[j] + kBM - 1) / kBM;
    }
}

// One wave per block. The positions are handed out query by query: one LDS instruction per query,
// executed by that query's lanes only. The slots that count name distinct chunks, so the lanes of
// one instruction never meet in a counter, and the instructions of consecutive queries reach the
// counters in program order. All 64 lanes then store their entries with one instruction.
__global__ __launch_bounds__(64) void list_fill_kernel(const int32_t *__restrict__ sel, int N, int topk, int C,
                                                       const uint32_t *__restrict__ vmask, int NB,
                                                       const int32_t *__restrict__ cnt_blk,
                                                       const int32_t *__restrict__ list_off,
                                                       int32_t *__restrict__ qlist) {
    extern __shared__ int32_t cursor[];  // [C]
    const int bh = blockIdx.y, blk = blockIdx.x, lane = threadIdx.x;
    const int i0 = blk * kRowsPerBlk, nrow = min(kRowsPerBlk, N - i0);
    const int32_t *base = cnt_blk + ((size_t)bh * NB + blk) * C;
    const int32_t *lo = list_off + (size_t)bh * (C + 1);
    for (int b = lane; b < C; b += 64) cursor[b] = lo[b] + base[b];
    __syncthreads();
    const int32_t *src = sel + ((size_t)bh * N + i0) * topk;
    const uint32_t *vm = vmask + (size_t)bh * N + i0;
    int32_t *ql = qlist + (size_t)bh * N * topk;
    const int rpb = 64 / topk;
    const int mu = lane / topk, r = lane - mu * topk;
    const bool lane_on = mu < rpb;
    constexpr int U = 4;                           // steps whose loads are in flight together
    for (int u0 = 0; u0 < nrow; u0 += U * rpb) {
        int j[U];
        bool ok[U];
#pragma unroll
        for (int t = 0; t < U; ++t) {
            const int u = u0 + t * rpb + mu;
            const bool in = lane_on && u < nrow;
            ok[t] = in && ((vm[in ? u : 0] >> r) & 1u);
            j[t] = in ? src[(size_t)u * topk + r] : 0;
        }
#pragma unroll
        for (int t = 0; t < U; ++t) {
            int pos = 0;
            for (int v = 0; v < rpb; ++v)
                if (ok[t] && mu == v) pos = atomicAdd(&cursor[j[t]], 1);
            if (ok[t]) ql[pos] = ((i0 + u0 + t * rpb + mu) << 5) | r;
        }
    }
}

hipError_t launch_build_lists(const moc_meta *m, int BH, int topk, const int32_t *sel, char *ws, const AttnWs &L,
                              hipStream_t st) {
    const int C = m->C, N = m->N;
    const int NB = (N + kRowsPerBlk - 1) / kRowsPerBlk;
    int32_t *cnt = reinterpret_cast<int32_t *>(ws + L.cnt);
    int32_t *cnt_blk = reinterpret_cast<int32_t *>(ws + L.cnt_blk);
    uint32_t *vmask = reinterpret_cast<uint32_t *>(ws + L.vmask);
    int32_t *list_off = reinterpret_cast<int32_t *>(ws + L.list_off);
    int32_t *tile_off = reinterpret_cast<int32_t *>(ws + L.tile_off);
    int32_t *qlist = reinterpret_cast<int32_t *>(ws + L.qlist);
    MOC_PROF("build_lists", st);
    const size_t shm_fill = (size_t)C * 4, shm_count = (size_t)C * 4;
    list_count_kernel<<<dim3(NB, BH), dim3(64), shm_count, st>>>(sel, N, topk, C, m->d_chunk_of, m->d_win, m->d_rwin, NB,
                                                                 vmask, cnt_blk);
    int32_t *gsum = reinterpret_cast<int32_t *>(ws + L.gsum);
    const dim3 sgrid((C + 255) / 256, kScanGroups, BH);
    list_group_sum_kernel<<<sgrid, dim3(256), 0, st>>>(cnt_blk, NB, C, gsum);
    list_block_scan_kernel<<<sgrid, dim3(256), 0, st>>>(cnt_blk, NB, C, gsum, cnt);
    list_scan_kernel<<<dim3(BH), dim3(256), 0, st>>>(cnt, C, list_off, tile_off);
    list_fill_kernel<<<dim3(NB, BH), dim3(64), shm_fill, st>>>(sel, N, topk, C, vmask, NB, cnt_blk, list_off, qlist);
    return hipGetLastError();
}

}  // namespace moc
