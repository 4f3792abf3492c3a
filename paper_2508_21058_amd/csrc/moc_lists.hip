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
//   count  one workgroup per block of kRowsPerBlk queries: which entries of a
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

// slot r of the row `row` (topk entries) of a query whose chunk lies in window wq
__device__ __forceinline__ bool entry_ok(const int32_t *row, int r, int C, const int32_t *kind, const int32_t *win,
                                         int wq) {
    const int j = row[r];
    if (j < 0 || j >= C) return false;
    if (kind[j] != 0 || win[j] == wq) return false;
    for (int p = 0; p < r; ++p)
        if (row[p] == j) return false;
    return true;
}

__global__ __launch_bounds__(256) void list_count_kernel(const int32_t *__restrict__ sel, int N, int topk, int C,
                                                         const int32_t *__restrict__ chunk_of,
                                                         const int32_t *__restrict__ kind,
                                                         const int32_t *__restrict__ win, int NB,
                                                         uint32_t *__restrict__ vmask, int32_t *__restrict__ cnt_blk) {
    extern __shared__ int32_t hist[];
    const int bh = blockIdx.y, blk = blockIdx.x;
    for (int b = threadIdx.x; b < C; b += 256) hist[b] = 0;
    __syncthreads();
    const int i0 = blk * kRowsPerBlk;
    for (int u = threadIdx.x; u < kRowsPerBlk; u += 256) {
        const int i = i0 + u;
        if (i >= N) break;
        const int32_t *row = sel + ((size_t)bh * N + i) * topk;
        const int wq = win[chunk_of[i]];
        uint32_t mask = 0;
        for (int r = 0; r < topk; ++r)
            if (entry_ok(row, r, C, kind, win, wq)) {
                mask |= 1u << r;
                atomicAdd(&hist[row[r]], 1);
            }
        vmask[(size_t)bh * N + i] = mask;
    }
    __syncthreads();
    int32_t *out = cnt_blk + ((size_t)bh * NB + blk) * C;
    for (int b = threadIdx.x; b < C; b += 256) out[b] = hist[b];
}

// down the blocks: cnt_blk[bh][blk][j] becomes the number of entries of chunk j in earlier blocks
__global__ __launch_bounds__(256) void list_block_scan_kernel(int32_t *__restrict__ cnt_blk, int NB, int C,
                                                              int32_t *__restrict__ cnt) {
    const int bh = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= C) return;
    int32_t *col = cnt_blk + (size_t)bh * NB * C + j;
    int run = 0;
    int b = 0;
    for (; b + 8 <= NB; b += 8) {
        int c[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) c[u] = col[(size_t)(b + u) * C];
#pragma unroll
        for (int u = 0; u < 8; ++u) { col[(size_t)(b + u) * C] = run; run += c[u]; }
    }
    for (; b < NB; ++b) { const int c = col[(size_t)b * C]; col[(size_t)b * C] = run; run += c; }
    cnt[(size_t)bh * C + j] = run;
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

// One wave per block of queries. Lane r holds slot r of the current query; the slots that count
// name distinct chunks, so the lanes of one LDS instruction never meet in a counter, and the
// instructions of consecutive queries reach the counters in program order.
__global__ __launch_bounds__(64) void list_fill_kernel(const int32_t *__restrict__ sel, int N, int topk, int C,
                                                       const uint32_t *__restrict__ vmask, int NB,
                                                       const int32_t *__restrict__ cnt_blk,
                                                       const int32_t *__restrict__ list_off,
                                                       int32_t *__restrict__ qlist) {
    extern __shared__ int32_t cursor[];
    const int bh = blockIdx.y, blk = blockIdx.x, lane = threadIdx.x;
    const int32_t *base = cnt_blk + ((size_t)bh * NB + blk) * C;
    const int32_t *lo = list_off + (size_t)bh * (C + 1);
    for (int b = lane; b < C; b += 64) cursor[b] = lo[b] + base[b];
    __syncthreads();
    const int i0 = blk * kRowsPerBlk, i1 = min(N, i0 + kRowsPerBlk);
    const int32_t *s = sel + (size_t)bh * N * topk;
    const uint32_t *vm = vmask + (size_t)bh * N;
    int32_t *ql = qlist + (size_t)bh * N * topk;
    const int r = lane & 31;
    constexpr int U = 8;       // queries in flight
    for (int i = i0; i < i1; i += U) {
        int j[U], pos[U];
        bool ok[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int q = min(i + u, i1 - 1);
            ok[u] = i + u < i1 && lane < topk && ((vm[q] >> r) & 1u);
            j[u] = ok[u] ? s[(size_t)q * topk + r] : 0;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            pos[u] = 0;
            if (ok[u]) pos[u] = atomicAdd(&cursor[j[u]], 1);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (ok[u]) ql[pos[u]] = ((i + u) << 5) | r;
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
    const size_t shm = (size_t)C * 4;
    list_count_kernel<<<dim3(NB, BH), dim3(256), shm, st>>>(sel, N, topk, C, m->d_chunk_of, m->d_kind, m->d_win, NB,
                                                            vmask, cnt_blk);
    list_block_scan_kernel<<<dim3((C + 255) / 256, BH), dim3(256), 0, st>>>(cnt_blk, NB, C, cnt);
    list_scan_kernel<<<dim3(BH), dim3(256), 0, st>>>(cnt, C, list_off, tile_off);
    list_fill_kernel<<<dim3(NB, BH), dim3(64), shm, st>>>(sel, N, topk, C, vmask, NB, cnt_blk, list_off, qlist);
    return hipGetLastError();
}

}  // namespace moc
