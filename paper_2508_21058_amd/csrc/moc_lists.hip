// Inverse routing lists: for every (head, chunk) the queries that routed to it.
//
// Routing is per query (Eq. 3), so under incoherent selections a tile of
// neighbouring queries touches far more chunks than k. The attention passes
// therefore visit routed work chunk-major: the rows gathered through these
// lists form dense query tiles against one chunk's keys - the packing the
// paper obtains from a variable-length attention call (Sec. 3.3).
//
// Counting sort on the device, no host synchronisation:
//   count (LDS histogram per workgroup, one global atomic per non-empty bin)
//   -> exclusive scan per head (list offsets and tile offsets)
//   -> fill (LDS ranks + one reservation per bin).
// An entry packs query and slot as (i << 5) | r (r < MOC_MAX_TOPK = 32).
#include "moc_device.h"
#include "moc_internal.h"

namespace moc {

constexpr int kEntPerThread = 16;
constexpr int kEntPerWg = 256 * kEntPerThread;
constexpr int kMaxLdsBins = 16384;

__global__ __launch_bounds__(256) void zero_i32_kernel(int32_t *p, size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = 0;
}

template <bool LDS_HIST>
__global__ __launch_bounds__(256) void list_count_kernel(const int32_t *__restrict__ sel, int NK, int C,
                                                         int32_t *__restrict__ cnt) {
    extern __shared__ int32_t hist[];
    const int bh = blockIdx.y;
    const int32_t *s = sel + (size_t)bh * NK;
    int32_t *c = cnt + (size_t)bh * C;
    if (LDS_HIST) {
        for (int b = threadIdx.x; b < C; b += 256) hist[b] = 0;
        __syncthreads();
    }
#pragma unroll 4
    for (int u = 0; u < kEntPerThread; ++u) {
        const int e = blockIdx.x * kEntPerWg + u * 256 + threadIdx.x;
        if (e < NK) {
            const int j = s[e];
            if (j >= 0 && j < C) {
                if (LDS_HIST) atomicAdd(&hist[j], 1); else atomicAdd(&c[j], 1);
            }
        }
    }
    if (LDS_HIST) {
        __syncthreads();
        for (int b = threadIdx.x; b < C; b += 256) {
            const int h = hist[b];
            if (h) atomicAdd(&c[b], h);
        }
    }
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

template <bool LDS_HIST>
__global__ __launch_bounds__(256) void list_fill_kernel(const int32_t *__restrict__ sel, int NK, int topk, int C,
                                                        const int32_t *__restrict__ list_off,
                                                        int32_t *__restrict__ cursor,
                                                        int32_t *__restrict__ qlist) {
    extern __shared__ int32_t hist[];
    const int bh = blockIdx.y;
    const int32_t *s = sel + (size_t)bh * NK;
    const int32_t *lo = list_off + (size_t)bh * (C + 1);
    int32_t *cur = cursor + (size_t)bh * C;
    int32_t *ql = qlist + (size_t)bh * NK;
    int jj[kEntPerThread], rk[kEntPerThread];
    if (LDS_HIST) {
        for (int b = threadIdx.x; b < C; b += 256) hist[b] = 0;
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < kEntPerThread; ++u) {
        const int e = blockIdx.x * kEntPerWg + u * 256 + threadIdx.x;
        int j = -1;
        if (e < NK) j = s[e];
        if (j >= C) j = -1;
        jj[u] = j;
        rk[u] = 0;
        if (j >= 0) rk[u] = LDS_HIST ? atomicAdd(&hist[j], 1) : atomicAdd(&cur[j], 1);
    }
    if (LDS_HIST) {
        __syncthreads();
        for (int b = threadIdx.x; b < C; b += 256) {
            const int h = hist[b];
            if (h) hist[b] = atomicAdd(&cur[b], h);   // bin now holds this workgroup's base
        }
        __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < kEntPerThread; ++u) {
        const int e = blockIdx.x * kEntPerWg + u * 256 + threadIdx.x;
        const int j = jj[u];
        if (j >= 0) {
            const int i = e / topk;
            ql[lo[j] + (LDS_HIST ? hist[j] : 0) + rk[u]] = (i << 5) | (e - i * topk);
        }
    }
}

hipError_t launch_build_lists(const moc_meta *m, int BH, int topk, const int32_t *sel, char *ws, const AttnWs &L,
                              hipStream_t st) {
    const int C = m->C;
    const int NK = m->N * topk;
    int32_t *cnt = reinterpret_cast<int32_t *>(ws + L.cnt);
    int32_t *list_off = reinterpret_cast<int32_t *>(ws + L.list_off);
    int32_t *tile_off = reinterpret_cast<int32_t *>(ws + L.tile_off);
    int32_t *cursor = reinterpret_cast<int32_t *>(ws + L.cursor);
    int32_t *qlist = reinterpret_cast<int32_t *>(ws + L.qlist);
    // cnt and cursor are adjacent sections; clear both (a fill kernel, so the
    // call can be captured into a graph)
    const size_t nz = (size_t)BH * C;
    MOC_PROF("build_lists", st);
    zero_i32_kernel<<<dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, st>>>(cnt, nz);
    zero_i32_kernel<<<dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, st>>>(cursor, nz);
    dim3 grid((NK + kEntPerWg - 1) / kEntPerWg, BH), block(256);
    const bool lds = C <= kMaxLdsBins;
    const size_t shm = lds ? (size_t)C * 4 : 0;
    if (lds) list_count_kernel<true><<<grid, block, shm, st>>>(sel, NK, C, cnt);
    else list_count_kernel<false><<<grid, block, 0, st>>>(sel, NK, C, cnt);
    list_scan_kernel<<<dim3(BH), dim3(256), 0, st>>>(cnt, C, list_off, tile_off);
    if (lds) list_fill_kernel<true><<<grid, block, shm, st>>>(sel, NK, topk, C, list_off, cursor, qlist);
    else list_fill_kernel<false><<<grid, block, 0, st>>>(sel, NK, topk, C, list_off, cursor, qlist);
    return hipGetLastError();
}

}  // namespace moc
