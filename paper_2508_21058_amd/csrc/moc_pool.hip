// Stage (a) device part (token -> chunk map) and stage (b1) mean pooling.
//
// Pooling (Sec. 3.1: the chunk descriptor is the arithmetic mean of its keys;
// Sec. 3.3: pooled on the fly per variable-length segment) is bandwidth bound:
// k is read exactly once, 16 bytes per lane, rows of a chunk are contiguous in
// the head-major layout so every wave reads whole 256-byte rows.
#include "moc_device.h"
#include "moc_internal.h"
#include "moc_pool_unit.h"

namespace moc {

// chunk_of[i] = j with off[j] <= i < off[j+1]  (the bucketize of Sec. 3.3)
__global__ __launch_bounds__(256) void chunk_of_kernel(const int32_t *__restrict__ off, int C, int N,
                                                       int32_t *__restrict__ chunk_of) {
    int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= N) return;
    int lo = 0, hi = C;  // invariant: off[lo] <= i < off[hi]
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (off[mid] <= i) lo = mid; else hi = mid;
    }
    chunk_of[i] = lo;
}

hipError_t launch_chunk_of(const moc_meta *m, hipStream_t st) {
    chunk_of_kernel<<<dim3((m->N + 255) / 256), dim3(256), 0, st>>>(m->d_off, m->C, m->N, m->d_chunk_of);
    return hipGetLastError();
}

// One workgroup per (chunk, head); see pool_unit.
template <int D, typename T>
__global__ __launch_bounds__(256) void pool_kernel(const T *__restrict__ k, const int32_t *__restrict__ off,
                                                   int N, int C, int Cpad, float *__restrict__ kbar,
                                                   bf16_t *__restrict__ split) {
    __shared__ float red[PoolShape<D, T>::kRedFloats];
    pool_unit<D, T>(k, off, N, C, Cpad, kbar, split, blockIdx.x, blockIdx.y, red);
}

hipError_t launch_pool(const moc_meta *m, int BH, int d, int dtype, const void *k, float *kbar, void *kb_split,
                       int Cpad, hipStream_t st) {
    dim3 grid(Cpad, BH), block(256);
    MOC_PROF("pool", st);
#define MOC_POOL(DD, TT) \
    pool_kernel<DD, TT><<<grid, block, 0, st>>>(static_cast<const TT *>(k), m->d_off, m->N, m->C, Cpad, kbar, \
                                                static_cast<bf16_t *>(kb_split))
    if (dtype == MOC_BF16) { if (d == 128) MOC_POOL(128, bf16_t); else MOC_POOL(64, bf16_t); }
    else { if (d == 128) MOC_POOL(128, float); else MOC_POOL(64, float); }
#undef MOC_POOL
    return hipGetLastError();
}

}  // namespace moc
