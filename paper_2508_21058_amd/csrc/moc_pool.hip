// Stage (a) device part (token -> chunk map) and stage (b1) mean pooling.
//
// Pooling (Sec. 3.1: the chunk descriptor is the arithmetic mean of its keys;
// Sec. 3.3: pooled on the fly per variable-length segment) is bandwidth bound:
// k is read exactly once, 16 bytes per lane, rows of a chunk are contiguous in
// the head-major layout so every wave reads whole 256-byte rows.
#include "moc_device.h"
#include "moc_internal.h"

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

// One workgroup per (chunk, head). Thread t owns 8 (bf16) or 4 (fp32) features
// of every (256/TPR)-th row; partial sums are combined through LDS in a fixed
// order, so the result does not depend on scheduling.
// Besides the fp32 mean the kernel writes its exact split into three bf16
// planes (hi + mid + lo == mean) for the matrix-core scoring pass; rows
// C .. Cpad-1 of the planes are zero.
template <int D, typename T>
__global__ __launch_bounds__(256) void pool_kernel(const T *__restrict__ k, const int32_t *__restrict__ off,
                                                   int N, int C, int Cpad, float *__restrict__ kbar,
                                                   bf16_t *__restrict__ split) {
    constexpr int VEC = 16 / sizeof(T);      // elements per 16-byte load
    constexpr int TPR = D / VEC;             // threads per row
    constexpr int RPP = 256 / TPR;           // rows per pass
    const int j = blockIdx.x, bh = blockIdx.y;
    if (j >= C) {
        if (threadIdx.x < D) {
#pragma unroll
            for (int p = 0; p < 3; ++p) split[(((size_t)bh * 3 + p) * Cpad + j) * D + threadIdx.x] = (bf16_t)0.f;
        }
        return;
    }
    const int t0 = off[j], t1 = off[j + 1];
    const int cg = threadIdx.x % TPR, r0 = threadIdx.x / TPR;
    const T *base = k + ((size_t)bh * N) * D + cg * VEC;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    int t = t0 + r0;
    // 4 independent loads in flight per lane
    for (; t + 3 * RPP < t1; t += 4 * RPP) {
        float f[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if constexpr (sizeof(T) == 2) {
                Io<T>::load8f(base + (size_t)(t + u * RPP) * D, f[u]);
            } else {
                f32x4 x = *reinterpret_cast<const f32x4 *>(base + (size_t)(t + u * RPP) * D);
                f[u][0] = x[0]; f[u][1] = x[1]; f[u][2] = x[2]; f[u][3] = x[3];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += f[u][e];
    }
    for (; t < t1; t += RPP) {
        float f[8];
        if constexpr (sizeof(T) == 2) {
            Io<T>::load8f(base + (size_t)t * D, f);
        } else {
            f32x4 x = *reinterpret_cast<const f32x4 *>(base + (size_t)t * D);
            f[0] = x[0]; f[1] = x[1]; f[2] = x[2]; f[3] = x[3];
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += f[e];
    }
    __shared__ float red[RPP][D + 4];
#pragma unroll
    for (int e = 0; e < VEC; ++e) red[r0][cg * VEC + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < D) {
        float s = 0.f;
#pragma unroll 4
        for (int r = 0; r < RPP; ++r) s += red[r][threadIdx.x];
        const float mean = s / (float)(t1 - t0);
        kbar[((size_t)bh * C + j) * D + threadIdx.x] = mean;
        const bf16_t hi = (bf16_t)mean;
        const float r1 = mean - (float)hi;
        const bf16_t mid = (bf16_t)r1;
        const bf16_t lo = (bf16_t)(r1 - (float)mid);
        split[(((size_t)bh * 3 + 0) * Cpad + j) * D + threadIdx.x] = hi;
        split[(((size_t)bh * 3 + 1) * Cpad + j) * D + threadIdx.x] = mid;
        split[(((size_t)bh * 3 + 2) * Cpad + j) * D + threadIdx.x] = lo;
    }
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
