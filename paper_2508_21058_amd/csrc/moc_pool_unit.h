// Mean pooling of one (chunk, head) by one workgroup of 256 threads (stage b1; Sec. 3.1: the
// chunk descriptor is the arithmetic mean of its keys). Shared by the pooling kernel and by the
// fused routing kernel.
#pragma once
#include "moc_device.h"

namespace moc {

template <int D, typename T> struct PoolShape {
    static constexpr int VEC = 16 / sizeof(T);      // elements per 16-byte load
    static constexpr int TPR = D / VEC;             // threads per row
    static constexpr int RPP = 256 / TPR;           // rows per pass
    static constexpr int kRedFloats = RPP * (D + 4);
};

// Thread t owns 8 (bf16) or 4 (fp32) features of every (256/TPR)-th row; partial sums are combined
// through `red` (LDS, PoolShape::kRedFloats floats) in a fixed order, so the result does not depend
// on scheduling. Besides the fp32 mean the unit writes its exact split into three bf16 planes
// (hi + mid + lo == mean) for the matrix-core scoring pass; rows C .. Cpad-1 of the planes are zero.
// Ends with a workgroup barrier, so `red` may be reused at once.
template <int D, typename T>
__device__ __forceinline__ void pool_unit(const T *__restrict__ k, const int32_t *__restrict__ off, int N, int C,
                                          int Cpad, float *__restrict__ kbar, bf16_t *__restrict__ split, int j, int bh,
                                          float *red) {
    constexpr int VEC = PoolShape<D, T>::VEC, TPR = PoolShape<D, T>::TPR, RPP = PoolShape<D, T>::RPP;
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
#pragma unroll
    for (int e = 0; e < VEC; ++e) red[r0 * (D + 4) + cg * VEC + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < D) {
        float s = 0.f;
#pragma unroll 4
        for (int r = 0; r < RPP; ++r) s += red[r * (D + 4) + threadIdx.x];
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
    __syncthreads();
}

}  // namespace moc
