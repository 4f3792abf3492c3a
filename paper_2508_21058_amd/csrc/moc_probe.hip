// Machine probes (measurement aids, not part of the layer): what one GPU
// sustains on a plain streaming copy and on a loop of independent bf16 MFMA
// chains. The bench reports the layer's kernels against these measured rates
// beside the published peaks.
#include "moc_internal.h"
#include "moc_device.h"

namespace moc {

// Each lane moves 16 bytes per iteration; the grid strides over the buffer.
__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                         size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// Eight waves per workgroup (two per SIMD), each running four independent
// accumulator chains of v_mfma_f32_32x32x16_bf16: 16 MFMAs per iteration per wave.
__global__ __launch_bounds__(512) void probe_mfma_kernel(float *__restrict__ out, int iters) {
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(1.f + 0.125f * ((threadIdx.x + i) & 3));
        b[i] = (__bf16)(0.0078125f * (1 + ((threadIdx.x * 3 + i) & 7)));
    }
    f32x16 c0 = zero16(), c1 = zero16(), c2 = zero16(), c3 = zero16();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            c0 = mfma32(a, b, c0);
            c1 = mfma32(b, a, c1);
            c2 = mfma32(a, a, c2);
            c3 = mfma32(b, b, c3);
        }
    }
    float s = 0.f;
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// Do matrix and vector instructions of different waves on one SIMD run at the same time? Eight
// waves per workgroup, one workgroup per compute unit (two waves per SIMD): waves 0-3 run MFMA
// chains (mode bit 0), waves 4-7 run independent fma / exp2 chains (mode bit 1). Timed with
// either role alone and with both, the three durations say whether the two kinds of work overlap
// (both = max of the two) or take turns (both = sum). Mode bit 2 puts the vector work into the
// MFMA waves themselves, interleaved with their matrix instructions (waves 4-7 idle).
__global__ __launch_bounds__(512) void probe_mix_kernel(float *__restrict__ out, int iters, int mode) {
    const int wave = threadIdx.x >> 6;
    float s = 0.f;
    if (wave < 4) {
        if (mode & 1) {
            bf16x8 a, b;
            for (int i = 0; i < 8; ++i) {
                a[i] = (__bf16)(1.f + 0.125f * ((threadIdx.x + i) & 3));
                b[i] = (__bf16)(0.0078125f * (1 + ((threadIdx.x * 3 + i) & 7)));
            }
            f32x16 c0 = zero16(), c1 = zero16();
            if (mode & 4) {
                // the same vector work inside the MFMA wave itself, six vector instructions behind every MFMA
                float x[16];
                for (int i = 0; i < 16; ++i) x[i] = threadIdx.x * 0.001f + i;
                for (int it = 0; it < iters; ++it) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        c0 = mfma32(a, b, c0);
                        c1 = mfma32(b, a, c1);
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int i = 0; i < 16; ++i) x[i] = __builtin_fmaf(x[i], 1.0001f, 0.5f);
#pragma unroll
                    for (int i = 0; i < 16; ++i) x[i] = __builtin_amdgcn_exp2f(x[i] * 0.001f);
#pragma unroll
                    for (int u = 0; u < 16; ++u) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);
                    }
                }
                for (int i = 0; i < 16; ++i) s += x[i];
            } else {
                for (int it = 0; it < iters; ++it) {
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        c0 = mfma32(a, b, c0);
                        c1 = mfma32(b, a, c1);
                    }
                }
            }
            for (int i = 0; i < 16; ++i) s += c0[i] + c1[i];
        }
    } else if (mode & 2) {
        float x[16];
        for (int i = 0; i < 16; ++i) x[i] = threadIdx.x * 0.001f + i;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < 16; ++i) x[i] = __builtin_fmaf(x[i], 1.0001f, 0.5f);
#pragma unroll
            for (int i = 0; i < 16; ++i) x[i] = __builtin_amdgcn_exp2f(x[i] * 0.001f);
        }
        for (int i = 0; i < 16; ++i) s += x[i];
    }
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// On-chip data paths of one compute unit, two workgroups of four waves per CU as in the query-stationary
// attention kernels. MODE 0 / 1: every wave re-reads its own 16 KB of LDS with ds_read_b128 /
// ds_read_b64_tr_b16 (the two operand reads of the attention kernels). MODE 2 / 3: every wave copies
// 16 KB per iteration from a cache-resident 64 KB of global memory into LDS, with the asynchronous
// global_load_lds_dwordx4 the kernels use, or through registers (global_load_dwordx4 + ds_write_b128).
template <int MODE>
__global__ __launch_bounds__(256) void probe_cu_path_kernel(const uint32_t *__restrict__ src, uint32_t *__restrict__ out,
                                                            int iters) {
    __shared__ __attribute__((aligned(1024))) uint32_t lds[16384];       // 64 KB
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 16384; i += 256) lds[i] = i;
    __syncthreads();
    uint32_t *mine = lds + wave * 4096;
    u32x4 acc = {0u, 0u, 0u, 0u};
    if (MODE == 0 || MODE == 1) {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                if (MODE == 0) {
                    acc += *reinterpret_cast<const u32x4 *>(mine + ((u * 256 + lane * 4) & 4095));
                } else {
                    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
                    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(mine + ((u * 128 + lane * 2) & 4095)));
                    acc[0] += (uint32_t)v[0];
                    acc[1] += (uint32_t)v[1];
                }
            }
            asm volatile("" : "+v"(acc));
        }
    } else {
        const uint32_t *g = src + wave * 4096 + lane * 4;
        for (int it = 0; it < iters; ++it) {
            if (MODE == 2) {
#pragma unroll
                for (int u = 0; u < 16; ++u) async_copy16_at(g + u * 256, lds_address(mine + u * 256));
                wait_vmcnt<0>();
            } else {
                u32x4 v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = *reinterpret_cast<const u32x4 *>(g + u * 256);
#pragma unroll
                for (int u = 0; u < 16; ++u) *reinterpret_cast<u32x4 *>(mine + u * 256 + lane * 4) = v[u];
                wait_lgkm0();
            }
            asm volatile("" ::: "memory");
        }
        __syncthreads();
        acc[0] = lds[threadIdx.x];
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = acc[0] + acc[1] + acc[2] + acc[3];
}

// Runs one probe on `st` bracketed by the two events; `units` receives the bytes
// moved (copy: read + written) or the flops issued (mfma) inside the bracket.
hipError_t launch_probe(int kind, void *buf, size_t bytes, int iters, hipStream_t st, hipEvent_t e0, hipEvent_t e1,
                        double *units) {
    if (kind == MOC_PROBE_COPY) {
        const size_t n16 = bytes / 32;                  // 16-byte words in each half
        const u32x4 *src = (const u32x4 *)buf;
        u32x4 *dst = (u32x4 *)buf + n16;
        const int grid = 256 * 16;
        probe_copy_kernel<<<grid, 256, 0, st>>>(src, dst, n16);          // untimed first pass
        (void)hipEventRecord(e0, st);
        for (int i = 0; i < iters; ++i) probe_copy_kernel<<<grid, 256, 0, st>>>(src, dst, n16);
        (void)hipEventRecord(e1, st);
        *units = 2.0 * 16.0 * (double)n16 * iters;
    } else if (kind >= MOC_PROBE_MFMA4 && kind <= MOC_PROBE_MFMA4_VALU_SAME_WAVE) {
        const int mode = kind == MOC_PROBE_MFMA4 ? 1 : (kind == MOC_PROBE_VALU4 ? 2 : (kind == MOC_PROBE_MFMA4_VALU4 ? 3 : 5));
        const int grid = kProbeMfmaGrid;
        probe_mix_kernel<<<grid, 512, 0, st>>>((float *)buf, 16, mode);  // untimed first pass
        (void)hipEventRecord(e0, st);
        probe_mix_kernel<<<grid, 512, 0, st>>>((float *)buf, iters, mode);
        (void)hipEventRecord(e1, st);
        // per iteration and wave: 16 MFMAs (waves 0-3), 64 fma + 16 mul + 16 exp2 (waves 4-7)
        *units = (double)iters;
    } else if (kind >= MOC_PROBE_LDS_READ && kind <= MOC_PROBE_COPY_VIA_REGISTERS) {
        const int grid = 2 * kProbeMfmaGrid;            // two workgroups per compute unit
        const uint32_t *src = static_cast<const uint32_t *>(buf);
        uint32_t *out = static_cast<uint32_t *>(buf) + 16384;            // behind the 64 KB that are read
        auto go = [&](int n) {
            if (kind == MOC_PROBE_LDS_READ) probe_cu_path_kernel<0><<<grid, 256, 0, st>>>(src, out, n);
            else if (kind == MOC_PROBE_LDS_READ_TRANSPOSED) probe_cu_path_kernel<1><<<grid, 256, 0, st>>>(src, out, n);
            else if (kind == MOC_PROBE_COPY_TO_LDS_ASYNC) probe_cu_path_kernel<2><<<grid, 256, 0, st>>>(src, out, n);
            else probe_cu_path_kernel<3><<<grid, 256, 0, st>>>(src, out, n);
        };
        go(4);                                          // untimed first pass
        (void)hipEventRecord(e0, st);
        go(iters);
        (void)hipEventRecord(e1, st);
        // per iteration a wave moves 16 KB (8 KB with the 8-byte transposed reads), 4 waves per workgroup
        *units = (double)grid * 4.0 * (kind == MOC_PROBE_LDS_READ_TRANSPOSED ? 8192.0 : 16384.0) * (double)iters;
    } else {
        const int grid = kProbeMfmaGrid;                // one workgroup per compute unit
        probe_mfma_kernel<<<grid, 512, 0, st>>>((float *)buf, 16);       // untimed first pass
        (void)hipEventRecord(e0, st);
        probe_mfma_kernel<<<grid, 512, 0, st>>>((float *)buf, iters);
        (void)hipEventRecord(e1, st);
        // 16 MFMAs per iteration per wave, 2*32*32*16 flops each, 8 waves per workgroup
        *units = 16.0 * 32768.0 * 8.0 * grid * (double)iters;
    }
    return hipGetLastError();
}

}  // namespace moc
