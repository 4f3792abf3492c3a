// Device-side building blocks shared by the MoC kernels (gfx950 only).
//
// MFMA operand/accumulator layouts used throughout (wave64):
//   v_mfma_f32_32x32x16_bf16  D[32x32] += A[32x16] * B[16x32]
//     A operand: lane l holds A[l%32][8*(l/32) .. +8]          (8 bf16 = 4 VGPRs)
//     B operand: lane l holds B[8*(l/32) .. +8][l%32]
//     accumulator: lane l, register i (0..15) holds
//                  D[(i/4)*8 + (l/32)*4 + i%4][l%32]
// A contraction index may be permuted freely as long as A and B use the same
// permutation; the kernels use that to feed an accumulator tile straight back
// in as the B operand of the next product (see acc_to_bfrag).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moc {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

// two floats -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2 v = {lo, hi};
    bf16x2 p = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, p);
}

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// Registers 8*s .. 8*s+7 of a 32x32 accumulator as one B (or A) operand whose
// contraction slot e of lane-half h corresponds to accumulator row
//   (2*s + e/4)*8 + 4*h + e%4.
__device__ __forceinline__ bf16x8 acc_to_frag(const f32x16 &acc, int s) {
    u32x4 r;
    r[0] = pack_bf16(acc[8 * s + 0], acc[8 * s + 1]);
    r[1] = pack_bf16(acc[8 * s + 2], acc[8 * s + 3]);
    r[2] = pack_bf16(acc[8 * s + 4], acc[8 * s + 5]);
    r[3] = pack_bf16(acc[8 * s + 6], acc[8 * s + 7]);
    return __builtin_bit_cast(bf16x8, r);
}

// 8 consecutive elements of a row, converted to bf16 if the storage is fp32.
template <typename T> struct Io;
template <> struct Io<bf16_t> {
    static __device__ __forceinline__ bf16x8 load8(const bf16_t *p) {
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(p));
    }
    static __device__ __forceinline__ void load8f(const bf16_t *p, float *f) {
        u32x4 u = *reinterpret_cast<const u32x4 *>(p);
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[2 * i] = bf16_lo(u[i]); f[2 * i + 1] = bf16_hi(u[i]); }
    }
    static __device__ __forceinline__ void store4(bf16_t *p, float a, float b, float c, float d) {
        u32x2 u = {pack_bf16(a, b), pack_bf16(c, d)};
        *reinterpret_cast<u32x2 *>(p) = u;
    }
    static __device__ __forceinline__ void store8(bf16_t *p, const float *f) {
        u32x4 u = {pack_bf16(f[0], f[1]), pack_bf16(f[2], f[3]), pack_bf16(f[4], f[5]), pack_bf16(f[6], f[7])};
        *reinterpret_cast<u32x4 *>(p) = u;
    }
};
template <> struct Io<float> {
    static __device__ __forceinline__ bf16x8 load8(const float *p) {
        f32x4 a = *reinterpret_cast<const f32x4 *>(p);
        f32x4 b = *reinterpret_cast<const f32x4 *>(p + 4);
        u32x4 r = {pack_bf16(a[0], a[1]), pack_bf16(a[2], a[3]), pack_bf16(b[0], b[1]), pack_bf16(b[2], b[3])};
        return __builtin_bit_cast(bf16x8, r);
    }
    static __device__ __forceinline__ void load8f(const float *p, float *f) {
        f32x4 a = *reinterpret_cast<const f32x4 *>(p);
        f32x4 b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) { f[i] = a[i]; f[4 + i] = b[i]; }
    }
    static __device__ __forceinline__ void store4(float *p, float a, float b, float c, float d) {
        f32x4 u = {a, b, c, d};
        *reinterpret_cast<f32x4 *>(p) = u;
    }
    static __device__ __forceinline__ void store8(float *p, const float *f) {
        f32x4 a = {f[0], f[1], f[2], f[3]}, b = {f[4], f[5], f[6], f[7]};
        *reinterpret_cast<f32x4 *>(p) = a;
        *reinterpret_cast<f32x4 *>(p + 4) = b;
    }
};

// exchange with the other half-wave (lane ^ 32)
__device__ __forceinline__ float xhalf(float v) { return __shfl_xor(v, 32, 64); }

// Row-major LDS tile [ROWS][D] of bf16 without padding; the 16-byte column
// groups of a row are XOR-swizzled by the row index so that BOTH access
// patterns below are bank-conflict free:
//   frag()   row operand: 16 consecutive rows read the same 16-byte group;
//   tfrag()  transposed operand through ds_read_b64_tr_b16: a 32-lane phase
//            reads a patch of 4 rows x 32 features.
// ds_read_b64_tr_b16 (gfx950): within each block of 16 lanes, lane i receives
// element (i & 3) of the 8-byte words addressed by lanes (i >> 2) + {0,4,8,12}.
// With lane j of a block pointing at (row R0 + j/4, features F0 + 4*(j%4) ..+4)
// lane i ends up with feature F0 + i of rows R0 .. R0+3: a 4 x 16 patch, transposed.
typedef short s16x4 __attribute__((ext_vector_type(4)));
template <int D> struct SwTile {
    static constexpr int CG = D / 8;
    static __device__ __forceinline__ int sw(int row) { return (((row & 3) << 2) | ((row >> 2) & 3)) & (CG - 1); }
    static __device__ __forceinline__ int off(int row, int cg) { return row * D + ((cg ^ sw(row)) << 3); }
    // row operand: row r, features [16*step + 8*half, +8)
    static __device__ __forceinline__ bf16x8 frag(const bf16_t *base, int r, int step, int half) {
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(base + off(r, 2 * step + half)));
    }
    // transposed operand for the lane's feature 32*db + (lane & 31): contraction
    // slots 0..3 -> rows 16*s + 4*half + {0..3}, slots 4..7 -> the same + 8
    // (the slot order of acc_to_frag).
    static __device__ __forceinline__ bf16x8 tfrag(const bf16_t *base, int lane, int db, int s) {
        const int i = lane & 15, bq = (lane >> 4) & 1, half = lane >> 5;
        const int x = 32 * db + 16 * bq + 4 * (i & 3);
        const int r0 = 16 * s + 4 * half + (i >> 2);
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const bf16_t *p0 = base + off(r0, x >> 3) + (x & 7);
        const bf16_t *p1 = base + off(r0 + 8, x >> 3) + (x & 7);
        s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p0);
        s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p1);
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        s16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
        return __builtin_bit_cast(bf16x8, r);
    }
};

// Lane-dependent byte offsets into a SwTile<D>. They do not depend on the tile's
// base address, on which 32-row block (row reads) or on which 16-row step
// (transposed reads) is addressed: all of that goes into the instruction's
// immediate offset, so one set of 8 + 8 registers serves every buffer.
// pin() hides the values from loop-invariant code motion; without it the
// compiler materialises one address register per (buffer, block, step).
template <int D> struct LaneOffs {
    static constexpr int KS = D / 16, DB = D / 32;
    int row[KS];        // row operand: row (lane & 31), features [16 s + 8 half, +8)
    int tr[2 * DB];     // transposed operand: [2 db + second]
    __device__ __forceinline__ void init(int lane) {
        const int half = lane >> 5, l32 = lane & 31;
#pragma unroll
        for (int s = 0; s < KS; ++s) row[s] = SwTile<D>::off(l32, 2 * s + half) * 2;
        const int i = lane & 15, bq = (lane >> 4) & 1;
#pragma unroll
        for (int u = 0; u < 2 * DB; ++u) {
            const int x = 32 * (u >> 1) + 16 * bq + 4 * (i & 3);
            const int r0 = 4 * half + (i >> 2) + 8 * (u & 1);
            tr[u] = (SwTile<D>::off(r0, x >> 3) + (x & 7)) * 2;
        }
    }
    __device__ __forceinline__ void pin() {
#pragma unroll
        for (int s = 0; s < KS; ++s) asm volatile("" : "+v"(row[s]));
#pragma unroll
        for (int u = 0; u < 2 * DB; ++u) asm volatile("" : "+v"(tr[u]));
    }
    // row operand of rows [row0, row0+32) (row0 a multiple of 32) of the tile at byte offset `tile`
    template <int TILE_ROW0_BYTES>
    __device__ __forceinline__ bf16x8 frag(const char *smem, int s) const {
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(smem + row[s] + TILE_ROW0_BYTES));
    }
    // transposed operand, feature block db, source rows [row0, row0+16) (row0 a multiple of 16)
    template <int TILE_ROW0_BYTES>
    __device__ __forceinline__ bf16x8 tfrag(const char *smem, int db) const {
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + tr[2 * db] + TILE_ROW0_BYTES));
        s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(smem + tr[2 * db + 1] + TILE_ROW0_BYTES));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        s16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
        return __builtin_bit_cast(bf16x8, r);
    }
};

// s_waitcnt that only bounds the number of outstanding vector-memory operations
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}
// s_waitcnt that only waits for the wave's LDS (and scalar-memory) operations
__device__ __forceinline__ void wait_lgkm0() { __builtin_amdgcn_s_waitcnt(0xC07F); }
// ... until at most N of them are outstanding. LDS operations complete in order, so this means: every LDS
// operation older than the N youngest is done (outstanding scalar loads only make the wait longer).
template <int N> __device__ __forceinline__ void wait_lgkm() {
    static_assert(N >= 0 && N < 16, "lgkmcnt range");
    __builtin_amdgcn_s_waitcnt(0xC07F | (N << 8));
}

// Asynchronous global -> LDS copies (global_load_lds): every lane moves BYTES
// bytes from its own global address to LDS address  base + lane * BYTES, where
// base is wave-uniform (it travels in M0). The copy completes out of sight of
// the wave; it counts in vmcnt like any vector-memory load.
// They are written as inline assembly on purpose. Given the intrinsic, the
// compiler treats every later LDS read as depending on the newest copy and
// puts an s_waitcnt vmcnt(0) in front of it, which drains the very prefetch
// the copy was issued for. Issued this way the compiler does not know about
// them, so the CALLER orders them: wait_vmcnt<N>() (N = copies this wave has
// issued since the ones it needs) and then a workgroup barrier before any lane
// reads what other waves copied.
// a pointer the caller knows to be wave-uniform, in scalar registers whatever the compiler's analysis says
__device__ __forceinline__ const void *uniform_ptr(const void *p) {
    const uint64_t b = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b), hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    return (const void *)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
// Read-only table word at a wave-uniform index through the scalar cache (s_load): unlike a vector
// load it does not enter the vector-memory counter that orders the asynchronous tile copies.
__device__ __forceinline__ uint32_t uniform_load_u32(const uint32_t *table, int idx) {
    const __attribute__((address_space(4))) uint32_t *t =
        (const __attribute__((address_space(4))) uint32_t *)(uintptr_t)table;
    return t[__builtin_amdgcn_readfirstlane(idx)];
}
__device__ __forceinline__ uint32_t lds_address(const void *p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char *)p;
}
__device__ __forceinline__ void async_copy16(const void *g, void *lds) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(g), "s"(__builtin_amdgcn_readfirstlane(lds_address(lds))) : "memory", "m0");
}
// wave-uniform base pointer + 32-bit unsigned byte offset per lane
__device__ __forceinline__ void async_copy16(const void *base, uint32_t off, void *lds) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(off), "s"(uniform_ptr(base)), "s"(__builtin_amdgcn_readfirstlane(lds_address(lds))) : "memory", "m0");
}
// the same with the LDS destination given as an address (see lds_address)
__device__ __forceinline__ void async_copy16_at(const void *g, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(g), "s"(__builtin_amdgcn_readfirstlane(lds)) : "memory", "m0");
}
__device__ __forceinline__ void async_copy16_at(const void *base, uint32_t off, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(off), "s"(uniform_ptr(base)), "s"(__builtin_amdgcn_readfirstlane(lds)) : "memory", "m0");
}
__device__ __forceinline__ void async_copy4_at(const void *g, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" :: "v"(g), "s"(__builtin_amdgcn_readfirstlane(lds)) : "memory", "m0");
}
__device__ __forceinline__ void async_copy4_at(const void *base, uint32_t off, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :: "v"(off), "s"(uniform_ptr(base)), "s"(__builtin_amdgcn_readfirstlane(lds)) : "memory", "m0");
}

// max (or sum) of a value with its counterpart in the other half-wave, in all
// lanes, without going through LDS (v_permlane32_swap)
__device__ __forceinline__ float xhalf_max(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

}  // namespace moc
