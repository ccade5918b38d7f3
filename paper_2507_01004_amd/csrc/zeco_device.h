// Device-side helpers shared by the gfx950 kernels: vector types, bf16 packing, MFMA tile traits.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "zeco_internal.h"

namespace zeco {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kChunk = 64;  // chunk length C; equals the wavefront width

// Two floats -> packed bf16 pair (round to nearest even), low half = a.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
    bf16x2 r;
    r[0] = (__bf16)a;
    r[1] = (__bf16)b;
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) {
    return __builtin_bit_cast(float, w & 0xffff0000u);
}

// Natural exponential through the hardware exp2 (relative error ~1e-6 over the ranges used here).
__device__ __forceinline__ float fast_exp(float x) { return __expf(x); }

// Traits of the two bf16 MFMA shapes used.  A wave computes D[M x N] += A[M x K] B[K x N] with
// M = N = TILE.  Lane l holds column (l % TILE) of D; with kg = l / TILE, accumulator register r
// holds row `row(r, kg)`.  For A (B) lane l holds row (column) l % TILE and the 8 consecutive
// k-slots 8*kg .. 8*kg+7.
template <int TILE> struct Mma;

template <> struct Mma<16> {
    typedef f32x4 acc_t;
    static constexpr int kAcc = 4;   // accumulator registers per tile
    static constexpr int kK = 32;    // K extent of one instruction
    static constexpr int kGroups = 4;
    __device__ static __forceinline__ acc_t run(bf16x8 a, bf16x8 b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ constexpr int row(int r, int kg) { return 4 * kg + r; }
};

template <> struct Mma<32> {
    typedef f32x16 acc_t;
    static constexpr int kAcc = 16;
    static constexpr int kK = 16;
    static constexpr int kGroups = 2;
    __device__ static __forceinline__ acc_t run(bf16x8 a, bf16x8 b, acc_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    __device__ static __forceinline__ constexpr int row(int r, int kg) {
        return 8 * (r / 4) + 4 * kg + (r % 4);
    }
};

// fp32 MFMA 16x16x4: lane l holds A[l%16][l/16], B[l/16][l%16]; D register r holds row 4*(l/16)+r,
// column l%16.
__device__ __forceinline__ f32x4 mma_f32(float a, float b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// 16-byte LDS / global accessors on raw byte pointers.
__device__ __forceinline__ bf16x8 lds_frag(const unsigned char *base, int byte_off) {
    return *reinterpret_cast<const bf16x8 *>(base + byte_off);
}

// Four consecutive gate values of one token, as loaded and as floats.
template <int GM> struct GateVal;
template <> struct GateVal<kGateF32> {
    typedef f32x4 raw_t;
    __device__ static __forceinline__ f32x4 get(raw_t r) { return r; }
};
template <> struct GateVal<kGateHead> {
    typedef float raw_t;
    __device__ static __forceinline__ f32x4 get(raw_t r) { return f32x4{r, r, r, r}; }
};
template <> struct GateVal<kGateBF16> {
    typedef u32x2 raw_t;
    __device__ static __forceinline__ f32x4 get(raw_t r) {
        return f32x4{bf16_lo(r[0]), bf16_hi(r[0]), bf16_lo(r[1]), bf16_hi(r[1])};
    }
};

// N consecutive bf16 values (two per word) stored as one LDS write.
template <int N> struct TokenRun;
template <> struct TokenRun<8> {
    uint32_t w[4];
    __device__ __forceinline__ void store(unsigned char *dst) const {
        *reinterpret_cast<u32x4 *>(dst) = u32x4{w[0], w[1], w[2], w[3]};
    }
};
template <> struct TokenRun<4> {
    uint32_t w[2];
    __device__ __forceinline__ void store(unsigned char *dst) const {
        *reinterpret_cast<u32x2 *>(dst) = u32x2{w[0], w[1]};
    }
};
template <> struct TokenRun<2> {
    uint32_t w[1];
    __device__ __forceinline__ void store(unsigned char *dst) const {
        *reinterpret_cast<uint32_t *>(dst) = w[0];
    }
};

// Low halves / high halves of two packed bf16 pairs: (x.lo, y.lo) and (x.hi, y.hi).
__device__ __forceinline__ uint32_t pair_lo(uint32_t x, uint32_t y) {
    return __builtin_amdgcn_perm(y, x, 0x05040100u);
}
__device__ __forceinline__ uint32_t pair_hi(uint32_t x, uint32_t y) {
    return __builtin_amdgcn_perm(y, x, 0x07060302u);
}

// MFMA operand fragment from a TOKEN-major bf16 tile through gfx950's transposing LDS read
// (ds_read_b64_tr_b16).  In every group of 16 lanes, lane 4 k + r supplies the address of four
// consecutive elements of tile row k (8 bytes), and lane 4 r' + e receives, as its element k, element e
// of what lane 4 k + r' supplied: the group turns a patch of 4 tokens x 16 channels into 16 lanes
// (channels) x 4 tokens.  `addr` is this lane's address for tokens row0 .. row0+3 (row0 + k for its
// k = (lane % 16) / 4, columns 4 r ..); the second read, `second` bytes further, fills the lane's
// other four k-slots, and the lane ends up with 8 tokens of its own channel, which is the operand
// layout of the 32x32x16 MFMA (lane = row or column lt, k-slots = 8 tokens).  Which tokens the rows are
// is up to the caller: a contraction does not care about the order of its k-slots as long as both
// operands agree.
typedef __attribute__((ext_vector_type(4))) short s16x4;
__device__ __forceinline__ bf16x8 lds_frag_tr(const unsigned char *addr, int second) {
    typedef __attribute__((address_space(3))) s16x4 *lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(addr));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(addr + second));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
}

}  // namespace zeco
