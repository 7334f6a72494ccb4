// Device-side building blocks shared by the gfx950 kernels: packed-layout geometry and the
// in-register unpack of 4-/8-bit codes to exact fp16 integers.
//
// Packed layout (layout version 1): tiles of 16 rows x TK columns (TK = 128 for 4-bit, 64 for
// 8-bit), 1024 bytes each, stored [N/16][K/TK]; lane l of a wavefront owns the 16-byte chunk l
// of a tile: row l % 16, column-quarter kq = l / 16; word/byte order as documented in rtn.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rtn {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

template <int BITS> struct Layout;
template <> struct Layout<4> {
    static constexpr int TK = 128;       // columns per 1 KiB tile
    static constexpr int MFMA_PER_TILE = 4;
    static constexpr int QMAX = 7;
    static constexpr int QMIN = -8;
    static constexpr int BIAS = 8;
};
template <> struct Layout<8> {
    static constexpr int TK = 64;
    static constexpr int MFMA_PER_TILE = 2;
    static constexpr int QMAX = 127;
    static constexpr int QMIN = -128;
    static constexpr int BIAS = 128;
};

__device__ __forceinline__ half2_t as_half2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }

union Half8Words {
    half8_t v;
    half2_t h2[4];
};

// fp16 1024.0 in both halves, materialised once in a vector register.  0x6400 is fp16 1024, whose
// ulp is 1: or-ing a nibble or byte into the mantissa gives 1024 + n exactly.
__device__ __forceinline__ uint32_t fp16_magic_vgpr() {
    uint32_t m;
    asm volatile("v_mov_b32 %0, 0x64006400" : "=v"(m));
    return m;
}

// (x & mask) | magic in one instruction.  gfx9-family VOP3 encodings take no literal and at most
// one scalar operand, so the mask lives in an SGPR and the magic in a VGPR; left to itself the
// compiler emits a separate and + or with two literals.
__device__ __forceinline__ uint32_t and_or(uint32_t x, uint32_t mask, uint32_t magic_v) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "s"(mask), "v"(magic_v));
    return r;
}

// One 32-bit word of 4-bit codes (offset binary, nibble order {0,4,1,5,2,6,3,7}) -> the 8 fp16
// values one lane feeds to one 16x16x32 MFMA: and_or puts two nibbles under the 1024 exponent
// (1024 + n, or 1024 + 16 n for a nibble sitting 4 bits up), one packed add / fma removes the
// offset exactly.  9 vector ops per 8 weights.
__device__ __forceinline__ half8_t unpack_word4_off(uint32_t w, uint32_t magic_v, half2_t sub_lo, half2_t add_hi) {
    const half2_t k16th = {(half_t)0.0625f, (half_t)0.0625f};
    const uint32_t w8 = w >> 8;
    Half8Words r;
    r.h2[0] = as_half2(and_or(w, 0x000F000Fu, magic_v)) - sub_lo;                                 // nibbles 0,4
    r.h2[1] = __builtin_elementwise_fma(as_half2(and_or(w, 0x00F000F0u, magic_v)), k16th, add_hi);   // nibbles 1,5
    r.h2[2] = as_half2(and_or(w8, 0x000F000Fu, magic_v)) - sub_lo;                                // nibbles 2,6
    r.h2[3] = __builtin_elementwise_fma(as_half2(and_or(w8, 0x00F000F0u, magic_v)), k16th, add_hi);  // nibbles 3,7
    return r.v;
}

__device__ __forceinline__ half8_t unpack_word4(uint32_t w, uint32_t magic_v) {
    const half2_t k1032 = {(half_t)1032.0f, (half_t)1032.0f};
    const half2_t k72 = {(half_t)-72.0f, (half_t)-72.0f};
    return unpack_word4_off(w, magic_v, k1032, k72);
}

// Two 32-bit words of 8-bit codes (offset binary, natural byte order) -> 8 fp16 values.
// A byte permute places each byte under a 0x64 exponent byte (1024 + byte), one packed add
// removes 1024 + 128.  8 vector ops per 8 weights.
__device__ __forceinline__ half8_t unpack_words8_off(uint32_t w0, uint32_t w1, half2_t sub) {
    const uint32_t E = 0x64646464u;
    Half8Words r;
    r.h2[0] = as_half2(__builtin_amdgcn_perm(E, w0, 0x04010400u)) - sub;
    r.h2[1] = as_half2(__builtin_amdgcn_perm(E, w0, 0x04030402u)) - sub;
    r.h2[2] = as_half2(__builtin_amdgcn_perm(E, w1, 0x04010400u)) - sub;
    r.h2[3] = as_half2(__builtin_amdgcn_perm(E, w1, 0x04030402u)) - sub;
    return r.v;
}

__device__ __forceinline__ half8_t unpack_words8(uint32_t w0, uint32_t w1) {
    const half2_t k1152 = {(half_t)1152.0f, (half_t)1152.0f};
    return unpack_words8_off(w0, w1, k1152);
}

// MFMA operand number i (0 .. MFMA_PER_TILE-1) of a 16-byte tile chunk.
template <int BITS>
__device__ __forceinline__ half8_t unpack_operand(const u32x4_t& chunk, int i, uint32_t magic_v) {
    if constexpr (BITS == 4) {
        return unpack_word4(chunk[i], magic_v);
    } else {
        return unpack_words8(chunk[2 * i], chunk[2 * i + 1]);
    }
}

// The same with a per-lane integer zero point Z (asymmetric variant): the operand holds q + Z, exact for |Z| <= 2^(BITS-1)
// (1024 + 2^(BITS-1) - Z and 64 + 2^(BITS-1) - Z are fp16 integers, so the subtraction is still exact).
template <int BITS>
__device__ __forceinline__ half8_t unpack_operand_zp(const u32x4_t& chunk, int i, uint32_t magic_v, float z) {
    if constexpr (BITS == 4) {
        const half_t lo = (half_t)(1032.0f - z), hi = (half_t)(z - 72.0f);
        return unpack_word4_off(chunk[i], magic_v, (half2_t){lo, lo}, (half2_t){hi, hi});
    } else {
        const half_t lo = (half_t)(1152.0f - z);
        return unpack_words8_off(chunk[2 * i], chunk[2 * i + 1], (half2_t){lo, lo});
    }
}

// Streaming (read-once) 16-byte load of packed weights.
__device__ __forceinline__ u32x4_t load_stream16(const void* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
}

}  // namespace rtn
