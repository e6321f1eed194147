// Register-level decoding of packed codes into FP16 MFMA operands (gfx950).
//
// A slot is 32 consecutive codes of one group: four 32-bit words (4-bit) or three words plus
// the group's tail word (3-bit).  Inside a word, even positions live in the low half-word and odd
// positions in the high half-word, so (word & mask) picks one code into each half.  OR-ing the
// bits of a power of two whose ulp equals the code's bit weight turns the pair into the two FP16
// numbers 2^e + q without any shift or conversion:
//      bits 0..3  | 0x6400 -> 1024 + q        bits 4..7 | 0x5400 -> 64 + q          (4-bit)
//      bits 0..2  | 0x6400 -> 1024 + q        bits 3..5 | 0x5800 -> 128 + q
//      bits 6..8  | 0x4C00 -> 16 + q                                                 (3-bit)
// One packed FP16 add of -(2^e + z) then gives the exact integers q - z (Sec. 3.2, Eq. 10 without
// the scale).  The constants -(2^e + z) are built with integer ops from z (z < 16 fits the mantissa).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gwq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// A constant the optimiser cannot see through.  With mask and magic in registers, (x & mask) | magic
// selects the single three-operand v_and_or_b32; as literals it would become two instructions.
__device__ inline uint32_t opaque(uint32_t c)
{
    uint32_t r;
    asm("s_mov_b32 %0, %1" : "=s"(r) : "i"(c));
    return r;
}
__device__ inline uint32_t opaque_v(uint32_t c)
{
    uint32_t r;
    asm("v_mov_b32 %0, %1" : "=v"(r) : "i"(c));
    return r;
}

// Sixteen bytes at 4-byte alignment (gfx950 global memory takes unaligned vector loads): the 3-bit
// slots start every 12 bytes.
struct __attribute__((packed, aligned(4))) U128a4 { uint32_t x, y, z, w; };

// Masks (SGPR) and magic numbers (VGPR) of the decoders, materialised once per kernel.
struct DecodeConsts {
    uint32_t m0, m1, m2, k1024, kmid, k16;
    __device__ inline explicit DecodeConsts(int bits)
    {
        if (bits == 4) {
            m0 = opaque(0x000F000Fu); m1 = opaque(0x00F000F0u); m2 = 0;
            k1024 = opaque_v(0x64006400u); kmid = opaque_v(0x54005400u); k16 = 0;
        } else {
            m0 = opaque(0x00070007u); m1 = opaque(0x00380038u); m2 = opaque(0x01C001C0u);
            k1024 = opaque_v(0x64006400u); kmid = opaque_v(0x58005800u); k16 = opaque_v(0x4C004C00u);
        }
    }
};

__device__ inline uint32_t and_or(uint32_t x, uint32_t mask, uint32_t magic) { return (x & mask) | magic; }

__device__ inline uint32_t pk_add(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2v, a) + __builtin_bit_cast(half2v, b));
}
__device__ inline uint32_t pk_mul(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2v, a) * __builtin_bit_cast(half2v, b));
}

// Per-group constants derived from the zero point: -(2^e + z) in both halves.
template <int BITS> struct ZeroConsts;
template <> struct ZeroConsts<4> {
    uint32_t c1024, c64;
    __device__ inline explicit ZeroConsts(uint32_t z)
    {
        // one 24-bit multiply-add each: the products never carry into the constants' set bits
        c1024 = z * 0x10001u + 0xE400E400u;    // -(1024 + z): ulp is 1 in [1024, 2048)
        c64 = z * 0x100010u + 0xD400D400u;     // -(64 + z):   ulp is 1/16 in [64, 128)
    }
};
template <> struct ZeroConsts<3> {
    uint32_t c1024, c128, c16;
    __device__ inline explicit ZeroConsts(uint32_t z)
    {
        c1024 = z * 0x10001u + 0xE400E400u;
        c128 = z * 0x80008u + 0xD800D800u;     // -(128 + z): ulp is 1/8 in [128, 256)
        c16 = z * 0x400040u + 0xCC00CC00u;     // -(16 + z):  ulp is 1/64 in [16, 32)
    }
};

// One 4-bit word (8 codes) -> 8 FP16 values q - z in position order.
__device__ inline u32x4 decode_word4(uint32_t x, const ZeroConsts<4> &c, const DecodeConsts &d)
{
    const uint32_t y = x >> 8;
    u32x4 r;
    r.x = pk_add(and_or(x, d.m0, d.k1024), c.c1024);
    r.y = pk_add(and_or(x, d.m1, d.kmid), c.c64);
    r.z = pk_add(and_or(y, d.m0, d.k1024), c.c1024);
    r.w = pk_add(and_or(y, d.m1, d.kmid), c.c64);
    return r;
}

// 4-bit slot: words w[0..3] -> operands f[0..3] (8 codes each).
__device__ inline void decode_slot4(const uint32_t w[4], uint32_t z, const DecodeConsts &d, u32x4 f[4])
{
    const ZeroConsts<4> c(z);
#pragma unroll
    for (int j = 0; j < 4; ++j) f[j] = decode_word4(w[j], c, d);
}

// The same for a slot whose two halves (codes 0..15 and 16..31) have zero points of their own: groups of 16.
__device__ inline void decode_slot4_halves(const uint32_t w[4], uint32_t z_lo, uint32_t z_hi, const DecodeConsts &d, u32x4 f[4])
{
    const ZeroConsts<4> c_lo(z_lo), c_hi(z_hi);
    f[0] = decode_word4(w[0], c_lo, d);
    f[1] = decode_word4(w[1], c_lo, d);
    f[2] = decode_word4(w[2], c_hi, d);
    f[3] = decode_word4(w[3], c_hi, d);
}

// 3-bit slot: words w[0..2] hold codes 0..29 (five pairs each), `tail_pair` holds codes 30, 31 in
// bits 0..2 and 16..18 (the caller shifts the group's tail word by 3 * slot).
__device__ inline void decode_slot3(const uint32_t w[3], uint32_t tail_pair, uint32_t z, const DecodeConsts &d,
                                    u32x4 f[4])
{
    const ZeroConsts<3> c(z);
    uint32_t p[16];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const uint32_t x = w[i], y = x >> 9;
        p[5 * i + 0] = pk_add(and_or(x, d.m0, d.k1024), c.c1024);
        p[5 * i + 1] = pk_add(and_or(x, d.m1, d.kmid), c.c128);
        p[5 * i + 2] = pk_add(and_or(x, d.m2, d.k16), c.c16);
        p[5 * i + 3] = pk_add(and_or(y, d.m0, d.k1024), c.c1024);
        p[5 * i + 4] = pk_add(and_or(y, d.m1, d.kmid), c.c128);
    }
    p[15] = pk_add(and_or(tail_pair, d.m0, d.k1024), c.c1024);
#pragma unroll
    for (int j = 0; j < 4; ++j) f[j] = u32x4{p[4 * j], p[4 * j + 1], p[4 * j + 2], p[4 * j + 3]};
}

// The same with one zero point for codes 0..15 (pairs 0..7: word 0 and the first three pairs of word 1) and
// one for codes 16..31.
__device__ inline void decode_slot3_halves(const uint32_t w[3], uint32_t tail_pair, uint32_t z_lo, uint32_t z_hi,
                                           const DecodeConsts &d, u32x4 f[4])
{
    const ZeroConsts<3> c_lo(z_lo), c_hi(z_hi);
    uint32_t p[16];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const uint32_t x = w[i], y = x >> 9;
        const ZeroConsts<3> &c0 = i == 0 ? c_lo : c_hi;                     // pairs 5i+3, 5i+4
        const ZeroConsts<3> &c1 = i <= 1 ? c_lo : c_hi;                     // pairs 5i .. 5i+2
        p[5 * i + 0] = pk_add(and_or(x, d.m0, d.k1024), c1.c1024);
        p[5 * i + 1] = pk_add(and_or(x, d.m1, d.kmid), c1.c128);
        p[5 * i + 2] = pk_add(and_or(x, d.m2, d.k16), c1.c16);
        p[5 * i + 3] = pk_add(and_or(y, d.m0, d.k1024), c0.c1024);
        p[5 * i + 4] = pk_add(and_or(y, d.m1, d.kmid), c0.c128);
    }
    p[15] = pk_add(and_or(tail_pair, d.m0, d.k1024), c_hi.c1024);
#pragma unroll
    for (int j = 0; j < 4; ++j) f[j] = u32x4{p[4 * j], p[4 * j + 1], p[4 * j + 2], p[4 * j + 3]};
}

// ---- bfloat16 operands -------------------------------------------------------------------------
// bfloat16 has 7 mantissa bits, so only a code that sits in bits 0..3 of its half-word can be turned into a number
// by an OR: ((x >> shift) & mask) | 0x4300 is 128 + q (ulp 1 in [128, 256)), one shift and one and-or per pair of
// codes.  gfx950 has no packed bfloat16 add to take 128 + z off again: the kernels multiply with 128 + q and
// subtract (128 + z) * sum_k x from the FP32 sum of the group, which they get from one more MFMA against ones.
struct DecodeConstsBf16 {
    uint32_t m, k128;
    __device__ inline explicit DecodeConstsBf16(int bits)
    {
        m = opaque(bits == 4 ? 0x000F000Fu : 0x00070007u);
        k128 = opaque_v(0x43004300u);
    }
};
constexpr uint32_t kBf16Ones = 0x3F803F80u;            // the pair (1.0, 1.0)

// 4-bit slot: words w[0..3] -> operands f[0..3], eight values 128 + q each in position order.
__device__ inline void decode_slot4_bf16(const uint32_t w[4], const DecodeConstsBf16 &d, u32x4 f[4])
{
#pragma unroll
    for (int j = 0; j < 4; ++j)
        f[j] = u32x4{and_or(w[j], d.m, d.k128), and_or(w[j] >> 4, d.m, d.k128), and_or(w[j] >> 8, d.m, d.k128),
                     and_or(w[j] >> 12, d.m, d.k128)};
}

// 3-bit slot (layout as decode_slot3): pair t of word i sits at bits 3t of both half-words.
__device__ inline void decode_slot3_bf16(const uint32_t w[3], uint32_t tail_pair, const DecodeConstsBf16 &d, u32x4 f[4])
{
    uint32_t p[16];
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int t = 0; t < 5; ++t) p[5 * i + t] = and_or(w[i] >> (3 * t), d.m, d.k128);
    p[15] = and_or(tail_pair, d.m, d.k128);
#pragma unroll
    for (int j = 0; j < 4; ++j) f[j] = u32x4{p[4 * j], p[4 * j + 1], p[4 * j + 2], p[4 * j + 3]};
}

// f[0], f[1] (codes 0..15 of a slot) times the packed FP16 pair s_lo, f[2], f[3] times s_hi.
__device__ inline void scale_halves(u32x4 f[4], uint32_t s_lo, uint32_t s_hi)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t s2 = j < 2 ? s_lo : s_hi;
        f[j].x = pk_mul(f[j].x, s2); f[j].y = pk_mul(f[j].y, s2);
        f[j].z = pk_mul(f[j].z, s2); f[j].w = pk_mul(f[j].w, s2);
    }
}

}  // namespace gwq
