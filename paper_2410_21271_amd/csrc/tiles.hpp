// Device-side decoding of the tile-major stored formats into MFMA operand fragments.
//
// A 16 x 16 x 32 fp16 MFMA takes, per lane l = 16*j + n, eight fp16 of operand row n for the
// k-slots 8*j .. 8*j+7.  The stored tiles give every lane exactly the words of its row n and its
// column quarter j, so a 32-bit word of eight codes becomes one fragment without any cross-lane
// traffic.  Codes are turned into the EXACT integers (code - zero) in fp16; the group scale is
// applied afterwards in fp32 on the accumulator, so the effective weight scale*(code-zero) carries
// no rounding (asymmetric group-wise quantisation, Sec. 4.1 / App. A.11 of the paper).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace eora {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));

union Frag {
    h8 v;
    h2 p[4];
    uint32_t u[4];
    u4 q;
};

__device__ __forceinline__ h2 as_h2(uint32_t v) { return __builtin_bit_cast(h2, v); }

__device__ __forceinline__ f4 mfma16(h8 a, h8 b, f4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// fp16 bit patterns of (base + z) replicated in both halves, for the small integer z < 16.
// base = 1024, 128, 64, 16 have a mantissa unit of 1, 1/8, 1/16, 1/64.
__device__ __forceinline__ uint32_t k1024(uint32_t z) { return 0x64006400u | (z * 0x00010001u); }
__device__ __forceinline__ uint32_t k128(uint32_t z) { return 0x58005800u | (z * 0x00080008u); }
__device__ __forceinline__ uint32_t k64(uint32_t z) { return 0x54005400u | (z * 0x00100010u); }
__device__ __forceinline__ uint32_t k16(uint32_t z) { return 0x4C004C00u | (z * 0x00400040u); }

constexpr uint32_t MAGIC = 0x64006400u;   // fp16 1024.0 twice: OR-ing a small integer into the mantissa adds it

// (w & mask) | base in one instruction.  The compiler splits this into v_and + v_or when both
// constants are literals (a three-operand instruction takes no literal on this target).  Hiding the
// constants' values behind empty asm statements (no instruction is emitted) makes it see a scalar and
// a vector REGISTER operand, for which it selects the single v_and_or_b32 itself: that halves the
// bit-field extraction work that bounds the decode kernels.  (Writing the instruction as inline asm
// is not an option: the compiler inserts no MFMA wait states around instructions it cannot see.)
__device__ __forceinline__ uint32_t in_sgpr(uint32_t v)
{
    asm("" : "+s"(v));
    return v;
}
__device__ __forceinline__ uint32_t in_vgpr(uint32_t v)
{
    asm("" : "+v"(v));
    return v;
}
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask, uint32_t base) { return (w & in_sgpr(mask)) | base; }

// Eight 4-bit codes of one word -> (code - z) as eight fp16, columns in natural order.
// Nibble e holds column 2*(e%4) + e/4, so each mask yields two adjacent columns.
__device__ __forceinline__ h8 dq4_word(uint32_t w, uint32_t c1024, uint32_t c64)
{
    const h2 sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    const uint32_t hi = w >> 8, magic = in_vgpr(MAGIC);
    Frag f;
    f.p[0] = as_h2(and_or(w, 0x000F000Fu, magic)) - as_h2(c1024);                                  // 1024+q
    f.p[1] = __builtin_elementwise_fma(as_h2(and_or(w, 0x00F000F0u, magic)), sixteenth, -as_h2(c64));   // 1024+16q
    f.p[2] = as_h2(and_or(hi, 0x000F000Fu, magic)) - as_h2(c1024);
    f.p[3] = __builtin_elementwise_fma(as_h2(and_or(hi, 0x00F000F0u, magic)), sixteenth, -as_h2(c64));
    return f.v;
}

// Sixteen 2-bit codes of one word -> (code - z) as two fragments of eight fp16, columns in natural order.
// Pair p of adjacent columns sits at bits 2p of both 16-bit halves: masked in place it reads 1024 + 4^p * q
// for p < 4 (bits 8..15 after a shift by 8), and one fused multiply-add brings it to q - z exactly.
__device__ __forceinline__ void dq2_word(uint32_t w, uint32_t z, h8& lo, h8& hi8)
{
    const h2 quarter = {(_Float16)0.25f, (_Float16)0.25f};
    const h2 sixteenth = {(_Float16)0.0625f, (_Float16)0.0625f};
    const h2 sixtyfourth = {(_Float16)0.015625f, (_Float16)0.015625f};
    const h2 c1024 = as_h2(k1024(z)), c256 = as_h2(0x5C005C00u | (z * 0x00040004u)), c64 = as_h2(k64(z)), c16 = as_h2(k16(z));
    const uint32_t magic = in_vgpr(MAGIC);
    const uint32_t half[2] = {w, w >> 8};
    Frag f[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        f[i].p[0] = as_h2(and_or(half[i], 0x00030003u, magic)) - c1024;                                        // 1024+q
        f[i].p[1] = __builtin_elementwise_fma(as_h2(and_or(half[i], 0x000C000Cu, magic)), quarter, -c256);      // 1024+4q
        f[i].p[2] = __builtin_elementwise_fma(as_h2(and_or(half[i], 0x00300030u, magic)), sixteenth, -c64);     // 1024+16q
        f[i].p[3] = __builtin_elementwise_fma(as_h2(and_or(half[i], 0x00C000C0u, magic)), sixtyfourth, -c16);   // 1024+64q
    }
    lo = f[0].v;
    hi8 = f[1].v;
}

// Thirty-two 3-bit codes of one lane (three words) -> four fragments of (code - z).
__device__ __forceinline__ void dq3_lane(uint32_t d0, uint32_t d1, uint32_t d2, uint32_t z, h8 out[4])
{
    const h2 eighth = {(_Float16)0.125f, (_Float16)0.125f};
    const h2 sixtyfourth = {(_Float16)0.015625f, (_Float16)0.015625f};
    const h2 c1024 = as_h2(k1024(z)), c128 = as_h2(k128(z)), c16 = as_h2(k16(z));
    h2 pr[16];
    const uint32_t d[3] = {d0, d1, d2};
    const uint32_t MAGICV = in_vgpr(MAGIC);
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const uint32_t w = d[i], hi = w >> 9;
        pr[5 * i + 0] = as_h2(and_or(w, 0x00070007u, MAGICV)) - c1024;                                      // 1024+q
        pr[5 * i + 1] = __builtin_elementwise_fma(as_h2(and_or(w, 0x00380038u, MAGICV)), eighth, -c128);        // 1024+8q
        pr[5 * i + 2] = __builtin_elementwise_fma(as_h2(and_or(w, 0x01C001C0u, MAGICV)), sixtyfourth, -c16);    // 1024+64q
        pr[5 * i + 3] = as_h2(and_or(hi, 0x00070007u, MAGICV)) - c1024;
        pr[5 * i + 4] = __builtin_elementwise_fma(as_h2(and_or(hi, 0x00380038u, MAGICV)), eighth, -c128);
    }
    uint32_t last = and_or(d0 >> 15, 0x00010001u, MAGICV);     // bit b of the last pair is bit 15 / 31 of word b
    last = and_or(d1 >> 14, 0x00020002u, last);
    last = and_or(d2 >> 13, 0x00040004u, last);
    pr[15] = as_h2(last) - c1024;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        Frag f;
        f.p[0] = pr[4 * t + 0];
        f.p[1] = pr[4 * t + 1];
        f.p[2] = pr[4 * t + 2];
        f.p[3] = pr[4 * t + 3];
        out[t] = f.v;
    }
}

// ------------------------------------------------------------------------------------------------
// Codes as fp16 SUBNORMALS (decode kernel for one to four tokens).  A b-bit code left in place at bit p
// (p + b <= 10) of a 16-bit half, everything else masked off, IS the fp16 subnormal code * 2^(p-24): one AND per
// two weights, no OR and no subtraction (the fp16 MFMAs of this chip honour subnormal inputs exactly; checked
// on the device).  The position factor 2^p is taken out by the activations, which the kernel stages
// multiplied column by column with 2^-p (xscale_chunk below; exact in fp16 down to its subnormals), the common
// 2^-24 by one multiplication of the finished accumulator, and the zero-point by
//      sum_i (q_i - z) x_i = sum_i q_i x_i - z sum_i x_i
// with sum_i x_i formed once per (token, group) when x is staged.
template <int WORDS>
__device__ __forceinline__ void raw_tile(const uint32_t (&w)[WORDS], h8 (&b)[4])
{
    Frag f[4];
    if constexpr (WORDS == 4) {                            // Q4: word t = columns 8t .. 8t+7, pairs at bits 0, 4, 8, 12
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const uint32_t hi = w[t] >> 8;
            f[t].u[0] = w[t] & 0x000F000Fu;                // 2^-24
            f[t].u[1] = w[t] & 0x00F000F0u;                // 2^-20
            f[t].u[2] = hi & 0x000F000Fu;
            f[t].u[3] = hi & 0x00F000F0u;
        }
    } else if constexpr (WORDS == 3) {                     // Q3: pair p < 15 in word p/5 at bits 3(p%5); pair 15 in bit 15 of the words
        uint32_t pr[16];
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const uint32_t hi = w[i] >> 9;
            pr[5 * i + 0] = w[i] & 0x00070007u;            // 2^-24
            pr[5 * i + 1] = w[i] & 0x00380038u;            // 2^-21
            pr[5 * i + 2] = w[i] & 0x01C001C0u;            // 2^-18
            pr[5 * i + 3] = hi & 0x00070007u;
            pr[5 * i + 4] = hi & 0x00380038u;
        }
        uint32_t last = (w[0] >> 15) & 0x00010001u;
        last = and_or(w[1] >> 14, 0x00020002u, last);
        last = and_or(w[2] >> 13, 0x00040004u, last);
        pr[15] = last;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) f[t].u[e] = pr[4 * t + e];
    } else {                                               // Q2: word u = columns 16u .. 16u+15, pairs at bits 2p
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const uint32_t half[2] = {w[u], w[u] >> 8};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f[2 * u + h].u[0] = half[h] & 0x00030003u; // 2^-24
                f[2 * u + h].u[1] = half[h] & 0x000C000Cu; // 2^-22
                f[2 * u + h].u[2] = half[h] & 0x00300030u; // 2^-20
                f[2 * u + h].u[3] = half[h] & 0x00C000C0u; // 2^-18
            }
        }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) b[t] = f[t].v;
}

// What the staged activations are multiplied with so that raw_tile's position factors cancel: the factors of
// the eight columns 8c .. 8c+7 (c = 0..3) of a lane's 32 columns of a tile, i.e. of the 16-byte chunk number
// 4j + c of the tile's 128 columns.
template <int WORDS>
__device__ __forceinline__ h8 xscale_chunk(int c)
{
    const _Float16 o = (_Float16)1.0f, e = (_Float16)0.125f, q = (_Float16)0.25f, s = (_Float16)0.0625f, x = (_Float16)0.015625f;
    if constexpr (WORDS == 4) {
        return h8{o, o, s, s, o, o, s, s};
    } else if constexpr (WORDS == 2) {
        return h8{o, o, q, q, s, s, x, x};
    } else {
        // pairs 4c .. 4c+3 of the lane; pair p < 15 has the factor {1, 1/8, 1/64, 1, 1/8}[p % 5], pair 15 the factor 1
        const h8 c0 = {o, o, e, e, x, x, o, o}, c1 = {e, e, o, o, e, e, x, x}, c2 = {o, o, e, e, o, o, e, e}, c3 = {x, x, o, o, e, e, o, o};
        h8 r = c0;
        r = c == 1 ? c1 : r;
        r = c == 2 ? c2 : r;
        r = c == 3 ? c3 : r;
        return r;
    }
}

// zero-point nibble of row n of (row block R, quantisation group q)
__device__ __forceinline__ uint32_t load_zero(const uint32_t* __restrict__ qzeros, size_t rq, int n)
{
    const uint32_t w = qzeros[2 * rq + (n >> 3)];
    return (w >> (4 * (n & 7))) & 0xFu;
}

}  // namespace eora
