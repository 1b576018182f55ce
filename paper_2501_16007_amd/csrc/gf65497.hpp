// Arithmetic in GF(p), p = 65497 = 2^16 - 39, for gfx950 integer ALUs.
//
// The field is the modulus M of the paper's polynomial congruence (Appendix C,
// Algorithms 3 and 5).  Every operand is < 2^16, so products fit 32 bits and the
// full-rate 24-bit multiplier (v_mul_u32_u24 / v_mad_u32_u24) is exact.
// Reduction folds the high half down with 2^16 = 39 (mod p): no division, no
// 32-bit multiply-high, no floating point.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace toploc {

constexpr uint32_t kPrime = 65497u;
constexpr uint32_t kFold16 = 39u;    // 2^16 mod p
constexpr uint32_t kFold32 = 1521u;  // 2^32 mod p = 39^2

// exact product of two operands < 2^24 whose product fits 32 bits, on the full-rate
// 24-bit multiplier (HIP declares __umul24 as returning int: keep it unsigned)
__device__ __forceinline__ uint32_t mul24(uint32_t a, uint32_t b)
{
    return (uint32_t)__umul24(a, b);
}

// (v >> 16) * 39 + (v & 0xFFFF): one folding step, congruent to v
__device__ __forceinline__ uint32_t fold16(uint32_t v)
{
    return mul24(v >> 16, kFold16) + (v & 0xFFFFu);
}

// v < 2p -> v mod p: v - p wraps to a huge value exactly when v < p
__device__ __forceinline__ uint32_t below_2p(uint32_t v)
{
    const uint32_t w = v - kPrime;
    return w < v ? w : v;
}

// any 32-bit v -> v mod p
__device__ __forceinline__ uint32_t reduce32(uint32_t v)
{
    v = fold16(v);  // < 40 * 2^16
    v = fold16(v);  // <= 39*39 + 65535 < 2p
    return below_2p(v);
}

// a, b < 2^16
__device__ __forceinline__ uint32_t mulmod(uint32_t a, uint32_t b)
{
    return reduce32(mul24(a, b));
}

// a*b + c with a, b, c < p: (p-1)^2 + (p-1) < 2^32, so one reduction suffices
// (this is one step of Horner's rule, Algorithm 5).
__device__ __forceinline__ uint32_t muladdmod(uint32_t a, uint32_t b, uint32_t c)
{
    return reduce32(mul24(a, b) + c);
}

__device__ __forceinline__ uint32_t submod(uint32_t a, uint32_t b)  // a, b < p
{
    return a >= b ? a - b : a + kPrime - b;
}

// a sum of fewer than 2^20 products of 16-bit operands -> mod p
__device__ __forceinline__ uint32_t reduce64(uint64_t acc)
{
    uint32_t lo = reduce32((uint32_t)acc);
    uint32_t hi = (uint32_t)(acc >> 32);                 // < 2^20
    return reduce32(lo + reduce32(hi) * kFold32);        // < p + p*1521 < 2^32
}

// a^(p-2): the inverse of a != 0 by Fermat's little theorem (replaces the
// extended Euclid of Algorithm 4; the inverse is unique, so the result is the same).
// p - 2 = 65495 = 0b1111111111010111, taken three bits at a time where they are 111:
// 16 squarings and 6 multiplications.
__device__ __forceinline__ uint32_t invmod(uint32_t a)
{
    const uint32_t a3 = mulmod(mulmod(a, a), a);
    const uint32_t a7 = mulmod(mulmod(a3, a3), a);
    auto sq3 = [](uint32_t r) { r = mulmod(r, r); r = mulmod(r, r); return mulmod(r, r); };
    uint32_t r = a7;                       // 111
    r = mulmod(sq3(r), a7);                // 111111
    r = mulmod(sq3(r), a7);                // 111111111
    r = mulmod(mulmod(r, r), a);           // 1111111111
    r = mulmod(r, r);                      // 11111111110
    r = mulmod(mulmod(r, r), a);           // 111111111101
    r = mulmod(r, r);                      // 1111111111010
    return mulmod(sq3(r), a7);             // 1111111111010111
}

// The field as the interpolation and evaluation code sees it.
struct Field16 {
    typedef uint16_t elem_t;                 // a residue in LDS
    static constexpr uint32_t P = kPrime;
    static constexpr int WORDS = 1;          // 16-bit words of an encoded coefficient

    static __device__ __forceinline__ uint32_t from_pattern(uint32_t bits) { return bits >= P ? bits - P : bits; }
    // (i mod m) < 65536 < 2p: residues 65497..65535 alias 0..38
    static __device__ __forceinline__ uint32_t from_residue(uint32_t x) { return x >= P ? x - P : x; }
    static __device__ __forceinline__ uint32_t mulmod(uint32_t a, uint32_t b) { return toploc::mulmod(a, b); }
    static __device__ __forceinline__ uint32_t muladdmod(uint32_t a, uint32_t b, uint32_t c)
    {
        return toploc::muladdmod(a, b, c);
    }
    static __device__ __forceinline__ uint32_t addmod(uint32_t a, uint32_t b)   // a, b < p
    {
        return below_2p(a + b);
    }
    static __device__ __forceinline__ uint32_t submod(uint32_t a, uint32_t b) { return toploc::submod(a, b); }
    static __device__ __forceinline__ uint32_t neg(uint32_t a) { return a ? P - a : 0u; }
    static __device__ __forceinline__ uint32_t inv(uint32_t a) { return invmod(a); }
    // sum of fewer than 2^20 products of residues, unreduced in 64 bits
    struct Acc {
        uint64_t v;
        __device__ __forceinline__ Acc() : v(0) {}
        __device__ __forceinline__ void mac(uint32_t a, uint32_t b) { v += (uint64_t)mul24(a, b); }
        __device__ __forceinline__ void add(uint32_t x) { v += x; }
        __device__ __forceinline__ uint32_t reduce() const { return reduce64(v); }
    };
};

}  // namespace toploc
