// Arithmetic in GF(p), p = 4294967291 = 2^32 - 5, for gfx950 integer ALUs: the field of
// the polynomial congruence when the encoded values are fp32 patterns (Appendix C bounds
// the modulus by 2^32 for 32-bit types).  Products are 64 bits (v_mul_lo_u32 +
// v_mul_hi_u32); reduction folds the high half down with 2^32 = 5 (mod p): no division.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace toploc {

constexpr uint32_t kPrime32 = 4294967291u;

// any 64-bit v -> v mod p
__device__ __forceinline__ uint32_t reduce64_p32(uint64_t v)
{
    uint64_t t = (uint64_t)((uint32_t)(v >> 32)) * 5u + (uint32_t)v;   // < 6 * 2^32
    t = (uint64_t)((uint32_t)(t >> 32) * 5u) + (uint32_t)t;            // <= 25 + 2^32 - 1 < 2p
    return t >= kPrime32 ? (uint32_t)(t - kPrime32) : (uint32_t)t;
}

// The field as the interpolation and evaluation code sees it.
struct Field32 {
    typedef uint32_t elem_t;                 // a residue in LDS
    static constexpr uint32_t P = kPrime32;
    static constexpr int WORDS = 2;          // 16-bit words of an encoded coefficient
    static constexpr int INV_BITS = 32;      // bits of P - 2

    static __device__ __forceinline__ uint32_t from_pattern(uint32_t bits) { return bits >= P ? bits - P : bits; }
    // (i mod m) with m <= 65536 is already a field element
    static __device__ __forceinline__ uint32_t from_residue(uint32_t x) { return x; }
    static __device__ __forceinline__ uint32_t mulmod(uint32_t a, uint32_t b) { return reduce64_p32((uint64_t)a * b); }
    // a*b + c with a, b, c < p: (p-1)^2 + (p-1) < 2^64 (one step of Horner's rule, Algorithm 5)
    static __device__ __forceinline__ uint32_t muladdmod(uint32_t a, uint32_t b, uint32_t c)
    {
        return reduce64_p32((uint64_t)a * b + c);
    }
    static __device__ __forceinline__ uint32_t addmod(uint32_t a, uint32_t b)   // a, b < p
    {
        const uint64_t s = (uint64_t)a + b;
        return s >= P ? (uint32_t)(s - P) : (uint32_t)s;
    }
    static __device__ __forceinline__ uint32_t submod(uint32_t a, uint32_t b) { return a >= b ? a - b : a + (P - b); }
    static __device__ __forceinline__ uint32_t neg(uint32_t a) { return a ? P - a : 0u; }
    // a^(p-2): the inverse of a != 0 (Fermat; the same unique inverse Algorithm 4 finds)
    static __device__ __forceinline__ uint32_t inv(uint32_t a)
    {
        constexpr uint32_t e = P - 2u;   // 0xFFFFFFF9
        uint32_t r = a;
#pragma unroll 1
        for (int bit = 30; bit >= 0; --bit) {
            r = mulmod(r, r);
            if ((e >> bit) & 1u) r = mulmod(r, a);
        }
        return r;
    }
    // sum of up to 2^32 products of residues: 96 bits
    struct Acc {
        uint64_t lo;
        uint32_t hi;
        __device__ __forceinline__ Acc() : lo(0), hi(0) {}
        __device__ __forceinline__ void mac(uint32_t a, uint32_t b)
        {
            const uint64_t p = (uint64_t)a * b;
            lo += p;
            hi += lo < p ? 1u : 0u;
        }
        __device__ __forceinline__ void add(uint32_t x)
        {
            lo += x;
            hi += lo < x ? 1u : 0u;
        }
        __device__ __forceinline__ uint32_t reduce() const   // 2^64 = 25 (mod p); hi < 2^27 keeps 25*hi in 32 bits
        {
            return addmod(reduce64_p32(lo), reduce64_p32((uint64_t)hi * 25u));
        }
    };
};

}  // namespace toploc
