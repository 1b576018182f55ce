// Residues of GF(65497) as BYTE PLANES: a residue a < 2^16 is a1*256 + a0, a vector of residues is one
// array of high bytes and one of low bytes.  For two vectors,
//     sum a*b = 2^16 * sum a1*b1 + 2^8 * (sum a1*b0 + sum a0*b1) + sum a0*b0,
// three 32-bit accumulators fed by four packed dot products (v_dot4_u32_u8: four 8x8-bit products and
// an add per lane and instruction) per four terms, folded once per sum with 2^16 = 39 (mod p).
// Used by the interpolation (the paper's Algorithm 3, interp16.hpp) and by the evaluation of the proof
// polynomial (Algorithm 5, verify.hpp).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gf65497.hpp"

namespace toploc {

typedef uint32_t u32v4 __attribute__((ext_vector_type(4)));

// three accumulators of a sum of products of byte-plane vectors
struct PlaneAcc {
    uint32_t hh, m, ll;
    __device__ __forceinline__ PlaneAcc() : hh(0), m(0), ll(0) {}
    // four terms: a and b each as a word of high bytes and a word of low bytes
    __device__ __forceinline__ void step(uint32_t a1, uint32_t a0, uint32_t b1, uint32_t b0)
    {
        hh = __builtin_amdgcn_udot4(a1, b1, hh, false);
        m = __builtin_amdgcn_udot4(a1, b0, m, false);
        m = __builtin_amdgcn_udot4(a0, b1, m, false);
        ll = __builtin_amdgcn_udot4(a0, b0, ll, false);
    }
    // (hh 2^16 + m 2^8 + ll) mod p for at most 128 steps: hh, ll < 2^25, m < 2^26
    __device__ __forceinline__ uint32_t value() const
    {
        const uint32_t h39 = (hh << 5) + (hh << 3) - hh;          // 39 hh < 2^31
        return reduce32(h39 + (reduce32(m) << 8) + ll);           // < 2^31 + 2^24 + 2^25
    }
    // the same for at most 28 steps: hh, ll < 28 * 2^18 < 2^23, m < 2^24, so 39 hh + 2^8 m + ll < 2^32 as it is
    __device__ __forceinline__ uint32_t value_short() const
    {
        return reduce32(mul24(hh, kFold16) + (m << 8) + ll);
    }
};

// the value the other lane of the pair (lane ^ 1) holds: a DPP move inside the quad, no LDS round trip
__device__ __forceinline__ uint32_t pair_swap(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);   // quad_perm:[1,0,3,2]
}

// a DPP move inside the quad: QP = 0xA0 gives both lanes of a pair the even lane's value, 0xF5 the odd lane's
template <int QP>
__device__ __forceinline__ uint32_t quad_from(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, QP, 0xF, 0xF, true);
}

// bytes sh .. sh+3 of the eight bytes {hi, lo}
__device__ __forceinline__ uint32_t byte_window(uint32_t hi, uint32_t lo, uint32_t sh)
{
    return __builtin_amdgcn_alignbyte(hi, lo, sh);
}

__device__ __forceinline__ uint32_t plane_get(const uint8_t* hi, const uint8_t* lo, uint32_t j)
{
    return ((uint32_t)hi[j] << 8) | (uint32_t)lo[j];
}
__device__ __forceinline__ void plane_put(uint8_t* hi, uint8_t* lo, uint32_t j, uint32_t v)
{
    hi[j] = (uint8_t)(v >> 8);
    lo[j] = (uint8_t)v;
}

// The powers 1, x, .., x^15 of a residue as packed planes (word w holds the bytes of x^(4w) .. x^(4w+3));
// returns x^16.
__device__ __forceinline__ uint32_t plane_powers16(uint32_t x, uint32_t (&pw1)[4], uint32_t (&pw0)[4])
{
    uint32_t pw[16];
    uint32_t p = 1u;
#pragma unroll
    for (uint32_t r0 = 0; r0 < 16u; ++r0) {
        pw[r0] = p;
        p = mulmod(p, x);
    }
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const uint32_t t0 = __builtin_amdgcn_perm(pw[4 * w + 1], pw[4 * w], 0x05010400u);   // a0 b0 a1 b1
        const uint32_t t1 = __builtin_amdgcn_perm(pw[4 * w + 3], pw[4 * w + 2], 0x05010400u);
        pw0[w] = __builtin_amdgcn_perm(t1, t0, 0x05040100u);
        pw1[w] = __builtin_amdgcn_perm(t1, t0, 0x07060302u);
    }
    return p;
}

}  // namespace toploc
