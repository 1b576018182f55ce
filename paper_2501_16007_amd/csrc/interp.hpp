// Steps 2-5 of the paper's Algorithm 1 for one chunk, one workgroup:
// findInjectiveModulus (Algorithm 6), i mod m, InterpolateModPolynomial (what
// Algorithm 3 returns, with the inverses of Algorithm 4) -- all in GF(p) on the integer
// ALUs, operands staged in LDS.  The field F is GF(65497) for bf16 patterns (gf65497.hpp)
// and GF(2^32 - 5) for fp32 patterns (gf32.hpp).
//
// The interpolating polynomial of degree < k through k points is unique, so any
// exact method yields the bytes the paper's Newton form would.  The Lagrange form
// is used here because each of its steps is k-wide parallel with short dependent
// chains:
//   W(X)  = prod_j (X - x_j)                       product tree, ceil(log2 k) levels
//   d_j   = W'(x_j) = sum_r W'_r x_j^r
//   a_j   = y_j / d_j                              inverse by Fermat's little theorem
//   S_r   = sum_j a_j x_j^r,  r = 0..k-1
//   c_i   = sum_{r=0}^{k-1-i} W_{i+1+r} S_r        (from P = sum_j a_j W/(X - x_j))
// Powers come from two small tables per point, x^r = x^(16 r1) * x^(r0) with r = 16 r1 + r0
// (baby steps B[j][r0], giant steps G[r1][j]): about 25 modular multiplications per point
// instead of k, and both matrix products (d and S) become sums of plain products, which
// are accumulated unreduced (64 bits, 96 bits in the larger field) and reduced once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gf32.hpp"
#include "gf65497.hpp"
#include "ticks.hpp"

#ifndef TOPLOC_TREE_LEAF
#define TOPLOC_TREE_LEAF 16   // 16: leaves of 16 points built by lane groups; 1: the plain tree from single points
#endif

namespace toploc {

constexpr uint32_t kModHigh = 65536u;
constexpr uint32_t kModLow = 32769u;  // 2^15 + 1
constexpr uint32_t kBaby = 16u;       // baby-step table width

template <int KMAX, typename F = Field16>
struct InterpShared {
    static_assert(KMAX % 16 == 0, "giant steps cover 16 powers each");
    typedef typename F::elem_t E;
    uint32_t idx[KMAX];       // top-k flat indices
    alignas(16) E xs[KMAX];   // (idx mod m) mod p (read 16 at a time)
    E ys[KMAX];               // pattern mod p
    E pa[KMAX + 2];           // product tree ping
    E pb[KMAX + 2];           // product tree pong
    alignas(16) E wder[KMAX]; // coefficients of W' (read 16 at a time)
    E S[KMAX];
    alignas(16) union {
        uint32_t bitmap[2048];                    // modulus search: one bit per residue below 65536
        struct {
            E B[KMAX * 16];                       // B[j][r0] = x_j^r0
            E G[(KMAX / 16) * KMAX];              // G[r1][j] = x_j^(16 r1), later a_j x_j^(16 r1)
        } pw;
    } u;
    uint32_t collide[2];
};

// Sixteen consecutive field elements from LDS (16-byte aligned) into registers with
// 16-byte loads: 2 loads for 16-bit elements, 4 for 32-bit ones, instead of 16.
template <typename E>
__device__ __forceinline__ void load16(const E* p, uint32_t (&out)[16])
{
    typedef uint32_t vec4 __attribute__((ext_vector_type(4)));
    const vec4* v = reinterpret_cast<const vec4*>(p);
    if (sizeof(E) == 2) {
        const vec4 a = v[0], b = v[1];
        const uint32_t w[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) { out[2 * i] = w[i] & 0xFFFFu; out[2 * i + 1] = w[i] >> 16; }
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const vec4 a = v[q];
            out[4 * q] = a.x; out[4 * q + 1] = a.y; out[4 * q + 2] = a.z; out[4 * q + 3] = a.w;
        }
    }
}

template <typename E>
__device__ __forceinline__ void store16(E* p, const uint32_t (&in)[16])
{
    typedef uint32_t vec4 __attribute__((ext_vector_type(4)));
    vec4* v = reinterpret_cast<vec4*>(p);
    if (sizeof(E) == 2) {
        uint32_t w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = in[2 * i] | (in[2 * i + 1] << 16);
        v[0] = vec4{w[0], w[1], w[2], w[3]};
        v[1] = vec4{w[4], w[5], w[6], w[7]};
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = vec4{in[4 * q], in[4 * q + 1], in[4 * q + 2], in[4 * q + 3]};
    }
}

// Algorithm 6 with the residues compared in the form Algorithms 3 and 5 consume them,
// (i mod m) mod p: the largest m in [2^15+1, 65536] for which the k points are
// distinct.  xs[j] receives the mapped index.  Returns 0 when no m works.
// All threads call; s.u.bitmap must be zero and is left zero; ends with a barrier.
template <int THREADS, int KMAX, typename F>
__device__ __forceinline__ uint32_t find_modulus(InterpShared<KMAX, F>& s, uint32_t k)
{
    const uint32_t tid = threadIdx.x;
    for (uint32_t m = kModHigh; m >= kModLow; --m) {
        uint32_t* flag = &s.collide[m & 1u];
        for (uint32_t j = tid; j < k; j += THREADS) {
            const uint32_t x = F::from_residue(s.idx[j] % m);  // < 65536
            s.xs[j] = (typename F::elem_t)x;
            const uint32_t bit = 1u << (x & 31u);
            if (atomicOr(&s.u.bitmap[x >> 5], bit) & bit) *flag = 1u;
        }
        __syncthreads();
        const uint32_t c = *flag;
        for (uint32_t j = tid; j < k; j += THREADS) s.u.bitmap[(uint32_t)s.xs[j] >> 5] = 0;
        if (tid == 0) s.collide[(m + 1u) & 1u] = 0;  // the next candidate's flag; last read one barrier ago
        __syncthreads();
        if (!c) return m;
    }
    return 0;
}

// coef_out[0..k) <- coefficients (ascending powers) of the polynomial through
// (s.xs[j], s.ys[j]); the xs must be distinct.  All threads call; ends with a barrier.
template <int THREADS, int KMAX, typename F>
__device__ __forceinline__ void interpolate(InterpShared<KMAX, F>& s, uint32_t k, uint32_t* coef_out)
{
    typedef typename F::elem_t E;
    typedef typename F::Acc Acc;
    // L lanes share a point or an output (alternate terms) when the workgroup has lanes to spare
    constexpr int L = (2 * KMAX <= THREADS) ? 2 : 1;
    constexpr int PPT = (KMAX * L + THREADS - 1) / THREADS;  // points per lane
    const uint32_t tid = threadIdx.x;
    const uint32_t h = (L == 2) ? (tid & 1u) : 0u;
    const uint32_t n_giant = (k + kBaby - 1u) / kBaby;

    // ---- W(X) = prod (X - x_j): pairwise products of monic polynomials ----
    TOPLOC_TICK_BEGIN(tree);
    E* src = s.pa;
    E* dst = s.pb;
#if TOPLOC_TREE_LEAF == 16
    // Leaves of 16 points, one lane per point: the 16 lanes of a group hold the coefficients
    // c_0..c_15 of the running product and multiply it by (X - x_s) sixteen times,
    // c_i <- c_{i-1} - x_s c_i (the coefficient 1 of the highest power is implied, as in the
    // levels above).  This replaces the four lowest levels, whose cost is all overhead.
    static_assert(KMAX <= THREADS && KMAX % 16 == 0, "one lane per point, whole groups");
    if (tid < ((k + 15u) & ~15u)) {  // whole groups of 16 lanes; a group never straddles a wave
        const uint32_t g0 = tid & ~15u, i = tid & 15u;
        const uint32_t cnt = (k - g0) < 16u ? (k - g0) : 16u;  // points of this group
        uint32_t xg[16];                   // the group's points: the same two LDS loads for its 16 lanes
        load16(&s.xs[g0], xg);
        uint32_t c = (i == 0u) ? 1u : 0u;  // the polynomial 1
#pragma unroll
        for (uint32_t step = 0; step < 16u; ++step) {
            // c_{i-1} from the lane below inside the row of 16 (DPP row_shr:1; lane 0 of a row gets 0)
            const uint32_t below = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0x111, 0xF, 0xF, false);
            const uint32_t next = F::submod(below, F::mulmod(xg[step], c));
            if (step < cnt) c = next;
        }
        if (i < cnt) src[tid] = (E)c;
    }
    __syncthreads();
    for (uint32_t d = 16u; d < k; d <<= 1) {
#else
    for (uint32_t j = tid; j < k; j += THREADS) src[j] = (E)F::neg(s.xs[j]);
    __syncthreads();
    for (uint32_t d = 1; d < k; d <<= 1) {
#endif
        for (uint32_t o = tid / L; o < k; o += THREADS / L) {
            const uint32_t start = o & ~(2u * d - 1u);
            const uint32_t t = o - start;
            const uint32_t df = (k - start) < d ? (k - start) : d;
            const uint32_t rem = k - start - df;
            const uint32_t dg = rem < d ? rem : d;
            const E* f = src + start;        // f_0..f_{df-1}, f_df = 1
            const E* g = src + start + df;   // g_0..g_{dg-1}, g_dg = 1
            // h_t = sum_i f_i g_{t-i}: the terms with both coefficients stored ...
            const uint32_t lo = t + 1u > dg ? t + 1u - dg : 0u;
            const uint32_t hi = t < df ? t + 1u : df;   // exclusive
            Acc acc;
#pragma unroll 4
            for (uint32_t i = lo + h; i < hi; i += L) acc.mac(f[i], g[t - i]);
            // ... and the two terms that meet a leading 1
            if (h == 0) {
                if (t >= df) acc.add(g[t - df]);
                if (t >= dg) acc.add(f[t - dg]);
            }
            uint32_t c = acc.reduce();
            if (L == 2) c = F::addmod(c, __shfl_xor(c, 1));
            if (h == 0) dst[o] = (E)c;
        }
        __syncthreads();
        E* tmp = src; src = dst; dst = tmp;
    }
    const E* W = src;  // W_0..W_{k-1}; W_k = 1
    TOPLOC_TICK_END(tree, 7);
    TOPLOC_TICK_BEGIN(tables);
    // ---- W'(X) coefficients: wder_r = (r+1) W_{r+1}; power tables of every point ----
    for (uint32_t r = tid; r < k; r += THREADS)
        s.wder[r] = (E)F::mulmod(r + 1, r + 1 == k ? 1u : (uint32_t)W[r + 1]);
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
        const uint32_t j = (tid + i * THREADS) / L;
        if (j < k) {
            const uint32_t x = s.xs[j];
            if (L == 1 || h == 0) {   // baby steps 1, x, .., x^15
                uint32_t pw[kBaby];
                uint32_t p = 1u;
#pragma unroll
                for (uint32_t r0 = 0; r0 < kBaby; ++r0) {
                    pw[r0] = p;
                    p = F::mulmod(p, x);
                }
                store16(&s.u.pw.B[j * kBaby], pw);
            }
            if (L == 1 || h == 1) {   // giant steps 1, x^16, x^32, ..
                uint32_t x16 = F::mulmod(x, x);
                x16 = F::mulmod(x16, x16);
                x16 = F::mulmod(x16, x16);
                x16 = F::mulmod(x16, x16);
                uint32_t p = 1u;
                for (uint32_t r1 = 0; r1 < n_giant; ++r1) {
                    s.u.pw.G[r1 * KMAX + j] = (E)p;
                    p = F::mulmod(p, x16);
                }
            }
        }
    }
    __syncthreads();
    TOPLOC_TICK_END(tables, 8);
    TOPLOC_TICK_BEGIN(denom);
    // ---- d_j = sum_r1 x_j^(16 r1) * (sum_r0 W'_(16 r1 + r0) x_j^r0); a_j = y_j / d_j; G <- a_j G ----
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
        const uint32_t j = (tid + i * THREADS) / L;
        if (j < k) {
            uint32_t brow[kBaby];
            load16(&s.u.pw.B[j * kBaby], brow);
            Acc dacc;   // sum over r1 of (inner sum mod p) * x_j^(16 r1)
            for (uint32_t r1 = h; r1 < n_giant; r1 += L) {
                const uint32_t rbase = r1 * kBaby;
                uint32_t wrow[kBaby];   // the same 16 coefficients for every lane: a broadcast read
                load16(&s.wder[rbase], wrow);
                Acc acc;
#pragma unroll
                for (uint32_t r0 = 0; r0 < kBaby; ++r0)
                    if (rbase + r0 < k) acc.mac(wrow[r0], brow[r0]);
                dacc.mac(acc.reduce(), s.u.pw.G[r1 * KMAX + j]);
            }
            uint32_t d = dacc.reduce();
            uint32_t a = 0;
            if (L == 2) {
                d = F::addmod(d, __shfl_xor(d, 1));
                if (h == 0) a = F::mulmod(s.ys[j], F::inv(d));
                a = __shfl(a, (int)(__lane_id() & ~1u));
            } else {
                a = F::mulmod(s.ys[j], F::inv(d));
            }
            for (uint32_t r1 = h; r1 < n_giant; r1 += L)
                s.u.pw.G[r1 * KMAX + j] = (E)F::mulmod(a, s.u.pw.G[r1 * KMAX + j]);
        }
    }
    __syncthreads();
    TOPLOC_TICK_END(denom, 9);
    TOPLOC_TICK_BEGIN(sums);
    // ---- S_r = sum_j (a_j x_j^(16 r1)) x_j^r0, r = 16 r1 + r0; lane h takes j = h mod L ----
    for (uint32_t r = tid / L; r < k; r += THREADS / L) {
        const E* arow = &s.u.pw.G[(r / kBaby) * KMAX];
        const E* bcol = &s.u.pw.B[r % kBaby];
        Acc acc;
#pragma unroll 8
        for (uint32_t j = h; j < k; j += L) acc.mac(arow[j], bcol[j * kBaby]);
        uint32_t v = acc.reduce();
        if (L == 2) v = F::addmod(v, __shfl_xor(v, 1));
        if (h == 0) s.S[r] = (E)v;
    }
    __syncthreads();
    TOPLOC_TICK_END(sums, 10);
    TOPLOC_TICK_BEGIN(coefs);
    // ---- c_i = sum_{r=0}^{k-1-i} W_{i+1+r} S_r, lane h takes r = h mod L ----
    for (uint32_t i = tid / L; i < k; i += THREADS / L) {
        Acc acc;
        const uint32_t last = k - 1u - i;                 // W_{i+1+last} = W_k = 1
#pragma unroll 4
        for (uint32_t r = h; r < last; r += L) acc.mac(W[i + 1u + r], s.S[r]);
        if ((last % L) == h) acc.add(s.S[last]);
        uint32_t c = acc.reduce();
        if (L == 2) c = F::addmod(c, __shfl_xor(c, 1));
        if (h == 0) coef_out[i] = c;
    }
    __syncthreads();
    TOPLOC_TICK_END(coefs, 11);
}

// Remaining steps of Algorithm 1 for one chunk whose top-k pairs sit in s.idx / s.ys
// (ys already reduced mod p): modulus, index map, interpolation, encode.  `proof`
// points at the chunk's 2 + 2k bytes (2 + 4k in the 32-bit field: a coefficient is written
// as F::WORDS 16-bit words, low word first), `status` at its status byte.
template <int THREADS, int KMAX, typename F>
__device__ __forceinline__ void finish_proof(InterpShared<KMAX, F>& s, uint32_t* coef, uint32_t k, uint16_t* proof,
                                             uint8_t* status)
{
    const uint32_t tid = threadIdx.x;
    for (uint32_t w = tid; w < 2048; w += THREADS) s.u.bitmap[w] = 0;
    if (tid == 0) { s.collide[0] = 0; s.collide[1] = 0; }
    __syncthreads();
    TOPLOC_TICK_BEGIN(modulus);
    const uint32_t m = find_modulus<THREADS>(s, k);
    TOPLOC_TICK_END(modulus, 6);
    if (m == 0) {  // uniform
        for (uint32_t j = tid; j <= k * F::WORDS; j += THREADS) proof[j] = 0;
        if (tid == 0) *status = 1;  // TOPLOC_CHUNK_NO_MODULUS
        return;
    }
    interpolate<THREADS>(s, k, coef);
    if (tid == 0) { proof[0] = (uint16_t)(m & 0xFFFFu); *status = 0; }
    for (uint32_t j = tid; j < k; j += THREADS) {
        proof[1 + j * F::WORDS] = (uint16_t)coef[j];
        if (F::WORDS == 2) proof[2 + j * F::WORDS] = (uint16_t)(coef[j] >> 16);
    }
}

}  // namespace toploc
