// Steps 2-5 of the paper's Algorithm 1 for one chunk, one workgroup:
// findInjectiveModulus (Algorithm 6), i mod m, InterpolateModPolynomial (what
// Algorithm 3 returns, with the inverses of Algorithm 4) -- all in GF(65497) on the
// integer ALUs, operands staged in LDS.
//
// The interpolating polynomial of degree < k through k points is unique, so any
// exact method yields the bytes the paper's Newton form would.  The Lagrange form
// is used here because each of its steps is k-wide parallel with short dependent
// chains:
//   W(X)  = prod_j (X - x_j)                       product tree, ceil(log2 k) levels
//   d_j   = W'(x_j)                                Horner in x_j^2, even and odd part
//   a_j   = y_j / d_j                              inverse by Fermat's little theorem
//   S_r   = sum_j a_j x_j^r,  r = 0..k-1           Vandermonde product, RB rows at a time
//   c_i   = sum_{r=0}^{k-1-i} W_{i+1+r} S_r        (from P = sum_j a_j W/(X - x_j))
// Sums of products are accumulated unreduced in 64 bits and reduced once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gf65497.hpp"

namespace toploc {

#ifdef TOPLOC_TIMING
__device__ unsigned long long g_tt[8];
#define TT_MARK(i) do { if (threadIdx.x == 0) { const uint64_t now_ = wall_clock64(); atomicAdd(&g_tt[i], (unsigned long long)(now_ - tt0_)); tt0_ = now_; } } while (0)
#define TT_START() uint64_t tt0_ = wall_clock64()
#else
#define TT_MARK(i) do { } while (0)
#define TT_START() do { } while (0)
#endif

constexpr uint32_t kModHigh = 65536u;
constexpr uint32_t kModLow = 32769u;  // 2^15 + 1

template <int KMAX, int RB>
struct InterpShared {
    uint32_t idx[KMAX];      // top-k flat indices
    uint32_t xs[KMAX];       // (idx mod m) mod p
    uint32_t ys[KMAX];       // bf16 pattern mod p
    uint32_t pa[KMAX + 1];   // product tree ping
    uint32_t pb[KMAX + 1];   // product tree pong
    uint32_t wder[KMAX];     // coefficients of W'
    uint32_t a[KMAX];
    uint32_t S[KMAX];
    union {
        uint32_t bitmap[2048];            // modulus search: one bit per field element
        uint16_t V[RB * (KMAX + 2)];      // V[r][j] = x_j^(r0 + r), row pitch KMAX + 2
    } u;
    uint32_t collide[2];
};

// Algorithm 6 with the residues compared in the form Algorithms 3 and 5 consume them,
// (i mod m) mod p: the largest m in [2^15+1, 65536] for which the k points are
// distinct.  xs[j] receives the mapped index.  Returns 0 when no m works.
// All threads call; s.u.bitmap must be zero and is left zero; ends with a barrier.
template <int THREADS, int KMAX, int RB>
__device__ __forceinline__ uint32_t find_modulus(InterpShared<KMAX, RB>& s, uint32_t k)
{
    const uint32_t tid = threadIdx.x;
    for (uint32_t m = kModHigh; m >= kModLow; --m) {
        uint32_t* flag = &s.collide[m & 1u];
        for (uint32_t j = tid; j < k; j += THREADS) {
            uint32_t x = s.idx[j] % m;
            x = x >= kPrime ? x - kPrime : x;  // x < 65536 < 2p
            s.xs[j] = x;
            const uint32_t bit = 1u << (x & 31u);
            if (atomicOr(&s.u.bitmap[x >> 5], bit) & bit) *flag = 1u;
        }
        __syncthreads();
        const uint32_t c = *flag;
        for (uint32_t j = tid; j < k; j += THREADS) s.u.bitmap[s.xs[j] >> 5] = 0;
        if (tid == 0) s.collide[(m + 1u) & 1u] = 0;  // the next candidate's flag; last read one barrier ago
        __syncthreads();
        if (!c) return m;
    }
    return 0;
}

// low coefficients f_0..f_{deg-1} of a monic polynomial of degree deg; f_deg = 1
__device__ __forceinline__ uint32_t monic_coef(const uint32_t* f, uint32_t deg, uint32_t i)
{
    return i == deg ? 1u : f[i];
}

// coef_out[0..k) <- coefficients (ascending powers) of the polynomial through
// (s.xs[j], s.ys[j]); the xs must be distinct.  All threads call; ends with a barrier.
template <int THREADS, int KMAX, int RB>
__device__ __forceinline__ void interpolate(InterpShared<KMAX, RB>& s, uint32_t k, uint32_t* coef_out)
{
    // L lanes share a point (even and odd powers) when the workgroup has lanes to spare
    constexpr int L = (2 * KMAX <= THREADS) ? 2 : 1;
    constexpr int PPT = (KMAX * L + THREADS - 1) / THREADS;  // points per lane
    const uint32_t tid = threadIdx.x;
    const uint32_t h = (L == 2) ? (tid & 1u) : 0u;
    TT_START();

    // ---- W(X) = prod (X - x_j): pairwise products of monic polynomials ----
    uint32_t* src = s.pa;
    uint32_t* dst = s.pb;
    for (uint32_t j = tid; j < k; j += THREADS) src[j] = s.xs[j] ? kPrime - s.xs[j] : 0u;
    __syncthreads();
    for (uint32_t d = 1; d < k; d <<= 1) {
        // lane pair (L = 2) or lane (L = 1) per output coefficient o; lane h takes every L-th term
        for (uint32_t o = tid / L; o < k; o += THREADS / L) {
            const uint32_t start = o & ~(2u * d - 1u);
            const uint32_t t = o - start;
            const uint32_t df = (k - start) < d ? (k - start) : d;
            const uint32_t rem = k - start - df;
            const uint32_t dg = rem < d ? rem : d;
            const uint32_t* f = src + start;        // f_0..f_{df-1}, f_df = 1
            const uint32_t* g = src + start + df;   // g_0..g_{dg-1}, g_dg = 1
            // h_t = sum_i f_i g_{t-i}: the terms with both coefficients stored ...
            const uint32_t lo = t + 1u > dg ? t + 1u - dg : 0u;
            const uint32_t hi = t < df ? t + 1u : df;   // exclusive
            uint64_t acc = 0;
#pragma unroll 4
            for (uint32_t i = lo + h; i < hi; i += L) acc += (uint64_t)mul24(f[i], g[t - i]);
            // ... and the two terms that meet a leading 1
            if (h == 0) {
                if (t >= df) acc += g[t - df];
                if (t >= dg) acc += f[t - dg];
            }
            uint32_t c = reduce64(acc);
            if (L == 2) {
                c += __shfl_xor(c, 1);
                c = c >= kPrime ? c - kPrime : c;
            }
            if (h == 0) dst[o] = c;
        }
        __syncthreads();
        uint32_t* tmp = src; src = dst; dst = tmp;
    }
    const uint32_t* W = src;  // W_0..W_{k-1}; W_k = 1
    TT_MARK(1);
    // ---- W'(X) coefficients: wder_r = (r+1) W_{r+1} ----
    for (uint32_t r = tid; r < k; r += THREADS) {
        s.wder[r] = mulmod(r + 1, monic_coef(W, k, r + 1));
        s.S[r] = 0;
    }
    __syncthreads();
    // ---- a_j = y_j / W'(x_j); W'(x) = E(x^2) + x O(x^2), lane h takes powers = h mod L ----
    uint32_t xj[PPT], x2[PPT];
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
        const uint32_t j = (tid + i * THREADS) / L;
        xj[i] = 0; x2[i] = 0;
        if (j < k) {
            const uint32_t x = s.xs[j];
            xj[i] = x;
            const uint32_t step = (L == 2) ? mulmod(x, x) : x;
            x2[i] = step;
            // highest power with the lane's parity
            int r = (int)k - 1;
            if (L == 2 && ((uint32_t)r & 1u) != h) r -= 1;
            uint32_t acc = 0;
            for (; r >= 0; r -= L) acc = muladdmod(acc, step, s.wder[r]);
            if (L == 2) {
                if (h) acc = mulmod(acc, x);
                acc += __shfl_xor(acc, 1);
                acc = acc >= kPrime ? acc - kPrime : acc;
            }
            if (h == 0) s.a[j] = mulmod(s.ys[j], invmod(acc));
        }
    }
    __syncthreads();
    TT_MARK(2);
    // ---- S_r = sum_j a_j x_j^r, RB rows of the Vandermonde matrix at a time ----
    constexpr uint32_t PITCH = KMAX + 2;
    uint32_t pw[PPT];
#pragma unroll
    for (int i = 0; i < PPT; ++i) pw[i] = h ? xj[i] : 1u;  // x_j^(r0 + h), carried from block to block
    constexpr uint32_t SLICES = THREADS / RB;
    const uint32_t r_local = tid % RB;
    const uint32_t slice = tid / RB;
    for (uint32_t r0 = 0; r0 < k; r0 += RB) {
#pragma unroll
        for (int i = 0; i < PPT; ++i) {
            const uint32_t j = (tid + i * THREADS) / L;
            if (j < k) {
                uint32_t p = pw[i];
                for (uint32_t r = h; r < RB; r += L) {
                    s.u.V[r * PITCH + j] = (uint16_t)p;
                    p = mulmod(p, x2[i]);
                }
                pw[i] = p;
            }
        }
        __syncthreads();
        if (r0 + r_local < k) {
            const uint32_t per = (k + SLICES - 1) / SLICES;
            const uint32_t j0 = slice * per;
            const uint32_t j1 = (j0 + per) < k ? (j0 + per) : k;
            uint64_t acc = 0;
            const uint16_t* row = &s.u.V[r_local * PITCH];
#pragma unroll 8
            for (uint32_t j = j0; j < j1; ++j) acc += (uint64_t)mul24(s.a[j], (uint32_t)row[j]);
            if (j0 < j1) atomicAdd(&s.S[r0 + r_local], reduce64(acc));
        }
        __syncthreads();
    }
    for (uint32_t r = tid; r < k; r += THREADS) s.S[r] = reduce32(s.S[r]);  // sums of SLICES partial results
    __syncthreads();
    TT_MARK(3);
    // ---- c_i = sum_{r=0}^{k-1-i} W_{i+1+r} S_r, lane h takes r = h mod L ----
#pragma unroll
    for (int n = 0; n < PPT; ++n) {
        const uint32_t i = (tid + n * THREADS) / L;
        if (i < k) {
            uint64_t acc = 0;
            const uint32_t last = k - 1u - i;                 // W_{i+1+last} = W_k = 1
#pragma unroll 4
            for (uint32_t r = h; r < last; r += L) acc += (uint64_t)mul24(W[i + 1u + r], s.S[r]);
            if ((last % L) == h) acc += s.S[last];
            uint32_t c = reduce64(acc);
            if (L == 2) {
                c += __shfl_xor(c, 1);
                c = c >= kPrime ? c - kPrime : c;
            }
            if (h == 0) coef_out[i] = c;
        }
    }
    __syncthreads();
    TT_MARK(4);
}

// Remaining steps of Algorithm 1 for one chunk whose top-k pairs sit in s.idx / s.ys
// (ys already reduced mod p): modulus, index map, interpolation, encode.  `proof`
// points at the chunk's 2 + 2k bytes, `status` at its status byte.
template <int THREADS, int KMAX, int RB>
__device__ __forceinline__ void finish_proof(InterpShared<KMAX, RB>& s, uint32_t* coef, uint32_t k, uint16_t* proof,
                                             uint8_t* status)
{
    const uint32_t tid = threadIdx.x;
    TT_START();
    for (uint32_t w = tid; w < 2048; w += THREADS) s.u.bitmap[w] = 0;
    if (tid == 0) { s.collide[0] = 0; s.collide[1] = 0; }
    __syncthreads();
    const uint32_t m = find_modulus<THREADS, KMAX, RB>(s, k);
    TT_MARK(0);
    if (m == 0) {  // uniform
        for (uint32_t j = tid; j <= k; j += THREADS) proof[j] = 0;
        if (tid == 0) *status = 1;  // TOPLOC_CHUNK_NO_MODULUS
        return;
    }
    interpolate<THREADS, KMAX, RB>(s, k, coef);
    if (tid == 0) { proof[0] = (uint16_t)(m & 0xFFFFu); *status = 0; }
    for (uint32_t j = tid; j < k; j += THREADS) proof[1 + j] = (uint16_t)coef[j];
    TT_MARK(5);
}

}  // namespace toploc
