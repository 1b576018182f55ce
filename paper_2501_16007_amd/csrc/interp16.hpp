// InterpolateModPolynomial (what the paper's Algorithm 3 returns) over GF(65497) with the field
// elements kept in LDS as BYTE PLANES, so that the sums of products that make up the Lagrange form
// run on the packed dot-product instruction (v_dot4_u32_u8: four 8x8-bit products and an add per
// lane and instruction) instead of one 16x16-bit multiply-add per term.
//
// A residue a < 2^16 is a1*256 + a0.  For two vectors,
//     sum a*b = 2^16 * sum a1*b1 + 2^8 * (sum a1*b0 + sum a0*b1) + sum a0*b0,
// three 32-bit accumulators fed by four dot4 per four terms; they are folded once per output with
// 2^16 = 39 (mod p).  A vector lives as two byte arrays ("planes"), high bytes and low bytes.
//
// The algorithm is the one of interp.hpp (product tree for W = prod (X - x_j), W'(x_j) and the
// power sums S_r from baby-step / giant-step power tables, a_j = y_j / W'(x_j) with Fermat
// inverses, c_i = sum_r W_{i+1+r} S_r); only the data layout and the inner loops differ:
//   * a polynomial product h_t = sum_i f_i g_{t-i} reads f forward and g from a plane stored in
//     REVERSED order with four zero bytes on either side, so that the four bytes g_{t-i} .. g_{t-i-3}
//     are consecutive in memory for every t and out-of-range terms read zeros; the window is not
//     4-byte aligned in general: two aligned words and v_alignbyte_b32;
//   * the baby-step table, scaled by a_j = y_j / W'(x_j), is kept transposed (BT[r0][j] = a_j x_j^r0, rows padded against bank
//     conflicts) so that S_r is a plain dot product over j of two contiguous planes;
//   * c_i reads W forward at byte offset i + 1 + r (unaligned window again) against S.
// The polynomial is unique, so the bytes are those of any exact method.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gf65497.hpp"
#include "interp.hpp"
#include "planes.hpp"

namespace toploc {

template <int KMAX>
struct InterpShared<KMAX, Field16> {
    static_assert(KMAX % 16 == 0, "giant steps cover 16 powers each");
    typedef uint16_t E;
    static constexpr int FLEN = KMAX + 16;       // forward planes: 16 bytes of room behind the last coefficient
    static constexpr int RLEN = KMAX + 16;       // reversed planes: regions of d + 8 bytes per pair of blocks (d >= 16)
    static constexpr int BT_STRIDE = KMAX + 16;  // bytes between rows of BT: 16 rows KMAX apart would share their banks
    uint32_t idx[KMAX];       // top-k flat indices
    alignas(16) E xs[KMAX];   // (idx mod m) mod p
    E ys[KMAX];               // pattern mod p
    alignas(16) uint8_t f_hi[2][FLEN], f_lo[2][FLEN];   // product tree, ping and pong: blocks that are the f of the next product
    alignas(16) uint8_t r_hi[2][RLEN], r_lo[2][RLEN];   //                              blocks that are the g, reversed and padded
    alignas(16) uint8_t wd_hi[KMAX], wd_lo[KMAX];       // coefficients of W'
    alignas(16) uint8_t s_hi[KMAX + 16], s_lo[KMAX + 16];   // S_r
    E dj[KMAX];               // W'(x_j), then a_j = y_j / W'(x_j): handed between the lanes that sum and the lanes that invert
    alignas(16) union {
        uint32_t bitmap[2048];                    // modulus search: one bit per residue below 65536
        struct {
            uint8_t bt_hi[16 * BT_STRIDE], bt_lo[16 * BT_STRIDE];       // BT[r0][j] = x_j^r0, later a_j x_j^r0
            uint8_t g_hi[(KMAX / 16) * KMAX], g_lo[(KMAX / 16) * KMAX]; // G[r1][j] = x_j^(16 r1)
        } pw;
    } u;
    uint32_t collide[2];
};

// Sum over `n` steps of four terms of a forward plane pair (aligned, from word a_w on) times a window
// that starts at byte position `p` of another plane pair and moves forward.
__device__ __forceinline__ void plane_dot_window(PlaneAcc& acc, const uint32_t* __restrict__ a1, const uint32_t* __restrict__ a0,
                                                 const uint32_t* __restrict__ b1, const uint32_t* __restrict__ b0, uint32_t p,
                                                 uint32_t n)
{
    const uint32_t w = p >> 2, sh = p & 3u;
    uint32_t c1 = b1[w], c0 = b0[w];
#pragma unroll 2
    for (uint32_t s = 0; s < n; ++s) {
        const uint32_t n1 = b1[w + 1u + s], n0 = b0[w + 1u + s];
        acc.step(a1[s], a0[s], byte_window(n1, c1, sh), byte_window(n0, c0, sh));
        c1 = n1;
        c0 = n0;
    }
}

// coef_out[0..k) <- coefficients (ascending powers) of the polynomial through (s.xs[j], s.ys[j]); the xs
// must be distinct.  All threads call; ends with a barrier.  THREADS = 2 KMAX: two lanes share a point
// or an output and take one half of its terms each.
template <int THREADS, int KMAX>
__device__ __forceinline__ void interpolate(InterpShared<KMAX, Field16>& s, uint32_t k, uint32_t* coef_out)
{
    typedef Field16 F;
    typedef InterpShared<KMAX, Field16> Sh;
    static_assert(THREADS == 2 * KMAX, "two lanes per point");
    const uint32_t tid = threadIdx.x;
    const uint32_t h = tid & 1u;          // which half of the terms
    const uint32_t o = tid >> 1;          // the point or output this lane works on
    const uint32_t n_giant = (k + kBaby - 1u) / kBaby;
    const uint32_t k16 = n_giant * kBaby;  // k rounded up to whole rows of 16

    // ---- leaves: W of 16 points by groups of 16 lanes (one lane per point), as in interp.hpp ----
    TOPLOC_TICK_BEGIN(tree);
    if (tid < k16) {
        const uint32_t g0 = tid & ~15u, i = tid & 15u, c = tid >> 4;
        const uint32_t cnt = (k - g0) < 16u ? (k - g0) : 16u;
        uint32_t xg[16];
        load16(&s.xs[g0], xg);
        uint32_t v = (i == 0u) ? 1u : 0u;
#pragma unroll
        for (uint32_t step = 0; step < 16u; ++step) {
            const uint32_t below = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);
            const uint32_t next = F::submod(below, F::mulmod(xg[step], v));
            if (step < cnt) v = next;
        }
        if (i >= cnt) v = 0;
        if ((c & 1u) == 0) {   // the f of pair c/2: forward, at its global position
            plane_put(s.f_hi[0], s.f_lo[0], tid, v);
        } else {               // the g of pair c/2: reversed inside its padded region
            const uint32_t region = (c >> 1) * (16u + 8u);
            plane_put(s.r_hi[0], s.r_lo[0], region + 4u + 15u - i, v);
            if (i < 2u) {      // the four zero bytes below and above
                const uint32_t pad = region + (i ? 20u : 0u);
                *reinterpret_cast<uint32_t*>(&s.r_hi[0][pad]) = 0;
                *reinterpret_cast<uint32_t*>(&s.r_lo[0][pad]) = 0;
            }
        }
    }
    __syncthreads();

    // ---- levels: blocks of d coefficients are multiplied in pairs ----
    uint32_t b = 0;   // buffer the level reads
    for (uint32_t ld = 4u; (1u << ld) < k; ++ld, b ^= 1u) {   // d = 2^ld
        const uint32_t d = 1u << ld, span = 2u * d;
        const uint32_t kceil = ((k + span - 1u) >> (ld + 1u)) << (ld + 1u);   // outputs: whole blocks of 2d (<= KMAX)
        if (o < kceil) {
            const uint32_t q = o >> (ld + 1u), t = o & (span - 1u), start = o & ~(span - 1u);
            const uint32_t df = (k - start) < d ? (k - start) : d;
            const uint32_t rem = k - start - df;
            const uint32_t dg = rem < d ? rem : d;
            const uint32_t len = df + dg;
            const uint8_t* F1 = s.f_hi[b] + start;
            const uint8_t* F0 = s.f_lo[b] + start;
            const uint8_t* R1 = s.r_hi[b] + q * (d + 8u);
            const uint8_t* R0 = s.r_lo[b] + q * (d + 8u);
            uint32_t val = 0;
            if (dg == 0) {   // uniform within the block: no partner, the block is handed on as it is
                if (t < df) val = plane_get(F1, F0, t);
            } else {         // df == d
                // terms i with 0 <= i < d and 0 <= t - i < dg; whole words of four, the padding reads as zero
                const uint32_t lo = t + 1u > dg ? t + 1u - dg : 0u;
                const uint32_t hi = t < d ? t + 1u : d;
                const uint32_t lo4 = lo & ~3u, hi4 = (hi + 3u) & ~3u;
                const uint32_t n4 = hi4 > lo4 ? (hi4 - lo4) >> 2 : 0u;
                const uint32_t half = (n4 + 1u) >> 1;
                const uint32_t first = lo4 + (h ? 4u * half : 0u);
                const uint32_t mine = h ? n4 - half : half;
                PlaneAcc acc;
                if (mine)
                    plane_dot_window(acc, reinterpret_cast<const uint32_t*>(F1) + (first >> 2),
                                     reinterpret_cast<const uint32_t*>(F0) + (first >> 2), reinterpret_cast<const uint32_t*>(R1),
                                     reinterpret_cast<const uint32_t*>(R0), 4u + (d - 1u - t) + first, mine);
                val = acc.value();
                val = F::addmod(val, pair_swap(val));
                if (t < len) {   // the two terms that meet a leading 1
                    if (t >= d) val = F::addmod(val, plane_get(R1, R0, 4u + d - 1u - (t - d)));
                    if (t >= dg) val = F::addmod(val, plane_get(F1, F0, t - dg));
                } else {
                    val = 0;
                }
            }
            if (h == 0) {
                if (span >= k || (q & 1u) == 0) {   // W itself, or the f of the next pair: forward
                    plane_put(s.f_hi[b ^ 1u], s.f_lo[b ^ 1u], o, val);
                } else {                            // the g of the next pair
                    const uint32_t region = (q >> 1) * (span + 8u);
                    plane_put(s.r_hi[b ^ 1u], s.r_lo[b ^ 1u], region + 4u + span - 1u - t, val);
                    if (t < 2u) {
                        const uint32_t pad = region + (t ? 4u + span : 0u);
                        *reinterpret_cast<uint32_t*>(&s.r_hi[b ^ 1u][pad]) = 0;
                        *reinterpret_cast<uint32_t*>(&s.r_lo[b ^ 1u][pad]) = 0;
                    }
                }
            }
        }
        __syncthreads();
    }
    uint8_t* W1 = s.f_hi[b];   // W_0 .. W_{k-1}; W_k = 1
    uint8_t* W0 = s.f_lo[b];
    TOPLOC_TICK_END(tree, 7);
    TOPLOC_TICK_BEGIN(tables);
    // ---- W' coefficients wder_r = (r+1) W_{r+1} (zero from k on), zeros behind W, power tables ----
    if (tid < k16) {
        uint32_t v = 0;
        if (tid < k) v = F::mulmod(tid + 1u, tid + 1u == k ? 1u : plane_get(W1, W0, tid + 1u));
        plane_put(s.wd_hi, s.wd_lo, tid, v);
    }
    uint32_t pw1[4], pw0[4];   // the point's baby steps 1, x, .., x^15 as planes, kept for the next phase
    {
        const uint32_t j = o;
        if (j < k16) {
            // the two lanes of a point take eight powers each: lane h computes x^(8h) .. x^(8h+7)
            const uint32_t x = j < k ? (uint32_t)s.xs[j] : 0u;
            const uint32_t x2 = F::mulmod(x, x), x4 = F::mulmod(x2, x2), x8 = F::mulmod(x4, x4);
            uint32_t q[8];
            uint32_t p = j < k ? (h ? x8 : 1u) : 0u;
#pragma unroll
            for (uint32_t i = 0; i < 8u; ++i) {
                q[i] = p;
                p = F::mulmod(p, x);
            }
            const uint32_t x16 = quad_from<0xF5>(p);   // the odd lane ends on x^16 (0 for a padding lane)
            const uint32_t ta = __builtin_amdgcn_perm(q[1], q[0], 0x05010400u);   // a0 b0 a1 b1
            const uint32_t tb = __builtin_amdgcn_perm(q[3], q[2], 0x05010400u);
            const uint32_t tc = __builtin_amdgcn_perm(q[5], q[4], 0x05010400u);
            const uint32_t td = __builtin_amdgcn_perm(q[7], q[6], 0x05010400u);
            const uint32_t lo_a = __builtin_amdgcn_perm(tb, ta, 0x05040100u), hi_a = __builtin_amdgcn_perm(tb, ta, 0x07060302u);
            const uint32_t lo_b = __builtin_amdgcn_perm(td, tc, 0x05040100u), hi_b = __builtin_amdgcn_perm(td, tc, 0x07060302u);
            // words 0, 1 come from the even lane of the pair, words 2, 3 from the odd one
            pw0[0] = quad_from<0xA0>(lo_a); pw0[1] = quad_from<0xA0>(lo_b); pw0[2] = quad_from<0xF5>(lo_a); pw0[3] = quad_from<0xF5>(lo_b);
            pw1[0] = quad_from<0xA0>(hi_a); pw1[1] = quad_from<0xA0>(hi_b); pw1[2] = quad_from<0xF5>(hi_a); pw1[3] = quad_from<0xF5>(hi_b);
            // giant steps 1, x^16, x^32, ..: the two lanes take alternate ones
            const uint32_t x32 = F::mulmod(x16, x16);
            uint32_t g = h ? x16 : (j < k ? 1u : 0u);
            for (uint32_t r1 = h; r1 < n_giant; r1 += 2u) {
                plane_put(s.u.pw.g_hi, s.u.pw.g_lo, r1 * KMAX + j, g);
                g = F::mulmod(g, x32);
            }
        }
    }
    if (tid < 16u) { W1[k + tid] = 0; W0[k + tid] = 0; }   // the window of the last phase reads a little past W_{k-1}
    __syncthreads();
    TOPLOC_TICK_END(tables, 8);
    TOPLOC_TICK_BEGIN(denom);
    // ---- d_j = sum_r1 x_j^(16 r1) * (sum_r0 W'_(16 r1 + r0) x_j^r0); a_j = y_j / d_j; BT[r0][j] <- a_j x_j^r0 ----
    {
        const uint32_t j = o;
        if (j < k) {
            uint64_t dacc = 0;
            for (uint32_t r1 = h; r1 < n_giant; r1 += 2u) {
                const u32v4 w1 = *reinterpret_cast<const u32v4*>(&s.wd_hi[r1 * kBaby]);   // the same 16 coefficients for every lane
                const u32v4 w0 = *reinterpret_cast<const u32v4*>(&s.wd_lo[r1 * kBaby]);
                PlaneAcc acc;
                acc.step(w1.x, w0.x, pw1[0], pw0[0]);
                acc.step(w1.y, w0.y, pw1[1], pw0[1]);
                acc.step(w1.z, w0.z, pw1[2], pw0[2]);
                acc.step(w1.w, w0.w, pw1[3], pw0[3]);
                dacc += (uint64_t)mul24(acc.value_short(), plane_get(s.u.pw.g_hi, s.u.pw.g_lo, r1 * KMAX + j));
            }
            uint32_t dsum = reduce64(dacc);
            dsum = F::addmod(dsum, pair_swap(dsum));
            if (h == 0) s.dj[j] = (typename Sh::E)dsum;
        }
    }
    __syncthreads();
    // The inverses: a quarter of the waves take two points per lane and invert the product of their two
    // denominators (1/d0 = d1/(d0 d1), 1/d1 = d0/(d0 d1)), so the exponentiation runs once per two points
    // and on a quarter of the waves only; which quarter rotates with the workgroup so that, with several
    // workgroups on a CU, the chains spread over the SIMDs.  The denominators of distinct points are
    // non-zero (products of differences), so the product has an inverse.
    {
        constexpr uint32_t LANES = KMAX / 2;                  // lanes that invert
        static_assert(LANES % 64 == 0, "whole waves invert");
        const uint32_t w0 = (blockIdx.x & 3u) * LANES;        // THREADS = 4 LANES
        if (tid - w0 < LANES) {                               // whole waves (LANES is a multiple of 64)
            const uint32_t j0 = 2u * (tid - w0), j1 = j0 + 1u;
            if (j0 < k) {
                const uint32_t d0 = s.dj[j0];
                const uint32_t d1 = j1 < k ? (uint32_t)s.dj[j1] : 1u;
                const uint32_t inv01 = F::inv(F::mulmod(d0, d1));
                s.dj[j0] = (typename Sh::E)F::mulmod(s.ys[j0], F::mulmod(inv01, d1));
                if (j1 < k) s.dj[j1] = (typename Sh::E)F::mulmod(s.ys[j1], F::mulmod(inv01, d0));
            }
        }
    }
    __syncthreads();
    // BT[r0][j] <- a_j x_j^r0 (the power sums then need no scaled copy of the giant steps): the two lanes of a
    // point take eight powers each, the second one starting from a_j x_j^8
    {
        const uint32_t j = o;
        if (j < k16) {   // the lanes of the padding points write the zeros the sums read there
            const uint32_t a = j < k ? (uint32_t)s.dj[j] : 0u;
            const uint32_t x = j < k ? (uint32_t)s.xs[j] : 0u;
            const uint32_t x8 = ((pw1[2] & 0xFFu) << 8) | (pw0[2] & 0xFFu);
            uint32_t p = h ? F::mulmod(a, x8) : a;
#pragma unroll
            for (uint32_t i = 0; i < kBaby / 2u; ++i) {
                const uint32_t at = (h * (kBaby / 2u) + i) * Sh::BT_STRIDE + j;
                s.u.pw.bt_hi[at] = (uint8_t)(p >> 8);
                s.u.pw.bt_lo[at] = (uint8_t)p;
                p = F::mulmod(p, x);
            }
        }
    }
    __syncthreads();
    TOPLOC_TICK_END(denom, 9);
    TOPLOC_TICK_BEGIN(sums);
    // ---- S_r = sum_j x_j^(16 r1) (a_j x_j^r0), r = 16 r1 + r0: a dot product of two contiguous planes ----
    {
        const uint32_t r = o;
        if (r < k) {
            const uint32_t r1 = r / kBaby, r0 = r % kBaby;
            const uint32_t half = (n_giant + 1u) >> 1;                 // rows of 16 bytes: this lane's share of j
            const uint32_t first = h ? half : 0u, mine = h ? n_giant - half : half;
            const u32v4* a1 = reinterpret_cast<const u32v4*>(&s.u.pw.g_hi[r1 * KMAX]) + first;
            const u32v4* a0 = reinterpret_cast<const u32v4*>(&s.u.pw.g_lo[r1 * KMAX]) + first;
            const u32v4* b1 = reinterpret_cast<const u32v4*>(&s.u.pw.bt_hi[r0 * Sh::BT_STRIDE]) + first;
            const u32v4* b0 = reinterpret_cast<const u32v4*>(&s.u.pw.bt_lo[r0 * Sh::BT_STRIDE]) + first;
            PlaneAcc acc;
#pragma unroll 2
            for (uint32_t q = 0; q < mine; ++q) {
                const u32v4 x1 = a1[q], x0 = a0[q], y1 = b1[q], y0 = b0[q];
                acc.step(x1.x, x0.x, y1.x, y0.x);
                acc.step(x1.y, x0.y, y1.y, y0.y);
                acc.step(x1.z, x0.z, y1.z, y0.z);
                acc.step(x1.w, x0.w, y1.w, y0.w);
            }
            uint32_t v = acc.value();
            v = F::addmod(v, pair_swap(v));
            if (h == 0) plane_put(s.s_hi, s.s_lo, r, v);
        }
    }
    __syncthreads();
    TOPLOC_TICK_END(sums, 10);
    TOPLOC_TICK_BEGIN(coefs);
    // ---- c_i = sum_{r=0}^{k-1-i} W_{i+1+r} S_r; the last term meets W_k = 1 ----
    {
        const uint32_t i = o;
        if (i < k) {
            const uint32_t last = k - 1u - i;
            const uint32_t n4 = (last + 3u) >> 2;    // words of four terms; W reads as zero from k on
            const uint32_t half = (n4 + 1u) >> 1;
            const uint32_t first = h ? half : 0u, mine = h ? n4 - half : half;
            PlaneAcc acc;
            if (mine)
                plane_dot_window(acc, reinterpret_cast<const uint32_t*>(s.s_hi) + first, reinterpret_cast<const uint32_t*>(s.s_lo) + first,
                                 reinterpret_cast<const uint32_t*>(W1), reinterpret_cast<const uint32_t*>(W0), i + 1u + 4u * first, mine);
            uint32_t c = acc.value();
            c = F::addmod(c, pair_swap(c));
            if (h == 0) coef_out[i] = F::addmod(c, plane_get(s.s_hi, s.s_lo, last));
        }
    }
    __syncthreads();
    TOPLOC_TICK_END(coefs, 11);
}

}  // namespace toploc
