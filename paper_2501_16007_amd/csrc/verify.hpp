// The paper's Algorithm 2 after topk(h, k) for one chunk, one workgroup: decode,
// index map, Horner evaluation of the proof polynomial at the k mapped indices
// (Algorithm 5), extractBits, the err_e / err_m statistics and the three thresholds
// (Section 5.2).  All integer arithmetic.  Over GF(65497) the evaluation groups the coefficients in
// blocks of sixteen (sums of products on the packed dot-product instruction, planes.hpp) and runs
// Horner over the blocks; the value is that of Algorithm 5.
//
// Two precisions meet here (Section 5.7): the proof's (its field F: GF(65497) carries
// bf16 patterns, GF(2^32 - 5) fp32 patterns) and the validator's (the format of the
// recomputed activations).  Exponent and mantissa are compared in the validator's
// precision: an fp32 proof value met by bf16 activations has its 23-bit mantissa scaled
// down to 7 bits (>> 16), a bf16 proof value met by fp32 activations gets 16 zero bits
// appended (<< 16).  With a bf16 validator err_m lies in [0, 127] and is kept as a
// histogram, so the mean test and the median are exact; with an fp32 validator the
// differences (< 2^23) are kept as a list and the lower median is found by rank.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/toploc.h"
#include "gf32.hpp"
#include "gf65497.hpp"
#include "interp.hpp"
#include "planes.hpp"
#include "select.hpp"

#ifndef TOPLOC_HORNER_LANES
#define TOPLOC_HORNER_LANES 2
#endif

namespace toploc {

template <int KMAX, bool WIDE = false>
struct VerifyShared {
    uint32_t coef[KMAX];                 // c_0..c_{k-1}  (proofs over GF(2^32 - 5); unused with GF(65497))
    alignas(16) uint8_t c_hi[KMAX], c_lo[KMAX];   // proofs over GF(65497): the coefficients as byte planes, zeros from k to the next multiple of 16
    uint32_t hist_d[128];                // bf16 validator: err_m as a histogram of |m_p - m_v| in [0, 127]
    uint32_t diffs[WIDE ? KMAX : 1];     // fp32 validator: err_m as a list
    uint32_t err_e, mant_sum, bad, m, n_match, median;
};

// The words of a proof as the lanes read them from global memory: issued early (before the
// chunk's first loads, which return in order behind them), used by verify_decode.
template <int THREADS, int KMAX>
struct ProofWords {
    static constexpr int PER_LANE = (KMAX + THREADS - 1) / THREADS;
    uint32_t mf;            // the 2-byte modulus field
    uint32_t c[PER_LANE];   // coefficients tid, tid + THREADS, ..
};

template <int THREADS, typename F, int KMAX>
__device__ __forceinline__ ProofWords<THREADS, KMAX> verify_load_proof(const uint16_t* __restrict__ proof, uint32_t k)
{
    ProofWords<THREADS, KMAX> w;
    w.mf = proof[0];
#pragma unroll
    for (int i = 0; i < ProofWords<THREADS, KMAX>::PER_LANE; ++i) {
        const uint32_t j = threadIdx.x + i * THREADS;
        uint32_t c = 0;
        if (j < k) {
            c = proof[1 + j * F::WORDS];
            if (F::WORDS == 2) c |= (uint32_t)proof[2 + j * F::WORDS] << 16;
        }
        w.c[i] = c;
    }
    return w;
}

// decode(p): coefficients and modulus into LDS.  Returns false (uniformly) for a
// malformed proof, after writing its result record.  All threads call; ends with a barrier.
template <int THREADS, typename F, int KMAX, bool WIDE>
__device__ __forceinline__ bool verify_decode(VerifyShared<KMAX, WIDE>& vs, const ProofWords<THREADS, KMAX>& w, uint32_t k,
                                              toploc_verify_result* __restrict__ result)
{
    const uint32_t tid = threadIdx.x;
    if (tid == 0) { vs.err_e = 0; vs.mant_sum = 0; vs.bad = 0; vs.n_match = 0; vs.median = 0; }
    for (uint32_t b = tid; b < 128; b += THREADS) vs.hist_d[b] = 0;
    __syncthreads();
    const uint32_t m = w.mf ? w.mf : kModHigh;   // the 2-byte field stores m mod 65536
    static_assert(KMAX % 16 == 0, "the coefficient planes are read 16 bytes at a time");
#pragma unroll
    for (int i = 0; i < ProofWords<THREADS, KMAX>::PER_LANE; ++i) {
        const uint32_t j = tid + i * THREADS;
        if (j < k) {
            if (F::WORDS == 1) { vs.c_hi[j] = (uint8_t)(w.c[i] >> 8); vs.c_lo[j] = (uint8_t)w.c[i]; }
            else vs.coef[j] = w.c[i];
            if (w.c[i] >= F::P) vs.bad = 1u;
        } else if (F::WORDS == 1 && j < ((k + 15u) & ~15u)) {
            vs.c_hi[j] = 0;
            vs.c_lo[j] = 0;
        }
    }
    if (tid == 0) {
        vs.m = m;
        if (m < kModLow) vs.bad = 1u;
    }
    __syncthreads();
    if (vs.bad) {  // uniform
        if (tid == 0) {
            toploc_verify_result r = {};
            r.status = TOPLOC_CHUNK_MALFORMED;
            *result = r;
        }
        return false;
    }
    return true;
}

template <int THREADS, typename F, int KMAX, bool WIDE>
__device__ __forceinline__ bool verify_decode(VerifyShared<KMAX, WIDE>& vs, const uint16_t* __restrict__ proof, uint32_t k,
                                              toploc_verify_result* __restrict__ result)
{
    return verify_decode<THREADS, F>(vs, verify_load_proof<THREADS, F, KMAX>(proof, k), k, result);
}

// extractBits of a proof value (a pattern of the field's precision), expressed in the
// validator's precision Fmt
template <typename F, typename Fmt>
__device__ __forceinline__ void extract_proof_bits(uint32_t p, uint32_t& e, uint32_t& mant)
{
    if (F::WORDS == 2) { e = (p >> 23) & 0xFFu; mant = p & 0x7FFFFFu; }
    else               { e = (p >> 7) & 0xFFu;  mant = p & 0x7Fu; }
    if (F::WORDS == 2 && Fmt::ELEMS == 8) mant >>= 16;   // fp32 mantissa scaled to bf16's width
    if (F::WORDS == 1 && Fmt::ELEMS == 4) mant <<= 16;   // 16 zero bits appended to the bf16 pattern
}

// The loop and the decision of Algorithm 2 over the k selected (index, pattern) pairs
// in LDS (any order).  All threads call.
template <int THREADS, typename F, typename Fmt, int KMAX, bool WIDE>
__device__ __forceinline__ void verify_tail(VerifyShared<KMAX, WIDE>& vs, const uint32_t* cand_idx,
                                            const typename Fmt::bits_t* cand_bits, uint32_t k, const toploc_thresholds& thr,
                                            toploc_verify_result* __restrict__ result)
{
    static_assert(WIDE == (Fmt::ELEMS == 4), "an fp32 validator keeps err_m as a list");
    const uint32_t tid = threadIdx.x;
    const uint32_t m = vs.m;
    // With lanes to spare two lanes share a point: P(x) = E(y) + x' O(y) with the terms split by parity, two
    // chains of half the length (the chain is the tail's critical path).
    constexpr int L = (2 * KMAX <= THREADS && TOPLOC_HORNER_LANES == 2) ? 2 : 1;
    const uint32_t h = (L == 2) ? (tid & 1u) : 0u;
    for (uint32_t j = tid / L; j < k; j += THREADS / L) {
        const uint32_t x = F::from_residue(cand_idx[j] % m);
        uint32_t acc;
        if (F::WORDS == 1) {
            // GF(65497): P(x) = sum_r1 X^r1 I_r1(x), X = x^16, I_r1(x) = sum_r0 c_(16 r1 + r0) x^r0 a 16-term sum of
            // products on the packed dot-product instruction (coefficients and powers as byte planes), Horner over r1
            // in X (two lanes: even and odd r1 in X^2): k/16 dependent steps instead of k
            uint32_t pw1[4], pw0[4];
            const uint32_t X = plane_powers16(x, pw1, pw0);
            const uint32_t step = (L == 2) ? mulmod(X, X) : X;
            const uint32_t n_giant = (k + 15u) >> 4;
            const int terms = (int)((n_giant - h + (uint32_t)L - 1u) / (uint32_t)L);   // r1 = h, h + L, ..
            acc = 0;
#pragma unroll 2
            for (int i = terms - 1; i >= 0; --i) {
                const uint32_t r1 = (uint32_t)i * (uint32_t)L + h;
                const u32v4 w1 = *reinterpret_cast<const u32v4*>(&vs.c_hi[r1 * 16u]);   // the same 16 coefficients for every lane
                const u32v4 w0 = *reinterpret_cast<const u32v4*>(&vs.c_lo[r1 * 16u]);
                PlaneAcc inner;
                inner.step(w1.x, w0.x, pw1[0], pw0[0]);
                inner.step(w1.y, w0.y, pw1[1], pw0[1]);
                inner.step(w1.z, w0.z, pw1[2], pw0[2]);
                inner.step(w1.w, w0.w, pw1[3], pw0[3]);
                acc = muladdmod(acc, step, inner.value_short());
            }
            if (L == 2) {
                const uint32_t odd = pair_swap(acc);          // the partner's chain
                acc = muladdmod(odd, X, acc);                 // meaningful in the even lane
                if (h) continue;
            }
        } else if (L == 2) {
            const uint32_t x2 = F::mulmod(x, x);
            const int terms = (int)((k - h + 1u) / 2u);   // coefficients h, h + 2, ...
            acc = 0;
#pragma unroll 8   // eight coefficient reads in flight per round trip to LDS instead of one
            for (int i = terms - 1; i >= 0; --i) acc = F::muladdmod(acc, x2, vs.coef[2 * i + (int)h]);
            const uint32_t odd = __shfl_xor(acc, 1);      // the partner's chain
            acc = F::muladdmod(odd, x, acc);              // meaningful in the even lane
            if (h) continue;
        } else {
            acc = vs.coef[k - 1];
#pragma unroll 8
            for (int i = (int)k - 2; i >= 0; --i) acc = F::muladdmod(acc, x, vs.coef[i]);
        }
        const uint32_t v = cand_bits[j];
        uint32_t e_p, m_p, e_v, m_v;
        extract_proof_bits<F, Fmt>(acc, e_p, m_p);
        if (Fmt::ELEMS == 4) { e_v = (v >> 23) & 0xFFu; m_v = v & 0x7FFFFFu; }
        else                 { e_v = (v >> 7) & 0xFFu;  m_v = v & 0x7Fu; }
        if (e_p == e_v) {
            const uint32_t d = m_p > m_v ? m_p - m_v : m_v - m_p;
            if (WIDE) vs.diffs[atomicAdd(&vs.n_match, 1u)] = d;
            else atomicAdd(&vs.hist_d[d], 1u);
            atomicAdd(&vs.mant_sum, d);   // k * (2^23 - 1) < 2^32 for k <= 512
        } else {
            atomicAdd(&vs.err_e, 1u);
        }
    }
    __syncthreads();
    uint32_t n, med = 0;
    if (WIDE) {
        // lower median by rank: the entry that floor((n-1)/2) entries precede, ties by slot
        n = vs.n_match;
        const uint32_t target = n ? (n - 1) / 2 : 0;
        for (uint32_t j = tid; j < n; j += THREADS) {
            const uint32_t mine = vs.diffs[j];
            uint32_t rank = 0;
            for (uint32_t u = 0; u < n; ++u) {
                const uint32_t o = vs.diffs[u];
                rank += (o < mine || (o == mine && u < j)) ? 1u : 0u;
            }
            if (rank == target) vs.median = mine;
        }
        __syncthreads();
        med = vs.median;
    } else if (tid < 64) {
        // |err_m| and its lower median from the histogram: the smallest d whose
        // cumulative count reaches floor((n-1)/2) + 1
        const uint32_t h0 = vs.hist_d[2 * tid], h1 = vs.hist_d[2 * tid + 1];
        const uint32_t v = wave_prefix_sum(h0 + h1);  // inclusive prefix sum over lanes
        n = (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
        const uint32_t target = n ? (n - 1) / 2 + 1 : 0;
        const uint32_t before = v - h0 - h1;
        med = 0xFFFFFFFFu;
        if (n && before < target && before + h0 >= target) med = 2 * tid;
        else if (n && before + h0 < target && v >= target) med = 2 * tid + 1;
        const uint64_t mask = __ballot(med != 0xFFFFFFFFu);
        const int srcl = mask ? (__ffsll((long long)mask) - 1) : 0;  // uniform
        med = (uint32_t)__builtin_amdgcn_readlane((int)med, srcl);
    } else {
        n = 0;
    }
    if (tid == 0) {
        toploc_verify_result r = {};
        r.err_exp = vs.err_e;
        r.n_match = n;
        r.mant_sum = vs.mant_sum;
        r.mant_median = n ? med : 0u;
        bool reject = vs.err_e > thr.t_exp;
        if (n) {
            if ((uint64_t)vs.mant_sum > (uint64_t)thr.t_mean * n) reject = true;   // mean(err_m) > T_mean
            if (r.mant_median > thr.t_median) reject = true;
        }
        r.accept = reject ? 0 : 1;
        r.status = TOPLOC_CHUNK_OK;
        *result = r;
    }
}

}  // namespace toploc
