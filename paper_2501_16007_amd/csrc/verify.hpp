// The paper's Algorithm 2 after topk(h, k) for one chunk, one workgroup: decode,
// index map, Horner evaluation of the proof polynomial at the k mapped indices
// (Algorithm 5), extractBits, the err_e / err_m statistics and the three thresholds
// (Section 5.2).  All integer arithmetic; err_m is kept as a 128-bin histogram so that
// the mean test and the median are exact.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/toploc.h"
#include "gf65497.hpp"
#include "interp.hpp"

namespace toploc {

template <int KMAX>
struct VerifyShared {
    uint32_t coef[KMAX];     // c_0..c_{k-1}
    uint32_t hist_d[128];    // err_m as a histogram of |m_p - m_v| in [0, 127]
    uint32_t err_e, mant_sum, bad, m;
};

// decode(p): coefficients and modulus into LDS.  Returns false (uniformly) for a
// malformed proof, after writing its result record.  All threads call; ends with a barrier.
template <int THREADS, int KMAX>
__device__ __forceinline__ bool verify_decode(VerifyShared<KMAX>& vs, const uint16_t* __restrict__ proof, uint32_t k,
                                              toploc_verify_result* __restrict__ result)
{
    const uint32_t tid = threadIdx.x;
    if (tid == 0) { vs.err_e = 0; vs.mant_sum = 0; vs.bad = 0; }
    for (uint32_t b = tid; b < 128; b += THREADS) vs.hist_d[b] = 0;
    __syncthreads();
    const uint32_t mf = proof[0];
    const uint32_t m = mf ? mf : kModHigh;   // the 2-byte field stores m mod 65536
    for (uint32_t j = tid; j < k; j += THREADS) {
        const uint32_t c = proof[1 + j];
        vs.coef[j] = c;
        if (c >= kPrime) vs.bad = 1u;
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

// The loop and the decision of Algorithm 2 over the k selected (index, pattern) pairs
// in LDS (any order).  All threads call.
template <int THREADS, int KMAX>
__device__ __forceinline__ void verify_tail(VerifyShared<KMAX>& vs, const uint32_t* cand_idx, const uint16_t* cand_bits,
                                            uint32_t k, const toploc_thresholds& thr,
                                            toploc_verify_result* __restrict__ result)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t m = vs.m;
    for (uint32_t j = tid; j < k; j += THREADS) {
        uint32_t x = cand_idx[j] % m;
        x = x >= kPrime ? x - kPrime : x;
        uint32_t acc = vs.coef[k - 1];
        for (int i = (int)k - 2; i >= 0; --i) acc = muladdmod(acc, x, vs.coef[i]);
        const uint32_t v = cand_bits[j];
        const uint32_t e_p = (acc >> 7) & 0xFFu, m_p = acc & 0x7Fu;
        const uint32_t e_v = (v >> 7) & 0xFFu, m_v = v & 0x7Fu;
        if (e_p == e_v) {
            const uint32_t d = m_p > m_v ? m_p - m_v : m_v - m_p;
            atomicAdd(&vs.hist_d[d], 1u);
            atomicAdd(&vs.mant_sum, d);
        } else {
            atomicAdd(&vs.err_e, 1u);
        }
    }
    __syncthreads();
    if (tid < 64) {
        // |err_m| and its lower median from the histogram: the smallest d whose
        // cumulative count reaches floor((n-1)/2) + 1
        const uint32_t h0 = vs.hist_d[2 * tid], h1 = vs.hist_d[2 * tid + 1];
        uint32_t v = h0 + h1;  // inclusive prefix sum over lanes
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(v, d);
            if ((int)tid >= d) v += o;
        }
        const uint32_t n = __shfl(v, 63);
        const uint32_t target = n ? (n - 1) / 2 + 1 : 0;
        const uint32_t before = v - h0 - h1;
        uint32_t med = 0xFFFFFFFFu;
        if (n && before < target && before + h0 >= target) med = 2 * tid;
        else if (n && before + h0 < target && v >= target) med = 2 * tid + 1;
        const uint64_t mask = __ballot(med != 0xFFFFFFFFu);
        const int srcl = mask ? (__ffsll((long long)mask) - 1) : 0;
        med = __shfl(med, srcl);
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
}

}  // namespace toploc
