// Exact top-k by magnitude over one chunk of bf16 patterns, one workgroup per
// chunk, one pass over HBM.  This is topk(h, k) of the paper's Algorithm 1 and
// Algorithm 2 ("top-k magnitude elements", Section 5.3) with the total order
//     a before b  <=>  |a| > |b|  or  (|a| == |b| and index(a) < index(b)),
// |x| taken as the integer (bits & 0x7FFF).
//
// Method (a streaming filter with a rising threshold, not a sort):
//   * every lane reads 16 bytes (8 values) per load, U loads per round;
//   * a value is a candidate when it comes before the current threshold element
//     (tm, ti); the first, coarse test is one packed 16-bit max over the 8 values
//     against tm, so in steady state a wave spends ~1.3 VALU ops per value;
//   * candidates go to an LDS buffer through a wave-aggregated counter;
//   * when the buffer passes its soft limit the workgroup prunes it to the exact
//     best k (radix select on the 8-bit exponent, then the 7-bit mantissa, then the
//     index among equal magnitudes) and the k-th survivor becomes the threshold;
//   * a buffer overflow loses nothing: the values of the round are still in
//     registers, the lanes that found no room retry after the prune.
// Since the threshold is always an element that k-1 seen elements precede, a value
// that fails the test can never belong to the top-k, so the result is exact and
// independent of the order in which waves append.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace toploc {

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int THREADS, int CAP>
struct SelectShared {
    uint32_t cand_idx[CAP];   // flat index of a candidate
    uint16_t cand_bits[CAP];  // its bf16 pattern
    uint16_t eq_slot[CAP];    // prune: slots whose magnitude equals the new threshold
    uint32_t hist_e[256];     // prune: exponent histogram
    uint32_t hist_m[128];     // prune: mantissa histogram inside the threshold exponent
    uint32_t count;           // slots handed out (may run past CAP on overflow)
    uint32_t eq_count;
    int32_t tm;               // threshold magnitude
    uint32_t ti;              // threshold index
    uint32_t flag[3];         // "buffer passed the soft limit" for barrier round r mod 3
};

__device__ __forceinline__ uint32_t lane_id() { return __lane_id(); }

// Suffix search over a histogram held 'BPL' bins per lane by one wave: returns the
// bin b (scanning from the highest bin down) at which the running count
// above0 + sum_{b' > b} hist[b'] first reaches k when hist[b] is added, and that
// running count ("above", the number of entries strictly above bin b).
template <int BPL>
__device__ __forceinline__ void find_bin(const uint32_t* hist, uint32_t above0, uint32_t k,
                                         uint32_t& bin, uint32_t& above)
{
    const uint32_t lane = lane_id();
    uint32_t own[BPL];
    uint32_t t = 0;
#pragma unroll
    for (int b = 0; b < BPL; ++b) { own[b] = hist[lane * BPL + b]; t += own[b]; }
    uint32_t v = t;  // inclusive suffix sum over lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        uint32_t o = __shfl_down(v, d);
        if (lane + d < 64) v += o;
    }
    uint32_t a = above0 + (v - t);
    uint32_t fbin = 0, fabove = 0;
    bool found = false;
#pragma unroll
    for (int b = BPL - 1; b >= 0; --b) {
        if (!found && a < k && a + own[b] >= k) { found = true; fbin = lane * BPL + b; fabove = a; }
        a += own[b];
    }
    uint64_t mask = __ballot(found);
    int src = mask ? (__ffsll((long long)mask) - 1) : 0;
    bin = __shfl(fbin, src);
    above = __shfl(fabove, src);
}

// Wave-aggregated append. Returns true for a lane that passed but found no room.
template <int THREADS, int CAP>
__device__ __forceinline__ bool append(SelectShared<THREADS, CAP>& s, bool pass, uint32_t idx, uint32_t bits,
                                       uint32_t soft, uint32_t* flag)
{
    const uint64_t mask = __ballot(pass);
    if (mask == 0) return false;
    const uint32_t lane = lane_id();
    const int leader = __ffsll((long long)mask) - 1;
    const uint32_t n = __popcll(mask);
    uint32_t base = 0;
    if ((int)lane == leader) {
        base = atomicAdd(&s.count, n);
        if (base + n > soft) *flag = 1u;
    }
    base = __shfl(base, leader);
    const uint32_t slot = base + __popcll(mask & ((1ull << lane) - 1ull));
    if (pass && slot < (uint32_t)CAP) {
        s.cand_idx[slot] = idx;
        s.cand_bits[slot] = (uint16_t)bits;
        return false;
    }
    return pass;
}

// Reduce the buffer to the exact best k entries and set the threshold to the k-th.
// Called by all threads. On return count == min(k, entries) and *overflow tells
// whether some lanes could not append in the round before.
template <int THREADS, int CAP>
__device__ __attribute__((noinline)) void prune(SelectShared<THREADS, CAP>& s, uint32_t k, int32_t& tm, uint32_t& ti, bool& overflow)
{
    constexpr int EPT = CAP / THREADS;
    const uint32_t tid = threadIdx.x;
    __syncthreads();  // appends of the round are visible
    const uint32_t raw = s.count;
    overflow = raw > (uint32_t)CAP;
    const uint32_t M = overflow ? (uint32_t)CAP : raw;
    if (M <= k) {  // nothing to drop (uniform decision)
        __syncthreads();
        return;
    }
    uint32_t idx[EPT];
    uint32_t bits[EPT];
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const uint32_t slot = tid + i * THREADS;
        idx[i] = 0; bits[i] = 0;
        if (slot < M) { idx[i] = s.cand_idx[slot]; bits[i] = s.cand_bits[slot]; }
    }
    for (uint32_t b = tid; b < 256; b += THREADS) s.hist_e[b] = 0;
    for (uint32_t b = tid; b < 128; b += THREADS) s.hist_m[b] = 0;
    __syncthreads();  // everyone holds its entries and has read `raw`
    if (tid == 0) { s.count = 0; s.eq_count = 0; }
#pragma unroll
    for (int i = 0; i < EPT; ++i)
        if (tid + i * THREADS < M) atomicAdd(&s.hist_e[(bits[i] & 0x7FFFu) >> 7], 1u);
    __syncthreads();
    uint32_t e_star, above_e;
    find_bin<4>(s.hist_e, 0u, k, e_star, above_e);
#pragma unroll
    for (int i = 0; i < EPT; ++i)
        if (tid + i * THREADS < M && ((bits[i] & 0x7FFFu) >> 7) == e_star) atomicAdd(&s.hist_m[bits[i] & 0x7Fu], 1u);
    __syncthreads();
    uint32_t m_star, g;
    find_bin<2>(s.hist_m, above_e, k, m_star, g);
    const uint32_t new_tm = (e_star << 7) | m_star;
    const uint32_t need = k - g;  // how many of the entries with magnitude new_tm survive (>= 1)
#pragma unroll
    for (int i = 0; i < EPT; ++i)
        if (tid + i * THREADS < M && (bits[i] & 0x7FFFu) == new_tm) {
            const uint32_t q = atomicAdd(&s.eq_count, 1u);
            s.eq_slot[q] = (uint16_t)(tid + i * THREADS);
        }
    __syncthreads();
    const uint32_t E = s.eq_count;
    // the need-th smallest index among the E equal-magnitude entries is the new threshold element
    for (uint32_t q = tid; q < E; q += THREADS) {
        const uint32_t mine = s.cand_idx[s.eq_slot[q]];
        uint32_t rank = 0;
        for (uint32_t u = 0; u < E; ++u) rank += (s.cand_idx[s.eq_slot[u]] < mine) ? 1u : 0u;
        if (rank == need - 1) { s.ti = mine; s.tm = (int32_t)new_tm; }
    }
    __syncthreads();
    tm = s.tm;
    ti = s.ti;
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        if (tid + i * THREADS < M) {
            const int32_t mag = (int32_t)(bits[i] & 0x7FFFu);
            if (mag > tm || (mag == tm && idx[i] <= ti)) {
                const uint32_t q = atomicAdd(&s.count, 1u);
                s.cand_idx[q] = idx[i];
                s.cand_bits[q] = (uint16_t)bits[i];
            }
        }
    }
    __syncthreads();
}

// Top-k of src[0 .. 8*nvec) into s.cand_idx / s.cand_bits [0 .. k), in the order
// (magnitude descending, index ascending).  Requires k <= 8*nvec, k <= CAP/2,
// 8*nvec < 2^32.  All threads of the workgroup call it; it ends with a barrier.
template <int THREADS, int U, int CAP>
__device__ void select_topk(const u32x4* __restrict__ src, uint32_t nvec, uint32_t k, SelectShared<THREADS, CAP>& s)
{
    static_assert(CAP % THREADS == 0, "CAP must be a multiple of THREADS");
    static_assert(U >= 1 && U <= 4, "pending mask holds 8 bits per load");
    constexpr uint32_t SOFT = CAP / 2;
    const uint32_t tid = threadIdx.x;
    if (tid == 0) {
        s.count = 0; s.eq_count = 0; s.tm = 0; s.ti = 0xFFFFFFFFu;
        s.flag[0] = 0; s.flag[1] = 0; s.flag[2] = 0;
    }
    __syncthreads();
    int32_t tm = 0;            // everything comes before (0, 0xFFFFFFFF): the buffer is empty
    uint32_t ti = 0xFFFFFFFFu;
    uint32_t round = 0;        // barrier rounds; flag[round % 3] belongs to the current one

    for (uint32_t base = 0; base < nvec; base += THREADS * U) {
        u32x4 r[U];
        uint32_t pend = 0;     // bit 8u+e: value e of load u still has to be placed
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t v = base + u * THREADS + tid;
            r[u] = u32x4{0u, 0u, 0u, 0u};
            if (v < nvec) { r[u] = __builtin_nontemporal_load(src + v); pend |= 0xFFu << (8 * u); }
        }
        // coarse filter: the largest of the 8 magnitudes against the threshold magnitude
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t a = r[u].x & 0x7FFF7FFFu, b = r[u].y & 0x7FFF7FFFu;
            const uint32_t c = r[u].z & 0x7FFF7FFFu, d = r[u].w & 0x7FFF7FFFu;
            u16x2 m01 = __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b));
            u16x2 m23 = __builtin_elementwise_max(__builtin_bit_cast(u16x2, c), __builtin_bit_cast(u16x2, d));
            u16x2 mm = __builtin_elementwise_max(m01, m23);
            const int32_t mx = (int32_t)(mm.x > mm.y ? mm.x : mm.y);
            if (mx < tm) pend &= ~(0xFFu << (8 * u));
        }
        while (true) {
            uint32_t* flag = &s.flag[round % 3u];
            if (__any(pend != 0)) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    uint32_t pu = (pend >> (8 * u)) & 0xFFu;
                    if (!__any(pu != 0)) continue;
                    const uint32_t ebase = (base + u * THREADS + tid) * 8u;
#pragma unroll 1
                    for (uint32_t e = 0; e < 8; ++e) {
                        const uint32_t q = e >> 1;
                        const uint32_t w = q == 0 ? r[u].x : q == 1 ? r[u].y : q == 2 ? r[u].z : r[u].w;
                        const uint32_t bits = (w >> (16u * (e & 1u))) & 0xFFFFu;
                        const int32_t mag = (int32_t)(bits & 0x7FFFu);
                        const uint32_t idx = ebase + e;
                        const bool pass = ((pu >> e) & 1u) && (mag > tm || (mag == tm && idx < ti));
                        const bool over = append<THREADS, CAP>(s, pass, idx, bits, SOFT, flag);
                        if (!over) pu &= ~(1u << e);
                    }
                    pend = (pend & ~(0xFFu << (8 * u))) | (pu << (8 * u));
                }
            }
            __syncthreads();
            const uint32_t f = *flag;
            if (tid == 0) s.flag[(round + 2u) % 3u] = 0;  // the previous round's flag: read by all before this barrier
            ++round;
            if (!f) break;
            bool overflow;
            prune<THREADS, CAP>(s, k, tm, ti, overflow);
            if (!overflow) break;
        }
    }
    __syncthreads();
    if (s.count > k) {  // uniform: nobody appends any more
        bool overflow;
        prune<THREADS, CAP>(s, k, tm, ti, overflow);
    }
    // order the k survivors: rank = number of survivors that come before
    constexpr int KPT = (CAP / 2 + THREADS - 1) / THREADS;
    uint32_t my_idx[KPT], my_bits[KPT], my_rank[KPT];
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const uint32_t t = tid + i * THREADS;
        my_idx[i] = 0; my_bits[i] = 0; my_rank[i] = 0;
        if (t < k) {
            my_idx[i] = s.cand_idx[t];
            my_bits[i] = s.cand_bits[t];
            const uint32_t mag = my_bits[i] & 0x7FFFu;
            uint32_t rank = 0;
            for (uint32_t u = 0; u < k; ++u) {
                const uint32_t om = s.cand_bits[u] & 0x7FFFu;
                const uint32_t oi = s.cand_idx[u];
                rank += (om > mag || (om == mag && oi < my_idx[i])) ? 1u : 0u;
            }
            my_rank[i] = rank;
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        if (tid + i * THREADS < k) {
            s.cand_idx[my_rank[i]] = my_idx[i];
            s.cand_bits[my_rank[i]] = (uint16_t)my_bits[i];
        }
    }
    __syncthreads();
}

}  // namespace toploc
