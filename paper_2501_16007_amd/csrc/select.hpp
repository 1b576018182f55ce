// Exact top-k by magnitude over one chunk of bf16 (or fp32) patterns, one workgroup per
// chunk, one pass over HBM.  This is topk(h, k) of the paper's Algorithm 1 and
// Algorithm 2 (Section 5.3 ranks the elements by magnitude) with the total order
//     a before b  <=>  |a| > |b|  or  (|a| == |b| and index(a) < index(b)),
// |x| taken as the integer (bits & 0x7FFF), for fp32 (bits & 0x7FFFFFFF).
//
// Method (a streaming filter with a rising threshold, not a sort):
//   * every lane reads 16 bytes (8 bf16 or 4 fp32 values) per load, U loads per round, and
//     the loads of the next round are issued before the current round is examined;
//   * the hot loop does one thing per vector: the largest of its magnitudes (a packed
//     16-bit max tree for bf16) against the threshold magnitude tm, about 1.3 VALU ops
//     per value.  A vector that passes is copied whole into an LDS queue, nothing else;
//   * when the queue passes its soft limit the workgroup drains it with all lanes
//     evenly loaded: every queued value that comes before the threshold element
//     (tm, ti) goes to the candidate buffer, and when that buffer passes its own
//     limit it is pruned to the exact best k (radix select on the 8-bit exponent,
//     then the mantissa, then the index among equal magnitudes); the k-th
//     survivor becomes the new threshold element;
//   * the first threshold is the k-th largest of the per-vector maxima of the first two rounds, so
//     nothing is ever flooded; a queue overflow loses nothing either: the vectors of
//     the round are still in registers and the lanes that found no room retry after
//     the drain; a candidate-buffer overflow (sorted data) is undone and redone against a bound
//     found from the queue's own values.
// The threshold is always either an element that k-1 seen elements precede or a magnitude
// that at least k seen elements reach, so a value that fails the test can never belong to
// the top-k: the result is exact and does not depend on the order in which waves run.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#ifndef TOPLOC_PRUNE_LIMIT
#define TOPLOC_PRUNE_LIMIT(cap, k) ((cap) / 2)
#endif

#include "ticks.hpp"

namespace toploc {

// prune: up to this many entries of the k-th magnitude are ranked against each other directly
// (E^2 / THREADS steps); more of them (tie-heavy data: all equal, a handful of distinct values)
// go through a radix descent over their indices
constexpr int kRankDirect = 256;

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// largest of the 8 bf16 magnitudes of a vector
__device__ __forceinline__ int32_t vec_max_mag(const u32x4& r)
{
    const uint32_t a = r.x & 0x7FFF7FFFu, b = r.y & 0x7FFF7FFFu;
    const uint32_t c = r.z & 0x7FFF7FFFu, d = r.w & 0x7FFF7FFFu;
    const u16x2 m01 = __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b));
    const u16x2 m23 = __builtin_elementwise_max(__builtin_bit_cast(u16x2, c), __builtin_bit_cast(u16x2, d));
    const u16x2 mm = __builtin_elementwise_max(m01, m23);
    return (int32_t)(mm.x > mm.y ? mm.x : mm.y);
}

// What the selection needs to know about the element type.  A 16-byte vector holds ELEMS
// patterns; the magnitude is (pattern & MAG_MASK); the prune resolves the magnitude in
// LEVELS radix digits, most significant first, digit l being width(l) bits at shift(l)
// (exponent, then mantissa pieces); half a vector (8 bytes) holds ELEMS/2 patterns.
struct Bf16Fmt {
    typedef uint16_t bits_t;
    static constexpr bool STATS = false;   // see Bf16FmtStats
    static constexpr int ELEMS = 8;
    static constexpr uint32_t MAG_MASK = 0x7FFFu;
    static constexpr int LEVELS = 2;
    static constexpr int shift(int l) { return l == 0 ? 7 : 0; }
    static constexpr int width(int l) { return l == 0 ? 8 : 7; }
    static __device__ __forceinline__ int32_t vec_max(const u32x4& r) { return vec_max_mag(r); }
    static __device__ __forceinline__ uint32_t half_elem(const u32x2& w, int e)
    {
        return (((e >> 1) ? w.y : w.x) >> (16 * (e & 1))) & 0xFFFFu;
    }
};
// The same format with the selection's event counters switched on (a measurement aid: how many
// drains and prunes a chunk costs, how many vectors were queued, how many candidates appended).
struct Bf16FmtStats : Bf16Fmt {
    static constexpr bool STATS = true;
};
struct F32Fmt {
    typedef uint32_t bits_t;
    static constexpr bool STATS = false;
    static constexpr int ELEMS = 4;
    static constexpr uint32_t MAG_MASK = 0x7FFFFFFFu;
    static constexpr int LEVELS = 4;
    static constexpr int shift(int l) { return l == 0 ? 23 : l == 1 ? 15 : l == 2 ? 7 : 0; }
    static constexpr int width(int l) { return l == 3 ? 7 : 8; }
    static __device__ __forceinline__ int32_t vec_max(const u32x4& r)
    {
        const uint32_t a = r.x & MAG_MASK, b = r.y & MAG_MASK, c = r.z & MAG_MASK, d = r.w & MAG_MASK;
        const uint32_t ab = a > b ? a : b, cd = c > d ? c : d;
        return (int32_t)(ab > cd ? ab : cd);
    }
    static __device__ __forceinline__ uint32_t half_elem(const u32x2& w, int e) { return e ? w.y : w.x; }
};

template <int THREADS, int CAP, int QCAP, typename Fmt = Bf16Fmt>
struct SelectShared {
    typedef Fmt fmt;
    u32x4 qvec[QCAP];         // queue: vectors holding at least one magnitude >= tm
    uint32_t qidx[QCAP];      // their vector index inside the chunk
    uint32_t cand_idx[CAP];   // candidates: flat index
    typename Fmt::bits_t cand_bits[CAP];  //     pattern
    uint16_t eq_slot[CAP];    // prune: slots whose magnitude equals the new threshold
    uint32_t hist[Fmt::LEVELS][256];  // prune: one histogram per radix digit
    uint32_t qcount[2];       // queue slots handed out (may run past QCAP on overflow); one counter per
                              // drain epoch, so that the next epoch's is cleared without a barrier of its own
    uint32_t count;           // candidate slots in use
    uint32_t count_base;      // `count` as the last prune (or the start) left it: what a sweep that ran past CAP
                              // falls back to.  Written by lane 0 behind a barrier, never while a sweep appends
    uint32_t eq_count;
    uint32_t found_bin, found_above;  // prune: what wave 0 found in a histogram, for the other waves
    uint32_t hole_count;      // prune: slots below k whose entry does not survive
    uint32_t move_count;      // prune: survivors at or above slot k, moved into the holes
    int32_t tm;               // threshold magnitude
    uint32_t ti;              // threshold index
    uint32_t flag[3];         // "queue passed its soft limit" for barrier round r mod 3
    uint32_t stats[Fmt::STATS ? 4 : 1];   // STATS only: drains, prunes, queued vectors, appended candidates
};
enum { kStatDrains = 0, kStatPrunes = 1, kStatQueued = 2, kStatAppended = 3 };

__device__ __forceinline__ uint32_t lane_id() { return __lane_id(); }

// A value every lane of the wave read from the same LDS word: keep it in a scalar register.
__device__ __forceinline__ uint32_t uniform(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

// Inclusive prefix sum over the 64 lanes of a wave with DPP adds: four shifts inside the
// rows of 16 lanes, then lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2
// and 3.  Lanes without a source add 0.  No LDS round trip, unlike the shuffle form.
// Every lane of the wave must be active (the callers run it in whole waves only).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, false);
}
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t v)
{
    v += dpp_or_zero<0x111, 0xF>(v);  // row_shr:1
    v += dpp_or_zero<0x112, 0xF>(v);  // row_shr:2
    v += dpp_or_zero<0x114, 0xF>(v);  // row_shr:4
    v += dpp_or_zero<0x118, 0xF>(v);  // row_shr:8
    v += dpp_or_zero<0x142, 0xA>(v);  // row_bcast:15
    v += dpp_or_zero<0x143, 0xC>(v);  // row_bcast:31
    return v;
}

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
    // entries in the lanes above this one: the wave's total minus the inclusive prefix sum
    const uint32_t incl = wave_prefix_sum(t);
    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    uint32_t a = above0 + (total - incl);
    uint32_t fbin = 0, fabove = 0;
    bool found = false;
#pragma unroll
    for (int b = BPL - 1; b >= 0; --b) {
        if (!found && a < k && a + own[b] >= k) { found = true; fbin = lane * BPL + b; fabove = a; }
        a += own[b];
    }
    const uint64_t mask = __ballot(found);
    const int src = mask ? (__ffsll((long long)mask) - 1) : 0;  // uniform
    bin = (uint32_t)__builtin_amdgcn_readlane((int)fbin, src);
    above = (uint32_t)__builtin_amdgcn_readlane((int)fabove, src);
}

// the threshold element as the lanes carry it
struct Threshold {
    int32_t tm;
    uint32_t ti;
    bool ties = false;   // uniform: the chunk has shown hundreds of values of one magnitude (set by the first threshold
                         // or by a prune; it only steers which way the overflow path goes first)
};

__device__ __forceinline__ bool before(int32_t mag, uint32_t idx, const Threshold& t)
{
    return mag > t.tm || (mag == t.tm && idx < t.ti);
}

// Prune, tie-heavy data (all equal, a handful of distinct values): the need-th smallest index among
// the E entries listed in eq_slot becomes the threshold index.  Ranking every entry against every other
// one would cost E^2 / THREADS steps; this is a radix descent over the complemented index instead (the
// need-th smallest index is the need-th largest complement), 8 bits per level.  All threads call.
template <int THREADS, int CAP, int QCAP, typename Fmt>
__device__ __forceinline__ void rank_by_radix(SelectShared<THREADS, CAP, QCAP, Fmt>& s, uint32_t E, uint32_t need,
                                           uint32_t new_tm)
{
    const uint32_t tid = threadIdx.x;
    uint32_t pre = 0, abv = 0;
#pragma unroll 1
    for (int sh = 24; sh >= 0; sh -= 8) {
        for (uint32_t b = tid; b < 256u; b += THREADS) s.hist[0][b] = 0;
        __syncthreads();
#pragma unroll 1
        for (uint32_t q = tid; q < E; q += THREADS) {
            const uint32_t ci = ~s.cand_idx[s.eq_slot[q]];
            if ((uint32_t)((uint64_t)ci >> (sh + 8)) == pre) atomicAdd(&s.hist[0][(ci >> sh) & 255u], 1u);
        }
        __syncthreads();
        if (tid < 64) {
            uint32_t d, a;
            find_bin<4>(s.hist[0], abv, need, d, a);
            if (tid == 0) { s.found_bin = d; s.found_above = a; }
        }
        __syncthreads();
        pre = (pre << 8) | uniform(s.found_bin);
        abv = uniform(s.found_above);
    }
    if (tid == 0) { s.ti = ~pre; s.tm = (int32_t)new_tm; }
}

// If the candidate buffer holds more than `limit` entries, reduce it to the exact
// best k and make the k-th the threshold element.  Called by all threads, starts with a
// barrier and, when it prunes, ends with one.  When it does not prune it ends with a
// barrier only if SYNC_AFTER: a caller whose next append to the buffer lies behind a
// barrier of its own anyway (the streaming loop: one per round) saves that one.  Returns the
// number of slots that had been handed out: a value above CAP means appends were dropped,
// and nothing is pruned then (the caller redoes them); a value in (limit, CAP] means it
// pruned and `t` is the new threshold.
template <bool SYNC_AFTER = true, int THREADS, int CAP, int QCAP, typename Fmt>
__device__ __forceinline__ uint32_t prune_if_above(SelectShared<THREADS, CAP, QCAP, Fmt>& s, uint32_t k, uint32_t limit,
                                                     Threshold& t)
{
    const uint32_t tid = threadIdx.x;
    __syncthreads();  // appends are visible
    const uint32_t M = uniform(s.count);
    if (M <= limit || M > (uint32_t)CAP) {  // uniform decision
        if (Fmt::STATS && tid == 0 && M <= (uint32_t)CAP) s.stats[kStatAppended] += M - s.count_base;
        if (tid == 0 && M <= (uint32_t)CAP) s.count_base = M;
        if (SYNC_AFTER) __syncthreads();  // everyone has read the count before anyone appends again
        return M;
    }
    for (uint32_t b = tid; b < 256u * Fmt::LEVELS; b += THREADS) (&s.hist[0][0])[b] = 0;
    if (tid == 0) { s.eq_count = 0; s.hole_count = 0; s.move_count = 0; }
    if (Fmt::STATS && tid == 0) { s.stats[kStatPrunes] += 1; s.stats[kStatAppended] += M - s.count_base; }
    __syncthreads();
    // radix descent: digit l of the k-th largest magnitude, among the entries that share its higher digits
    uint32_t prefix = 0, above = 0;
#pragma unroll
    for (int l = 0; l < Fmt::LEVELS; ++l) {
        const int sh = Fmt::shift(l), w = Fmt::width(l);  // constants once the loop is unrolled
#pragma unroll 1
        for (uint32_t slot = tid; slot < M; slot += THREADS) {
            const uint32_t mag = (uint32_t)s.cand_bits[slot] & Fmt::MAG_MASK;
            if (l == 0 || (mag >> (sh + w)) == prefix) atomicAdd(&s.hist[l][(mag >> sh) & ((1u << w) - 1u)], 1u);
        }
        __syncthreads();
        if (tid < 64) {  // one wave searches the histogram; the others only wait
            uint32_t d, a;
            if (w == 8) find_bin<4>(s.hist[l], above, k, d, a);
            else find_bin<2>(s.hist[l], above, k, d, a);
            if (tid == 0) { s.found_bin = d; s.found_above = a; }
        }
        __syncthreads();
        const uint32_t digit = uniform(s.found_bin);
        above = uniform(s.found_above);
        prefix = (prefix << w) | digit;
    }
    const uint32_t new_tm = prefix;
    const uint32_t need = k - above;  // how many of the entries with magnitude new_tm survive (>= 1)
#pragma unroll 1
    for (uint32_t slot = tid; slot < M; slot += THREADS)
        if (((uint32_t)s.cand_bits[slot] & Fmt::MAG_MASK) == new_tm) {
            const uint32_t q = atomicAdd(&s.eq_count, 1u);
            s.eq_slot[q] = (uint16_t)slot;
        }
    __syncthreads();
    const uint32_t E = uniform(s.eq_count);
    if (E > (uint32_t)kRankDirect) t.ties = true;
    // the need-th smallest index among the E equal-magnitude entries is the new threshold element
    // uniform; the usual case: a few dozen entries share the k-th magnitude
    if (E <= (uint32_t)kRankDirect) {
        for (uint32_t q = tid; q < E; q += THREADS) {
            const uint32_t mine = s.cand_idx[s.eq_slot[q]];
            uint32_t rank = 0;
            for (uint32_t u = 0; u < E; ++u) rank += (s.cand_idx[s.eq_slot[u]] < mine) ? 1u : 0u;
            if (rank == need - 1) { s.ti = mine; s.tm = (int32_t)new_tm; }
        }
    } else {
        rank_by_radix(s, E, need, new_tm);
    }
    __syncthreads();
    t.tm = (int32_t)uniform((uint32_t)s.tm);
    t.ti = uniform(s.ti);
    // Compact in place: exactly k entries survive.  Survivors already below slot k stay;
    // every survivor at or above slot k moves into a slot below k that lost its entry.
#pragma unroll 1
    for (uint32_t slot = tid; slot < k; slot += THREADS) {
        const int32_t mag = (int32_t)((uint32_t)s.cand_bits[slot] & Fmt::MAG_MASK);
        if (!(mag > t.tm || (mag == t.tm && s.cand_idx[slot] <= t.ti)))
            s.eq_slot[atomicAdd(&s.hole_count, 1u)] = (uint16_t)slot;  // eq_slot is free again: list of holes
    }
    __syncthreads();
#pragma unroll 1
    for (uint32_t slot = k + tid; slot < M; slot += THREADS) {
        const uint32_t bits = s.cand_bits[slot];
        const uint32_t idx = s.cand_idx[slot];
        const int32_t mag = (int32_t)(bits & Fmt::MAG_MASK);
        if (mag > t.tm || (mag == t.tm && idx <= t.ti)) {
            const uint32_t dest = s.eq_slot[atomicAdd(&s.move_count, 1u)];
            s.cand_idx[dest] = idx;
            s.cand_bits[dest] = (typename Fmt::bits_t)bits;
        }
    }
    if (tid == 0) { s.count = k; s.count_base = k; }
    __syncthreads();
    return M;
}

// Exact test of the queued vectors [q0, q1): two lanes share a vector (half of its values each); a value that comes
// before the threshold element takes a candidate slot (slots past CAP are counted but
// not written).
template <int THREADS, int CAP, int QCAP, typename Fmt>
__device__ __forceinline__ void drain_range(SelectShared<THREADS, CAP, QCAP, Fmt>& s, uint32_t q0, uint32_t q1,
                                            const Threshold& t)
{
    constexpr int HALF = Fmt::ELEMS / 2;
    const uint32_t tid = threadIdx.x;
    const uint32_t half = tid & 1u;
    for (uint32_t q = q0 + (tid >> 1); q < q1; q += THREADS / 2) {
        const u32x2 w = reinterpret_cast<const u32x2*>(&s.qvec[q])[half];
        const uint32_t ebase = s.qidx[q] * (uint32_t)Fmt::ELEMS + half * (uint32_t)HALF;
#pragma unroll
        for (int e = 0; e < HALF; ++e) {
            const uint32_t bits = Fmt::half_elem(w, e);
            const int32_t mag = (int32_t)(bits & Fmt::MAG_MASK);
            if (before(mag, ebase + e, t)) {
                const uint32_t slot = atomicAdd(&s.count, 1u);
                if (slot < (uint32_t)CAP) {
                    s.cand_idx[slot] = ebase + e;
                    s.cand_bits[slot] = (typename Fmt::bits_t)bits;
                }
            }
        }
    }
}

// The overflow path's first resort: when one sweep over the queue would hand out more candidate slots
// than there are (sorted or otherwise adversarial data: nearly every queued value passes), find the k-th
// largest magnitude among the candidates kept so far and ALL queued values by a radix descent over both
// (the same histograms as the prune, fed from the queue two lanes per vector).  At least k real elements
// reach that magnitude, so it is a valid bound; it becomes the threshold (without an index: equal magnitudes
// still pass) and the queue is then swept once.  Returns false, and leaves the threshold alone, when
// even that sweep might not fit: many values share the k-th magnitude (tie-heavy data), which the batches
// handle.  All threads call, after a barrier behind which s.count is the count before the sweep.
template <int THREADS, int CAP, int QCAP, typename Fmt>
__device__ __forceinline__ bool bound_from_queue(SelectShared<THREADS, CAP, QCAP, Fmt>& s, uint32_t k, uint32_t nq, Threshold& t)
{
    constexpr int HALF = Fmt::ELEMS / 2;
    const uint32_t tid = threadIdx.x;
    const uint32_t M0 = uniform(s.count);
    for (uint32_t b = tid; b < 256u * Fmt::LEVELS; b += THREADS) (&s.hist[0][0])[b] = 0;
    if (Fmt::STATS && tid == 0) s.stats[kStatPrunes] += 1;   // counted with the prunes: it is the same radix descent
    __syncthreads();
    uint32_t prefix = 0, above = 0, in_bin = 0;
#pragma unroll
    for (int l = 0; l < Fmt::LEVELS; ++l) {
        const int sh = Fmt::shift(l), w = Fmt::width(l);
#pragma unroll 1
        for (uint32_t slot = tid; slot < M0; slot += THREADS) {
            const uint32_t mag = (uint32_t)s.cand_bits[slot] & Fmt::MAG_MASK;
            if (l == 0 || (mag >> (sh + w)) == prefix) atomicAdd(&s.hist[l][(mag >> sh) & ((1u << w) - 1u)], 1u);
        }
#pragma unroll 1
        for (uint32_t q = tid >> 1; q < nq; q += THREADS / 2) {
            const u32x2 wv = reinterpret_cast<const u32x2*>(&s.qvec[q])[tid & 1u];
#pragma unroll
            for (int e = 0; e < HALF; ++e) {
                const uint32_t mag = Fmt::half_elem(wv, e) & Fmt::MAG_MASK;
                if (l == 0 || (mag >> (sh + w)) == prefix) atomicAdd(&s.hist[l][(mag >> sh) & ((1u << w) - 1u)], 1u);
            }
        }
        __syncthreads();
        if (tid < 64) {
            uint32_t d, a;
            if (w == 8) find_bin<4>(s.hist[l], above, k, d, a);
            else find_bin<2>(s.hist[l], above, k, d, a);
            if (tid == 0) { s.found_bin = d; s.found_above = a; }
        }
        __syncthreads();
        const uint32_t digit = uniform(s.found_bin);
        above = uniform(s.found_above);
        in_bin = uniform(s.hist[l][digit]);   // values that share every digit so far
        prefix = (prefix << w) | digit;
    }
    // the sweep appends at most the queued values that reach the bound: above + in_bin of them
    if (M0 + above + in_bin > (uint32_t)CAP) return false;
    if ((int32_t)prefix > t.tm) {
        t.tm = (int32_t)prefix;
        t.ti = 0xFFFFFFFFu;
    }
    return true;
}

// Move every queued value that comes before the threshold element into the candidate
// buffer, prune that buffer when it holds more than `limit` (CAP/2 while streaming, k
// at the end), then empty the queue.  Two lanes share
// a vector.  The whole queue is taken in one sweep; should that ever hand out more than
// CAP slots (the excess is dropped, not written), the sweep is undone; then either the threshold is
// raised from the queue's own values so that one sweep fits (bound_from_queue), or, on tie-heavy
// data, the sweep is repeated in batches of at most CAP/16 vectors with a prune check after each: a
// batch adds at most CAP/2 values to a buffer holding at most CAP/2.
// Called by all threads after a barrier that made the queue writes visible.  `epoch`
// (uniform) says which queue counter the pushes used; the drain clears the other one and
// switches to it, so the usual drain costs one barrier: the caller must pass one more
// barrier before it touches the candidate buffer again (the streaming loop has one per
// round; select_topk_from ends with one).  Returns true when lanes are still waiting for
// room in the queue.
template <int THREADS, int CAP, int QCAP, typename Fmt>
__device__ __forceinline__ bool drain(SelectShared<THREADS, CAP, QCAP, Fmt>& s, uint32_t k, uint32_t limit, Threshold& t,
                                        uint32_t& epoch)
{
    constexpr uint32_t BATCH = (CAP / 16 < THREADS / 2) ? CAP / 16 : THREADS / 2;  // vectors: ELEMS * BATCH <= CAP / 2
    const uint32_t tid = threadIdx.x;
    const uint32_t raw = uniform(s.qcount[epoch & 1u]);
    const uint32_t nq = raw < (uint32_t)QCAP ? raw : (uint32_t)QCAP;
    if (tid == 0) s.qcount[(epoch + 1u) & 1u] = 0;  // last read one drain ago; visible after the barrier below
    if (Fmt::STATS && tid == 0) { s.stats[kStatDrains] += 1; s.stats[kStatQueued] += nq; }
    ++epoch;
    limit = limit < (uint32_t)(CAP / 2) ? limit : (uint32_t)(CAP / 2);
    drain_range(s, 0u, nq, t);
    if (prune_if_above<false>(s, k, limit, t) > (uint32_t)CAP) {  // uniform; rare
        // Undo the sweep: back to the count the last prune left (count_base; <= CAP/2).  It is not read
        // from s.count at the start of this function, where a wave that runs ahead may already be appending.
        __syncthreads();  // everyone has read the count
        if (tid == 0) s.count = s.count_base;
        __syncthreads();
        if (!t.ties && bound_from_queue(s, k, nq, t)) {  // uniform
            drain_range(s, 0u, nq, t);
        } else {
            for (uint32_t b0 = 0; b0 < nq; b0 += BATCH) {
                const uint32_t b1 = b0 + BATCH < nq ? b0 + BATCH : nq;
                drain_range(s, b0, b1, t);
                (void)prune_if_above(s, k, CAP / 2, t);
            }
        }
        (void)prune_if_above(s, k, limit, t);
    }
    return raw > (uint32_t)QCAP;
}

// number of set bits of `mask` below the calling lane
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// One round of loads: vectors b + u*THREADS + tid, u < U, of a range whose vector v0 sits at src
// (vector v is read from src + (v - v0)).  A round that lies wholly inside [.., v1) is loaded
// without per-lane tests; vectors past v1 read as zero.
template <int THREADS, int U>
__device__ __forceinline__ void load_round(u32x4 (&buf)[U], const u32x4* __restrict__ src, uint32_t v0, uint32_t b,
                                           uint32_t v1)
{
    const uint32_t tid = threadIdx.x;
    const u32x4* p = src + (b - v0);   // uniform
    if (b + THREADS * U <= v1) {  // uniform
#pragma unroll
        for (int u = 0; u < U; ++u) buf[u] = __builtin_nontemporal_load(p + u * THREADS + tid);
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            buf[u] = u32x4{0u, 0u, 0u, 0u};
            if (b + u * THREADS + tid < v1) buf[u] = __builtin_nontemporal_load(p + u * THREADS + tid);
        }
    }
}

// Examine the round held in buf (vectors b + u*THREADS + tid): every vector that may hold a value
// coming before the threshold element goes to the queue.  A vector's largest magnitude decides:
// above the threshold's it goes, below it does not, and a vector that only equals it goes when its
// first index is below the threshold's index.  The threshold element usually lies before the round
// (it was read in an earlier one); then "equal" never goes and one compare against tm + 1 settles it:
// the four compares leave their lane masks in scalar registers, and a wave whose masks are all
// empty goes straight to the barrier.  Otherwise the wave takes all its queue slots with one LDS
// atomic (slot of a lane = the wave's first slot + set bits of the masks below it), and lane 0 raises
// the round's flag when the queue passed its soft limit.  One barrier per pass; the workgroup drains
// the queue when the flag is up.  Lanes that found the queue full (rare: the wave's slots ran past the
// end) remember their vectors in `pend` and try again after the drain, against the new threshold.
template <int THREADS, int U, int CAP, int QCAP, typename Fmt, bool PLAIN>
__device__ __forceinline__ uint32_t queue_first_pass(const u32x4 (&buf)[U], const int32_t (&m)[U], const uint64_t (&want)[U],
                                                     uint32_t thr, uint32_t b, SelectShared<THREADS, CAP, QCAP, Fmt>& s,
                                                     uint32_t* flag, uint32_t epoch)
{
    constexpr uint32_t QSOFT = QCAP / 2;
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = lane_id();
    uint32_t total = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) total += (uint32_t)__popcll(want[u]);
    uint32_t first = 0;
    if (lane == 0) first = atomicAdd(&s.qcount[epoch & 1u], total);
    first = __builtin_amdgcn_readfirstlane(first);
    if (first + total > QSOFT && lane == 0) *flag = 1u;       // some slot at or past the soft limit was handed out
    const bool spill = first + total > (uint32_t)QCAP;         // uniform: some lane finds no room
    uint32_t pend = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (want[u] != 0) {  // uniform
            // the lane's bit of want[u]: in a plain round the compare that made the mask, evaluated again
            const bool mine = PLAIN ? ((uint32_t)m[u] >= thr) : (((want[u] >> lane) & 1ull) != 0);
            if (mine) {
                const uint32_t slot = first + lanes_below(want[u]);
                if (!spill || slot < (uint32_t)QCAP) {
                    s.qvec[slot] = buf[u];
                    s.qidx[slot] = b + u * THREADS + tid;
                } else {
                    pend |= 1u << u;
                }
            }
            first += (uint32_t)__popcll(want[u]);
        }
    }
    return pend;
}

template <int THREADS, int U, int CAP, int QCAP, typename Fmt>
__device__ __forceinline__ void examine_round(const u32x4 (&buf)[U], uint32_t b, uint32_t v1, uint32_t k,
                                              SelectShared<THREADS, CAP, QCAP, Fmt>& s, Threshold& t, uint32_t& round,
                                              uint32_t& epoch)
{
    constexpr uint32_t QSOFT = QCAP / 2;
    const uint32_t tid = threadIdx.x;
    int32_t m[U];
#pragma unroll
    for (int u = 0; u < U; ++u) m[u] = Fmt::vec_max(buf[u]);
    // uniform: is there a threshold element yet (before the first prune tm is only a bound that at least k
    // values reach: equal magnitudes count), and if so, does it lie inside or behind this round?
    const bool element = t.ti != 0xFFFFFFFFu;
    const bool by_index = element && t.ti > b * (uint32_t)Fmt::ELEMS;
    const uint32_t thr = (uint32_t)t.tm + (element && !by_index ? 1u : 0u);  // magnitudes are below 2^31: no wrap
    const bool plain = !by_index && b + THREADS * U <= v1;        // uniform: one compare per vector decides
    uint64_t want[U];   // lanes whose vector u goes to the queue
    uint64_t any = 0;
    if (plain) {
#pragma unroll
        for (int u = 0; u < U; ++u) { want[u] = __ballot((uint32_t)m[u] >= thr); any |= want[u]; }
    } else {
        // the ragged last round, and rounds that may hold the threshold element itself: without the index rule
        // data with many equal magnitudes would queue every vector of every round
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t v = b + u * THREADS + tid;
            want[u] = __ballot((uint32_t)m[u] >= thr && v < v1 && !(m[u] == t.tm && v * (uint32_t)Fmt::ELEMS >= t.ti));
            any |= want[u];
        }
    }
    uint32_t pend = 0;  // bit u: vector u found the queue full and still has to be queued
    if (any != 0) {     // uniform within the wave
        uint32_t* flag = &s.flag[round % 3u];
        pend = plain ? queue_first_pass<THREADS, U, CAP, QCAP, Fmt, true>(buf, m, want, thr, b, s, flag, epoch)
                     : queue_first_pass<THREADS, U, CAP, QCAP, Fmt, false>(buf, m, want, thr, b, s, flag, epoch);
    }
    while (true) {
        __syncthreads();
        const uint32_t f = uniform(s.flag[round % 3u]);
        if (tid == 0) s.flag[(round + 2u) % 3u] = 0;  // the previous round's flag: read by all before this barrier
        ++round;
        if (!f) break;  // no slot at or past the soft limit was handed out: nothing is pending either
        TOPLOC_TICK_BEGIN(drain);
        const bool again = drain(s, k, TOPLOC_PRUNE_LIMIT(CAP, k), t, epoch);
        TOPLOC_TICK_END(drain, 2);
        if (!again) break;
        // The queue was full for some lanes: they queue what still comes before the new threshold element,
        // which may be one of this round's.
        uint32_t* flag = &s.flag[round % 3u];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (m[u] < t.tm || (m[u] == t.tm && (b + u * THREADS + tid) * (uint32_t)Fmt::ELEMS >= t.ti)) pend &= ~(1u << u);
        if (__ballot(pend != 0u)) {  // uniform within the wave
            uint64_t left[U];
            uint32_t total = 0;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                left[u] = __ballot((pend >> u) & 1u);
                total += (uint32_t)__popcll(left[u]);
            }
            uint32_t first = 0;
            if (lane_id() == 0) first = atomicAdd(&s.qcount[epoch & 1u], total);
            first = __builtin_amdgcn_readfirstlane(first);
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if ((pend >> u) & 1u) {
                    const uint32_t slot = first + lanes_below(left[u]);
                    if (slot >= QSOFT) *flag = 1u;
                    if (slot < (uint32_t)QCAP) {
                        s.qvec[slot] = buf[u];
                        s.qidx[slot] = b + u * THREADS + tid;
                        pend &= ~(1u << u);
                    }
                }
                first += (uint32_t)__popcll(left[u]);
            }
        }
    }
}

// What a selection starts from.  A plain selection starts from nothing; the online path
// continues an earlier one (one token row per call): its seed() puts the n survivors of the
// earlier calls (n <= k) into s.cand_idx / s.cand_bits [0, n) and reports the threshold
// those calls ended with, and k then counts seeds and new values together.  seed() runs
// after the loads of the first two rounds were issued, so that its own global reads overlap
// them (the verify kernel decodes its proof there for the same reason).
struct SelectStart {
    uint32_t n;   // seeds placed in the candidate buffer
    Threshold t;  // first threshold; (0, 0xFFFFFFFF): everything comes before it, nothing seen yet
    uint32_t k;   // how many to select
};
struct NoSeed {
    uint32_t k;
    template <typename Shared>
    __device__ __forceinline__ SelectStart seed(Shared&) const { return SelectStart{0u, Threshold{0, 0xFFFFFFFFu}, k}; }
};

// Top-k of the vectors [v0, v1) of a chunk, vector v0 being the one at src (8 values per vector,
// flat index of value e of vector v is ELEMS*v + e) into s.cand_idx / s.cand_bits [0 .. k), in no
// particular order (order_topk sorts them).
// Requires k <= seeds + ELEMS*(v1 - v0), k <= CAP/4, ELEMS*v1 < 2^32.  All threads of the workgroup
// call it; it ends with a barrier.  Returns k and the threshold the selection ended with:
// (0, 0xFFFFFFFF) as long as nothing had to be pruned, else the k-th element.
template <int THREADS, int U, int DEPTH = 2, int CAP, int QCAP, typename Fmt, typename Seed>
__device__ __forceinline__ SelectStart select_topk_from(const u32x4* __restrict__ src, uint32_t v0, uint32_t v1,
                                                        SelectShared<THREADS, CAP, QCAP, Fmt>& s, const Seed& seeder)
{
    static_assert(DEPTH == 2 || DEPTH == 3, "two or three rounds of loads in registers");
    constexpr uint32_t ROUND = THREADS * U;
    const uint32_t tid = threadIdx.x;
    TOPLOC_TICK_BEGIN(boot);
    // DEPTH rounds in registers: one is examined while the loads of the others fly.  Three cost 16 more
    // registers than two (one workgroup per CU less): worth it only for a launch that fits the chip in one
    // generation, where nobody else's streaming covers a workgroup's pauses.
    u32x4 even[U], odd[U], third[DEPTH == 3 ? U : 1];
    load_round<THREADS, U>(even, src, v0, v0, v1);
    load_round<THREADS, U>(odd, src, v0, v0 + ROUND, v1);   // in flight while the first threshold is found
    if (DEPTH == 3) load_round<THREADS, U>(reinterpret_cast<u32x4(&)[U]>(third), src, v0, v0 + 2u * ROUND, v1);
    const SelectStart start = seeder.seed(s);
    const uint32_t k = start.k;
    const uint32_t n_seed = start.n;
    if (tid == 0) {
        s.qcount[0] = 0; s.qcount[1] = 0; s.count = n_seed; s.count_base = n_seed; s.eq_count = 0; s.tm = start.t.tm; s.ti = start.t.ti;
        s.flag[0] = 0; s.flag[1] = 0; s.flag[2] = 0;
        if (Fmt::STATS) { s.stats[0] = 0; s.stats[1] = 0; s.stats[2] = 0; s.stats[3] = 0; }
    }
    Threshold t = start.t;
    uint32_t round = 0;    // barrier rounds; flag[round % 3] belongs to the current one
    uint32_t epoch = 0;    // drains so far; qcount[epoch % 2] counts the current pushes

    // First threshold: the largest magnitude of every vector of the first two rounds (both are on
    // their way by now) belongs to a distinct real element, so the k-th largest of those maxima is a
    // magnitude that at least k elements reach: nothing below it can be in the top-k.  Two radix
    // digits of the maxima (exponent, then the next digit among the maxima that share the k-th's
    // exponent) find it: exactly for bf16, to 16 of the 31 magnitude bits for fp32.  Exact
    // thresholds follow from the first prune.
    const uint32_t first = (v1 - v0) < 2u * ROUND ? (v1 - v0) : 2u * ROUND;
    if (n_seed == 0 && first >= k) {  // uniform
        constexpr int S0 = Fmt::shift(0), S1 = Fmt::shift(1), W1 = Fmt::width(1);
        for (uint32_t b = tid; b < 512u; b += THREADS) (&s.hist[0][0])[b] = 0;
        __syncthreads();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (v0 + u * THREADS + tid < v1) atomicAdd(&s.hist[0][(uint32_t)Fmt::vec_max(even[u]) >> S0], 1u);
            if (v0 + ROUND + u * THREADS + tid < v1) atomicAdd(&s.hist[0][(uint32_t)Fmt::vec_max(odd[u]) >> S0], 1u);
        }
        __syncthreads();
        uint32_t e_star, above;   // every wave searches for itself: no broadcast, no barrier
        find_bin<4>(s.hist[0], 0u, k, e_star, above);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t me = (uint32_t)Fmt::vec_max(even[u]), mo = (uint32_t)Fmt::vec_max(odd[u]);
            if (v0 + u * THREADS + tid < v1 && (me >> S0) == e_star) atomicAdd(&s.hist[1][(me >> S1) & ((1u << W1) - 1u)], 1u);
            if (v0 + ROUND + u * THREADS + tid < v1 && (mo >> S0) == e_star)
                atomicAdd(&s.hist[1][(mo >> S1) & ((1u << W1) - 1u)], 1u);
        }
        __syncthreads();
        uint32_t digit, above1;
        if (W1 == 8) find_bin<4>(s.hist[1], above, k, digit, above1);
        else find_bin<2>(s.hist[1], above, k, digit, above1);
        t.tm = (int32_t)((e_star << S0) | (digit << S1));
        t.ties = uniform(s.hist[1][digit]) > (uint32_t)kRankDirect;   // that many maxima share the k-th's digits
    }
    __syncthreads();

    TOPLOC_TICK_END(boot, 0);
    TOPLOC_TICK_BEGIN(stream);
    uint32_t base = v0;  // v1 - v0 >= 1
    constexpr uint32_t AHEAD = (DEPTH - 1) * ROUND;   // the buffer just examined takes the round this far ahead
    while (true) {
        examine_round<THREADS, U>(even, base, v1, k, s, t, round, epoch);
        base += ROUND;
        if (base >= v1) break;
        load_round<THREADS, U>(even, src, v0, base + AHEAD, v1);
        examine_round<THREADS, U>(odd, base, v1, k, s, t, round, epoch);
        base += ROUND;
        if (base >= v1) break;
        load_round<THREADS, U>(odd, src, v0, base + AHEAD, v1);
        if (DEPTH == 3) {
            examine_round<THREADS, U>(reinterpret_cast<const u32x4(&)[U]>(third), base, v1, k, s, t, round, epoch);
            base += ROUND;
            if (base >= v1) break;
            load_round<THREADS, U>(reinterpret_cast<u32x4(&)[U]>(third), src, v0, base + AHEAD, v1);
        }
    }
    __syncthreads();
    TOPLOC_TICK_END(stream, 1);
    TOPLOC_TICK_BEGIN(fin);
    (void)drain(s, k, k, t, epoch);  // prunes to exactly k
    __syncthreads();
    TOPLOC_TICK_END(fin, 3);
    return SelectStart{k, t, k};
}

template <int THREADS, int U, int DEPTH = 2, int CAP, int QCAP, typename Fmt>
__device__ __forceinline__ void select_topk(const u32x4* __restrict__ src, uint32_t v0, uint32_t v1, uint32_t k,
                                            SelectShared<THREADS, CAP, QCAP, Fmt>& s)
{
    (void)select_topk_from<THREADS, U, DEPTH>(src, v0, v1, s, NoSeed{k});
}

// Top-k of candidate lists: `n` (index, pattern) pairs in global memory, entries whose
// index is 0xFFFFFFFF are padding.  They are loaded in batches of CAP/2 with a prune
// after each, so any n fits.  Leaves min(k, valid entries) survivors in
// s.cand_idx / s.cand_bits, unordered.  All threads call; ends with a barrier.
template <int THREADS, int CAP, int QCAP, typename Fmt>
__device__ __forceinline__ void merge_topk(const uint32_t* __restrict__ c_idx,
                                           const typename Fmt::bits_t* __restrict__ c_bits, uint32_t n, uint32_t k,
                                           SelectShared<THREADS, CAP, QCAP, Fmt>& s)
{
    const uint32_t tid = threadIdx.x;
    if (tid == 0) { s.count = 0; s.count_base = 0; s.eq_count = 0; s.tm = 0; s.ti = 0xFFFFFFFFu; }
    __syncthreads();
    Threshold t;
    t.tm = 0;
    t.ti = 0xFFFFFFFFu;
    for (uint32_t b0 = 0; b0 < n; b0 += CAP / 2) {
        const uint32_t b1 = b0 + CAP / 2 < n ? b0 + CAP / 2 : n;
        for (uint32_t i = b0 + tid; i < b1; i += THREADS) {
            const uint32_t idx = c_idx[i];
            if (idx != 0xFFFFFFFFu) {
                const uint32_t slot = atomicAdd(&s.count, 1u);
                s.cand_idx[slot] = idx;
                s.cand_bits[slot] = c_bits[i];
            }
        }
        (void)prune_if_above(s, k, b1 == n ? k : (uint32_t)(CAP / 2), t);
    }
}

// Put the k survivors of select_topk into the order (magnitude descending, index
// ascending): rank = number of survivors that come before.  All threads call; ends
// with a barrier.
template <int THREADS, int CAP, int QCAP, typename Fmt>
__device__ __forceinline__ void order_topk(SelectShared<THREADS, CAP, QCAP, Fmt>& s, uint32_t k)
{
    const uint32_t tid = threadIdx.x;
    constexpr int KPT = (CAP / 2 + THREADS - 1) / THREADS;
    uint32_t my_idx[KPT], my_bits[KPT], my_rank[KPT];
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const uint32_t j = tid + i * THREADS;
        my_idx[i] = 0; my_bits[i] = 0; my_rank[i] = 0;
        if (j < k) {
            my_idx[i] = s.cand_idx[j];
            my_bits[i] = s.cand_bits[j];
            const uint32_t mag = my_bits[i] & Fmt::MAG_MASK;
            uint32_t rank = 0;
            for (uint32_t u = 0; u < k; ++u) {
                const uint32_t om = s.cand_bits[u] & Fmt::MAG_MASK;
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
            s.cand_bits[my_rank[i]] = (typename Fmt::bits_t)my_bits[i];
        }
    }
    __syncthreads();
}

}  // namespace toploc
