// TopLoc proof build / verify for MI355X (gfx950): kernels and the C ABI of
// include/toploc.h.  Chunks (and segments) are independent.
//
// Large batches, one 256-lane workgroup per chunk, one launch:
//   build_kernel    all of Algorithm 1 (k <= 128): topk, then findInjectiveModulus,
//                   i mod m, InterpolateModPolynomial, encode out of LDS while other
//                   workgroups of the compute unit keep streaming
//   verify_kernel   all of Algorithm 2: decode, topk, i mod m, Horner at the k points,
//                   extractBits, err_e / err_m statistics, thresholds
//   select_kernel   topk(h, k) alone, ordered (toploc_topk)
// Small batches, long segments, k > 128: a chunk is cut into parts so that the launch
// fills the chip, and a second launch merges the parts' candidates:
//   part_kernel          topk of one part of one chunk / segment -> k candidates
//   build_merge_kernel   topk of the candidates, then the rest of Algorithm 1
//   verify_merge_kernel  topk of the candidates, then the rest of Algorithm 2
//   ring_kernel          provider-side ring of the last chunk_tokens hidden vectors
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <atomic>
#include <mutex>
#include <vector>

#include "../../include/toploc.h"
#include "gf65497.hpp"
#include "interp.hpp"
#ifndef TOPLOC_INTERP_PLANES
#define TOPLOC_INTERP_PLANES 1   // 1: GF(65497) interpolation on byte planes and packed dot products (interp16.hpp)
#endif
#if TOPLOC_INTERP_PLANES
#include "interp16.hpp"
#endif
#include "plan.hpp"
#include "select.hpp"
#include "verify.hpp"

#ifndef TOPLOC_QCAP
#define TOPLOC_QCAP 512
#endif
#ifndef TOPLOC_MIN_WAVES
#define TOPLOC_MIN_WAVES 6  // waves per SIMD the streaming kernels must reach: 80 VGPRs, which 4 loads per lane just fit
#endif

namespace toploc {

constexpr int kThreads = (int)plan::kThreads;   // lanes per streaming workgroup
constexpr int kLoads = (int)plan::kLoads;       // 16-byte loads in flight per lane and round
constexpr int kQcap = TOPLOC_QCAP;        // queue entries (16-byte vectors)
#ifndef TOPLOC_CAP_SMALL
#define TOPLOC_CAP_SMALL 1024
#endif
constexpr int kCapSmall = TOPLOC_CAP_SMALL;  // candidate buffer for k <= 128
constexpr int kCapLarge = 2048;           // candidate buffer for k <= TOPLOC_MAX_K
constexpr int kCapMerge = 4096;           // candidate buffer of the merge kernels: few workgroups, LDS to spare, and a long segment
                                          // brings dozens of parts: 2048 candidates per batch and prune instead of 512
constexpr int kCapWide = 16384;           // candidate buffer of the selection alone up to TOPLOC_MAX_K_TOPK (140 KB of LDS:
                                          // one workgroup per compute unit; an aid for statistics, not a fast path)
// The larger candidate buffer (k > 128) costs registers in the prune and the ordering: one wave per SIMD less.
constexpr int waves_for(int cap) { return cap > kCapSmall ? TOPLOC_MIN_WAVES - 1 : TOPLOC_MIN_WAVES; }
// A fused launch of at most this many chunks fits the chip in one generation even at 5 workgroups per CU (256 CUs):
// it runs the kernels that keep three rounds of loads in flight (95 VGPRs, 5 waves per SIMD).
#ifndef TOPLOC_ONE_GENERATION
#define TOPLOC_ONE_GENERATION 1280
#endif
constexpr uint64_t kOneGeneration = TOPLOC_ONE_GENERATION;
static_assert(kCapLarge >= 4 * (int)TOPLOC_MAX_K && kCapSmall >= 4 * 128 && kCapWide >= 4 * (int)TOPLOC_MAX_K_TOPK,
              "soft limit CAP/2 must leave room above k");
static_assert(kCapWide <= 65536, "prune keeps slot numbers in 16 bits");

// Where a workgroup of a split launch finds its piece.  Fixed chunks need no table:
// chunk = block / parts, part = block % parts.  Segments: the row offsets are a device
// array; segment i starts at vector a_i = row_offsets[i] * row_vecs of the matrix, is cut into
// parts of part_vecs vectors and owns the candidate slots from a_i / part_vecs + i on (see
// plan.hpp).  A small planning kernel turns that into one PartDesc per slot.
struct PartDesc {          // one per workgroup of part_kernel
    uint64_t seg_vec;      // first vector of the segment, from the tensor base; kIdlePart: nothing to do
    uint32_t v0, v1;       // vectors [v0, v1) of the segment
};
static_assert(sizeof(PartDesc) == plan::kPartDescBytes, "workspace layout");
constexpr uint64_t kIdlePart = ~0ull;
struct Layout {
    const PartDesc* part_table;   // NULL: fixed chunks
    const uint64_t* row_offsets;  // segments: device, n_segments + 1 row numbers
    uint64_t total_rows;          // segments: rows of the matrix
    uint32_t row_vecs;            // segments: 16-byte vectors per row
    uint32_t row_values;          // segments: values per row (hidden)
    uint32_t nvec;                // fixed chunks: vectors per chunk
    uint32_t parts;               // fixed chunks: parts per chunk
    uint32_t part_vecs;           // vectors per part
};

// One segment as the kernels see it.  status is TOPLOC_CHUNK_OK, TOPLOC_CHUNK_SHORT (fewer than k
// values) or TOPLOC_CHUNK_BAD_SEGMENT (offsets that decrease, leave the matrix, or span 2^32 values
// or more); only an OK segment has parts.
struct SegInfo {
    uint64_t a_vec;        // first vector, from the tensor base
    uint32_t nvec;         // vectors
    uint32_t n_parts;
    uint64_t first_slot;
    uint32_t status;
};
__device__ __forceinline__ SegInfo segment_info(const Layout& lay, uint64_t i, uint32_t k)
{
    SegInfo g = {0, 0, 0, 0, TOPLOC_CHUNK_BAD_SEGMENT};
    const uint64_t r0 = lay.row_offsets[i], r1 = lay.row_offsets[i + 1];
    if (r1 < r0 || r1 > lay.total_rows) return g;
    const uint64_t values = (r1 - r0) * lay.row_values;   // < 2^62: total_rows * hidden is
    if (values >= (1ull << 32)) return g;
    if (values < k) { g.status = TOPLOC_CHUNK_SHORT; return g; }
    g.a_vec = r0 * lay.row_vecs;
    g.nvec = (uint32_t)((r1 - r0) * lay.row_vecs);
    g.n_parts = (g.nvec + lay.part_vecs - 1) / lay.part_vecs;
    g.first_slot = g.a_vec / lay.part_vecs + i;
    g.status = TOPLOC_CHUNK_OK;
    return g;
}

// Planning kernel of the segment calls, one thread per slot: which part of which segment the slot
// holds.  The first slot of segment i, a_i / part_vecs + i, grows strictly with i (offsets do not
// decrease), so the owner of slot p is the last segment whose first slot is <= p, found by bisection
// over the offsets; p is idle when it lies behind that segment's parts.  Offsets are clamped to the
// matrix before use, so whatever they hold no part ever points outside it.
__global__ __launch_bounds__(256) void plan_segments_kernel(Layout lay, uint64_t n_segments, uint64_t slots, uint32_t k,
                                                            PartDesc* __restrict__ table)
{
    const uint64_t p = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (p >= slots) return;
    PartDesc d = {kIdlePart, 0u, 0u};
    uint64_t lo = 0, hi = n_segments;   // invariant: first_slot(lo) <= p (checked below for lo = 0), first_slot(hi) > p
    while (hi - lo > 1) {
        const uint64_t mid = lo + (hi - lo) / 2;
        uint64_t r = lay.row_offsets[mid];
        r = r < lay.total_rows ? r : lay.total_rows;
        if (r * lay.row_vecs / lay.part_vecs + mid <= p) lo = mid; else hi = mid;
    }
    if (n_segments) {
        const SegInfo g = segment_info(lay, lo, k);
        if (g.status == TOPLOC_CHUNK_OK && p >= g.first_slot && p - g.first_slot < g.n_parts) {
            const uint32_t j = (uint32_t)(p - g.first_slot);
            d.seg_vec = g.a_vec;
            d.v0 = j * lay.part_vecs;
            d.v1 = d.v0 + lay.part_vecs < g.nvec ? d.v0 + lay.part_vecs : g.nvec;
        }
    }
    table[p] = d;
}

// Which chunk a workgroup takes.  Workgroups go to the 8 XCDs round-robin by block index,
// so with chunk = block index consecutive chunks land on different XCDs and every XCD's
// reads spread over all HBM channels.  The alternative, one contiguous eighth of the
// tensor per XCD (TOPLOC_XCD_CONTIGUOUS), was measured 5 % slower on the 70B shape: chunks
// are read once, so there is no reuse for an XCD's L2 to keep.
__device__ __forceinline__ uint64_t chunk_of_block()
{
#ifdef TOPLOC_XCD_CONTIGUOUS
    const uint32_t b = blockIdx.x, per = gridDim.x / 8u;
    return b < per * 8u ? (uint64_t)(b % 8u) * per + b / 8u : b;
#else
    return blockIdx.x;
#endif
}

// ---------------------------------------------------------------------------
// topk(h, k) alone: writes the ordered (index, value) pairs of every chunk
// ---------------------------------------------------------------------------
template <int CAP, int WAVES = waves_for(CAP)>
__global__ __launch_bounds__(kThreads, WAVES) void select_kernel(const u32x4* __restrict__ hidden, uint32_t nvec,
                                                                 uint32_t k, uint32_t* __restrict__ out_idx,
                                                                 uint16_t* __restrict__ out_val)
{
    __shared__ SelectShared<kThreads, CAP, kQcap> s;
    const uint64_t chunk = chunk_of_block();
    select_topk<kThreads, kLoads, 2, CAP, kQcap>(hidden + chunk * nvec, 0u, nvec, k, s);
    order_topk(s, k);
    for (uint32_t t = threadIdx.x; t < k; t += kThreads) {
        out_idx[chunk * k + t] = s.cand_idx[t];
        out_val[chunk * k + t] = s.cand_bits[t];
    }
}

// Measurement aid: the same selection with its event counters on; writes, per chunk, the number of
// drains and prunes, of queued vectors and of candidates appended (the final drain and prune included).
template <int CAP>
__global__ __launch_bounds__(kThreads) void select_stats_kernel(const u32x4* __restrict__ hidden, uint32_t nvec, uint32_t k,
                                                                uint32_t* __restrict__ out_stats)
{
    __shared__ SelectShared<kThreads, CAP, kQcap, Bf16FmtStats> s;
    const uint64_t chunk = blockIdx.x;
    select_topk<kThreads, kLoads, 2, CAP, kQcap>(hidden + chunk * nvec, 0u, nvec, k, s);
    if (threadIdx.x < 4) out_stats[chunk * 4 + threadIdx.x] = s.stats[threadIdx.x];
}

// ---------------------------------------------------------------------------
// Algorithm 1 in one launch, k <= KMAX <= kThreads: the selection streams the chunk,
// then the same workgroup turns its k pairs into the proof out of LDS (the selection's
// buffers are dead by then and are reused).
// ---------------------------------------------------------------------------
template <int KMAX, int CAP, typename F = Field16, typename Fmt = Bf16Fmt, int U = kLoads, int WAVES = waves_for(CAP), int DEPTH = 2>
__global__ __launch_bounds__(kThreads, WAVES) void build_kernel(const u32x4* __restrict__ hidden, uint32_t nvec,
                                                                           uint32_t k, uint8_t* __restrict__ proofs,
                                                                           uint8_t* __restrict__ status,
                                                                           uint32_t* __restrict__ out_idx)
{
    static_assert(KMAX <= kThreads, "one pair per lane is carried across the phase change");
    __shared__ union BuildShared {
        SelectShared<kThreads, CAP, kQcap, Fmt> sel;
        InterpShared<KMAX, F> itp;
    } sh;
    __shared__ uint32_t coef[KMAX];
    const uint32_t tid = threadIdx.x;
    const uint64_t chunk = chunk_of_block();
    select_topk<kThreads, U, DEPTH>(hidden + chunk * nvec, 0u, nvec, k, sh.sel);
    if (out_idx) {  // uniform: the caller wants the ordered indices
        order_topk(sh.sel, k);
        if (tid < k) out_idx[chunk * k + tid] = sh.sel.cand_idx[tid];
    }
    uint32_t my_idx = 0, my_y = 0;
    if (tid < k) { my_idx = sh.sel.cand_idx[tid]; my_y = sh.sel.cand_bits[tid]; }
    __syncthreads();  // the selection's LDS is dead from here on
    if (tid < k) {
        sh.itp.idx[tid] = my_idx;
        sh.itp.ys[tid] = (typename F::elem_t)F::from_pattern(my_y);
    }
    TOPLOC_TICK_BEGIN(tail);
    finish_proof<kThreads>(sh.itp, coef, k,
                           reinterpret_cast<uint16_t*>(proofs + chunk * (2 + 2 * (uint64_t)F::WORDS * k)), status + chunk);
    TOPLOC_TICK_END(tail, 5);
}

// ---------------------------------------------------------------------------
// Algorithm 2, fused: one pass over the recomputed chunk
// ---------------------------------------------------------------------------
// decode(p) as the first thing a selection does after issuing its first loads
template <typename F, int KMAX, bool WIDE>
struct DecodeFirst {
    VerifyShared<KMAX, WIDE>& vs;
    const ProofWords<kThreads, KMAX>& words;  // read from global memory before the chunk's first loads
    uint32_t k;
    toploc_verify_result* result;
    bool* ok;
    template <typename Shared>
    __device__ __forceinline__ SelectStart seed(Shared&) const
    {
        *ok = verify_decode<kThreads, F>(vs, words, k, result);
        return SelectStart{0u, Threshold{0, 0xFFFFFFFFu}, k};
    }
};

// F is the proof's field, Fmt the format of the recomputed activations (Section 5.7
// validates across the two precisions).
template <int KMAX, int CAP, typename F = Field16, typename Fmt = Bf16Fmt, int U = kLoads, int WAVES = waves_for(CAP), int DEPTH = 2>
__global__ __launch_bounds__(kThreads, WAVES) void verify_kernel(const u32x4* __restrict__ hidden, uint32_t nvec,
                                                                            uint32_t k, const uint8_t* __restrict__ proofs,
                                                                            toploc_thresholds thr,
                                                                            toploc_verify_result* __restrict__ results)
{
    __shared__ SelectShared<kThreads, CAP, kQcap, Fmt> s;
    __shared__ VerifyShared<KMAX, Fmt::ELEMS == 4> vs;
    const uint64_t chunk = chunk_of_block();
    const uint16_t* proof = reinterpret_cast<const uint16_t*>(proofs + chunk * (2 + 2 * (uint64_t)F::WORDS * k));
    // The proof's words are requested first and the chunk's first loads right behind them; decode(p)
    // runs while those are in flight.  A malformed proof has its record written there and the
    // selection's result is dropped
    bool ok = true;
    const ProofWords<kThreads, KMAX> words = verify_load_proof<kThreads, F, KMAX>(proof, k);
    const DecodeFirst<F, KMAX, Fmt::ELEMS == 4> first{vs, words, k, results + chunk, &ok};
    (void)select_topk_from<kThreads, U, DEPTH>(hidden + chunk * nvec, 0u, nvec, s, first);  // order is irrelevant here
    if (!ok) return;  // uniform
    TOPLOC_TICK_BEGIN(tail);
    verify_tail<kThreads, F, Fmt>(vs, s.cand_idx, s.cand_bits, k, thr, results + chunk);
    TOPLOC_TICK_END(tail, 4);
}

// ---------------------------------------------------------------------------
// Split path, first launch: top-k of one part.  Writes k candidate slots per part,
// the unused ones (part shorter than k values) padded with index 0xFFFFFFFF.
// ---------------------------------------------------------------------------
template <int CAP, typename Fmt = Bf16Fmt, int DEPTH = 2>
__global__ __launch_bounds__(kThreads, DEPTH == 3 ? TOPLOC_MIN_WAVES - 1 : waves_for(CAP)) void part_kernel(const u32x4* __restrict__ hidden, Layout lay,
                                                                          uint32_t k, uint32_t* __restrict__ c_idx,
                                                                          typename Fmt::bits_t* __restrict__ c_bits)
{
    __shared__ SelectShared<kThreads, CAP, kQcap, Fmt> s;
    const uint32_t tid = threadIdx.x;
    const uint64_t slot = blockIdx.x;
    const u32x4* src;
    uint32_t v0, v1;
    if (lay.part_table) {
        const PartDesc d = lay.part_table[slot];
        if (d.seg_vec == kIdlePart) return;  // uniform: a slot no segment owns
        src = hidden + d.seg_vec;
        v0 = d.v0;
        v1 = d.v1;
    } else {
        const uint64_t chunk = slot / lay.parts;
        const uint32_t part = (uint32_t)(slot - chunk * lay.parts);
        src = hidden + chunk * lay.nvec;
        v0 = part * lay.part_vecs;
        v1 = v0 + lay.part_vecs < lay.nvec ? v0 + lay.part_vecs : lay.nvec;
        if (v0 > v1) v0 = v1;
    }
    const uint32_t have = (v1 - v0) * (uint32_t)Fmt::ELEMS;
    const uint32_t k_eff = have < k ? have : k;
    if (k_eff) select_topk<kThreads, kLoads, DEPTH>(src + v0, v0, v1, k_eff, s);
    for (uint32_t t = tid; t < k; t += kThreads) {
        c_idx[slot * k + t] = t < k_eff ? s.cand_idx[t] : 0xFFFFFFFFu;
        c_bits[slot * k + t] = t < k_eff ? s.cand_bits[t] : (typename Fmt::bits_t)0;
    }
}

// candidate slots of the chunk / segment a merge workgroup owns; status as in SegInfo
__device__ __forceinline__ uint32_t merge_range(const Layout& lay, uint64_t unit, uint32_t k, uint64_t& first,
                                                uint32_t& n_parts)
{
    if (lay.row_offsets) {
        const SegInfo g = segment_info(lay, unit, k);
        first = g.first_slot;
        n_parts = g.n_parts;
        return g.status;
    }
    first = unit * lay.parts;
    n_parts = lay.parts;
    return TOPLOC_CHUNK_OK;
}

// ---------------------------------------------------------------------------
// Split path, second launch of a build: top-k of the candidates, then the rest of
// Algorithm 1 (interp.hpp).
// ---------------------------------------------------------------------------
template <int THREADS, int KMAX, int CAP, typename F = Field16, typename Fmt = Bf16Fmt>
__global__ __launch_bounds__(THREADS) void build_merge_kernel(Layout lay, uint32_t k, const uint32_t* __restrict__ c_idx,
                                                              const typename Fmt::bits_t* __restrict__ c_bits,
                                                              uint8_t* __restrict__ proofs, uint8_t* __restrict__ status,
                                                              uint32_t* __restrict__ out_idx)
{
    static_assert(KMAX <= THREADS, "one pair per lane is carried across the phase change");
    __shared__ union MergeShared {
        SelectShared<THREADS, CAP, 1, Fmt> sel;
        InterpShared<KMAX, F> itp;
    } sh;
    __shared__ uint32_t coef[KMAX];
    const uint32_t tid = threadIdx.x;
    const uint64_t unit = blockIdx.x;
    uint64_t first;
    uint32_t n_parts;
    const uint32_t seg_status = merge_range(lay, unit, k, first, n_parts);
    if (seg_status != TOPLOC_CHUNK_OK) {  // uniform: a segment without a proof
        uint16_t* proof = reinterpret_cast<uint16_t*>(proofs + unit * (2 + 2 * (uint64_t)F::WORDS * k));
        for (uint32_t j = tid; j <= k * F::WORDS; j += THREADS) proof[j] = 0;
        if (out_idx)
            for (uint32_t j = tid; j < k; j += THREADS) out_idx[unit * k + j] = 0xFFFFFFFFu;
        if (tid == 0) status[unit] = (uint8_t)seg_status;
        return;
    }
    merge_topk(c_idx + first * k, c_bits + first * k, n_parts * k, k, sh.sel);
    if (out_idx) {
        order_topk(sh.sel, k);
        if (tid < k) out_idx[unit * k + tid] = sh.sel.cand_idx[tid];
    }
    uint32_t my_idx = 0, my_y = 0;
    if (tid < k) { my_idx = sh.sel.cand_idx[tid]; my_y = sh.sel.cand_bits[tid]; }
    __syncthreads();
    if (tid < k) {
        sh.itp.idx[tid] = my_idx;
        sh.itp.ys[tid] = (typename F::elem_t)F::from_pattern(my_y);
    }
    finish_proof<THREADS>(sh.itp, coef, k,
                          reinterpret_cast<uint16_t*>(proofs + unit * (2 + 2 * (uint64_t)F::WORDS * k)), status + unit);
}

// ---------------------------------------------------------------------------
// Split path, second launch of a verify: top-k of the candidates, then the rest of
// Algorithm 2 (verify.hpp).
// ---------------------------------------------------------------------------
template <int THREADS, int KMAX, int CAP, typename F = Field16, typename Fmt = Bf16Fmt>
__global__ __launch_bounds__(THREADS) void verify_merge_kernel(Layout lay, uint32_t k, const uint32_t* __restrict__ c_idx,
                                                               const typename Fmt::bits_t* __restrict__ c_bits,
                                                               const uint8_t* __restrict__ proofs, toploc_thresholds thr,
                                                               toploc_verify_result* __restrict__ results)
{
    __shared__ SelectShared<THREADS, CAP, 1, Fmt> s;
    __shared__ VerifyShared<KMAX, Fmt::ELEMS == 4> vs;
    const uint64_t unit = blockIdx.x;
    const uint16_t* proof = reinterpret_cast<const uint16_t*>(proofs + unit * (2 + 2 * (uint64_t)F::WORDS * k));
    uint64_t first;
    uint32_t n_parts;
    const uint32_t seg_status = merge_range(lay, unit, k, first, n_parts);
    if (seg_status != TOPLOC_CHUNK_OK) {  // uniform: nothing to validate against
        if (threadIdx.x == 0) {
            toploc_verify_result r = {};
            r.status = (uint8_t)seg_status;
            results[unit] = r;
        }
        return;
    }
    if (!verify_decode<THREADS, F>(vs, proof, k, results + unit)) return;
    merge_topk(c_idx + first * k, c_bits + first * k, n_parts * k, k, s);
    verify_tail<THREADS, F, Fmt>(vs, s.cand_idx, s.cand_bits, k, thr, results + unit);
}

// ---------------------------------------------------------------------------
// Online path without the ring: per sequence the running top-k of the rows appended so
// far.  State of one sequence: header, k indices, k patterns (each part 16-byte aligned).
// ---------------------------------------------------------------------------
struct StreamHeader {
    uint32_t count;  // pairs held (<= k)
    int32_t tm;      // threshold element the selection ended with
    uint32_t ti;
    uint32_t rows;   // rows appended since the last emission
};
static_assert(sizeof(StreamHeader) == 16, "state layout");

static_assert(sizeof(StreamHeader) == plan::kStreamHeaderBytes, "state layout");
__host__ __device__ __forceinline__ size_t stream_idx_bytes(uint32_t k) { return ((size_t)k * 4 + 15) & ~(size_t)15; }

__global__ __launch_bounds__(256) void stream_reset_kernel(char* __restrict__ state, uint32_t n_seq, size_t stride)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_seq) *reinterpret_cast<StreamHeader*>(state + (size_t)i * stride) = StreamHeader{0u, 0, 0xFFFFFFFFu, 0u};
}

// What a sequence holds enters the selection of its next row: all k slots are read
// before the header says how many of them count, so that header, pairs and the row's
// first vectors are in flight together.
template <int CAP, typename Fmt = Bf16Fmt>
struct StreamSeed {
    const StreamHeader* hdr;
    const uint32_t* g_idx;
    const typename Fmt::bits_t* g_bits;
    uint32_t k, row_values;
    __device__ __forceinline__ SelectStart seed(SelectShared<kThreads, CAP, kQcap, Fmt>& s) const
    {
        constexpr int SPT = (CAP / 4 + kThreads - 1) / kThreads;  // k <= CAP/4 slots over the lanes
        uint32_t si[SPT], sb[SPT];
#pragma unroll
        for (int j = 0; j < SPT; ++j) {
            const uint32_t i = threadIdx.x + j * kThreads;
            si[j] = 0; sb[j] = 0;
            if (i < k) { si[j] = g_idx[i]; sb[j] = g_bits[i]; }
        }
        const StreamHeader h = *hdr;
#pragma unroll
        for (int j = 0; j < SPT; ++j) {
            const uint32_t i = threadIdx.x + j * kThreads;
            if (i < h.count) { s.cand_idx[i] = si[j]; s.cand_bits[i] = (typename Fmt::bits_t)sb[j]; }
        }
        const uint64_t have = (uint64_t)h.count + row_values;
        return SelectStart{h.count, Threshold{h.tm, h.ti}, have < k ? (uint32_t)have : k};
    }
};

// One appended row per sequence: the selection of select.hpp over the row's vectors,
// seeded with the pairs and the threshold the sequence holds.  The row is the vector range
// [v0, v0 + hvec) of the chunk, v0 = token*hvec, so flat indices come out as token*hidden + channel.
// With `slots` (continuous batching: the rows of a step belong to any subset of the
// sequences, each at its own position) row r goes to sequence slots[r] as token tokens[r];
// a row whose slot or token is out of range is skipped.
template <int CAP, typename Fmt = Bf16Fmt>
__global__ __launch_bounds__(kThreads, waves_for(CAP)) void stream_append_kernel(char* __restrict__ state, size_t stride,
                                                                                   const u32x4* __restrict__ step_vec,
                                                                                   uint32_t hvec, uint32_t v0, uint32_t k,
                                                                                   const uint32_t* __restrict__ slots,
                                                                                   const uint32_t* __restrict__ tokens,
                                                                                   uint32_t n_slots, uint32_t chunk_tokens)
{
    __shared__ SelectShared<kThreads, CAP, kQcap, Fmt> s;
    typedef typename Fmt::bits_t bits_t;
    const uint32_t tid = threadIdx.x;
    uint32_t seq = blockIdx.x;
    if (slots) {  // uniform
        seq = slots[blockIdx.x];
        const uint32_t token = tokens[blockIdx.x];
        if (seq >= n_slots || token >= chunk_tokens) return;
        v0 = token * hvec;
    }
    char* st = state + (size_t)seq * stride;
    StreamHeader* hdr = reinterpret_cast<StreamHeader*>(st);
    uint32_t* g_idx = reinterpret_cast<uint32_t*>(st + sizeof(StreamHeader));
    bits_t* g_bits = reinterpret_cast<bits_t*>(st + sizeof(StreamHeader) + stream_idx_bytes(k));
    const u32x4* row = step_vec + (size_t)blockIdx.x * hvec;
    const uint32_t rows = hdr->rows;
    const SelectStart end = select_topk_from<kThreads, kLoads, 2, CAP, kQcap>(
        row, v0, v0 + hvec, s, StreamSeed<CAP, Fmt>{hdr, g_idx, g_bits, k, hvec * (uint32_t)Fmt::ELEMS});
    for (uint32_t i = tid; i < end.k; i += kThreads) {
        g_idx[i] = s.cand_idx[i];
        g_bits[i] = s.cand_bits[i];
    }
    if (tid == 0) *hdr = StreamHeader{end.k, end.t.tm, end.t.ti, rows + 1u};
}

// Emission: steps 2-5 of Algorithm 1 on the k pairs a sequence holds, then the state is emptied.
template <int THREADS, int KMAX, int CAP, typename F = Field16, typename Fmt = Bf16Fmt>
__global__ __launch_bounds__(THREADS) void stream_emit_kernel(char* __restrict__ state, size_t stride, uint32_t k,
                                                              uint8_t* __restrict__ proofs, uint8_t* __restrict__ status,
                                                              uint32_t* __restrict__ out_idx,
                                                              const uint32_t* __restrict__ slots, uint32_t n_slots)
{
    static_assert(KMAX <= THREADS, "one pair per lane is carried across the phase change");
    __shared__ union EmitShared {
        SelectShared<THREADS, CAP, 1, Fmt> sel;
        InterpShared<KMAX, F> itp;
    } sh;
    __shared__ uint32_t coef[KMAX];
    typedef typename Fmt::bits_t bits_t;
    const uint32_t tid = threadIdx.x;
    const uint64_t seq = blockIdx.x;  // output row; with `slots` the state of sequence slots[seq]
    const uint64_t owner = slots ? slots[seq] : seq;
    const bool known = owner < n_slots;  // uniform
    char* st = state + (known ? owner : 0) * stride;
    StreamHeader* hdr = reinterpret_cast<StreamHeader*>(st);
    const uint32_t* g_idx = reinterpret_cast<const uint32_t*>(st + sizeof(StreamHeader));
    const bits_t* g_bits = reinterpret_cast<const bits_t*>(st + sizeof(StreamHeader) + stream_idx_bytes(k));
    const uint32_t count = known ? hdr->count : 0u;
    uint16_t* proof = reinterpret_cast<uint16_t*>(proofs + seq * (2 + 2 * (uint64_t)F::WORDS * k));
    __syncthreads();  // every lane has read the header
    if (tid == 0 && known) *hdr = StreamHeader{0u, 0, 0xFFFFFFFFu, 0u};
    if (count < k) {  // uniform
        for (uint32_t j = tid; j <= k * F::WORDS; j += THREADS) proof[j] = 0;
        if (out_idx)
            for (uint32_t j = tid; j < k; j += THREADS) out_idx[seq * k + j] = 0xFFFFFFFFu;
        if (tid == 0) status[seq] = TOPLOC_CHUNK_SHORT;
        return;
    }
    uint32_t my_idx = 0, my_y = 0;
    if (out_idx) {  // uniform: the caller wants the ordered indices
        for (uint32_t j = tid; j < k; j += THREADS) { sh.sel.cand_idx[j] = g_idx[j]; sh.sel.cand_bits[j] = g_bits[j]; }
        __syncthreads();
        order_topk(sh.sel, k);
        if (tid < k) { out_idx[seq * k + tid] = sh.sel.cand_idx[tid]; my_idx = sh.sel.cand_idx[tid]; my_y = sh.sel.cand_bits[tid]; }
        __syncthreads();
    } else if (tid < k) {
        my_idx = g_idx[tid];
        my_y = g_bits[tid];
    }
    if (tid < k) {
        sh.itp.idx[tid] = my_idx;
        sh.itp.ys[tid] = (typename F::elem_t)F::from_pattern(my_y);
    }
    finish_proof<THREADS>(sh.itp, coef, k, proof, status + seq);
}

// ---------------------------------------------------------------------------
// ring[s][step mod T][:] = step_vec[s][:]
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ring_kernel(u32x4* __restrict__ ring, const u32x4* __restrict__ step_vec,
                                                   uint32_t n_seq, uint32_t hvec, uint32_t chunk_tokens, uint32_t slot)
{
    const uint64_t total = (uint64_t)n_seq * hvec;
    for (uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; i < total; i += (uint64_t)gridDim.x * blockDim.x) {
        const uint64_t sidx = i / hvec;
        const uint64_t v = i - sidx * hvec;
        ring[(sidx * chunk_tokens + slot) * hvec + v] = step_vec[i];
    }
}

// ---------------------------------------------------------------------------
// Measurement aid: the same access pattern as the selection (one workgroup per
// chunk, 16-byte non-temporal loads, kLoads per lane and round) with nothing
// but a running maximum, to show what a pure read of the tensor achieves.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void read_kernel(const u32x4* __restrict__ hidden, uint32_t nvec,
                                                        uint32_t* __restrict__ out)
{
    const u32x4* src = hidden + (uint64_t)blockIdx.x * nvec;
    uint32_t m = 0;
    for (uint32_t base = 0; base < nvec; base += kThreads * kLoads) {
        u32x4 r[kLoads];
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            const uint32_t v = base + u * kThreads + threadIdx.x;
            r[u] = u32x4{0u, 0u, 0u, 0u};
            if (v < nvec) r[u] = __builtin_nontemporal_load(src + v);
        }
#pragma unroll
        for (int u = 0; u < kLoads; ++u) m = max(m, max(max(r[u].x, r[u].y), max(r[u].z, r[u].w)));
    }
    if (m == 0xFFFFFFFFu) out[blockIdx.x] = m;  // practically never: keeps the loads alive
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
// Process-wide state: entry points may be called from several host threads at once.
static std::atomic<int> g_last_hip_error{0};
static std::atomic<int> g_profile_on{0};
static std::atomic<uint32_t> g_force_parts{0};  // toploc_set_split: 0 = choose, n = cut every chunk into n parts
struct ProfRec { int slot; hipEvent_t a, b; };
static std::mutex g_prof_mutex;
static std::vector<ProfRec> g_prof;            // recorded, not yet read
static std::vector<hipEvent_t> g_event_pool;   // created by toploc_profile_enable, never by a launch
constexpr size_t kProfPairs = 8192;            // launches that can be timed between two reads

static bool hip_ok(hipError_t e)
{
    if (e != hipSuccess) { g_last_hip_error = (int)e; return false; }
    return true;
}

// Brackets one kernel launch with two events of the pool while timing is enabled.  With timing
// off (the default) it does nothing; with the pool empty the launch simply goes untimed: a launch
// never creates or destroys an event.
struct ProfScope {
    int slot; hipStream_t st; hipEvent_t a = nullptr, b = nullptr; bool on;
    ProfScope(int slot_, hipStream_t st_) : slot(slot_), st(st_), on(g_profile_on != 0)
    {
        if (!on) return;
        {
            std::lock_guard<std::mutex> lock(g_prof_mutex);
            on = g_event_pool.size() >= 2;
            if (on) {
                a = g_event_pool.back(); g_event_pool.pop_back();
                b = g_event_pool.back(); g_event_pool.pop_back();
            }
        }
        if (on && !hip_ok(hipEventRecord(a, st))) give_back();
    }
    ~ProfScope()
    {
        if (!on) return;
        if (!hip_ok(hipEventRecord(b, st))) { give_back(); return; }
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        g_prof.push_back({slot, a, b});
    }
    void give_back()
    {
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        g_event_pool.push_back(a);
        g_event_pool.push_back(b);
        on = false;
    }
};

using plan::aligned16;
using plan::bits_size_of;
using plan::cand_bytes;
using plan::chunk_len;
using plan::chunk_len_mixed;
using plan::FixedPlan;
using plan::up16;

// the cut of a batch of fixed chunks; the split switch is read once per plan: another thread may change it
static FixedPlan plan_fixed(uint64_t n_chunks, uint64_t nvec) { return plan::plan_fixed(n_chunks, nvec, g_force_parts.load()); }

static void launch_part(hipStream_t st, const void* d_hidden, const Layout& lay, uint64_t slots, uint32_t k, uint32_t* c_idx,
                        void* c_bits_any, uint32_t hidden_dtype = TOPLOC_DTYPE_BF16)
{
    ProfScope ps(TOPLOC_KERNEL_PART, st);
    if (hidden_dtype == TOPLOC_DTYPE_F32) {
        if (k <= 128)
            hipLaunchKernelGGL((part_kernel<kCapSmall, F32Fmt>), dim3((uint32_t)slots), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden, lay, k, c_idx, (uint32_t*)c_bits_any);
        else
            hipLaunchKernelGGL((part_kernel<kCapLarge, F32Fmt>), dim3((uint32_t)slots), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden, lay, k, c_idx, (uint32_t*)c_bits_any);
        return;
    }
    uint16_t* c_bits = (uint16_t*)c_bits_any;
    const bool one_generation = slots <= kOneGeneration;   // every part resident at once: three rounds of loads in flight each
    if (k <= 128 && one_generation)
        hipLaunchKernelGGL((part_kernel<kCapSmall, Bf16Fmt, 3>), dim3((uint32_t)slots), dim3(kThreads), 0, st, (const u32x4*)d_hidden,
                           lay, k, c_idx, c_bits);
    else if (k <= 128)
        hipLaunchKernelGGL((part_kernel<kCapSmall>), dim3((uint32_t)slots), dim3(kThreads), 0, st, (const u32x4*)d_hidden, lay,
                           k, c_idx, c_bits);
    else   // the wide candidate buffer allows 5 workgroups per CU anyway: the third round of loads is free
        hipLaunchKernelGGL((part_kernel<kCapLarge, Bf16Fmt, 3>), dim3((uint32_t)slots), dim3(kThreads), 0, st, (const u32x4*)d_hidden,
                           lay, k, c_idx, c_bits);
}

static void launch_build_merge(hipStream_t st, const Layout& lay, uint64_t units, uint32_t k, const uint32_t* c_idx,
                               const void* c_bits_any, uint8_t* d_proofs, uint8_t* d_status, uint32_t* d_topk_idx_opt,
                               uint32_t dtype = TOPLOC_DTYPE_BF16)
{
    ProfScope ps(TOPLOC_KERNEL_BUILD_MERGE, st);
    if (dtype == TOPLOC_DTYPE_F32) {
        if (k <= 128)
            hipLaunchKernelGGL((build_merge_kernel<256, 128, kCapMerge, Field32, F32Fmt>), dim3((uint32_t)units), dim3(256), 0,
                               st, lay, k, c_idx, (const uint32_t*)c_bits_any, d_proofs, d_status, d_topk_idx_opt);
        else
            hipLaunchKernelGGL((build_merge_kernel<1024, 512, kCapMerge, Field32, F32Fmt>), dim3((uint32_t)units), dim3(1024),
                               0, st, lay, k, c_idx, (const uint32_t*)c_bits_any, d_proofs, d_status, d_topk_idx_opt);
        return;
    }
    const uint16_t* c_bits = (const uint16_t*)c_bits_any;
    if (k <= 128)
        hipLaunchKernelGGL((build_merge_kernel<256, 128, kCapMerge>), dim3((uint32_t)units), dim3(256), 0, st, lay, k, c_idx,
                           c_bits, d_proofs, d_status, d_topk_idx_opt);
    else
        hipLaunchKernelGGL((build_merge_kernel<1024, 512, kCapMerge>), dim3((uint32_t)units), dim3(1024), 0, st, lay, k, c_idx,
                           c_bits, d_proofs, d_status, d_topk_idx_opt);
}

static void launch_verify_merge(hipStream_t st, const Layout& lay, uint64_t units, uint32_t k, const uint32_t* c_idx,
                                const void* c_bits_any, const uint8_t* d_proofs, const toploc_thresholds& thr,
                                toploc_verify_result* d_results, uint32_t hidden_dtype = TOPLOC_DTYPE_BF16,
                                uint32_t proof_dtype = TOPLOC_DTYPE_BF16)
{
    ProfScope ps(TOPLOC_KERNEL_VERIFY_MERGE, st);
    const dim3 grid((uint32_t)units), block(256), block_wide(512);
    const bool wide = k > 128;   // the larger candidate buffer and 512 lanes
    if (hidden_dtype == TOPLOC_DTYPE_F32 && proof_dtype == TOPLOC_DTYPE_F32) {
        if (!wide)
            hipLaunchKernelGGL((verify_merge_kernel<256, 128, kCapMerge, Field32, F32Fmt>), grid, block, 0, st, lay, k, c_idx,
                               (const uint32_t*)c_bits_any, d_proofs, thr, d_results);
        else
            hipLaunchKernelGGL((verify_merge_kernel<512, 512, kCapMerge, Field32, F32Fmt>), grid, block_wide, 0, st, lay, k,
                               c_idx, (const uint32_t*)c_bits_any, d_proofs, thr, d_results);
        return;
    }
    if (hidden_dtype == TOPLOC_DTYPE_F32) {  // bf16 proof, fp32 validator
        if (!wide)
            hipLaunchKernelGGL((verify_merge_kernel<256, 128, kCapMerge, Field16, F32Fmt>), grid, block, 0, st, lay, k, c_idx,
                               (const uint32_t*)c_bits_any, d_proofs, thr, d_results);
        else
            hipLaunchKernelGGL((verify_merge_kernel<512, 512, kCapMerge, Field16, F32Fmt>), grid, block_wide, 0, st, lay, k,
                               c_idx, (const uint32_t*)c_bits_any, d_proofs, thr, d_results);
        return;
    }
    const uint16_t* c_bits = (const uint16_t*)c_bits_any;
    if (proof_dtype == TOPLOC_DTYPE_F32) {   // fp32 proof, bf16 validator
        if (!wide)
            hipLaunchKernelGGL((verify_merge_kernel<256, 128, kCapMerge, Field32, Bf16Fmt>), grid, block, 0, st, lay, k, c_idx,
                               c_bits, d_proofs, thr, d_results);
        else
            hipLaunchKernelGGL((verify_merge_kernel<512, 512, kCapMerge, Field32, Bf16Fmt>), grid, block_wide, 0, st, lay, k,
                               c_idx, c_bits, d_proofs, thr, d_results);
        return;
    }
    if (!wide)
        hipLaunchKernelGGL((verify_merge_kernel<256, 128, kCapMerge>), grid, block, 0, st, lay, k, c_idx, c_bits, d_proofs, thr,
                           d_results);
    else
        hipLaunchKernelGGL((verify_merge_kernel<512, 512, kCapMerge>), grid, block_wide, 0, st, lay, k, c_idx, c_bits, d_proofs,
                           thr, d_results);
}

// Segments: the host plans from sizes alone (plan.hpp); the part table is built on the device from the
// row offsets, behind the candidate arrays of the workspace.
static plan::SegmentPlan plan_segments(uint64_t n_segments, uint64_t total_rows, uint32_t hidden, uint32_t k,
                                       uint32_t hidden_dtype, uint32_t proof_dtype)
{
    if (hidden_dtype > TOPLOC_DTYPE_F32 || proof_dtype > TOPLOC_DTYPE_F32) return plan::SegmentPlan{false, 0, 0, 0};
    return plan::plan_segments(n_segments, total_rows, hidden, k, hidden_dtype, plan::max_k_of(hidden_dtype, proof_dtype),
                               g_force_parts.load());
}

// Lays the workspace out, enqueues the planning kernel and the part launch of a segment call.
static int launch_segment_parts(const plan::SegmentPlan& pl, const void* d_hidden, uint64_t total_rows,
                                const uint64_t* d_row_offsets, uint64_t n_segments, uint32_t hidden, uint32_t k,
                                uint32_t hidden_dtype, void* d_workspace, hipStream_t st, Layout& lay, uint32_t*& c_idx,
                                void*& c_bits)
{
    char* w = (char*)d_workspace;
    const size_t bits_size = bits_size_of(hidden_dtype);
    c_idx = (uint32_t*)w;
    c_bits = w + up16((size_t)pl.slots * k * sizeof(uint32_t));
    PartDesc* table = (PartDesc*)(w + cand_bytes(pl.slots, k, bits_size));
    lay.part_table = table;
    lay.row_offsets = d_row_offsets;
    lay.total_rows = total_rows;
    lay.row_vecs = pl.row_vecs;
    lay.row_values = hidden;
    lay.nvec = 0;
    lay.parts = 0;
    lay.part_vecs = (uint32_t)pl.part_vecs;
    {
        ProfScope ps(TOPLOC_KERNEL_PLAN, st);
        hipLaunchKernelGGL(plan_segments_kernel, dim3((uint32_t)((pl.slots + 255) / 256)), dim3(256), 0, st, lay, n_segments,
                           pl.slots, k, table);
    }
    if (!hip_ok(hipGetLastError())) return TOPLOC_EHIP;
    launch_part(st, d_hidden, lay, pl.slots, k, c_idx, c_bits, hidden_dtype);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

}  // namespace toploc

using namespace toploc;

extern "C" {

size_t toploc_proof_bytes(uint32_t k) { return 2 + 2 * (size_t)k; }

int toploc_workspace_query(const toploc_params* params, uint64_t n_chunks, size_t* bytes)
{
    if (!bytes) return TOPLOC_EINVAL;
    *bytes = 0;
    const uint64_t n = chunk_len(params);
    if (n == 0 || n_chunks >= (1ull << 31)) return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    const FixedPlan f = plan_fixed(n_chunks, n / 8);
    if (f.parts == 1 && params->k <= 128) return TOPLOC_OK;  // one fused kernel, everything stays on chip
    if (n_chunks * f.parts >= (1ull << 31)) return TOPLOC_EINVAL;
    *bytes = cand_bytes(n_chunks * f.parts, params->k);
    return TOPLOC_OK;
}

size_t toploc_workspace_bytes(const toploc_params* params, uint64_t n_chunks)
{
    size_t bytes = 0;
    (void)toploc_workspace_query(params, n_chunks, &bytes);
    return bytes;
}

int toploc_set_split(uint32_t parts_per_chunk)
{
    if (parts_per_chunk > 4096) return TOPLOC_EINVAL;
    g_force_parts = parts_per_chunk;
    return TOPLOC_OK;
}

int toploc_topk(const void* d_hidden_bf16, uint64_t n_chunks, const toploc_params* params, uint32_t* d_topk_idx,
                uint16_t* d_topk_val, void* hip_stream)
{
    const uint64_t n = chunk_len(params, TOPLOC_MAX_K_TOPK);
    const int chk = plan::check_fixed(n, n_chunks, d_hidden_bf16, d_topk_idx, 4, d_topk_val, 2, nullptr);
    if (chk != plan::kGo) return chk;
    hipStream_t st = (hipStream_t)hip_stream;
    {
        ProfScope ps(TOPLOC_KERNEL_SELECT, st);
        if (params->k <= 128)
            hipLaunchKernelGGL((select_kernel<kCapSmall>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden_bf16, (uint32_t)(n / 8), params->k, d_topk_idx, d_topk_val);
        else if (params->k <= TOPLOC_MAX_K)
            hipLaunchKernelGGL((select_kernel<kCapLarge>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden_bf16, (uint32_t)(n / 8), params->k, d_topk_idx, d_topk_val);
        else
            hipLaunchKernelGGL((select_kernel<kCapWide, 1>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden_bf16, (uint32_t)(n / 8), params->k, d_topk_idx, d_topk_val);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

// Algorithm 1 over fixed chunks with the cut already chosen (`f`): one fused launch, or the split pair
// of launches with the candidates in `d_workspace`.  Arguments are checked by the callers.
static int build_fixed(const FixedPlan& f, const void* d_hidden, uint64_t n_chunks, uint32_t nvec, uint32_t k,
                       uint8_t* d_proofs, uint8_t* d_status, uint32_t* d_topk_idx_opt, void* d_workspace,
                       size_t workspace_bytes, hipStream_t st, uint32_t dtype = TOPLOC_DTYPE_BF16)
{
    const void* d_hidden_bf16 = d_hidden;
    const size_t bits_size = bits_size_of(dtype);
    const bool have_ws = d_workspace && workspace_bytes >= cand_bytes(n_chunks * f.parts, k, bits_size);
    if (k <= 128 && (f.parts == 1 || !have_ws)) {  // one launch; also the answer to a missing workspace
        ProfScope ps(TOPLOC_KERNEL_BUILD, st);
        if (dtype == TOPLOC_DTYPE_F32)
            hipLaunchKernelGGL((build_kernel<128, kCapSmall, Field32, F32Fmt>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden, nvec, k, d_proofs, d_status, d_topk_idx_opt);
        else if (n_chunks <= kOneGeneration)   // every workgroup resident at once: three rounds of loads in flight each
            hipLaunchKernelGGL((build_kernel<128, kCapSmall, Field16, Bf16Fmt, kLoads, TOPLOC_MIN_WAVES - 1, 3>), dim3((uint32_t)n_chunks),
                               dim3(kThreads), 0, st, (const u32x4*)d_hidden_bf16, nvec, k, d_proofs, d_status, d_topk_idx_opt);
        else
            hipLaunchKernelGGL((build_kernel<128, kCapSmall>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden_bf16, nvec, k, d_proofs, d_status, d_topk_idx_opt);
        return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
    }
    if (!have_ws) return d_workspace ? TOPLOC_EWORKSPACE : TOPLOC_EINVAL;
    const uint64_t slots = n_chunks * f.parts;
    if (slots >= (1ull << 31)) return TOPLOC_EINVAL;
    Layout lay = {nullptr, nullptr, 0, 0, 0, nvec, f.parts, f.part_vecs};
    uint32_t* c_idx = (uint32_t*)d_workspace;
    void* c_bits = (char*)d_workspace + up16((size_t)slots * k * sizeof(uint32_t));
    launch_part(st, d_hidden, lay, slots, k, c_idx, c_bits, dtype);
    if (!hip_ok(hipGetLastError())) return TOPLOC_EHIP;
    launch_build_merge(st, lay, n_chunks, k, c_idx, c_bits, d_proofs, d_status, d_topk_idx_opt, dtype);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_build_proofs(const void* d_hidden_bf16, uint64_t n_chunks, const toploc_params* params, uint8_t* d_proofs,
                        uint8_t* d_status, uint32_t* d_topk_idx_opt, void* d_workspace, size_t workspace_bytes,
                        void* hip_stream)
{
    const uint64_t n = chunk_len(params);
    const int chk = plan::check_fixed(n, n_chunks, d_hidden_bf16, d_proofs, 2, d_status, 1, d_workspace);
    if (chk != plan::kGo) return chk;
    const uint32_t nvec = (uint32_t)(n / 8);
    return build_fixed(plan_fixed(n_chunks, nvec), d_hidden_bf16, n_chunks, nvec, params->k, d_proofs, d_status,
                       d_topk_idx_opt, d_workspace, workspace_bytes, (hipStream_t)hip_stream);
}

// ---------------------------------------------------------------------------
// toploc_build_proofs for callers that cannot allocate: the candidates of a split launch go to a
// fixed array in device memory that belongs to the library (one copy per GPU, at its own address,
// held until the process ends).  Host code never passes the array by name: the name is only the
// host-side handle hipGetSymbolAddress turns into the device address, once per device.
// ---------------------------------------------------------------------------
constexpr size_t kScratchBytes = (size_t)TOPLOC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device i, once looked up

// the current device's copy of the scratch array
static int scratch_of_current_device(void** out)
{
    int dev = -1;
    if (!hip_ok(hipGetDevice(&dev))) return TOPLOC_EHIP;
    if (dev < 0 || dev >= kMaxDevices) return TOPLOC_EINVAL;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (!hip_ok(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch))) || !ptr) return TOPLOC_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return TOPLOC_OK;
}

int toploc_build_proofs_static(const void* d_hidden_bf16, uint64_t n_chunks, const toploc_params* params,
                               uint8_t* d_proofs, uint8_t* d_status, uint32_t* d_topk_idx_opt, void* hip_stream)
{
    const uint64_t n = chunk_len(params);
    const int chk = plan::check_fixed(n, n_chunks, d_hidden_bf16, d_proofs, 2, d_status, 1, nullptr);
    if (chk != plan::kGo) return chk;
    const uint32_t nvec = (uint32_t)(n / 8);
    const FixedPlan f = plan_fixed(n_chunks, nvec);
    const bool fused = plan::fixed_plan_is_fused(f, params->k);   // no scratch at all
    const int fits = plan::check_static_scratch(f, n_chunks, params->k, kScratchBytes);
    if (fits != plan::kGo) return fits;
    void* ptr = nullptr;
    if (!fused) {
        const int rc = scratch_of_current_device(&ptr);
        if (rc != TOPLOC_OK) return rc;
    }
    return build_fixed(f, d_hidden_bf16, n_chunks, nvec, params->k, d_proofs, d_status, d_topk_idx_opt, ptr,
                       fused ? 0 : kScratchBytes, (hipStream_t)hip_stream);
}

int toploc_verify_proofs(const void* d_hidden_bf16, uint64_t n_chunks, const toploc_params* params,
                         const uint8_t* d_proofs, const toploc_thresholds* thresholds, toploc_verify_result* d_results,
                         void* d_workspace, size_t workspace_bytes, void* hip_stream)
{
    const uint64_t n = chunk_len(params);
    if (!thresholds) return TOPLOC_EINVAL;
    const int chk = plan::check_fixed(n, n_chunks, d_hidden_bf16, d_proofs, 2, d_results, 4, d_workspace);
    if (chk != plan::kGo) return chk;
    const uint32_t k = params->k;
    const uint32_t nvec = (uint32_t)(n / 8);
    hipStream_t st = (hipStream_t)hip_stream;
    FixedPlan f = plan_fixed(n_chunks, nvec);
    const uint64_t slots = n_chunks * f.parts;
    const bool split = f.parts > 1 && d_workspace && workspace_bytes >= cand_bytes(slots, k) && slots < (1ull << 31);
    if (!split) {  // one launch; a missing workspace only costs speed on small batches
        ProfScope ps(TOPLOC_KERNEL_VERIFY, st);
        if (k <= 128 && n_chunks <= kOneGeneration)
            hipLaunchKernelGGL((verify_kernel<128, kCapSmall, Field16, Bf16Fmt, kLoads, TOPLOC_MIN_WAVES - 1, 3>), dim3((uint32_t)n_chunks),
                               dim3(kThreads), 0, st, (const u32x4*)d_hidden_bf16, nvec, k, d_proofs, *thresholds, d_results);
        else if (k <= 128)
            hipLaunchKernelGGL((verify_kernel<128, kCapSmall>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden_bf16, nvec, k, d_proofs, *thresholds, d_results);
        else   // 5 workgroups per CU either way (LDS): the third round of loads is free
            hipLaunchKernelGGL((verify_kernel<512, kCapLarge, Field16, Bf16Fmt, kLoads, TOPLOC_MIN_WAVES - 1, 3>), dim3((uint32_t)n_chunks),
                               dim3(kThreads), 0, st, (const u32x4*)d_hidden_bf16, nvec, k, d_proofs, *thresholds, d_results);
        return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
    }
    Layout lay = {nullptr, nullptr, 0, 0, 0, nvec, f.parts, f.part_vecs};
    uint32_t* c_idx = (uint32_t*)d_workspace;
    uint16_t* c_bits = (uint16_t*)((char*)d_workspace + up16((size_t)slots * k * sizeof(uint32_t)));
    launch_part(st, d_hidden_bf16, lay, slots, k, c_idx, c_bits);
    if (!hip_ok(hipGetLastError())) return TOPLOC_EHIP;
    launch_verify_merge(st, lay, n_chunks, k, c_idx, c_bits, d_proofs, *thresholds, d_results);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

size_t toploc_segments_workspace_bytes_dtype(uint64_t n_segments, uint64_t total_rows, uint32_t hidden, uint32_t k,
                                             uint32_t hidden_dtype)
{
    const plan::SegmentPlan pl = plan_segments(n_segments, total_rows, hidden, k, hidden_dtype, hidden_dtype);
    if (!pl.ok || n_segments == 0) return 0;
    return plan::segments_workspace_bytes(pl, k, bits_size_of(hidden_dtype));
}

size_t toploc_segments_workspace_bytes(uint64_t n_segments, uint64_t total_rows, uint32_t hidden, uint32_t k)
{
    return toploc_segments_workspace_bytes_dtype(n_segments, total_rows, hidden, k, TOPLOC_DTYPE_BF16);
}

// Algorithm 1 over segments, activations of `hidden_dtype` (the proof has the same precision)
static int build_segments(const void* d_hidden, uint32_t hidden_dtype, uint64_t total_rows, const uint64_t* d_row_offsets,
                          uint64_t n_segments, uint32_t hidden, uint32_t k, uint8_t* d_proofs, uint8_t* d_status,
                          uint32_t* d_topk_idx_opt, void* d_workspace, size_t workspace_bytes, void* hip_stream)
{
    const plan::SegmentPlan pl = plan_segments(n_segments, total_rows, hidden, k, hidden_dtype, hidden_dtype);
    const int chk = plan::check_segments(pl, n_segments, k, hidden_dtype, d_hidden, d_row_offsets, d_proofs, d_status, 1, d_workspace,
                                   workspace_bytes);
    if (chk != plan::kGo) return chk;
    hipStream_t st = (hipStream_t)hip_stream;
    Layout lay;
    uint32_t* c_idx;
    void* c_bits;
    const int rc = launch_segment_parts(pl, d_hidden, total_rows, d_row_offsets, n_segments, hidden, k, hidden_dtype,
                                        d_workspace, st, lay, c_idx, c_bits);
    if (rc != TOPLOC_OK) return rc;
    launch_build_merge(st, lay, n_segments, k, c_idx, c_bits, d_proofs, d_status, d_topk_idx_opt, hidden_dtype);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_build_proofs_segments(const void* d_hidden_bf16, uint64_t total_rows, const uint64_t* d_row_offsets,
                                 uint64_t n_segments, uint32_t hidden, uint32_t k, uint8_t* d_proofs, uint8_t* d_status,
                                 uint32_t* d_topk_idx_opt, void* d_workspace, size_t workspace_bytes, void* hip_stream)
{
    return build_segments(d_hidden_bf16, TOPLOC_DTYPE_BF16, total_rows, d_row_offsets, n_segments, hidden, k, d_proofs,
                          d_status, d_topk_idx_opt, d_workspace, workspace_bytes, hip_stream);
}

int toploc_build_proofs_segments_f32(const void* d_hidden_f32, uint64_t total_rows, const uint64_t* d_row_offsets,
                                     uint64_t n_segments, uint32_t hidden, uint32_t k, uint8_t* d_proofs, uint8_t* d_status,
                                     uint32_t* d_topk_idx_opt, void* d_workspace, size_t workspace_bytes,
                                     void* hip_stream)
{
    return build_segments(d_hidden_f32, TOPLOC_DTYPE_F32, total_rows, d_row_offsets, n_segments, hidden, k, d_proofs,
                          d_status, d_topk_idx_opt, d_workspace, workspace_bytes, hip_stream);
}

int toploc_verify_proofs_segments_mixed(const void* d_hidden, uint32_t hidden_dtype, uint64_t total_rows,
                                        const uint64_t* d_row_offsets, uint64_t n_segments, uint32_t hidden, uint32_t k,
                                        const uint8_t* d_proofs, uint32_t proof_dtype, const toploc_thresholds* thresholds,
                                        toploc_verify_result* d_results, void* d_workspace, size_t workspace_bytes,
                                        void* hip_stream)
{
    const plan::SegmentPlan pl = plan_segments(n_segments, total_rows, hidden, k, hidden_dtype, proof_dtype);
    if (!thresholds) return TOPLOC_EINVAL;
    const int chk = plan::check_segments(pl, n_segments, k, hidden_dtype, d_hidden, d_row_offsets, d_proofs, d_results, 4,
                                   d_workspace, workspace_bytes);
    if (chk != plan::kGo) return chk;
    hipStream_t st = (hipStream_t)hip_stream;
    Layout lay;
    uint32_t* c_idx;
    void* c_bits;
    const int rc = launch_segment_parts(pl, d_hidden, total_rows, d_row_offsets, n_segments, hidden, k, hidden_dtype,
                                        d_workspace, st, lay, c_idx, c_bits);
    if (rc != TOPLOC_OK) return rc;
    launch_verify_merge(st, lay, n_segments, k, c_idx, c_bits, d_proofs, *thresholds, d_results, hidden_dtype, proof_dtype);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_verify_proofs_segments(const void* d_hidden_bf16, uint64_t total_rows, const uint64_t* d_row_offsets,
                                  uint64_t n_segments, uint32_t hidden, uint32_t k, const uint8_t* d_proofs,
                                  const toploc_thresholds* thresholds, toploc_verify_result* d_results, void* d_workspace,
                                  size_t workspace_bytes, void* hip_stream)
{
    return toploc_verify_proofs_segments_mixed(d_hidden_bf16, TOPLOC_DTYPE_BF16, total_rows, d_row_offsets, n_segments,
                                               hidden, k, d_proofs, TOPLOC_DTYPE_BF16, thresholds, d_results, d_workspace,
                                               workspace_bytes, hip_stream);
}

size_t toploc_proof_bytes_dtype(uint32_t k, uint32_t dtype)
{
    return 2 + (size_t)k * (dtype == TOPLOC_DTYPE_F32 ? 4 : 2);
}

size_t toploc_workspace_bytes_f32(const toploc_params* params, uint64_t n_chunks)
{
    const uint64_t n = chunk_len_mixed(params, TOPLOC_DTYPE_F32, TOPLOC_DTYPE_F32);
    if (n == 0 || n_chunks == 0 || n_chunks >= (1ull << 31)) return 0;
    const FixedPlan f = plan_fixed(n_chunks, n / 4);
    if (plan::fixed_plan_is_fused(f, params->k) || n_chunks * f.parts >= (1ull << 31)) return 0;
    return cand_bytes(n_chunks * f.parts, params->k, sizeof(uint32_t));
}

int toploc_build_proofs_f32(const void* d_hidden_f32, uint64_t n_chunks, const toploc_params* params, uint8_t* d_proofs,
                            uint8_t* d_status, uint32_t* d_topk_idx_opt, void* d_workspace, size_t workspace_bytes,
                            void* hip_stream)
{
    const uint64_t n = chunk_len_mixed(params, TOPLOC_DTYPE_F32, TOPLOC_DTYPE_F32);
    const int chk = plan::check_fixed(n, n_chunks, d_hidden_f32, d_proofs, 2, d_status, 1, d_workspace);
    if (chk != plan::kGo) return chk;
    const uint32_t nvec = (uint32_t)(n / 4);
    return build_fixed(plan_fixed(n_chunks, nvec), d_hidden_f32, n_chunks, nvec, params->k, d_proofs, d_status, d_topk_idx_opt,
                       d_workspace, workspace_bytes, (hipStream_t)hip_stream, TOPLOC_DTYPE_F32);
}

int toploc_verify_proofs_mixed(const void* d_hidden, uint32_t hidden_dtype, uint64_t n_chunks, const toploc_params* params,
                               const uint8_t* d_proofs, uint32_t proof_dtype, const toploc_thresholds* thresholds,
                               toploc_verify_result* d_results, void* hip_stream)
{
    const uint64_t n = chunk_len_mixed(params, hidden_dtype, proof_dtype);
    if (!thresholds) return TOPLOC_EINVAL;
    const int chk = plan::check_fixed(n, n_chunks, d_hidden, d_proofs, 2, d_results, 4, nullptr);
    if (chk != plan::kGo) return chk;
    if (hidden_dtype == TOPLOC_DTYPE_BF16 && proof_dtype == TOPLOC_DTYPE_BF16)
        return toploc_verify_proofs(d_hidden, n_chunks, params, d_proofs, thresholds, d_results, nullptr, 0, hip_stream);
    hipStream_t st = (hipStream_t)hip_stream;
    const uint32_t k = params->k;
    const dim3 grid((uint32_t)n_chunks), block(kThreads);
    const u32x4* h = (const u32x4*)d_hidden;
    {
        ProfScope ps(TOPLOC_KERNEL_VERIFY, st);
        const bool wide = k > 128;   // the larger candidate buffer
        if (hidden_dtype == TOPLOC_DTYPE_F32 && proof_dtype == TOPLOC_DTYPE_F32) {
            if (!wide)
                hipLaunchKernelGGL((verify_kernel<128, kCapSmall, Field32, F32Fmt>), grid, block, 0, st, h, (uint32_t)(n / 4), k,
                                   d_proofs, *thresholds, d_results);
            else
                hipLaunchKernelGGL((verify_kernel<512, kCapLarge, Field32, F32Fmt>), grid, block, 0, st, h, (uint32_t)(n / 4), k,
                                   d_proofs, *thresholds, d_results);
        } else if (hidden_dtype == TOPLOC_DTYPE_F32) {   // bf16 proof, fp32 validator
            if (!wide)
                hipLaunchKernelGGL((verify_kernel<128, kCapSmall, Field16, F32Fmt>), grid, block, 0, st, h, (uint32_t)(n / 4), k,
                                   d_proofs, *thresholds, d_results);
            else
                hipLaunchKernelGGL((verify_kernel<512, kCapLarge, Field16, F32Fmt>), grid, block, 0, st, h, (uint32_t)(n / 4), k,
                                   d_proofs, *thresholds, d_results);
        } else {                                          // fp32 proof, bf16 validator
            if (!wide)
                hipLaunchKernelGGL((verify_kernel<128, kCapSmall, Field32, Bf16Fmt>), grid, block, 0, st, h, (uint32_t)(n / 8), k,
                                   d_proofs, *thresholds, d_results);
            else
                hipLaunchKernelGGL((verify_kernel<512, kCapLarge, Field32, Bf16Fmt>), grid, block, 0, st, h, (uint32_t)(n / 8), k,
                                   d_proofs, *thresholds, d_results);
        }
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

size_t toploc_stream_state_bytes_dtype(uint32_t n_seq, uint32_t k, uint32_t dtype)
{
    if (!plan::stream_k_ok(k, dtype)) return 0;
    return (size_t)n_seq * plan::stream_stride(k, dtype);
}

int toploc_stream_reset_dtype(void* d_state, uint32_t n_seq, uint32_t k, uint32_t dtype, void* hip_stream)
{
    if (!plan::stream_k_ok(k, dtype)) return TOPLOC_EINVAL;
    if (n_seq == 0) return TOPLOC_OK;
    if (!d_state || !aligned16(d_state)) return TOPLOC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    hipLaunchKernelGGL(stream_reset_kernel, dim3((n_seq + 255) / 256), dim3(256), 0, st, (char*)d_state, n_seq,
                       plan::stream_stride(k, dtype));
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_stream_append_dtype(void* d_state, uint32_t n_slots, const void* d_step, uint32_t dtype, const uint32_t* d_slots,
                               const uint32_t* d_tokens, uint32_t n_rows, uint32_t hidden, uint32_t chunk_tokens,
                               uint32_t token, uint32_t k, void* hip_stream)
{
    const int chk = plan::check_stream_append(d_state, n_slots, d_step, d_slots, d_tokens, n_rows, hidden, chunk_tokens, token,
                                              k, dtype);
    if (chk != plan::kGo) return chk;
    hipStream_t st = (hipStream_t)hip_stream;
    const bool f32 = dtype == TOPLOC_DTYPE_F32;
    const uint32_t hvec = hidden / plan::elems_per_vec(dtype);
    const uint32_t v0 = d_slots ? 0u : token * hvec;
    const uint32_t n_known = d_slots ? n_slots : n_rows;
    const size_t stride = plan::stream_stride(k, dtype);
    const u32x4* step = (const u32x4*)d_step;
    {
        ProfScope ps(TOPLOC_KERNEL_STREAM_APPEND, st);
        const dim3 grid(n_rows), block(kThreads);
        if (!f32 && k <= 128)
            hipLaunchKernelGGL((stream_append_kernel<kCapSmall>), grid, block, 0, st, (char*)d_state, stride, step, hvec, v0, k,
                               d_slots, d_tokens, n_known, chunk_tokens);
        else if (!f32)
            hipLaunchKernelGGL((stream_append_kernel<kCapLarge>), grid, block, 0, st, (char*)d_state, stride, step, hvec, v0, k,
                               d_slots, d_tokens, n_known, chunk_tokens);
        else if (k <= 128)
            hipLaunchKernelGGL((stream_append_kernel<kCapSmall, F32Fmt>), grid, block, 0, st, (char*)d_state, stride, step, hvec,
                               v0, k, d_slots, d_tokens, n_known, chunk_tokens);
        else
            hipLaunchKernelGGL((stream_append_kernel<kCapLarge, F32Fmt>), grid, block, 0, st, (char*)d_state, stride, step, hvec,
                               v0, k, d_slots, d_tokens, n_known, chunk_tokens);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_stream_emit_dtype(void* d_state, uint32_t n_slots, uint32_t dtype, const uint32_t* d_slots, uint32_t n_rows,
                             uint32_t k, uint8_t* d_proofs, uint8_t* d_status, uint32_t* d_topk_idx_opt, void* hip_stream)
{
    const int chk = plan::check_stream_emit(d_state, n_rows, k, d_proofs, d_status, d_slots != nullptr, d_slots, n_slots, dtype);
    if (chk != plan::kGo) return chk;
    hipStream_t st = (hipStream_t)hip_stream;
    const bool f32 = dtype == TOPLOC_DTYPE_F32;
    const uint32_t n_known = d_slots ? n_slots : n_rows;
    const size_t stride = plan::stream_stride(k, dtype);
    {
        ProfScope ps(TOPLOC_KERNEL_STREAM_EMIT, st);
        const dim3 grid(n_rows);
        if (!f32 && k <= 128)
            hipLaunchKernelGGL((stream_emit_kernel<256, 128, kCapSmall>), grid, dim3(256), 0, st, (char*)d_state, stride, k,
                               d_proofs, d_status, d_topk_idx_opt, d_slots, n_known);
        else if (!f32)
            hipLaunchKernelGGL((stream_emit_kernel<1024, 512, kCapLarge>), grid, dim3(1024), 0, st, (char*)d_state, stride, k,
                               d_proofs, d_status, d_topk_idx_opt, d_slots, n_known);
        else if (k <= 128)
            hipLaunchKernelGGL((stream_emit_kernel<256, 128, kCapSmall, Field32, F32Fmt>), grid, dim3(256), 0, st,
                               (char*)d_state, stride, k, d_proofs, d_status, d_topk_idx_opt, d_slots, n_known);
        else
            hipLaunchKernelGGL((stream_emit_kernel<1024, 512, kCapLarge, Field32, F32Fmt>), grid, dim3(1024), 0, st,
                               (char*)d_state, stride, k, d_proofs, d_status, d_topk_idx_opt, d_slots, n_known);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

// the bf16 calls of the running top-k
size_t toploc_stream_state_bytes(uint32_t n_seq, uint32_t k) { return toploc_stream_state_bytes_dtype(n_seq, k, TOPLOC_DTYPE_BF16); }

int toploc_stream_reset(void* d_state, uint32_t n_seq, uint32_t k, void* hip_stream)
{
    return toploc_stream_reset_dtype(d_state, n_seq, k, TOPLOC_DTYPE_BF16, hip_stream);
}

int toploc_stream_append(void* d_state, const void* d_step_bf16, uint32_t n_seq, uint32_t hidden, uint32_t chunk_tokens,
                         uint32_t token, uint32_t k, void* hip_stream)
{
    return toploc_stream_append_dtype(d_state, n_seq, d_step_bf16, TOPLOC_DTYPE_BF16, nullptr, nullptr, n_seq, hidden,
                                      chunk_tokens, token, k, hip_stream);
}

int toploc_stream_append_rows(void* d_state, uint32_t n_slots, const void* d_step_bf16, const uint32_t* d_slots,
                              const uint32_t* d_tokens, uint32_t n_rows, uint32_t hidden, uint32_t chunk_tokens,
                              uint32_t k, void* hip_stream)
{
    if (n_rows != 0 && (!d_slots || !d_tokens)) return TOPLOC_EINVAL;
    return toploc_stream_append_dtype(d_state, n_slots, d_step_bf16, TOPLOC_DTYPE_BF16, d_slots, d_tokens, n_rows, hidden,
                                      chunk_tokens, 0, k, hip_stream);
}

int toploc_stream_emit(void* d_state, uint32_t n_seq, uint32_t k, uint8_t* d_proofs, uint8_t* d_status,
                       uint32_t* d_topk_idx_opt, void* hip_stream)
{
    return toploc_stream_emit_dtype(d_state, n_seq, TOPLOC_DTYPE_BF16, nullptr, n_seq, k, d_proofs, d_status, d_topk_idx_opt,
                                    hip_stream);
}

int toploc_stream_emit_rows(void* d_state, uint32_t n_slots, const uint32_t* d_slots, uint32_t n_rows, uint32_t k,
                            uint8_t* d_proofs, uint8_t* d_status, uint32_t* d_topk_idx_opt, void* hip_stream)
{
    if (n_rows != 0 && !d_slots) return TOPLOC_EINVAL;
    return toploc_stream_emit_dtype(d_state, n_slots, TOPLOC_DTYPE_BF16, d_slots, n_rows, k, d_proofs, d_status,
                                    d_topk_idx_opt, hip_stream);
}

int toploc_ring_append(void* d_ring_bf16, const void* d_step_bf16, uint32_t n_seq, uint32_t hidden,
                       uint32_t chunk_tokens, uint32_t step, void* hip_stream)
{
    const int chk = plan::check_ring_append(d_ring_bf16, d_step_bf16, n_seq, hidden, chunk_tokens);
    if (chk != plan::kGo) return chk;
    hipStream_t st = (hipStream_t)hip_stream;
    const uint32_t hvec = hidden / 8;
    const uint64_t total = (uint64_t)n_seq * hvec;
    uint64_t blocks = (total + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    {
        ProfScope ps(TOPLOC_KERNEL_RING, st);
        hipLaunchKernelGGL(ring_kernel, dim3((uint32_t)blocks), dim3(256), 0, st, (u32x4*)d_ring_bf16,
                           (const u32x4*)d_step_bf16, n_seq, hvec, chunk_tokens, step % chunk_tokens);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_bench_read(const void* d_hidden_bf16, uint64_t n_chunks, uint64_t chunk_values, uint32_t* d_out,
                      void* hip_stream)
{
    if (chunk_values == 0 || chunk_values % 8 != 0 || chunk_values >= (1ull << 32) || n_chunks >= (1ull << 31))
        return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    if (!d_hidden_bf16 || !d_out || !aligned16(d_hidden_bf16)) return TOPLOC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    {
        ProfScope ps(TOPLOC_KERNEL_READ, st);
        hipLaunchKernelGGL(read_kernel, dim3((uint32_t)n_chunks), dim3(kThreads), 0, st, (const u32x4*)d_hidden_bf16,
                           (uint32_t)(chunk_values / 8), d_out);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_selection_stats(const void* d_hidden_bf16, uint64_t n_chunks, const toploc_params* params, uint32_t* d_stats,
                           void* hip_stream)
{
    const uint64_t n = chunk_len(params);
    const int chk = plan::check_fixed(n, n_chunks, d_hidden_bf16, d_stats, 4, d_stats, 4, nullptr);
    if (chk != plan::kGo) return chk;
    hipStream_t st = (hipStream_t)hip_stream;
    if (params->k <= 128)
        hipLaunchKernelGGL((select_stats_kernel<kCapSmall>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                           (const u32x4*)d_hidden_bf16, (uint32_t)(n / 8), params->k, d_stats);
    else
        hipLaunchKernelGGL((select_stats_kernel<kCapLarge>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                           (const u32x4*)d_hidden_bf16, (uint32_t)(n / 8), params->k, d_stats);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_profile_enable(int on)
{
    if (on) {  // the only place events are created: up to kProfPairs launches can be timed between two reads
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        while (g_event_pool.size() + 2 * g_prof.size() < 2 * kProfPairs) {
            hipEvent_t e;
            if (!hip_ok(hipEventCreate(&e))) return TOPLOC_EHIP;
            g_event_pool.push_back(e);
        }
    }
    g_profile_on = on ? 1 : 0;
    return TOPLOC_OK;
}

int toploc_profile_read(uint32_t* launches, float* total_ms)
{
    if (!launches || !total_ms) return TOPLOC_EINVAL;
    for (int i = 0; i < TOPLOC_KERNEL_COUNT; ++i) { launches[i] = 0; total_ms[i] = 0.f; }
    int rc = TOPLOC_OK;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    for (auto& r : g_prof) {
        float ms = 0.f;
        if (hip_ok(hipEventSynchronize(r.b)) && hip_ok(hipEventElapsedTime(&ms, r.a, r.b))) {
            launches[r.slot] += 1;
            total_ms[r.slot] += ms;
        } else {
            rc = TOPLOC_EHIP;
        }
        g_event_pool.push_back(r.a);   // back to the pool: events live until the process ends
        g_event_pool.push_back(r.b);
    }
    g_prof.clear();
    return rc;
}

const char* toploc_strerror(int code)
{
    switch (code) {
    case TOPLOC_OK: return "ok";
    case TOPLOC_EINVAL: return "invalid argument (null or misaligned pointer, k = 0, k > chunk length, k > TOPLOC_MAX_K, "
                               "chunk length not a multiple of 8 or >= 2^32, prime != 65497, workspace missing where needed)";
    case TOPLOC_EWORKSPACE: return "workspace smaller than the workspace_bytes function reports";
    case TOPLOC_EHIP: return "a HIP runtime call failed (see toploc_last_hip_error)";
    case TOPLOC_ESCRATCH: return "the batch needs more scratch than the library's fixed array holds "
                                 "(TOPLOC_STATIC_SCRATCH_BYTES): use toploc_build_proofs with a workspace";
    default: return "unknown toploc error code";
    }
}

int toploc_last_hip_error(void) { return g_last_hip_error; }

#ifndef TOPLOC_BUILD_ID
#define TOPLOC_BUILD_ID "unstamped"
#endif
const char* toploc_build_id(void) { return TOPLOC_BUILD_ID; }

#ifdef TOPLOC_TIMING
// debug builds only: read (out != NULL) or clear the per-phase tick sums
int toploc_debug_ticks(unsigned long long* out)
{
    unsigned long long z[16] = {0};
    if (out) return hip_ok(hipMemcpyFromSymbol(out, HIP_SYMBOL(g_toploc_ticks), sizeof(z))) ? TOPLOC_OK : TOPLOC_EHIP;
    return hip_ok(hipMemcpyToSymbol(HIP_SYMBOL(g_toploc_ticks), z, sizeof(z))) ? TOPLOC_OK : TOPLOC_EHIP;
}
#endif

}  // extern "C"
