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
#include "select.hpp"
#include "verify.hpp"

#ifndef TOPLOC_LOADS
#define TOPLOC_LOADS 4
#endif
#ifndef TOPLOC_QCAP
#define TOPLOC_QCAP 512
#endif
#ifndef TOPLOC_MIN_WAVES
#define TOPLOC_MIN_WAVES 6  // waves per SIMD the streaming kernels must reach: 80 VGPRs, which 4 loads per lane just fit
#endif

namespace toploc {

constexpr int kThreads = 256;             // lanes per streaming workgroup
constexpr int kLoads = TOPLOC_LOADS;      // 16-byte loads in flight per lane and round
constexpr int kQcap = TOPLOC_QCAP;        // queue entries (16-byte vectors)
#ifndef TOPLOC_CAP_SMALL
#define TOPLOC_CAP_SMALL 1024
#endif
constexpr int kCapSmall = TOPLOC_CAP_SMALL;  // candidate buffer for k <= 128
constexpr int kCapLarge = 2048;           // candidate buffer for k <= TOPLOC_MAX_K
constexpr int kCapWide = 16384;           // candidate buffer of the selection alone up to TOPLOC_MAX_K_TOPK (140 KB of LDS:
                                          // one workgroup per compute unit; an aid for statistics, not a fast path)
constexpr uint32_t kRoundVecs = kThreads * kLoads;
// The larger candidate buffer (k > 128) costs registers in the prune and the ordering: one wave per SIMD less.
constexpr int waves_for(int cap) { return cap > kCapSmall ? TOPLOC_MIN_WAVES - 1 : TOPLOC_MIN_WAVES; }
static_assert(kCapLarge >= 4 * (int)TOPLOC_MAX_K && kCapSmall >= 4 * 128 && kCapWide >= 4 * (int)TOPLOC_MAX_K_TOPK,
              "soft limit CAP/2 must leave room above k");
static_assert(kCapWide <= 65536, "prune keeps slot numbers in 16 bits");

// Where a workgroup of a split launch finds its piece.  Fixed chunks need no table:
// chunk = block / parts, part = block % parts.  Segments come with two tables.
struct PartDesc {          // one per workgroup of part_kernel
    uint64_t seg_vec;      // first vector of the segment, from the tensor base
    uint32_t v0, v1;       // vectors [v0, v1) of the segment
};
struct SegDesc {           // one per workgroup of a merge kernel
    uint32_t first_part;   // candidate slots first_part .. first_part + n_parts - 1
    uint32_t n_parts;
};
struct Layout {
    const PartDesc* part_table;  // NULL: fixed chunks
    const SegDesc* seg_table;    // NULL: fixed chunks
    uint32_t nvec;               // fixed chunks: vectors per chunk
    uint32_t parts;              // fixed chunks: parts per chunk
    uint32_t part_vecs;          // fixed chunks: vectors per part
};

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
    select_topk<kThreads, kLoads, CAP, kQcap>(hidden + chunk * nvec, 0u, nvec, k, s);
    order_topk(s, k);
    for (uint32_t t = threadIdx.x; t < k; t += kThreads) {
        out_idx[chunk * k + t] = s.cand_idx[t];
        out_val[chunk * k + t] = s.cand_bits[t];
    }
}

// ---------------------------------------------------------------------------
// Algorithm 1 in one launch, k <= KMAX <= kThreads: the selection streams the chunk,
// then the same workgroup turns its k pairs into the proof out of LDS (the selection's
// buffers are dead by then and are reused).
// ---------------------------------------------------------------------------
template <int KMAX, int CAP, typename F = Field16, typename Fmt = Bf16Fmt, int U = kLoads, int WAVES = waves_for(CAP)>
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
    select_topk<kThreads, U>(hidden + chunk * nvec, 0u, nvec, k, sh.sel);
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
template <int KMAX, int CAP, typename F = Field16, typename Fmt = Bf16Fmt, int U = kLoads, int WAVES = waves_for(CAP)>
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
    (void)select_topk_from<kThreads, U>(hidden + chunk * nvec, 0u, nvec, s, first);  // order is irrelevant here
    if (!ok) return;  // uniform
    TOPLOC_TICK_BEGIN(tail);
    verify_tail<kThreads, F, Fmt>(vs, s.cand_idx, s.cand_bits, k, thr, results + chunk);
    TOPLOC_TICK_END(tail, 4);
}

// ---------------------------------------------------------------------------
// Split path, first launch: top-k of one part.  Writes k candidate slots per part,
// the unused ones (part shorter than k values) padded with index 0xFFFFFFFF.
// ---------------------------------------------------------------------------
template <int CAP, typename Fmt = Bf16Fmt>
__global__ __launch_bounds__(kThreads, waves_for(CAP)) void part_kernel(const u32x4* __restrict__ hidden, Layout lay,
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
    if (k_eff) select_topk<kThreads, kLoads>(src, v0, v1, k_eff, s);
    for (uint32_t t = tid; t < k; t += kThreads) {
        c_idx[slot * k + t] = t < k_eff ? s.cand_idx[t] : 0xFFFFFFFFu;
        c_bits[slot * k + t] = t < k_eff ? s.cand_bits[t] : (typename Fmt::bits_t)0;
    }
}

// candidate slots of the chunk / segment a merge workgroup owns
__device__ __forceinline__ void merge_range(const Layout& lay, uint64_t unit, uint64_t& first, uint32_t& n_parts)
{
    if (lay.seg_table) {
        const SegDesc d = lay.seg_table[unit];
        first = d.first_part;
        n_parts = d.n_parts;
    } else {
        first = unit * lay.parts;
        n_parts = lay.parts;
    }
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
    merge_range(lay, unit, first, n_parts);
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
    if (!verify_decode<THREADS, F>(vs, proof, k, results + unit)) return;
    uint64_t first;
    uint32_t n_parts;
    merge_range(lay, unit, first, n_parts);
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

__host__ __device__ __forceinline__ size_t stream_idx_bytes(uint32_t k) { return ((size_t)k * 4 + 15) & ~(size_t)15; }
__host__ __device__ __forceinline__ size_t stream_stride(uint32_t k)
{
    return sizeof(StreamHeader) + stream_idx_bytes(k) + (((size_t)k * 2 + 15) & ~(size_t)15);
}

__global__ __launch_bounds__(256) void stream_reset_kernel(char* __restrict__ state, uint32_t n_seq, size_t stride)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_seq) *reinterpret_cast<StreamHeader*>(state + (size_t)i * stride) = StreamHeader{0u, 0, 0xFFFFFFFFu, 0u};
}

// What a sequence holds enters the selection of its next row: all k slots are read
// before the header says how many of them count, so that header, pairs and the row's
// first vectors are in flight together.
template <int CAP>
struct StreamSeed {
    const StreamHeader* hdr;
    const uint32_t* g_idx;
    const uint16_t* g_bits;
    uint32_t k, row_values;
    __device__ __forceinline__ SelectStart seed(SelectShared<kThreads, CAP, kQcap>& s) const
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
            if (i < h.count) { s.cand_idx[i] = si[j]; s.cand_bits[i] = (uint16_t)sb[j]; }
        }
        const uint64_t have = (uint64_t)h.count + row_values;
        return SelectStart{h.count, Threshold{h.tm, h.ti}, have < k ? (uint32_t)have : k};
    }
};

// One appended row per sequence: the selection of select.hpp over the row's vectors,
// seeded with the pairs and the threshold the sequence holds.  `row_base` is the
// sequence's row pointer moved back by v0 vectors, so that vector v0 + j of the
// selection is vector j of the row and flat indices come out as token*hidden + channel.
// With `slots` (continuous batching: the rows of a step belong to any subset of the
// sequences, each at its own position) row r goes to sequence slots[r] as token tokens[r];
// a row whose slot or token is out of range is skipped.
template <int CAP>
__global__ __launch_bounds__(kThreads, waves_for(CAP)) void stream_append_kernel(char* __restrict__ state, size_t stride,
                                                                                   const u32x4* __restrict__ step_vec,
                                                                                   uint32_t hvec, uint32_t v0, uint32_t k,
                                                                                   const uint32_t* __restrict__ slots,
                                                                                   const uint32_t* __restrict__ tokens,
                                                                                   uint32_t n_slots, uint32_t chunk_tokens)
{
    __shared__ SelectShared<kThreads, CAP, kQcap> s;
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
    uint16_t* g_bits = reinterpret_cast<uint16_t*>(st + sizeof(StreamHeader) + stream_idx_bytes(k));
    const u32x4* row_base = reinterpret_cast<const u32x4*>(
        reinterpret_cast<uintptr_t>(step_vec + (size_t)blockIdx.x * hvec) - (uintptr_t)v0 * sizeof(u32x4));
    const uint32_t rows = hdr->rows;
    const SelectStart end = select_topk_from<kThreads, kLoads, CAP, kQcap>(
        row_base, v0, v0 + hvec, s, StreamSeed<CAP>{hdr, g_idx, g_bits, k, hvec * 8u});
    for (uint32_t i = tid; i < end.k; i += kThreads) {
        g_idx[i] = s.cand_idx[i];
        g_bits[i] = s.cand_bits[i];
    }
    if (tid == 0) *hdr = StreamHeader{end.k, end.t.tm, end.t.ti, rows + 1u};
}

// Emission: steps 2-5 of Algorithm 1 on the k pairs a sequence holds, then the state is emptied.
template <int THREADS, int KMAX, int CAP>
__global__ __launch_bounds__(THREADS) void stream_emit_kernel(char* __restrict__ state, size_t stride, uint32_t k,
                                                              uint8_t* __restrict__ proofs, uint8_t* __restrict__ status,
                                                              uint32_t* __restrict__ out_idx,
                                                              const uint32_t* __restrict__ slots, uint32_t n_slots)
{
    static_assert(KMAX <= THREADS, "one pair per lane is carried across the phase change");
    __shared__ union EmitShared {
        SelectShared<THREADS, CAP, 1> sel;
        InterpShared<KMAX> itp;
    } sh;
    __shared__ uint32_t coef[KMAX];
    const uint32_t tid = threadIdx.x;
    const uint64_t seq = blockIdx.x;  // output row; with `slots` the state of sequence slots[seq]
    const uint64_t owner = slots ? slots[seq] : seq;
    const bool known = owner < n_slots;  // uniform
    char* st = state + (known ? owner : 0) * stride;
    StreamHeader* hdr = reinterpret_cast<StreamHeader*>(st);
    const uint32_t* g_idx = reinterpret_cast<const uint32_t*>(st + sizeof(StreamHeader));
    const uint16_t* g_bits = reinterpret_cast<const uint16_t*>(st + sizeof(StreamHeader) + stream_idx_bytes(k));
    const uint32_t count = known ? hdr->count : 0u;
    uint16_t* proof = reinterpret_cast<uint16_t*>(proofs + seq * (2 + 2 * (uint64_t)k));
    __syncthreads();  // every lane has read the header
    if (tid == 0 && known) *hdr = StreamHeader{0u, 0, 0xFFFFFFFFu, 0u};
    if (count < k) {  // uniform
        for (uint32_t j = tid; j <= k; j += THREADS) proof[j] = 0;
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
        sh.itp.ys[tid] = (uint16_t)(my_y >= kPrime ? my_y - kPrime : my_y);
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

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static size_t up16(size_t b) { return (b + 15) & ~(size_t)15; }

// N (values per chunk) when the parameters are usable, else 0
static uint64_t chunk_len(const toploc_params* p, uint32_t max_k = TOPLOC_MAX_K)
{
    if (!p || p->k == 0 || p->k > max_k || p->prime != TOPLOC_PRIME) return 0;
    if (p->chunk_tokens == 0 || p->hidden == 0) return 0;
    const uint64_t n = (uint64_t)p->chunk_tokens * p->hidden;
    if (n % 8 != 0 || n >= (1ull << 32) || p->k > n) return 0;
    return n;
}

// How a launch is cut.  One workgroup keeps about 16 KB of loads in flight, so roughly a
// thousand streaming workgroups are needed to saturate HBM: a batch with fewer chunks is
// cut into parts until there are that many, but a part still streams a few rounds (every
// part pays for finding its own threshold), and no part is longer than kMaxPartVecs so
// that one long segment cannot become the launch's straggler.
constexpr uint64_t kTargetGroups = 1024;
constexpr uint64_t kMinPartVecs = 4 * kRoundVecs;
constexpr uint64_t kMaxPartVecs = 64 * kRoundVecs;

static uint64_t clamp_part_vecs(uint64_t pv)
{
    pv = (pv + kRoundVecs - 1) / kRoundVecs * kRoundVecs;
    return pv < kMinPartVecs ? kMinPartVecs : pv > kMaxPartVecs ? kMaxPartVecs : pv;
}

struct FixedPlan { uint32_t parts; uint32_t part_vecs; };
static FixedPlan plan_fixed(uint64_t n_chunks, uint64_t nvec)
{
    uint64_t pv;
    const uint64_t forced = g_force_parts.load();  // read once: another thread may change it
    if (forced) {
        pv = (nvec + forced - 1) / forced;
        pv = pv ? pv : 1;
    } else {
        const uint64_t want = n_chunks < kTargetGroups ? kTargetGroups / n_chunks : 1;  // parts per chunk
        pv = clamp_part_vecs((nvec + want - 1) / want);
    }
    FixedPlan f;
    f.parts = (uint32_t)((nvec + pv - 1) / pv);
    f.part_vecs = (uint32_t)(pv < nvec ? pv : nvec);
    return f;
}

// vectors per part for segments: `total_vecs` vectors in `n_units` segments, the longest of `max_unit_vecs`
static uint64_t pick_part_vecs(uint64_t total_vecs, uint64_t max_unit_vecs, uint64_t n_units)
{
    const uint64_t forced = g_force_parts.load();  // read once: another thread may change it
    if (forced) {
        const uint64_t pv = (max_unit_vecs + forced - 1) / forced;
        return pv ? pv : 1;
    }
    const uint64_t groups = n_units > kTargetGroups ? n_units : kTargetGroups;
    return clamp_part_vecs((total_vecs + groups - 1) / groups);
}

// candidate arrays for `slots` parts: [slots*k] uint32 indices, then [slots*k] patterns of
// `bits_size` bytes (2: bf16, 4: fp32), each array 16-byte aligned
static size_t cand_bytes(uint64_t slots, uint32_t k, size_t bits_size = sizeof(uint16_t))
{
    return up16((size_t)slots * k * sizeof(uint32_t)) + up16((size_t)slots * k * bits_size);
}
static size_t bits_size_of(uint32_t dtype) { return dtype == TOPLOC_DTYPE_F32 ? sizeof(uint32_t) : sizeof(uint16_t); }

static void launch_part(hipStream_t st, const void* d_hidden, const Layout& lay, uint64_t slots, uint32_t k, uint32_t* c_idx,
                        void* c_bits_any, uint32_t hidden_dtype = TOPLOC_DTYPE_BF16)
{
    ProfScope ps(TOPLOC_KERNEL_PART, st);
    if (hidden_dtype == TOPLOC_DTYPE_F32) {  // k <= TOPLOC_MAX_K_F32
        hipLaunchKernelGGL((part_kernel<kCapSmall, F32Fmt>), dim3((uint32_t)slots), dim3(kThreads), 0, st,
                           (const u32x4*)d_hidden, lay, k, c_idx, (uint32_t*)c_bits_any);
        return;
    }
    uint16_t* c_bits = (uint16_t*)c_bits_any;
    if (k <= 128)
        hipLaunchKernelGGL((part_kernel<kCapSmall>), dim3((uint32_t)slots), dim3(kThreads), 0, st, (const u32x4*)d_hidden, lay,
                           k, c_idx, c_bits);
    else
        hipLaunchKernelGGL((part_kernel<kCapLarge>), dim3((uint32_t)slots), dim3(kThreads), 0, st, (const u32x4*)d_hidden, lay,
                           k, c_idx, c_bits);
}

static void launch_build_merge(hipStream_t st, const Layout& lay, uint64_t units, uint32_t k, const uint32_t* c_idx,
                               const void* c_bits_any, uint8_t* d_proofs, uint8_t* d_status, uint32_t* d_topk_idx_opt,
                               uint32_t dtype = TOPLOC_DTYPE_BF16)
{
    ProfScope ps(TOPLOC_KERNEL_BUILD_MERGE, st);
    if (dtype == TOPLOC_DTYPE_F32) {  // k <= TOPLOC_MAX_K_F32
        hipLaunchKernelGGL((build_merge_kernel<256, 128, kCapSmall, Field32, F32Fmt>), dim3((uint32_t)units), dim3(256), 0, st,
                           lay, k, c_idx, (const uint32_t*)c_bits_any, d_proofs, d_status, d_topk_idx_opt);
        return;
    }
    const uint16_t* c_bits = (const uint16_t*)c_bits_any;
    if (k <= 128)
        hipLaunchKernelGGL((build_merge_kernel<256, 128, kCapSmall>), dim3((uint32_t)units), dim3(256), 0, st, lay, k, c_idx,
                           c_bits, d_proofs, d_status, d_topk_idx_opt);
    else
        hipLaunchKernelGGL((build_merge_kernel<1024, 512, kCapLarge>), dim3((uint32_t)units), dim3(1024), 0, st, lay, k, c_idx,
                           c_bits, d_proofs, d_status, d_topk_idx_opt);
}

static void launch_verify_merge(hipStream_t st, const Layout& lay, uint64_t units, uint32_t k, const uint32_t* c_idx,
                                const void* c_bits_any, const uint8_t* d_proofs, const toploc_thresholds& thr,
                                toploc_verify_result* d_results, uint32_t hidden_dtype = TOPLOC_DTYPE_BF16,
                                uint32_t proof_dtype = TOPLOC_DTYPE_BF16)
{
    ProfScope ps(TOPLOC_KERNEL_VERIFY_MERGE, st);
    const dim3 grid((uint32_t)units), block(256);
    if (hidden_dtype == TOPLOC_DTYPE_F32 && proof_dtype == TOPLOC_DTYPE_F32) {
        hipLaunchKernelGGL((verify_merge_kernel<256, 128, kCapSmall, Field32, F32Fmt>), grid, block, 0, st, lay, k, c_idx,
                           (const uint32_t*)c_bits_any, d_proofs, thr, d_results);
        return;
    }
    if (hidden_dtype == TOPLOC_DTYPE_F32) {  // bf16 proof, fp32 validator
        hipLaunchKernelGGL((verify_merge_kernel<256, 128, kCapSmall, Field16, F32Fmt>), grid, block, 0, st, lay, k, c_idx,
                           (const uint32_t*)c_bits_any, d_proofs, thr, d_results);
        return;
    }
    const uint16_t* c_bits = (const uint16_t*)c_bits_any;
    if (proof_dtype == TOPLOC_DTYPE_F32) {   // fp32 proof, bf16 validator
        hipLaunchKernelGGL((verify_merge_kernel<256, 128, kCapSmall, Field32, Bf16Fmt>), grid, block, 0, st, lay, k, c_idx,
                           c_bits, d_proofs, thr, d_results);
        return;
    }
    if (k <= 128)
        hipLaunchKernelGGL((verify_merge_kernel<256, 128, kCapSmall>), dim3((uint32_t)units), dim3(256), 0, st, lay, k, c_idx,
                           c_bits, d_proofs, thr, d_results);
    else
        hipLaunchKernelGGL((verify_merge_kernel<512, 512, kCapLarge>), dim3((uint32_t)units), dim3(512), 0, st, lay, k, c_idx,
                           c_bits, d_proofs, thr, d_results);
}

// Segments: tables of parts and of segments, laid out behind the candidate arrays.
struct SegPlan {
    std::vector<PartDesc> parts;
    std::vector<SegDesc> segs;
    bool ok = false;
};
static SegPlan plan_segments(const uint64_t* h_row_offsets, uint64_t n_segments, uint32_t hidden, uint32_t k,
                             uint32_t hidden_dtype = TOPLOC_DTYPE_BF16, uint32_t k_max = TOPLOC_MAX_K)
{
    SegPlan pl;
    if (!h_row_offsets || hidden == 0 || hidden % 8 != 0 || k == 0 || k > k_max || n_segments >= (1ull << 31)) return pl;
    const uint64_t hv = hidden / (hidden_dtype == TOPLOC_DTYPE_F32 ? 4 : 8);  // 16-byte vectors per row
    uint64_t max_vecs = 0;
    for (uint64_t i = 0; i < n_segments; ++i) {
        if (h_row_offsets[i + 1] < h_row_offsets[i]) return pl;
        const uint64_t rows = h_row_offsets[i + 1] - h_row_offsets[i];
        if (rows * hidden < k || rows * hidden >= (1ull << 32)) return pl;
        if (rows * hv > max_vecs) max_vecs = rows * hv;
    }
    const uint64_t total_vecs = n_segments ? (h_row_offsets[n_segments] - h_row_offsets[0]) * hv : 0;
    const uint64_t pv = pick_part_vecs(total_vecs, max_vecs, n_segments);
    pl.segs.reserve(n_segments);
    for (uint64_t i = 0; i < n_segments; ++i) {
        const uint64_t nvec = (h_row_offsets[i + 1] - h_row_offsets[i]) * hv;
        SegDesc sd;
        sd.first_part = (uint32_t)pl.parts.size();
        sd.n_parts = (uint32_t)((nvec + pv - 1) / pv);
        for (uint64_t v0 = 0; v0 < nvec; v0 += pv) {
            PartDesc pd;
            pd.seg_vec = h_row_offsets[i] * hv;
            pd.v0 = (uint32_t)v0;
            pd.v1 = (uint32_t)(v0 + pv < nvec ? v0 + pv : nvec);
            pl.parts.push_back(pd);
        }
        pl.segs.push_back(sd);
        if (pl.parts.size() >= (1ull << 31)) return pl;
    }
    pl.ok = true;
    return pl;
}

static size_t seg_workspace_bytes(const SegPlan& pl, uint32_t k, size_t bits_size = sizeof(uint16_t))
{
    return cand_bytes(pl.parts.size(), k, bits_size) + up16(pl.parts.size() * sizeof(PartDesc)) +
           up16(pl.segs.size() * sizeof(SegDesc));
}

// copies the tables behind the candidate arrays and fills the layout
template <typename Bits>
static bool stage_segments(const SegPlan& pl, uint32_t k, void* d_workspace, hipStream_t st, Layout& lay, uint32_t*& c_idx,
                           Bits*& c_bits)
{
    char* w = (char*)d_workspace;
    c_idx = (uint32_t*)w;
    c_bits = (Bits*)(w + up16(pl.parts.size() * (size_t)k * sizeof(uint32_t)));
    char* t_parts = w + cand_bytes(pl.parts.size(), k, sizeof(Bits));
    char* t_segs = t_parts + up16(pl.parts.size() * sizeof(PartDesc));
    if (!hip_ok(hipMemcpyAsync(t_parts, pl.parts.data(), pl.parts.size() * sizeof(PartDesc), hipMemcpyHostToDevice, st)))
        return false;
    if (!hip_ok(hipMemcpyAsync(t_segs, pl.segs.data(), pl.segs.size() * sizeof(SegDesc), hipMemcpyHostToDevice, st)))
        return false;
    lay.part_table = (const PartDesc*)t_parts;
    lay.seg_table = (const SegDesc*)t_segs;
    lay.nvec = 0; lay.parts = 0; lay.part_vecs = 0;
    return true;
}

}  // namespace toploc

using namespace toploc;

extern "C" {

size_t toploc_proof_bytes(uint32_t k) { return 2 + 2 * (size_t)k; }

size_t toploc_workspace_bytes(const toploc_params* params, uint64_t n_chunks)
{
    const uint64_t n = chunk_len(params);
    if (n == 0 || n_chunks == 0) return 0;
    const FixedPlan f = plan_fixed(n_chunks, n / 8);
    if (f.parts == 1 && params->k <= 128) return 0;  // one fused kernel, everything stays on chip
    return cand_bytes(n_chunks * f.parts, params->k);
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
    if (n == 0 || n_chunks >= (1ull << 31)) return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    if (!d_hidden_bf16 || !d_topk_idx || !d_topk_val || !aligned16(d_hidden_bf16)) return TOPLOC_EINVAL;
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
static int build_fixed(const FixedPlan& f, const void* d_hidden_bf16, uint64_t n_chunks, uint32_t nvec, uint32_t k,
                       uint8_t* d_proofs, uint8_t* d_status, uint32_t* d_topk_idx_opt, void* d_workspace,
                       size_t workspace_bytes, hipStream_t st)
{
    const bool have_ws = d_workspace && workspace_bytes >= cand_bytes(n_chunks * f.parts, k);
    if (k <= 128 && (f.parts == 1 || !have_ws)) {  // one launch; also the answer to a missing workspace
        ProfScope ps(TOPLOC_KERNEL_BUILD, st);
        hipLaunchKernelGGL((build_kernel<128, kCapSmall>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                           (const u32x4*)d_hidden_bf16, nvec, k, d_proofs, d_status, d_topk_idx_opt);
        return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
    }
    if (!have_ws) return d_workspace ? TOPLOC_EWORKSPACE : TOPLOC_EINVAL;
    const uint64_t slots = n_chunks * f.parts;
    if (slots >= (1ull << 31)) return TOPLOC_EINVAL;
    Layout lay = {nullptr, nullptr, nvec, f.parts, f.part_vecs};
    uint32_t* c_idx = (uint32_t*)d_workspace;
    uint16_t* c_bits = (uint16_t*)((char*)d_workspace + up16((size_t)slots * k * sizeof(uint32_t)));
    launch_part(st, d_hidden_bf16, lay, slots, k, c_idx, c_bits);
    if (!hip_ok(hipGetLastError())) return TOPLOC_EHIP;
    launch_build_merge(st, lay, n_chunks, k, c_idx, c_bits, d_proofs, d_status, d_topk_idx_opt);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_build_proofs(const void* d_hidden_bf16, uint64_t n_chunks, const toploc_params* params, uint8_t* d_proofs,
                        uint8_t* d_status, uint32_t* d_topk_idx_opt, void* d_workspace, size_t workspace_bytes,
                        void* hip_stream)
{
    const uint64_t n = chunk_len(params);
    if (n == 0 || n_chunks >= (1ull << 31)) return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    if (!d_hidden_bf16 || !d_proofs || !d_status || !aligned16(d_hidden_bf16)) return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0) return TOPLOC_EINVAL;
    if (d_workspace && !aligned16(d_workspace)) return TOPLOC_EINVAL;
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
    if (n == 0 || n_chunks >= (1ull << 31)) return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    if (!d_hidden_bf16 || !d_proofs || !d_status || !aligned16(d_hidden_bf16)) return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0) return TOPLOC_EINVAL;
    const uint32_t nvec = (uint32_t)(n / 8);
    const FixedPlan f = plan_fixed(n_chunks, nvec);
    const bool fused = f.parts == 1 && params->k <= 128;   // no scratch at all
    if (!fused && cand_bytes(n_chunks * f.parts, params->k) > kScratchBytes) return TOPLOC_ESCRATCH;
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
    if (n == 0 || n_chunks >= (1ull << 31) || !thresholds) return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    if (!d_hidden_bf16 || !d_proofs || !d_results || !aligned16(d_hidden_bf16)) return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0 || (reinterpret_cast<uintptr_t>(d_results) & 3u) != 0)
        return TOPLOC_EINVAL;
    if (d_workspace && !aligned16(d_workspace)) return TOPLOC_EINVAL;
    const uint32_t k = params->k;
    const uint32_t nvec = (uint32_t)(n / 8);
    hipStream_t st = (hipStream_t)hip_stream;
    FixedPlan f = plan_fixed(n_chunks, nvec);
    const uint64_t slots = n_chunks * f.parts;
    const bool split = f.parts > 1 && d_workspace && workspace_bytes >= cand_bytes(slots, k) && slots < (1ull << 31);
    if (!split) {  // one launch; a missing workspace only costs speed on small batches
        ProfScope ps(TOPLOC_KERNEL_VERIFY, st);
        if (k <= 128)
            hipLaunchKernelGGL((verify_kernel<128, kCapSmall>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden_bf16, nvec, k, d_proofs, *thresholds, d_results);
        else
            hipLaunchKernelGGL((verify_kernel<512, kCapLarge>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden_bf16, nvec, k, d_proofs, *thresholds, d_results);
        return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
    }
    Layout lay = {nullptr, nullptr, nvec, f.parts, f.part_vecs};
    uint32_t* c_idx = (uint32_t*)d_workspace;
    uint16_t* c_bits = (uint16_t*)((char*)d_workspace + up16((size_t)slots * k * sizeof(uint32_t)));
    launch_part(st, d_hidden_bf16, lay, slots, k, c_idx, c_bits);
    if (!hip_ok(hipGetLastError())) return TOPLOC_EHIP;
    launch_verify_merge(st, lay, n_chunks, k, c_idx, c_bits, d_proofs, *thresholds, d_results);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

size_t toploc_segments_workspace_bytes(const uint64_t* h_row_offsets, uint64_t n_segments, uint32_t hidden, uint32_t k)
{
    const SegPlan pl = plan_segments(h_row_offsets, n_segments, hidden, k);
    if (!pl.ok || n_segments == 0) return 0;
    return seg_workspace_bytes(pl, k);
}

int toploc_build_proofs_segments(const void* d_hidden_bf16, const uint64_t* h_row_offsets, uint64_t n_segments,
                                 uint32_t hidden, uint32_t k, uint8_t* d_proofs, uint8_t* d_status,
                                 uint32_t* d_topk_idx_opt, void* d_workspace, size_t workspace_bytes, void* hip_stream)
{
    const SegPlan pl = plan_segments(h_row_offsets, n_segments, hidden, k);
    if (!pl.ok) return TOPLOC_EINVAL;
    if (n_segments == 0) return TOPLOC_OK;
    if (!d_hidden_bf16 || !d_proofs || !d_status || !d_workspace || !aligned16(d_hidden_bf16) || !aligned16(d_workspace))
        return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0) return TOPLOC_EINVAL;
    if (workspace_bytes < seg_workspace_bytes(pl, k)) return TOPLOC_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    Layout lay;
    uint32_t* c_idx;
    uint16_t* c_bits;
    if (!stage_segments(pl, k, d_workspace, st, lay, c_idx, c_bits)) return TOPLOC_EHIP;
    launch_part(st, d_hidden_bf16, lay, pl.parts.size(), k, c_idx, c_bits);
    if (!hip_ok(hipGetLastError())) return TOPLOC_EHIP;
    launch_build_merge(st, lay, n_segments, k, c_idx, c_bits, d_proofs, d_status, d_topk_idx_opt);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_verify_proofs_segments(const void* d_hidden_bf16, const uint64_t* h_row_offsets, uint64_t n_segments,
                                  uint32_t hidden, uint32_t k, const uint8_t* d_proofs,
                                  const toploc_thresholds* thresholds, toploc_verify_result* d_results, void* d_workspace,
                                  size_t workspace_bytes, void* hip_stream)
{
    const SegPlan pl = plan_segments(h_row_offsets, n_segments, hidden, k);
    if (!pl.ok || !thresholds) return TOPLOC_EINVAL;
    if (n_segments == 0) return TOPLOC_OK;
    if (!d_hidden_bf16 || !d_proofs || !d_results || !d_workspace || !aligned16(d_hidden_bf16) || !aligned16(d_workspace))
        return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0 || (reinterpret_cast<uintptr_t>(d_results) & 3u) != 0)
        return TOPLOC_EINVAL;
    if (workspace_bytes < seg_workspace_bytes(pl, k)) return TOPLOC_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    Layout lay;
    uint32_t* c_idx;
    uint16_t* c_bits;
    if (!stage_segments(pl, k, d_workspace, st, lay, c_idx, c_bits)) return TOPLOC_EHIP;
    launch_part(st, d_hidden_bf16, lay, pl.parts.size(), k, c_idx, c_bits);
    if (!hip_ok(hipGetLastError())) return TOPLOC_EHIP;
    launch_verify_merge(st, lay, n_segments, k, c_idx, c_bits, d_proofs, *thresholds, d_results);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

// N (values per chunk) for the calls that involve fp32: k <= TOPLOC_MAX_K_F32, the chunk a
// whole number of 16-byte vectors in both formats
static uint64_t chunk_len_mixed(const toploc_params* p, uint32_t hidden_dtype, uint32_t proof_dtype)
{
    if (!p || hidden_dtype > TOPLOC_DTYPE_F32 || proof_dtype > TOPLOC_DTYPE_F32) return 0;
    if (p->prime != (proof_dtype == TOPLOC_DTYPE_F32 ? TOPLOC_PRIME32 : TOPLOC_PRIME)) return 0;
    const uint32_t kmax = (hidden_dtype == TOPLOC_DTYPE_F32 || proof_dtype == TOPLOC_DTYPE_F32) ? TOPLOC_MAX_K_F32 : TOPLOC_MAX_K;
    if (p->k == 0 || p->k > kmax || p->chunk_tokens == 0 || p->hidden == 0) return 0;
    const uint64_t n = (uint64_t)p->chunk_tokens * p->hidden;
    if (n % 8 != 0 || n >= (1ull << 32) || p->k > n) return 0;
    return n;
}

size_t toploc_proof_bytes_dtype(uint32_t k, uint32_t dtype)
{
    return 2 + (size_t)k * (dtype == TOPLOC_DTYPE_F32 ? 4 : 2);
}

int toploc_build_proofs_f32(const void* d_hidden_f32, uint64_t n_chunks, const toploc_params* params, uint8_t* d_proofs,
                            uint8_t* d_status, uint32_t* d_topk_idx_opt, void* hip_stream)
{
    const uint64_t n = chunk_len_mixed(params, TOPLOC_DTYPE_F32, TOPLOC_DTYPE_F32);
    if (n == 0 || n_chunks >= (1ull << 31)) return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    if (!d_hidden_f32 || !d_proofs || !d_status || !aligned16(d_hidden_f32)) return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0) return TOPLOC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    {
        ProfScope ps(TOPLOC_KERNEL_BUILD, st);
        hipLaunchKernelGGL((build_kernel<128, kCapSmall, Field32, F32Fmt>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                           (const u32x4*)d_hidden_f32, (uint32_t)(n / 4), params->k, d_proofs, d_status, d_topk_idx_opt);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_verify_proofs_mixed(const void* d_hidden, uint32_t hidden_dtype, uint64_t n_chunks, const toploc_params* params,
                               const uint8_t* d_proofs, uint32_t proof_dtype, const toploc_thresholds* thresholds,
                               toploc_verify_result* d_results, void* hip_stream)
{
    const uint64_t n = chunk_len_mixed(params, hidden_dtype, proof_dtype);
    if (n == 0 || n_chunks >= (1ull << 31) || !thresholds) return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    if (!d_hidden || !d_proofs || !d_results || !aligned16(d_hidden)) return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0 || (reinterpret_cast<uintptr_t>(d_results) & 3u) != 0)
        return TOPLOC_EINVAL;
    if (hidden_dtype == TOPLOC_DTYPE_BF16 && proof_dtype == TOPLOC_DTYPE_BF16)
        return toploc_verify_proofs(d_hidden, n_chunks, params, d_proofs, thresholds, d_results, nullptr, 0, hip_stream);
    hipStream_t st = (hipStream_t)hip_stream;
    const uint32_t k = params->k;
    const dim3 grid((uint32_t)n_chunks), block(kThreads);
    const u32x4* h = (const u32x4*)d_hidden;
    {
        ProfScope ps(TOPLOC_KERNEL_VERIFY, st);
        if (hidden_dtype == TOPLOC_DTYPE_F32 && proof_dtype == TOPLOC_DTYPE_F32)
            hipLaunchKernelGGL((verify_kernel<128, kCapSmall, Field32, F32Fmt>), grid, block, 0, st, h, (uint32_t)(n / 4), k,
                               d_proofs, *thresholds, d_results);
        else if (hidden_dtype == TOPLOC_DTYPE_F32)   // bf16 proof, fp32 validator
            hipLaunchKernelGGL((verify_kernel<128, kCapSmall, Field16, F32Fmt>), grid, block, 0, st, h, (uint32_t)(n / 4), k,
                               d_proofs, *thresholds, d_results);
        else                                          // fp32 proof, bf16 validator
            hipLaunchKernelGGL((verify_kernel<128, kCapSmall, Field32, Bf16Fmt>), grid, block, 0, st, h, (uint32_t)(n / 8), k,
                               d_proofs, *thresholds, d_results);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

// k limit and table plan of the segment calls that involve fp32
static SegPlan plan_segments_mixed(const uint64_t* h_row_offsets, uint64_t n_segments, uint32_t hidden, uint32_t k,
                                   uint32_t hidden_dtype, uint32_t proof_dtype)
{
    if (hidden_dtype > TOPLOC_DTYPE_F32 || proof_dtype > TOPLOC_DTYPE_F32) return SegPlan();
    const bool any32 = hidden_dtype == TOPLOC_DTYPE_F32 || proof_dtype == TOPLOC_DTYPE_F32;
    return plan_segments(h_row_offsets, n_segments, hidden, k, hidden_dtype, any32 ? TOPLOC_MAX_K_F32 : TOPLOC_MAX_K);
}

size_t toploc_segments_workspace_bytes_dtype(const uint64_t* h_row_offsets, uint64_t n_segments, uint32_t hidden,
                                             uint32_t k, uint32_t hidden_dtype)
{
    const SegPlan pl = plan_segments_mixed(h_row_offsets, n_segments, hidden, k, hidden_dtype, hidden_dtype);
    if (!pl.ok || n_segments == 0) return 0;
    return seg_workspace_bytes(pl, k, bits_size_of(hidden_dtype));
}

int toploc_build_proofs_segments_f32(const void* d_hidden_f32, const uint64_t* h_row_offsets, uint64_t n_segments,
                                     uint32_t hidden, uint32_t k, uint8_t* d_proofs, uint8_t* d_status,
                                     uint32_t* d_topk_idx_opt, void* d_workspace, size_t workspace_bytes,
                                     void* hip_stream)
{
    const SegPlan pl = plan_segments_mixed(h_row_offsets, n_segments, hidden, k, TOPLOC_DTYPE_F32, TOPLOC_DTYPE_F32);
    if (!pl.ok) return TOPLOC_EINVAL;
    if (n_segments == 0) return TOPLOC_OK;
    if (!d_hidden_f32 || !d_proofs || !d_status || !d_workspace || !aligned16(d_hidden_f32) || !aligned16(d_workspace))
        return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0) return TOPLOC_EINVAL;
    if (workspace_bytes < seg_workspace_bytes(pl, k, sizeof(uint32_t))) return TOPLOC_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    Layout lay;
    uint32_t* c_idx;
    uint32_t* c_bits;
    if (!stage_segments(pl, k, d_workspace, st, lay, c_idx, c_bits)) return TOPLOC_EHIP;
    launch_part(st, d_hidden_f32, lay, pl.parts.size(), k, c_idx, c_bits, TOPLOC_DTYPE_F32);
    if (!hip_ok(hipGetLastError())) return TOPLOC_EHIP;
    launch_build_merge(st, lay, n_segments, k, c_idx, c_bits, d_proofs, d_status, d_topk_idx_opt, TOPLOC_DTYPE_F32);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_verify_proofs_segments_mixed(const void* d_hidden, uint32_t hidden_dtype, const uint64_t* h_row_offsets,
                                        uint64_t n_segments, uint32_t hidden, uint32_t k, const uint8_t* d_proofs,
                                        uint32_t proof_dtype, const toploc_thresholds* thresholds,
                                        toploc_verify_result* d_results, void* d_workspace, size_t workspace_bytes,
                                        void* hip_stream)
{
    const SegPlan pl = plan_segments_mixed(h_row_offsets, n_segments, hidden, k, hidden_dtype, proof_dtype);
    if (!pl.ok || !thresholds) return TOPLOC_EINVAL;
    if (n_segments == 0) return TOPLOC_OK;
    if (!d_hidden || !d_proofs || !d_results || !d_workspace || !aligned16(d_hidden) || !aligned16(d_workspace))
        return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0 || (reinterpret_cast<uintptr_t>(d_results) & 3u) != 0)
        return TOPLOC_EINVAL;
    if (workspace_bytes < seg_workspace_bytes(pl, k, bits_size_of(hidden_dtype))) return TOPLOC_EWORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    Layout lay;
    uint32_t* c_idx;
    void* c_bits;
    if (hidden_dtype == TOPLOC_DTYPE_F32) {
        uint32_t* b32;
        if (!stage_segments(pl, k, d_workspace, st, lay, c_idx, b32)) return TOPLOC_EHIP;
        c_bits = b32;
    } else {
        uint16_t* b16;
        if (!stage_segments(pl, k, d_workspace, st, lay, c_idx, b16)) return TOPLOC_EHIP;
        c_bits = b16;
    }
    launch_part(st, d_hidden, lay, pl.parts.size(), k, c_idx, c_bits, hidden_dtype);
    if (!hip_ok(hipGetLastError())) return TOPLOC_EHIP;
    launch_verify_merge(st, lay, n_segments, k, c_idx, c_bits, d_proofs, *thresholds, d_results, hidden_dtype, proof_dtype);
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

size_t toploc_stream_state_bytes(uint32_t n_seq, uint32_t k)
{
    if (k == 0 || k > TOPLOC_MAX_K) return 0;
    return (size_t)n_seq * stream_stride(k);
}

int toploc_stream_reset(void* d_state, uint32_t n_seq, uint32_t k, void* hip_stream)
{
    if (k == 0 || k > TOPLOC_MAX_K) return TOPLOC_EINVAL;
    if (n_seq == 0) return TOPLOC_OK;
    if (!d_state || !aligned16(d_state)) return TOPLOC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    hipLaunchKernelGGL(stream_reset_kernel, dim3((n_seq + 255) / 256), dim3(256), 0, st, (char*)d_state, n_seq,
                       stream_stride(k));
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_stream_append(void* d_state, const void* d_step_bf16, uint32_t n_seq, uint32_t hidden, uint32_t chunk_tokens,
                         uint32_t token, uint32_t k, void* hip_stream)
{
    if (k == 0 || k > TOPLOC_MAX_K || hidden == 0 || hidden % 8 != 0 || chunk_tokens == 0 || token >= chunk_tokens)
        return TOPLOC_EINVAL;
    const uint64_t chunk_values = (uint64_t)chunk_tokens * hidden;
    if (chunk_values >= (1ull << 32)) return TOPLOC_EINVAL;
    if (n_seq == 0) return TOPLOC_OK;
    if (!d_state || !d_step_bf16 || !aligned16(d_state) || !aligned16(d_step_bf16)) return TOPLOC_EINVAL;
    if (reinterpret_cast<uintptr_t>(d_step_bf16) < chunk_values * 2) return TOPLOC_EINVAL;  // the kernel forms row - v0
    hipStream_t st = (hipStream_t)hip_stream;
    const uint32_t hvec = hidden / 8;
    {
        ProfScope ps(TOPLOC_KERNEL_STREAM_APPEND, st);
        if (k <= 128)
            hipLaunchKernelGGL((stream_append_kernel<kCapSmall>), dim3(n_seq), dim3(kThreads), 0, st, (char*)d_state,
                               stream_stride(k), (const u32x4*)d_step_bf16, hvec, token * hvec, k, nullptr, nullptr, n_seq,
                               chunk_tokens);
        else
            hipLaunchKernelGGL((stream_append_kernel<kCapLarge>), dim3(n_seq), dim3(kThreads), 0, st, (char*)d_state,
                               stream_stride(k), (const u32x4*)d_step_bf16, hvec, token * hvec, k, nullptr, nullptr, n_seq,
                               chunk_tokens);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_stream_append_rows(void* d_state, uint32_t n_slots, const void* d_step_bf16, const uint32_t* d_slots,
                              const uint32_t* d_tokens, uint32_t n_rows, uint32_t hidden, uint32_t chunk_tokens,
                              uint32_t k, void* hip_stream)
{
    if (k == 0 || k > TOPLOC_MAX_K || hidden == 0 || hidden % 8 != 0 || chunk_tokens == 0) return TOPLOC_EINVAL;
    const uint64_t chunk_values = (uint64_t)chunk_tokens * hidden;
    if (chunk_values >= (1ull << 32)) return TOPLOC_EINVAL;
    if (n_rows == 0) return TOPLOC_OK;
    if (!d_state || !d_step_bf16 || !d_slots || !d_tokens || n_slots == 0) return TOPLOC_EINVAL;
    if (!aligned16(d_state) || !aligned16(d_step_bf16)) return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_slots) & 3u) != 0 || (reinterpret_cast<uintptr_t>(d_tokens) & 3u) != 0)
        return TOPLOC_EINVAL;
    if (reinterpret_cast<uintptr_t>(d_step_bf16) < chunk_values * 2) return TOPLOC_EINVAL;  // the kernel forms row - v0
    hipStream_t st = (hipStream_t)hip_stream;
    const uint32_t hvec = hidden / 8;
    {
        ProfScope ps(TOPLOC_KERNEL_STREAM_APPEND, st);
        if (k <= 128)
            hipLaunchKernelGGL((stream_append_kernel<kCapSmall>), dim3(n_rows), dim3(kThreads), 0, st, (char*)d_state,
                               stream_stride(k), (const u32x4*)d_step_bf16, hvec, 0u, k, d_slots, d_tokens, n_slots,
                               chunk_tokens);
        else
            hipLaunchKernelGGL((stream_append_kernel<kCapLarge>), dim3(n_rows), dim3(kThreads), 0, st, (char*)d_state,
                               stream_stride(k), (const u32x4*)d_step_bf16, hvec, 0u, k, d_slots, d_tokens, n_slots,
                               chunk_tokens);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_stream_emit(void* d_state, uint32_t n_seq, uint32_t k, uint8_t* d_proofs, uint8_t* d_status,
                       uint32_t* d_topk_idx_opt, void* hip_stream)
{
    if (k == 0 || k > TOPLOC_MAX_K) return TOPLOC_EINVAL;
    if (n_seq == 0) return TOPLOC_OK;
    if (!d_state || !d_proofs || !d_status || !aligned16(d_state)) return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0) return TOPLOC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    {
        ProfScope ps(TOPLOC_KERNEL_STREAM_EMIT, st);
        if (k <= 128)
            hipLaunchKernelGGL((stream_emit_kernel<256, 128, kCapSmall>), dim3(n_seq), dim3(256), 0, st, (char*)d_state,
                               stream_stride(k), k, d_proofs, d_status, d_topk_idx_opt, nullptr, n_seq);
        else
            hipLaunchKernelGGL((stream_emit_kernel<1024, 512, kCapLarge>), dim3(n_seq), dim3(1024), 0, st, (char*)d_state,
                               stream_stride(k), k, d_proofs, d_status, d_topk_idx_opt, nullptr, n_seq);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_stream_emit_rows(void* d_state, uint32_t n_slots, const uint32_t* d_slots, uint32_t n_rows, uint32_t k,
                            uint8_t* d_proofs, uint8_t* d_status, uint32_t* d_topk_idx_opt, void* hip_stream)
{
    if (k == 0 || k > TOPLOC_MAX_K) return TOPLOC_EINVAL;
    if (n_rows == 0) return TOPLOC_OK;
    if (!d_state || !d_slots || !d_proofs || !d_status || n_slots == 0 || !aligned16(d_state)) return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0 || (reinterpret_cast<uintptr_t>(d_slots) & 3u) != 0)
        return TOPLOC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    {
        ProfScope ps(TOPLOC_KERNEL_STREAM_EMIT, st);
        if (k <= 128)
            hipLaunchKernelGGL((stream_emit_kernel<256, 128, kCapSmall>), dim3(n_rows), dim3(256), 0, st, (char*)d_state,
                               stream_stride(k), k, d_proofs, d_status, d_topk_idx_opt, d_slots, n_slots);
        else
            hipLaunchKernelGGL((stream_emit_kernel<1024, 512, kCapLarge>), dim3(n_rows), dim3(1024), 0, st, (char*)d_state,
                               stream_stride(k), k, d_proofs, d_status, d_topk_idx_opt, d_slots, n_slots);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_ring_append(void* d_ring_bf16, const void* d_step_bf16, uint32_t n_seq, uint32_t hidden,
                       uint32_t chunk_tokens, uint32_t step, void* hip_stream)
{
    if (hidden == 0 || hidden % 8 != 0 || chunk_tokens == 0) return TOPLOC_EINVAL;
    if (n_seq == 0) return TOPLOC_OK;
    if (!d_ring_bf16 || !d_step_bf16 || !aligned16(d_ring_bf16) || !aligned16(d_step_bf16)) return TOPLOC_EINVAL;
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
