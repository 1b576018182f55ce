// Host-side planning and argument validation of the C ABI: how a batch is cut into parts, how
// much scratch a call needs, which parameter combinations are refused.  Plain C++ with no HIP
// types or calls, so that the same code the library runs can be compiled for the host alone
// (with the address and undefined-behaviour sanitizers) and driven without a GPU.
//
// The operations being planned are the paper's Algorithm 1 and Algorithm 2 over chunks of
// chunk_tokens * hidden values (Section 5.6, 5.8) and over row ranges of unequal length (the
// whole prompt's proof, Section 5.6).
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "../../include/toploc.h"

namespace toploc {
namespace plan {

constexpr uint32_t kThreads = 256;   // lanes per streaming workgroup
#ifndef TOPLOC_LOADS
#define TOPLOC_LOADS 4
#endif
constexpr uint32_t kLoads = TOPLOC_LOADS;               // 16-byte loads in flight per lane and round
constexpr uint32_t kRoundVecs = kThreads * kLoads;      // vectors a workgroup examines per round

// How a launch is cut.  One workgroup keeps about 16 KB of loads in flight, so roughly a
// thousand streaming workgroups are needed to saturate HBM: a batch with fewer chunks is
// cut into parts until there are that many, but a part still streams a few rounds (every
// part pays for finding its own threshold), and no part is longer than kMaxPartVecs so
// that one long segment cannot become the launch's straggler.
constexpr uint64_t kTargetGroups = 1024;
constexpr uint64_t kMinPartVecs = 4 * (uint64_t)kRoundVecs;
constexpr uint64_t kMaxPartVecs = 64 * (uint64_t)kRoundVecs;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline size_t up16(size_t b) { return (b + 15) & ~(size_t)15; }

inline size_t bits_size_of(uint32_t dtype) { return dtype == TOPLOC_DTYPE_F32 ? sizeof(uint32_t) : sizeof(uint16_t); }
inline uint32_t elems_per_vec(uint32_t dtype) { return dtype == TOPLOC_DTYPE_F32 ? 4u : 8u; }

// N (values per chunk) when the parameters are usable for bf16 activations and proofs, else 0
inline uint64_t chunk_len(const toploc_params* p, uint32_t max_k = TOPLOC_MAX_K)
{
    if (!p || p->k == 0 || p->k > max_k || p->prime != TOPLOC_PRIME) return 0;
    if (p->chunk_tokens == 0 || p->hidden == 0) return 0;
    const uint64_t n = (uint64_t)p->chunk_tokens * p->hidden;
    if (n % 8 != 0 || n >= (1ull << 32) || p->k > n) return 0;
    return n;
}

// the largest k of a call with activations of `hidden_dtype` and proofs of `proof_dtype`
inline uint32_t max_k_of(uint32_t hidden_dtype, uint32_t proof_dtype)
{
    return (hidden_dtype == TOPLOC_DTYPE_F32 || proof_dtype == TOPLOC_DTYPE_F32) ? TOPLOC_MAX_K_F32 : TOPLOC_MAX_K;
}

// N for the calls that involve fp32: the chunk a whole number of 16-byte vectors in both formats
inline uint64_t chunk_len_mixed(const toploc_params* p, uint32_t hidden_dtype, uint32_t proof_dtype)
{
    if (!p || hidden_dtype > TOPLOC_DTYPE_F32 || proof_dtype > TOPLOC_DTYPE_F32) return 0;
    if (p->prime != (proof_dtype == TOPLOC_DTYPE_F32 ? TOPLOC_PRIME32 : TOPLOC_PRIME)) return 0;
    if (p->k == 0 || p->k > max_k_of(hidden_dtype, proof_dtype) || p->chunk_tokens == 0 || p->hidden == 0) return 0;
    const uint64_t n = (uint64_t)p->chunk_tokens * p->hidden;
    if (n % 8 != 0 || n >= (1ull << 32) || p->k > n) return 0;
    return n;
}

inline uint64_t clamp_part_vecs(uint64_t pv)
{
    pv = (pv + kRoundVecs - 1) / kRoundVecs * kRoundVecs;
    return pv < kMinPartVecs ? kMinPartVecs : pv > kMaxPartVecs ? kMaxPartVecs : pv;
}

// Fixed chunks of `nvec` vectors: parts per chunk and vectors per part.  `forced` is the
// toploc_set_split knob (0: choose).
struct FixedPlan { uint32_t parts; uint32_t part_vecs; };
inline FixedPlan plan_fixed(uint64_t n_chunks, uint64_t nvec, uint64_t forced)
{
    uint64_t pv;
    if (forced) {
        pv = (nvec + forced - 1) / forced;
        pv = pv ? pv : 1;
    } else {
        const uint64_t want = n_chunks < kTargetGroups ? kTargetGroups / (n_chunks ? n_chunks : 1) : 1;  // parts per chunk
        pv = clamp_part_vecs((nvec + want - 1) / want);
    }
    FixedPlan f;
    f.parts = (uint32_t)((nvec + pv - 1) / pv);
    f.part_vecs = (uint32_t)(pv < nvec ? pv : nvec);
    return f;
}

// candidate arrays for `slots` parts: [slots*k] uint32 indices, then [slots*k] patterns of
// `bits_size` bytes (2: bf16, 4: fp32), each array 16-byte aligned
inline size_t cand_bytes(uint64_t slots, uint32_t k, size_t bits_size = sizeof(uint16_t))
{
    return up16((size_t)slots * k * sizeof(uint32_t)) + up16((size_t)slots * k * bits_size);
}

// Segments.  The row offsets live in device memory (a serving engine's cumulative sequence
// lengths), so the host plans from sizes alone: `total_rows` rows of `hidden` values hold all
// segments.  Every segment is cut into parts of `part_vecs` vectors (the last one shorter);
// segment i, starting at vector a_i of the matrix, owns the candidate slots from
// floor(a_i / part_vecs) + i on.  It needs ceil(len_i / part_vecs) of them, which is at most the
// number of part_vecs-sized blocks of the matrix it touches, so the slot ranges of different
// segments never overlap and a slot's owner follows from the offsets without a prefix sum; the
// launch has blocks + n_segments slots, some of them idle.
constexpr uint64_t kMaxSegmentVecs = 1ull << 30;   // a segment holds fewer than 2^32 values: fewer vectors than this
struct SegmentPlan {
    bool ok;              // parameters usable
    uint32_t row_vecs;    // 16-byte vectors per row
    uint64_t part_vecs;   // vectors per part
    uint64_t slots;       // workgroups of the part launch = candidate slots = part table entries
};
inline SegmentPlan plan_segments(uint64_t n_segments, uint64_t total_rows, uint32_t hidden, uint32_t k, uint32_t hidden_dtype,
                                 uint32_t k_max, uint64_t forced)
{
    SegmentPlan pl = {false, 0, 0, 0};
    if (hidden == 0 || hidden % 8 != 0 || k == 0 || k > k_max || hidden_dtype > TOPLOC_DTYPE_F32) return pl;
    if (n_segments >= (1ull << 31) || total_rows > (1ull << 62) / hidden) return pl;   // value counts stay in 64 bits
    pl.row_vecs = hidden / elems_per_vec(hidden_dtype);
    const uint64_t total_vecs = total_rows * pl.row_vecs;
    if (forced) {   // `forced` parts per segment of average length
        const uint64_t units = n_segments ? n_segments : 1;
        const uint64_t pv = (total_vecs + forced * units - 1) / (forced * units);
        pl.part_vecs = pv == 0 ? 1 : pv > kMaxSegmentVecs ? kMaxSegmentVecs : pv;
    } else {
        const uint64_t groups = n_segments > kTargetGroups ? n_segments : kTargetGroups;
        pl.part_vecs = clamp_part_vecs((total_vecs + groups - 1) / groups);
    }
    pl.slots = (total_vecs + pl.part_vecs - 1) / pl.part_vecs + n_segments;
    pl.ok = pl.slots < (1ull << 31);
    return pl;
}

// part table entry (16 bytes per slot), behind the candidate arrays
constexpr size_t kPartDescBytes = 16;
inline size_t segments_workspace_bytes(const SegmentPlan& pl, uint32_t k, size_t bits_size)
{
    return cand_bytes(pl.slots, k, bits_size) + up16((size_t)pl.slots * kPartDescBytes);
}

// ---------------------------------------------------------------------------
// Argument checks of the entry points.  Each returns kGo when the call may launch, TOPLOC_OK when
// there is nothing to do (an empty batch), or the TOPLOC_E* code the entry point returns.
// ---------------------------------------------------------------------------
constexpr int kGo = 1;

// Calls over fixed chunks: `n` is what chunk_len / chunk_len_mixed made of the parameters; `a` and `b`
// are the call's two other required device pointers with the alignment each needs (1: any).
inline int check_fixed(uint64_t n, uint64_t n_chunks, const void* d_hidden, const void* a, uintptr_t a_align, const void* b,
                       uintptr_t b_align, const void* d_workspace)
{
    if (n == 0 || n_chunks >= (1ull << 31)) return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    if (!d_hidden || !a || !b || !aligned16(d_hidden)) return TOPLOC_EINVAL;
    if (!aligned(a, a_align) || !aligned(b, b_align)) return TOPLOC_EINVAL;
    if (d_workspace && !aligned16(d_workspace)) return TOPLOC_EINVAL;
    return kGo;
}

// toploc_build_proofs_static: does the cut `f` of the batch fit the library's fixed scratch array?
inline bool fixed_plan_is_fused(const FixedPlan& f, uint32_t k) { return f.parts == 1 && k <= 128; }
inline int check_static_scratch(const FixedPlan& f, uint64_t n_chunks, uint32_t k, size_t scratch_bytes)
{
    if (fixed_plan_is_fused(f, k)) return kGo;
    if (n_chunks * (uint64_t)f.parts >= (1ull << 31)) return TOPLOC_EINVAL;
    return cand_bytes(n_chunks * f.parts, k) > scratch_bytes ? TOPLOC_ESCRATCH : kGo;
}

// The segment calls: `out` is the status array (alignment 1) or the result records (4).
inline int check_segments(const SegmentPlan& pl, uint64_t n_segments, uint32_t k, uint32_t hidden_dtype, const void* d_hidden,
                          const uint64_t* d_row_offsets, const void* d_proofs, const void* d_out, uintptr_t out_align,
                          const void* d_workspace, size_t workspace_bytes)
{
    if (!pl.ok) return TOPLOC_EINVAL;
    if (n_segments == 0) return TOPLOC_OK;
    if (!d_hidden || !d_row_offsets || !d_proofs || !d_out || !d_workspace) return TOPLOC_EINVAL;
    if (!aligned16(d_hidden) || !aligned16(d_workspace) || !aligned(d_row_offsets, 8)) return TOPLOC_EINVAL;
    if (!aligned(d_proofs, 2) || !aligned(d_out, out_align)) return TOPLOC_EINVAL;
    if (workspace_bytes < segments_workspace_bytes(pl, k, bits_size_of(hidden_dtype))) return TOPLOC_EWORKSPACE;
    return kGo;
}

// The running top-k calls.  State of one sequence: a 16-byte header, k indices, k patterns (2 bytes
// each for bf16, 4 for fp32), each part rounded up to 16 bytes.
constexpr size_t kStreamHeaderBytes = 16;
inline size_t stream_idx_bytes(uint32_t k) { return ((size_t)k * 4 + 15) & ~(size_t)15; }
inline size_t stream_stride(uint32_t k, uint32_t dtype = TOPLOC_DTYPE_BF16)
{
    return kStreamHeaderBytes + stream_idx_bytes(k) + (((size_t)k * bits_size_of(dtype) + 15) & ~(size_t)15);
}
inline bool stream_k_ok(uint32_t k, uint32_t dtype = TOPLOC_DTYPE_BF16)
{
    return dtype <= TOPLOC_DTYPE_F32 && k != 0 && k <= max_k_of(dtype, dtype);
}

inline int check_stream_rows(uint32_t k, uint32_t hidden, uint32_t chunk_tokens, uint32_t dtype = TOPLOC_DTYPE_BF16)
{
    if (!stream_k_ok(k, dtype) || hidden == 0 || hidden % 8 != 0 || chunk_tokens == 0) return TOPLOC_EINVAL;
    if ((uint64_t)chunk_tokens * hidden >= (1ull << 32)) return TOPLOC_EINVAL;
    return kGo;
}
// one row per sequence (d_slots and d_tokens NULL: row r is token `token` of sequence r, n_rows sequences)
// or rows of any subset of the sequences (both given: row r is token d_tokens[r] of sequence d_slots[r])
inline int check_stream_append(const void* d_state, uint32_t n_slots, const void* d_step, const void* d_slots,
                               const void* d_tokens, uint32_t n_rows, uint32_t hidden, uint32_t chunk_tokens, uint32_t token,
                               uint32_t k, uint32_t dtype = TOPLOC_DTYPE_BF16)
{
    if (check_stream_rows(k, hidden, chunk_tokens, dtype) != kGo) return TOPLOC_EINVAL;
    const bool indexed = d_slots || d_tokens;
    if (!indexed && token >= chunk_tokens) return TOPLOC_EINVAL;
    if (n_rows == 0) return TOPLOC_OK;
    if (!d_state || !d_step || !aligned16(d_state) || !aligned16(d_step)) return TOPLOC_EINVAL;
    if (indexed && (!d_slots || !d_tokens || n_slots == 0 || !aligned(d_slots, 4) || !aligned(d_tokens, 4))) return TOPLOC_EINVAL;
    return kGo;
}
inline int check_stream_emit(const void* d_state, uint32_t n_rows, uint32_t k, const void* d_proofs, const void* d_status,
                             bool indexed, const void* d_slots, uint32_t n_slots, uint32_t dtype = TOPLOC_DTYPE_BF16)
{
    if (!stream_k_ok(k, dtype)) return TOPLOC_EINVAL;
    if (n_rows == 0) return TOPLOC_OK;
    if (!d_state || !d_proofs || !d_status || !aligned16(d_state) || !aligned(d_proofs, 2)) return TOPLOC_EINVAL;
    if (indexed && (!d_slots || n_slots == 0 || !aligned(d_slots, 4))) return TOPLOC_EINVAL;
    return kGo;
}
inline int check_ring_append(const void* d_ring, const void* d_step, uint32_t n_seq, uint32_t hidden, uint32_t chunk_tokens)
{
    if (hidden == 0 || hidden % 8 != 0 || chunk_tokens == 0) return TOPLOC_EINVAL;
    if (n_seq == 0) return TOPLOC_OK;
    if (!d_ring || !d_step || !aligned16(d_ring) || !aligned16(d_step)) return TOPLOC_EINVAL;
    return kGo;
}

}  // namespace plan
}  // namespace toploc
