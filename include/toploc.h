/*
 * toploc.h -- C ABI of the MI355X (gfx950) TopLoc proof build / verify library.
 *
 * The paper states the problem as two functions applied once per chunk of 32
 * new tokens (Section 4; Section 5.6 and 5.8 for the 32-token sampling):
 *   Algorithm 1:  (hidden state tensor h, k)      -> encoded proof p
 *   Algorithm 2:  (hidden state tensor h, proof p) -> accept / reject
 * with the three thresholds of Section 5.2 as fixed parameters.  The entry
 * points below are those two functions over a batch of independent chunks.
 *
 * Conventions common to every entry point
 *  - Pointers named d_* are DEVICE pointers (HIP global memory of the current
 *    device); everything else is a host pointer read during the call only.
 *  - The caller owns every buffer.  The library allocates no device memory and
 *    keeps no reference after the work it enqueued has finished.
 *  - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *    the default stream).  No entry point synchronises or copies: every call only
 *    launches kernels (so it can be captured into a HIP graph); results are valid
 *    once the stream has reached the end of the enqueued work.
 *  - bf16 values are read and written as their 16-bit patterns.  No floating
 *    point arithmetic happens anywhere on the path.
 *  - Return value: TOPLOC_OK (0) when the work was enqueued, a negative
 *    TOPLOC_E* code when the call was rejected (nothing was enqueued then).
 *    Data-dependent per-chunk conditions never fail the call; they are reported
 *    per chunk in `d_status` / `toploc_verify_result.status`.
 *  - Host threads: entry points may be called from several threads at once, each
 *    on its own stream and buffers.  toploc_set_split and toploc_profile_enable
 *    set process-wide switches that calls in flight on other threads may or may
 *    not see yet.
 *
 * Layout of a chunk: `chunk_tokens` consecutive token rows of `hidden` bf16
 * values, row major, so the flat index of (token t, channel c) is t*hidden + c
 * and chunk j starts at element j*chunk_tokens*hidden.  The chunk length
 * N = chunk_tokens*hidden must be a multiple of 8 and `d_hidden_bf16` 16-byte
 * aligned (the kernels read 16 bytes per lane).
 *
 * Layout of a proof (2 + 2k bytes; 258 for k = 128 as in the paper's abstract):
 *   bytes 0..1     m mod 65536, little endian (0 stands for m = 65536), where m
 *                  is the injective modulus of Algorithm 6
 *   bytes 2+2j..   coefficient c_j of x^j of the interpolated polynomial over
 *                  GF(65497) (Algorithm 3's output), little endian, j = 0..k-1
 */
#ifndef TOPLOC_H
#define TOPLOC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TOPLOC_PRIME 65497u     /* the field modulus M of Algorithms 3 and 5            */
#define TOPLOC_MAX_K 512u       /* largest supported top-k parameter                    */
#define TOPLOC_MAX_K_TOPK 4096u /* largest k of toploc_topk alone (Table 1 looks at k up to 4096) */

/* Precisions (Section 5.7 validates across fp32 and bf16).  An fp32 value enters the
 * polynomial as its 32-bit pattern over GF(TOPLOC_PRIME32); such a proof is 2 + 4k bytes:
 * the same 2-byte modulus field, then 4-byte little-endian coefficients. */
#define TOPLOC_DTYPE_BF16 0u
#define TOPLOC_DTYPE_F32 1u
#define TOPLOC_PRIME32 4294967291u  /* 2^32 - 5: the field modulus when fp32 patterns are encoded */
#define TOPLOC_MAX_K_F32 512u       /* largest k of the calls that involve fp32                    */

/* call-level return codes */
#define TOPLOC_OK 0
#define TOPLOC_EINVAL (-1)      /* null / misaligned pointer, k = 0, k > N, k > MAX_K,   */
                                /* N not a multiple of 8, N >= 2^32, prime != 65497      */
#define TOPLOC_EWORKSPACE (-2)  /* workspace smaller than toploc_workspace_bytes()       */
#define TOPLOC_EHIP (-3)        /* a HIP runtime call failed; see toploc_last_hip_error  */
#define TOPLOC_ESCRATCH (-4)    /* toploc_build_proofs_static: the batch needs more than */
                                /* TOPLOC_STATIC_SCRATCH_BYTES of scratch                */

/* per-chunk status codes */
#define TOPLOC_CHUNK_OK 0
#define TOPLOC_CHUNK_NO_MODULUS 1   /* Algorithm 6 exhausted [2^15+1, 65536]             */
/* 2 is not used: Algorithm 4's error exit (no inverse) cannot be reached once the modulus   */
/* makes the points distinct in GF(p)                                                        */
#define TOPLOC_CHUNK_MALFORMED 3    /* verify: decoded m < 2^15+1 or a coefficient >= p  */
#define TOPLOC_CHUNK_SHORT 4        /* fewer than k values: a streaming emit before k    */
                                    /* values were appended, a segment shorter than k    */
#define TOPLOC_CHUNK_BAD_SEGMENT 5  /* segment calls: row offsets that decrease, leave   */
                                    /* the matrix, or span 2^32 values or more           */

typedef struct {
    uint32_t k;             /* top-k parameter of Algorithms 1 and 2 (128 in the paper) */
    uint32_t chunk_tokens;  /* tokens per proof (32 in the paper)                       */
    uint32_t hidden;        /* hidden size of the model                                 */
    uint32_t prime;         /* must be TOPLOC_PRIME                                     */
} toploc_params;

/* T_exp, T_mean, T_median of Algorithm 2; Section 5.2 gives {38, 10, 8} for bf16. */
typedef struct {
    uint32_t t_exp, t_mean, t_median;
} toploc_thresholds;

/* What Algorithm 2 computes for one chunk. 20 bytes. */
typedef struct {
    uint32_t err_exp;      /* err_e: top-k entries whose exponent differs from P(x)'s     */
    uint32_t n_match;      /* |err_m|: entries whose exponent matched                     */
    uint32_t mant_sum;     /* sum of err_m (mean = mant_sum / n_match, kept exact)        */
    uint32_t mant_median;  /* lower median of err_m, 0 when err_m is empty                */
    uint8_t accept;        /* 1 unless err_e > T_exp or mean > T_mean or median > T_median */
    uint8_t status;        /* TOPLOC_CHUNK_OK or TOPLOC_CHUNK_MALFORMED (then accept = 0) */
    uint8_t _pad[2];
} toploc_verify_result;

/* Size of one encoded proof: 2 + 2k (Sections 4 and 5.8: two bytes per coefficient
 * plus the modulus). Host only. */
size_t toploc_proof_bytes(uint32_t k);

/* Bytes of device scratch that toploc_build_proofs / toploc_verify_proofs use for
 * `n_chunks` chunks with these parameters.  A batch too small to fill the chip with one
 * workgroup per chunk is cut into parts (first launch: top-k of every part into this
 * scratch, second launch: merge and finish), and so is every build with k > 128.
 * 0 means one fused launch needs no scratch (large batches, k <= 128), or invalid
 * parameters.  Host only. */
size_t toploc_workspace_bytes(const toploc_params *params, uint64_t n_chunks);
/* The same with the two meanings of 0 told apart: TOPLOC_EINVAL for unusable parameters (then
 * *bytes = 0), TOPLOC_OK with *bytes = 0 when no scratch is needed.  The cut (and with it the size)
 * depends on toploc_set_split: do not change that switch between the query and the call it sizes
 * (a build with k > 128 would be refused with TOPLOC_EWORKSPACE, other calls fall back to the
 * fused launch). */
int toploc_workspace_query(const toploc_params *params, uint64_t n_chunks, size_t *bytes);

/* Tuning / test knob: 0 (default) lets the library choose into how many parts a chunk
 * is cut, n >= 1 forces n parts per chunk (for the *_segments calls: n parts per segment
 * of average length).  Affects later calls, including the workspace_bytes functions. */
int toploc_set_split(uint32_t parts_per_chunk);

/* Algorithm 1 over n_chunks chunks: top-k by magnitude, injective modulus
 * (Algorithm 6), index map, interpolation over GF(p) (Algorithm 3), encode.
 *   d_hidden_bf16   in,  device, [n_chunks][chunk_tokens*hidden] bf16
 *   d_proofs        out, device, n_chunks * (2+2k) bytes (zero-filled for a chunk
 *                   whose status is not TOPLOC_CHUNK_OK)
 *   d_status        out, device, n_chunks bytes, TOPLOC_CHUNK_*
 *   d_topk_idx_opt  out, device, n_chunks*k uint32 flat indices in the order
 *                   (magnitude descending, index ascending); NULL to skip
 *   d_workspace     device scratch, 16-byte aligned, >= toploc_workspace_bytes().
 *                   For k <= 128 it may be NULL or too small: the fused launch is used
 *                   then (slower on small batches only).  For k > 128 it is required
 *                   (TOPLOC_EINVAL when NULL, TOPLOC_EWORKSPACE when too small).
 * n_chunks = 0 is valid and enqueues nothing. */
int toploc_build_proofs(const void *d_hidden_bf16, uint64_t n_chunks, const toploc_params *params,
                        uint8_t *d_proofs, uint8_t *d_status, uint32_t *d_topk_idx_opt,
                        void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* toploc_build_proofs for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same outputs, same bytes as toploc_build_proofs; the scratch that small batches and k > 128
 * need (top-k candidates of the parts a chunk is cut into) is a fixed array of
 * TOPLOC_STATIC_SCRATCH_BYTES in device memory that belongs to the library: every GPU the
 * library runs on holds its own copy until the process ends.  The call allocates nothing, on
 * the host or on the device.
 *  - A batch whose cut needs more than TOPLOC_STATIC_SCRATCH_BYTES (6 bytes per candidate: k per
 *    part; what toploc_workspace_bytes reports) is rejected with TOPLOC_ESCRATCH, nothing enqueued.
 *    Large batches with k <= 128 run as one fused launch and use no scratch at all.
 *  - All calls on one GPU share that GPU's array: calls whose work overlaps in time on one GPU
 *    (different streams, or several host threads) race on it.  Order them on one stream.  Nothing
 *    in the array needs to start at zero: every slot a merge reads was written by the same call.
 *  - The first call on a device looks up the array's device address (hipGetSymbolAddress) and
 *    keeps it; make that first call outside a graph capture. */
#define TOPLOC_STATIC_SCRATCH_BYTES (8u << 20)
int toploc_build_proofs_static(const void *d_hidden_bf16, uint64_t n_chunks, const toploc_params *params,
                               uint8_t *d_proofs, uint8_t *d_status, uint32_t *d_topk_idx_opt, void *hip_stream);

/* Algorithm 2 over n_chunks chunks: decode, top-k of the recomputed tensor,
 * index map, Horner evaluation (Algorithm 5) at the k mapped indices,
 * exponent / mantissa comparison, thresholds.
 *   d_hidden_bf16   in,  device, recomputed activations, same layout as above
 *   d_proofs        in,  device, n_chunks * (2+2k) bytes
 *   thresholds      in,  host
 *   d_results       out, device, n_chunks records
 *   d_workspace     device scratch as above; NULL or too small selects the fused launch */
int toploc_verify_proofs(const void *d_hidden_bf16, uint64_t n_chunks, const toploc_params *params,
                         const uint8_t *d_proofs, const toploc_thresholds *thresholds,
                         toploc_verify_result *d_results, void *d_workspace, size_t workspace_bytes,
                         void *hip_stream);

/* The first step of both algorithms alone (topk(h, k) of Algorithm 1 / 2), for
 * k <= TOPLOC_MAX_K_TOPK (above TOPLOC_MAX_K at a fraction of the speed: one workgroup
 * per compute unit):
 *   d_topk_idx   out, device, n_chunks*k uint32, (magnitude desc, index asc)
 *   d_topk_val   out, device, n_chunks*k uint16 bf16 patterns, same order */
int toploc_topk(const void *d_hidden_bf16, uint64_t n_chunks, const toploc_params *params,
                uint32_t *d_topk_idx, uint16_t *d_topk_val, void *hip_stream);

/* The same two algorithms over SEGMENTS of unequal length: the proof over a whole
 * prompt (Section 5.6: a set of top-k values is also kept for the activations of the
 * input prompt) and the ragged last chunk of a generation.  The activations are one
 * [total_rows][hidden] bf16 matrix; segment i is rows d_row_offsets[i] ..
 * d_row_offsets[i+1]-1, its flat index is (row - first row) * hidden + channel.
 *   total_rows      rows of the matrix: no segment may reach beyond it
 *   d_row_offsets   in, DEVICE, n_segments + 1 non-decreasing uint64 row numbers (a serving
 *                   engine's cumulative sequence lengths), 8-byte aligned.  The host never
 *                   reads them: the cut into parts is planned from n_segments, total_rows and
 *                   hidden alone and a small kernel derives every part from the offsets, so
 *                   the calls only launch kernels and can be captured into a HIP graph; a
 *                   replay uses whatever the array holds then
 *   hidden          a multiple of 8
 * Proofs, status, results and the optional indices are laid out per segment exactly as per
 * chunk above; prime and proof layout are the same.  Per segment, not per call: a segment
 * with fewer than k values gets TOPLOC_CHUNK_SHORT, one whose offsets decrease, leave the
 * matrix or span 2^32 values or more gets TOPLOC_CHUNK_BAD_SEGMENT; both get a zero-filled
 * proof (indices 0xFFFFFFFF) from a build and accept = 0 from a verify.  Offsets that are
 * not monotonic as a whole leave the other segments' results undefined, but never lead to
 * an access outside the matrix or the workspace.  Long segments are cut into parts like
 * small batches.  d_workspace (required, 16-byte aligned) must hold
 * toploc_segments_workspace_bytes() bytes. */
size_t toploc_segments_workspace_bytes(uint64_t n_segments, uint64_t total_rows, uint32_t hidden, uint32_t k);
int toploc_build_proofs_segments(const void *d_hidden_bf16, uint64_t total_rows, const uint64_t *d_row_offsets,
                                 uint64_t n_segments, uint32_t hidden, uint32_t k, uint8_t *d_proofs, uint8_t *d_status,
                                 uint32_t *d_topk_idx_opt, void *d_workspace, size_t workspace_bytes,
                                 void *hip_stream);
int toploc_verify_proofs_segments(const void *d_hidden_bf16, uint64_t total_rows, const uint64_t *d_row_offsets,
                                  uint64_t n_segments, uint32_t hidden, uint32_t k, const uint8_t *d_proofs,
                                  const toploc_thresholds *thresholds, toploc_verify_result *d_results,
                                  void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* Provider-side ring of the last chunk_tokens hidden vectors per sequence
 * (Section 5.8, Table 6: the provider keeps the last hidden states until the
 * proof is cut).  Copies d_step_bf16 [n_seq][hidden] into row (step mod
 * chunk_tokens) of d_ring_bf16 [n_seq][chunk_tokens][hidden]; after every
 * chunk_tokens-th step the ring is a valid input of toploc_build_proofs with
 * n_chunks = n_seq.  hidden must be a multiple of 8, both pointers 16-byte
 * aligned. */
int toploc_ring_append(void *d_ring_bf16, const void *d_step_bf16, uint32_t n_seq, uint32_t hidden,
                       uint32_t chunk_tokens, uint32_t step, void *hip_stream);

/* fp32 activations and validation across precisions (Section 5.7, Table 5; fp32 thresholds
 * {8, 256, 128} in Section 5.2).  Top-k ranks fp32 values by (pattern & 0x7FFFFFFF).
 *   toploc_proof_bytes_dtype   2 + 2k (TOPLOC_DTYPE_BF16) or 2 + 4k (TOPLOC_DTYPE_F32)
 *   toploc_build_proofs_f32    Algorithm 1 over [n_chunks][chunk_tokens*hidden] fp32 values;
 *                              params->prime must be TOPLOC_PRIME32, k <= TOPLOC_MAX_K_F32;
 *                              proofs are 2 + 4k bytes each; other arguments as toploc_build_proofs,
 *                              the workspace (toploc_workspace_bytes_f32; candidates carry 4-byte
 *                              patterns) being required for k > 128 and optional otherwise
 *   toploc_verify_proofs_mixed Algorithm 2 with activations of `hidden_dtype` and proofs of
 *                              `proof_dtype` (params->prime: the proof's field).  Exponent and
 *                              mantissa are compared in the validator's (the activations')
 *                              precision: an fp32 proof's mantissa is scaled to bf16's 7 bits
 *                              (>> 16) for a bf16 validator, a bf16 proof's value gets 16 zero
 *                              bits appended for an fp32 validator.  Thresholds are the caller's
 *                              (the paper uses the validator's precision's).
 * The validation runs as one fused launch per call and needs no workspace.
 *   toploc_build_proofs_segments_f32, toploc_verify_proofs_segments_mixed
 *                              the same two over segments of unequal length (the whole prompt,
 *                              a ragged last chunk), arguments as toploc_build_proofs_segments /
 *                              toploc_verify_proofs_segments; d_workspace must hold
 *                              toploc_segments_workspace_bytes_dtype(..., hidden_dtype) bytes
 *                              (candidates carry 4-byte patterns when the activations are fp32) */
size_t toploc_proof_bytes_dtype(uint32_t k, uint32_t dtype);
size_t toploc_workspace_bytes_f32(const toploc_params *params, uint64_t n_chunks);
int toploc_build_proofs_f32(const void *d_hidden_f32, uint64_t n_chunks, const toploc_params *params, uint8_t *d_proofs,
                            uint8_t *d_status, uint32_t *d_topk_idx_opt, void *d_workspace, size_t workspace_bytes,
                            void *hip_stream);
int toploc_verify_proofs_mixed(const void *d_hidden, uint32_t hidden_dtype, uint64_t n_chunks, const toploc_params *params,
                               const uint8_t *d_proofs, uint32_t proof_dtype, const toploc_thresholds *thresholds,
                               toploc_verify_result *d_results, void *hip_stream);
size_t toploc_segments_workspace_bytes_dtype(uint64_t n_segments, uint64_t total_rows, uint32_t hidden, uint32_t k,
                                             uint32_t hidden_dtype);
int toploc_build_proofs_segments_f32(const void *d_hidden_f32, uint64_t total_rows, const uint64_t *d_row_offsets,
                                     uint64_t n_segments, uint32_t hidden, uint32_t k, uint8_t *d_proofs,
                                     uint8_t *d_status, uint32_t *d_topk_idx_opt, void *d_workspace,
                                     size_t workspace_bytes, void *hip_stream);
int toploc_verify_proofs_segments_mixed(const void *d_hidden, uint32_t hidden_dtype, uint64_t total_rows,
                                        const uint64_t *d_row_offsets, uint64_t n_segments, uint32_t hidden, uint32_t k,
                                        const uint8_t *d_proofs, uint32_t proof_dtype,
                                        const toploc_thresholds *thresholds, toploc_verify_result *d_results,
                                        void *d_workspace, size_t workspace_bytes, void *hip_stream);

/* Online path without the ring (a design of this build; the paper's provider keeps the
 * last hidden states, Table 6, only to take their top-k when the proof is cut).  Per
 * sequence the library keeps the running top-k of the rows appended so far -- at most k
 * (flat index, bf16 pattern) pairs and the k-th element as threshold, 16 + 6k bytes
 * with each part rounded up to 16 bytes -- so a decode step costs one read of its
 * [n_seq][hidden] vectors and the emission never re-reads activations.  The proofs are
 * byte for byte those toploc_build_proofs gives for the chunk made of the appended rows.
 *   toploc_stream_state_bytes   size of d_state for n_seq sequences (0: invalid k)
 *   toploc_stream_reset         empties every sequence's state
 *   toploc_stream_append        row `token` (0-based position inside the chunk, each
 *                               position at most once per chunk, any order) of every
 *                               sequence: d_step_bf16 [n_seq][hidden]; the flat index of
 *                               channel c is token*hidden + c.  hidden % 8 == 0,
 *                               chunk_tokens*hidden < 2^32, d_step_bf16 16-byte aligned
 *   toploc_stream_emit          Algorithm 1 steps 2-5 on every sequence's k pairs: proofs,
 *                               status (TOPLOC_CHUNK_SHORT when fewer than k values were
 *                               appended) and optionally the ordered indices, laid out as by
 *                               toploc_build_proofs; then empties the states
 *   toploc_stream_append_rows   the same for a serving loop with continuous batching, where a
 *                               step carries rows of any subset of the sequences, each at its
 *                               own position: row r of d_step_bf16 [n_rows][hidden] enters the
 *                               state of sequence d_slots[r] (< n_slots) as token d_tokens[r]
 *                               (< chunk_tokens); d_slots, d_tokens: device, n_rows uint32.
 *                               The slots of one call must be distinct; a row whose slot or
 *                               token is out of range is skipped
 *   toploc_stream_emit_rows     emission for the sequences d_slots[0..n_rows): output row r
 *                               (proof, status, indices) belongs to sequence d_slots[r], whose
 *                               state is emptied; an out-of-range slot reads as an empty state
 *                               (TOPLOC_CHUNK_SHORT).  Slots must be distinct
 * d_state is 16-byte aligned device memory owned by the caller; calls on one state must
 * be ordered on one stream. */
size_t toploc_stream_state_bytes(uint32_t n_seq, uint32_t k);
int toploc_stream_reset(void *d_state, uint32_t n_seq, uint32_t k, void *hip_stream);
int toploc_stream_append(void *d_state, const void *d_step_bf16, uint32_t n_seq, uint32_t hidden, uint32_t chunk_tokens,
                         uint32_t token, uint32_t k, void *hip_stream);
int toploc_stream_emit(void *d_state, uint32_t n_seq, uint32_t k, uint8_t *d_proofs, uint8_t *d_status,
                       uint32_t *d_topk_idx_opt, void *hip_stream);
int toploc_stream_append_rows(void *d_state, uint32_t n_slots, const void *d_step_bf16, const uint32_t *d_slots,
                              const uint32_t *d_tokens, uint32_t n_rows, uint32_t hidden, uint32_t chunk_tokens,
                              uint32_t k, void *hip_stream);
int toploc_stream_emit_rows(void *d_state, uint32_t n_slots, const uint32_t *d_slots, uint32_t n_rows, uint32_t k,
                            uint8_t *d_proofs, uint8_t *d_status, uint32_t *d_topk_idx_opt, void *hip_stream);

/* The running top-k for either precision (Section 5.7: fp32 inference): the same four operations
 * with the element type as an argument; the calls above are these with TOPLOC_DTYPE_BF16.  With
 * TOPLOC_DTYPE_F32 a state holds 4-byte patterns (16 + 8k bytes per sequence, parts rounded up to
 * 16), rows are fp32, proofs are 2 + 4k bytes over GF(TOPLOC_PRIME32), k <= TOPLOC_MAX_K_F32.
 *   toploc_stream_append_dtype  d_slots and d_tokens both NULL: row r of d_step [n_rows][hidden] is
 *                               token `token` of sequence r (n_slots is ignored); both given: row r
 *                               is token d_tokens[r] of sequence d_slots[r] < n_slots (`token` is
 *                               ignored)
 *   toploc_stream_emit_dtype    d_slots NULL: output row r is sequence r; else sequence d_slots[r] */
size_t toploc_stream_state_bytes_dtype(uint32_t n_seq, uint32_t k, uint32_t dtype);
int toploc_stream_reset_dtype(void *d_state, uint32_t n_seq, uint32_t k, uint32_t dtype, void *hip_stream);
int toploc_stream_append_dtype(void *d_state, uint32_t n_slots, const void *d_step, uint32_t dtype,
                               const uint32_t *d_slots, const uint32_t *d_tokens, uint32_t n_rows, uint32_t hidden,
                               uint32_t chunk_tokens, uint32_t token, uint32_t k, void *hip_stream);
int toploc_stream_emit_dtype(void *d_state, uint32_t n_slots, uint32_t dtype, const uint32_t *d_slots, uint32_t n_rows,
                             uint32_t k, uint8_t *d_proofs, uint8_t *d_status, uint32_t *d_topk_idx_opt,
                             void *hip_stream);

/* Measurement aid, not part of the method: reads n_chunks * chunk_values bf16
 * values with the access pattern of the selection kernel (one workgroup per
 * chunk, 16-byte loads) and keeps only a running maximum, to show what a pure
 * read of the tensor achieves on the device.  d_out: device, n_chunks uint32
 * (written only for a chunk holding an all-ones word).  chunk_values must be a
 * multiple of 8 and < 2^32. */
int toploc_bench_read(const void *d_hidden_bf16, uint64_t n_chunks, uint64_t chunk_values, uint32_t *d_out,
                      void *hip_stream);

/* Measurement aid, not part of the method: what the selection (the top-k step of Algorithm 1 / 2)
 * did on every chunk.  d_stats: out, device, n_chunks * 4 uint32: drains of the queue, prunes of
 * the candidate buffer, vectors queued, candidates appended (the final drain and prune of a chunk
 * included).  Parameters as toploc_build_proofs.  Input laws differ in exactly these numbers. */
int toploc_selection_stats(const void *d_hidden_bf16, uint64_t n_chunks, const toploc_params *params,
                           uint32_t *d_stats, void *hip_stream);

/* Kernel timing for benchmarks.  toploc_profile_enable(1) creates a pool of HIP events (the only
 * place the library creates any; they live until the process ends); while enabled, every kernel
 * launch is bracketed by two events of the pool on the caller's stream, and a launch that finds the
 * pool empty (more than 8192 timed launches since the last read) goes untimed.
 * toploc_profile_read synchronises those events and returns, per kernel slot
 * (TOPLOC_KERNEL_*), the number of launches and their summed duration in
 * milliseconds since the last reset, then resets.  The list of events is shared by
 * all threads: one thread reads it, after the others' timed calls have returned. */
#define TOPLOC_KERNEL_SELECT 0        /* topk alone (toploc_topk)                        */
#define TOPLOC_KERNEL_PART 1          /* split path: top-k of one part                   */
#define TOPLOC_KERNEL_BUILD_MERGE 2   /* split path: merge, modulus, interpolation       */
#define TOPLOC_KERNEL_VERIFY_MERGE 3  /* split path: merge, evaluation, statistics       */
#define TOPLOC_KERNEL_BUILD 4         /* fused build kernel (k <= 128)                   */
#define TOPLOC_KERNEL_VERIFY 5        /* fused verify kernel                             */
#define TOPLOC_KERNEL_RING 6          /* ring append kernel                              */
#define TOPLOC_KERNEL_READ 7          /* toploc_bench_read                               */
#define TOPLOC_KERNEL_STREAM_APPEND 8 /* toploc_stream_append, toploc_stream_append_rows  */
#define TOPLOC_KERNEL_STREAM_EMIT 9   /* toploc_stream_emit, toploc_stream_emit_rows      */
#define TOPLOC_KERNEL_PLAN 10         /* segment calls: the part table from the row offsets */
#define TOPLOC_KERNEL_COUNT 11
int toploc_profile_enable(int on);
int toploc_profile_read(uint32_t *launches /*[TOPLOC_KERNEL_COUNT]*/, float *total_ms /*[TOPLOC_KERNEL_COUNT]*/);

/* Text for a TOPLOC_E* code; never NULL. */
const char *toploc_strerror(int code);

/* hipError_t (as int) of the last failed HIP call in this process, 0 if none. */
int toploc_last_hip_error(void);

/* Identifies the sources and compiler flags this library was built from (a hash the in-tree build
 * stamps in; "unstamped" otherwise).  Profile summaries record it, so that a reader of a number can
 * tell whether it was measured on this code.  Never NULL. */
const char *toploc_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* TOPLOC_H */
