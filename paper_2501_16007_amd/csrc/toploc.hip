// TopLoc proof build / verify for MI355X (gfx950): kernels and the C ABI of
// include/toploc.h.  One workgroup per chunk everywhere; chunks are independent.
//
//   build_kernel    all of Algorithm 1 in one launch (k <= 128): topk, then
//                   findInjectiveModulus, i mod m, InterpolateModPolynomial, encode
//                   while other workgroups of the compute unit keep streaming
//   select_kernel   topk(h, k)                       (Algorithm 1 / 2, first step)
//   interp_kernel   findInjectiveModulus, i mod m, InterpolateModPolynomial, encode
//                   (Algorithm 1, remaining steps; Algorithms 3, 4, 6), k > 128
//   verify_kernel   decode, topk, i mod m, Horner at the k points, extractBits,
//                   err_e / err_m statistics, thresholds (Algorithm 2, Algorithm 5)
//   ring_kernel     provider-side ring of the last chunk_tokens hidden vectors
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <vector>

#include "../../include/toploc.h"
#include "gf65497.hpp"
#include "interp.hpp"
#include "select.hpp"

namespace toploc {

#ifndef TOPLOC_THREADS
#define TOPLOC_THREADS 256
#endif
#ifndef TOPLOC_LOADS
#define TOPLOC_LOADS 4
#endif
#ifndef TOPLOC_CAP
#define TOPLOC_CAP 1024
#endif
#ifndef TOPLOC_MIN_WAVES
#define TOPLOC_MIN_WAVES 6  // waves per SIMD the streaming kernels must reach (bounds their VGPRs)
#endif
#ifndef TOPLOC_QCAP
#define TOPLOC_QCAP 512
#endif
constexpr int kThreads = TOPLOC_THREADS;  // threads per workgroup (one chunk each)
constexpr int kLoads = TOPLOC_LOADS;      // 16-byte loads in flight per lane and round
constexpr int kCap = TOPLOC_CAP;          // candidate buffer entries
constexpr int kQcap = TOPLOC_QCAP;        // queue entries (16-byte vectors)
static_assert(kCap >= 2 * (int)TOPLOC_MAX_K, "the soft limit CAP/2 must not be below k");

typedef SelectShared<kThreads, kCap, kQcap> SelShared;

// ---------------------------------------------------------------------------
// topk(h, k) alone: writes the ordered (index, value) pairs of every chunk
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads, TOPLOC_MIN_WAVES) void select_kernel(const u32x4* __restrict__ hidden, uint32_t nvec, uint32_t k,
                                                          uint32_t* __restrict__ out_idx, uint16_t* __restrict__ out_val,
                                                          uint32_t* __restrict__ out_idx2)
{
    __shared__ SelShared s;
    const uint64_t chunk = blockIdx.x;
    select_topk<kThreads, kLoads, kCap, kQcap>(hidden + chunk * nvec, nvec, k, s);
    order_topk<kThreads, kCap, kQcap>(s, k);
    for (uint32_t t = threadIdx.x; t < k; t += kThreads) {
        const uint32_t i = s.cand_idx[t];
        out_idx[chunk * k + t] = i;
        out_val[chunk * k + t] = s.cand_bits[t];
        if (out_idx2) out_idx2[chunk * k + t] = i;
    }
}

// ---------------------------------------------------------------------------
// Algorithm 1 after the selection (interp.hpp), as its own kernel for k > 128
// ---------------------------------------------------------------------------
template <int KMAX>
__global__ __launch_bounds__(kThreads) void interp_kernel(const uint32_t* __restrict__ topk_idx,
                                                          const uint16_t* __restrict__ topk_val, uint32_t k,
                                                          uint8_t* __restrict__ proofs, uint8_t* __restrict__ status)
{
    __shared__ InterpShared<KMAX> s;
    __shared__ uint32_t coef[KMAX];
    const uint32_t tid = threadIdx.x;
    const uint64_t chunk = blockIdx.x;
    for (uint32_t j = tid; j < k; j += kThreads) {
        s.idx[j] = topk_idx[chunk * k + j];
        const uint32_t y = topk_val[chunk * k + j];
        s.ys[j] = (uint16_t)(y >= kPrime ? y - kPrime : y);
    }
    finish_proof<kThreads, KMAX>(s, coef, k, reinterpret_cast<uint16_t*>(proofs + chunk * (2 + 2 * (uint64_t)k)),
                                     status + chunk);
}

// Algorithm 1 in one launch, k <= KMAX <= kThreads: the selection streams the chunk,
// then the same workgroup turns its k pairs into the proof out of LDS (the selection's
// buffers are dead by then and are reused).
template <int KMAX>
__global__ __launch_bounds__(kThreads, TOPLOC_MIN_WAVES) void build_kernel(const u32x4* __restrict__ hidden, uint32_t nvec,
                                                                           uint32_t k, uint8_t* __restrict__ proofs,
                                                                           uint8_t* __restrict__ status,
                                                                           uint32_t* __restrict__ out_idx)
{
    static_assert(KMAX <= kThreads, "one pair per lane is carried across the phase change");
    __shared__ union BuildShared {
        SelShared sel;
        InterpShared<KMAX> itp;
    } sh;
    __shared__ uint32_t coef[KMAX];
    const uint32_t tid = threadIdx.x;
    const uint64_t chunk = blockIdx.x;
    select_topk<kThreads, kLoads, kCap, kQcap>(hidden + chunk * nvec, nvec, k, sh.sel);
    if (out_idx) {  // uniform: the caller wants the ordered indices
        order_topk<kThreads, kCap, kQcap>(sh.sel, k);
        if (tid < k) out_idx[chunk * k + tid] = sh.sel.cand_idx[tid];
    }
#ifdef TOPLOC_TAIL_PRIO
    __builtin_amdgcn_s_setprio(TOPLOC_TAIL_PRIO);  // the arithmetic tail goes ahead of streaming waves
#endif
    uint32_t my_idx = 0, my_y = 0;
    if (tid < k) { my_idx = sh.sel.cand_idx[tid]; my_y = sh.sel.cand_bits[tid]; }
    __syncthreads();  // the selection's LDS is dead from here on
    if (tid < k) {
        sh.itp.idx[tid] = my_idx;
        sh.itp.ys[tid] = (uint16_t)(my_y >= kPrime ? my_y - kPrime : my_y);
    }
    finish_proof<kThreads, KMAX>(sh.itp, coef, k,
                                     reinterpret_cast<uint16_t*>(proofs + chunk * (2 + 2 * (uint64_t)k)), status + chunk);
}

// ---------------------------------------------------------------------------
// Algorithm 2, fused: one pass over the recomputed chunk
// ---------------------------------------------------------------------------
template <int KMAX>
__global__ __launch_bounds__(kThreads, TOPLOC_MIN_WAVES) void verify_kernel(const u32x4* __restrict__ hidden, uint32_t nvec, uint32_t k,
                                                          const uint8_t* __restrict__ proofs, toploc_thresholds thr,
                                                          toploc_verify_result* __restrict__ results)
{
    __shared__ SelShared s;
    __shared__ uint32_t coef[KMAX];
    __shared__ uint32_t hist_d[128];   // err_m as a histogram of |m_p - m_v| in [0, 127]
    __shared__ uint32_t err_e, mant_sum, bad;
    const uint32_t tid = threadIdx.x;
    const uint64_t chunk = blockIdx.x;
    // decode(p)
    const uint16_t* proof = reinterpret_cast<const uint16_t*>(proofs + chunk * (2 + 2 * (uint64_t)k));
    if (tid == 0) { err_e = 0; mant_sum = 0; bad = 0; }
    for (uint32_t b = tid; b < 128; b += kThreads) hist_d[b] = 0;
    __syncthreads();
    const uint32_t mf = proof[0];
    const uint32_t m = mf ? mf : kModHigh;
    for (uint32_t j = tid; j < k; j += kThreads) {
        const uint32_t c = proof[1 + j];
        coef[j] = c;
        if (c >= kPrime) bad = 1u;
    }
    if (tid == 0 && m < kModLow) bad = 1u;
    __syncthreads();
    if (bad) {  // uniform
        if (tid == 0) {
            toploc_verify_result r = {};
            r.status = TOPLOC_CHUNK_MALFORMED;
            results[chunk] = r;
        }
        return;
    }
    // topk(h, k)
    select_topk<kThreads, kLoads, kCap, kQcap>(hidden + chunk * nvec, nvec, k, s);  // order is irrelevant here
    // P(i mod m) by Horner, extractBits, compare
    for (uint32_t j = tid; j < k; j += kThreads) {
        uint32_t x = s.cand_idx[j] % m;
        x = x >= kPrime ? x - kPrime : x;
        uint32_t acc = coef[k - 1];
        for (int i = (int)k - 2; i >= 0; --i) acc = muladdmod(acc, x, coef[i]);
        const uint32_t v = s.cand_bits[j];
        const uint32_t e_p = (acc >> 7) & 0xFFu, m_p = acc & 0x7Fu;
        const uint32_t e_v = (v >> 7) & 0xFFu, m_v = v & 0x7Fu;
        if (e_p == e_v) {
            const uint32_t d = m_p > m_v ? m_p - m_v : m_v - m_p;
            atomicAdd(&hist_d[d], 1u);
            atomicAdd(&mant_sum, d);
        } else {
            atomicAdd(&err_e, 1u);
        }
    }
    __syncthreads();
    if (tid < 64) {
        // |err_m| and its lower median from the histogram: the smallest d whose
        // cumulative count reaches floor((n-1)/2) + 1
        const uint32_t h0 = hist_d[2 * tid], h1 = hist_d[2 * tid + 1];
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
            r.err_exp = err_e;
            r.n_match = n;
            r.mant_sum = mant_sum;
            r.mant_median = n ? med : 0u;
            bool reject = err_e > thr.t_exp;
            if (n) {
                if ((uint64_t)mant_sum > (uint64_t)thr.t_mean * n) reject = true;   // mean(err_m) > T_mean
                if (r.mant_median > thr.t_median) reject = true;
            }
            r.accept = reject ? 0 : 1;
            r.status = TOPLOC_CHUNK_OK;
            results[chunk] = r;
        }
    }
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
static int g_last_hip_error = 0;
static int g_profile_on = 0;
struct ProfRec { int slot; hipEvent_t a, b; };
static std::vector<ProfRec> g_prof;

static bool hip_ok(hipError_t e)
{
    if (e != hipSuccess) { g_last_hip_error = (int)e; return false; }
    return true;
}

struct ProfScope {
    int slot; hipStream_t st; hipEvent_t a = nullptr, b = nullptr; bool on;
    ProfScope(int slot_, hipStream_t st_) : slot(slot_), st(st_), on(g_profile_on != 0)
    {
        if (on) {
            on = hip_ok(hipEventCreate(&a)) && hip_ok(hipEventCreate(&b)) && hip_ok(hipEventRecord(a, st));
        }
    }
    ~ProfScope()
    {
        if (on && hip_ok(hipEventRecord(b, st))) g_prof.push_back({slot, a, b});
    }
};

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// N (values per chunk) when the parameters are usable, else 0
static uint64_t chunk_len(const toploc_params* p)
{
    if (!p || p->k == 0 || p->k > TOPLOC_MAX_K || p->prime != TOPLOC_PRIME) return 0;
    if (p->chunk_tokens == 0 || p->hidden == 0) return 0;
    const uint64_t n = (uint64_t)p->chunk_tokens * p->hidden;
    if (n % 8 != 0 || n >= (1ull << 32) || p->k > n) return 0;
    return n;
}

static size_t idx_bytes(uint64_t n_chunks, uint32_t k)
{
    const size_t b = (size_t)n_chunks * k * sizeof(uint32_t);
    return (b + 15) & ~(size_t)15;
}

}  // namespace toploc

using namespace toploc;

extern "C" {

size_t toploc_proof_bytes(uint32_t k) { return 2 + 2 * (size_t)k; }

size_t toploc_workspace_bytes(const toploc_params* params, uint64_t n_chunks)
{
    if (chunk_len(params) == 0) return 0;
    if (params->k <= 128) return 0;  // one fused kernel, everything stays on chip
    const size_t vb = ((size_t)n_chunks * params->k * sizeof(uint16_t) + 15) & ~(size_t)15;
    return idx_bytes(n_chunks, params->k) + vb;
}

int toploc_topk(const void* d_hidden_bf16, uint64_t n_chunks, const toploc_params* params, uint32_t* d_topk_idx,
                uint16_t* d_topk_val, void* hip_stream)
{
    const uint64_t n = chunk_len(params);
    if (n == 0 || n_chunks >= (1ull << 31)) return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    if (!d_hidden_bf16 || !d_topk_idx || !d_topk_val || !aligned16(d_hidden_bf16)) return TOPLOC_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    {
        ProfScope ps(TOPLOC_KERNEL_SELECT, st);
        hipLaunchKernelGGL(select_kernel, dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                           (const u32x4*)d_hidden_bf16, (uint32_t)(n / 8), params->k, d_topk_idx, d_topk_val,
                           (uint32_t*)nullptr);
    }
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
    const size_t need = toploc_workspace_bytes(params, n_chunks);
    if (need && (!d_workspace || !aligned16(d_workspace))) return TOPLOC_EINVAL;
    if (workspace_bytes < need) return TOPLOC_EWORKSPACE;
    const uint32_t k = params->k;
    hipStream_t st = (hipStream_t)hip_stream;
    if (k <= 128) {
        ProfScope ps(TOPLOC_KERNEL_BUILD, st);
        hipLaunchKernelGGL((build_kernel<128>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                           (const u32x4*)d_hidden_bf16, (uint32_t)(n / 8), k, d_proofs, d_status, d_topk_idx_opt);
        return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
    }
    uint32_t* ws_idx = (uint32_t*)d_workspace;
    uint16_t* ws_val = (uint16_t*)((char*)d_workspace + idx_bytes(n_chunks, k));
    {
        ProfScope ps(TOPLOC_KERNEL_SELECT, st);
        hipLaunchKernelGGL(select_kernel, dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                           (const u32x4*)d_hidden_bf16, (uint32_t)(n / 8), k, ws_idx, ws_val, d_topk_idx_opt);
    }
    if (!hip_ok(hipGetLastError())) return TOPLOC_EHIP;
    {
        ProfScope ps(TOPLOC_KERNEL_INTERP, st);
        hipLaunchKernelGGL((interp_kernel<512>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                           (const uint32_t*)ws_idx, (const uint16_t*)ws_val, k, d_proofs, d_status);
    }
    return hip_ok(hipGetLastError()) ? TOPLOC_OK : TOPLOC_EHIP;
}

int toploc_verify_proofs(const void* d_hidden_bf16, uint64_t n_chunks, const toploc_params* params,
                         const uint8_t* d_proofs, const toploc_thresholds* thresholds, toploc_verify_result* d_results,
                         void* d_workspace, size_t workspace_bytes, void* hip_stream)
{
    (void)d_workspace; (void)workspace_bytes;  // the fused kernel keeps everything on chip
    const uint64_t n = chunk_len(params);
    if (n == 0 || n_chunks >= (1ull << 31) || !thresholds) return TOPLOC_EINVAL;
    if (n_chunks == 0) return TOPLOC_OK;
    if (!d_hidden_bf16 || !d_proofs || !d_results || !aligned16(d_hidden_bf16)) return TOPLOC_EINVAL;
    if ((reinterpret_cast<uintptr_t>(d_proofs) & 1u) != 0 || (reinterpret_cast<uintptr_t>(d_results) & 3u) != 0)
        return TOPLOC_EINVAL;
    const uint32_t k = params->k;
    hipStream_t st = (hipStream_t)hip_stream;
    {
        ProfScope ps(TOPLOC_KERNEL_VERIFY, st);
        if (k <= 128)
            hipLaunchKernelGGL((verify_kernel<128>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden_bf16, (uint32_t)(n / 8), k, d_proofs, *thresholds, d_results);
        else
            hipLaunchKernelGGL((verify_kernel<512>), dim3((uint32_t)n_chunks), dim3(kThreads), 0, st,
                               (const u32x4*)d_hidden_bf16, (uint32_t)(n / 8), k, d_proofs, *thresholds, d_results);
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

#ifdef TOPLOC_TIMING
int toploc_debug_timing(uint64_t* out8, int reset)
{
    if (reset) { uint64_t z[8] = {0,0,0,0,0,0,0,0}; return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_tt), z, sizeof(z)); }
    return (int)hipMemcpyFromSymbol(out8, HIP_SYMBOL(g_tt), 64);
}
#endif

int toploc_profile_enable(int on)
{
    g_profile_on = on ? 1 : 0;
    return TOPLOC_OK;
}

int toploc_profile_read(uint32_t* launches, float* total_ms)
{
    if (!launches || !total_ms) return TOPLOC_EINVAL;
    for (int i = 0; i < TOPLOC_KERNEL_COUNT; ++i) { launches[i] = 0; total_ms[i] = 0.f; }
    int rc = TOPLOC_OK;
    for (auto& r : g_prof) {
        float ms = 0.f;
        if (hip_ok(hipEventSynchronize(r.b)) && hip_ok(hipEventElapsedTime(&ms, r.a, r.b))) {
            launches[r.slot] += 1;
            total_ms[r.slot] += ms;
        } else {
            rc = TOPLOC_EHIP;
        }
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_prof.clear();
    return rc;
}

const char* toploc_strerror(int code)
{
    switch (code) {
    case TOPLOC_OK: return "ok";
    case TOPLOC_EINVAL: return "invalid argument (null or misaligned pointer, k = 0, k > chunk length, k > TOPLOC_MAX_K, "
                               "chunk length not a multiple of 8 or >= 2^32, prime != 65497)";
    case TOPLOC_EWORKSPACE: return "workspace smaller than toploc_workspace_bytes()";
    case TOPLOC_EHIP: return "a HIP runtime call failed (see toploc_last_hip_error)";
    default: return "unknown toploc error code";
    }
}

int toploc_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
