/*
 * The C ABI used from plain C, without Python or PyTorch: device memory from the HIP
 * runtime, toploc_build_proofs / toploc_verify_proofs / toploc_topk through include/toploc.h,
 * and the CPU oracle (linked directly, this is a test) as the reference.  Prints one line per
 * check and exits 0 when every byte matches.
 *
 * Built by tests/cabi/build_cabi.py with gcc (host code only).
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "toploc.h"

/* the oracle's entry points (oracle/toploc_oracle.c) */
int toploc_oracle_build(const uint16_t *h, uint64_t n_chunks, uint64_t n, uint32_t k, uint32_t M, uint8_t *proofs,
                        uint8_t *status, uint32_t *topk_idx_opt, int n_threads);
int toploc_oracle_verify(const uint16_t *h, uint64_t n_chunks, uint64_t n, uint32_t k, uint32_t M, const uint8_t *proofs,
                         uint32_t t_exp, uint32_t t_mean, uint32_t t_median, toploc_verify_result *results, int n_threads);

#define CK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
    fprintf(stderr, "HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__); return 2; } } while (0)
#define TL(call) do { int rc_ = (call); if (rc_ != TOPLOC_OK) { \
    fprintf(stderr, "toploc error %d (%s) at line %d\n", rc_, toploc_strerror(rc_), __LINE__); return 3; } } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}

int main(void)
{
    const uint32_t k = 128, tokens = 32, hidden = 1024;
    const uint64_t n_chunks = 12, n = (uint64_t)tokens * hidden;
    const size_t pb = toploc_proof_bytes(k);
    if (pb != 258) { fprintf(stderr, "proof size %zu\n", pb); return 1; }

    /* finite bf16 patterns: small magnitudes everywhere, 8 channels of large ones */
    uint16_t *h = (uint16_t *)malloc(n_chunks * n * 2);
    uint16_t *rec = (uint16_t *)malloc(n_chunks * n * 2);
    for (uint64_t i = 0; i < n_chunks * n; ++i) {
        const uint32_t r = rnd();
        const uint32_t c = (uint32_t)(i % hidden);
        const uint32_t mag = (c % 128 == 5) ? 0x4100u + (r % 0x300u) : 0x3000u + (r % 0x0F00u);
        h[i] = (uint16_t)(mag | ((r >> 31) << 15));
        rec[i] = (uint16_t)(h[i] ^ ((r >> 8) % 97 == 0 ? 1u : 0u));   /* a few one-ulp moves */
    }

    void *d_h, *d_rec; uint8_t *d_proofs, *d_status; uint32_t *d_idx; uint16_t *d_val; toploc_verify_result *d_res;
    CK(hipMalloc(&d_h, n_chunks * n * 2));
    CK(hipMalloc(&d_rec, n_chunks * n * 2));
    CK(hipMalloc((void **)&d_proofs, n_chunks * pb));
    CK(hipMalloc((void **)&d_status, n_chunks));
    CK(hipMalloc((void **)&d_idx, n_chunks * k * 4));
    CK(hipMalloc((void **)&d_val, n_chunks * k * 2));
    CK(hipMalloc((void **)&d_res, n_chunks * sizeof(toploc_verify_result)));
    CK(hipMemcpy(d_h, h, n_chunks * n * 2, hipMemcpyHostToDevice));
    CK(hipMemcpy(d_rec, rec, n_chunks * n * 2, hipMemcpyHostToDevice));

    const toploc_params params = {k, tokens, hidden, TOPLOC_PRIME};
    const toploc_thresholds thr = {38, 10, 8};
    const size_t ws_bytes = toploc_workspace_bytes(&params, n_chunks);
    void *d_ws = NULL;
    if (ws_bytes) CK(hipMalloc(&d_ws, ws_bytes));
    TL(toploc_build_proofs(d_h, n_chunks, &params, d_proofs, d_status, d_idx, d_ws, ws_bytes, NULL));
    TL(toploc_verify_proofs(d_rec, n_chunks, &params, d_proofs, &thr, d_res, d_ws, ws_bytes, NULL));
    TL(toploc_topk(d_h, n_chunks, &params, d_idx, d_val, NULL));
    CK(hipDeviceSynchronize());

    uint8_t *proofs = (uint8_t *)malloc(n_chunks * pb), *status = (uint8_t *)malloc(n_chunks);
    uint32_t *idx = (uint32_t *)malloc(n_chunks * k * 4);
    toploc_verify_result *res = (toploc_verify_result *)malloc(n_chunks * sizeof(*res));
    CK(hipMemcpy(proofs, d_proofs, n_chunks * pb, hipMemcpyDeviceToHost));
    CK(hipMemcpy(status, d_status, n_chunks, hipMemcpyDeviceToHost));
    CK(hipMemcpy(idx, d_idx, n_chunks * k * 4, hipMemcpyDeviceToHost));
    CK(hipMemcpy(res, d_res, n_chunks * sizeof(*res), hipMemcpyDeviceToHost));

    uint8_t *o_proofs = (uint8_t *)malloc(n_chunks * pb), *o_status = (uint8_t *)malloc(n_chunks);
    uint32_t *o_idx = (uint32_t *)malloc(n_chunks * k * 4);
    toploc_verify_result *o_res = (toploc_verify_result *)calloc(n_chunks, sizeof(*o_res));
    if (toploc_oracle_build(h, n_chunks, n, k, TOPLOC_PRIME, o_proofs, o_status, o_idx, 4)) return 4;
    if (toploc_oracle_verify(rec, n_chunks, n, k, TOPLOC_PRIME, o_proofs, 38, 10, 8, o_res, 4)) return 4;

    int bad = 0;
    bad |= memcmp(proofs, o_proofs, n_chunks * pb) != 0;       printf("proof bytes   %s\n", bad ? "DIFFER" : "equal");
    int b2 = memcmp(status, o_status, n_chunks) != 0;          printf("status        %s\n", b2 ? "DIFFER" : "equal");
    int b3 = memcmp(idx, o_idx, n_chunks * k * 4) != 0;        printf("top-k indices %s\n", b3 ? "DIFFER" : "equal");
    int b4 = 0;
    for (uint64_t c = 0; c < n_chunks; ++c)
        b4 |= res[c].err_exp != o_res[c].err_exp || res[c].n_match != o_res[c].n_match || res[c].mant_sum != o_res[c].mant_sum ||
              res[c].mant_median != o_res[c].mant_median || res[c].accept != o_res[c].accept || res[c].status != o_res[c].status;
    printf("verify records %s (chunk 0: err_e %u, n %u, sum %u, median %u, accept %u)\n", b4 ? "DIFFER" : "equal",
           res[0].err_exp, res[0].n_match, res[0].mant_sum, res[0].mant_median, res[0].accept);
    bad |= b2 | b3 | b4;
    printf(bad ? "cabi FAILED\n" : "cabi ok\n");
    return bad ? 1 : 0;
}
