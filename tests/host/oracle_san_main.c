/* Driver that runs the CPU oracle inside a host program built with the address and
 * undefined-behaviour sanitizers (a sanitized shared object cannot be loaded into an
 * unsanitized Python).  It reads one request file, calls the oracle's batch entry points on
 * it, and writes what they returned; the test feeds the same bytes to the ordinary build of
 * the oracle and compares.  Any sanitizer finding ends the program with a report and a
 * non-zero exit status.
 *
 * Request: 16 little-endian uint64 words, then the payload.
 *   word 0 magic 0x544F504C4F43, 1 op, 2 h_dtype (0 bf16, 1 fp32), 3 p_dtype, 4 n_chunks, 5 n,
 *   6 k, 7 M (field modulus; 0 = Algorithm 6 to the letter where the oracle supports it),
 *   8..10 thresholds, 11 threads, 12..15 unused
 *   op 0 build (payload: activations)             -> proofs, status, top-k indices
 *   op 1 verify (payload: activations, proofs)    -> result records
 *   op 2 subroutines on the payload's index sets  -> moduli, status; inverse / Horner sums
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { uint32_t err_exp, n_match, mant_sum, mant_median; uint8_t accept, status, pad[2]; } result_rec;

int toploc_oracle_build(const uint16_t *h, uint64_t n_chunks, uint64_t n, uint32_t k, uint32_t M, uint8_t *proofs,
                        uint8_t *status, uint32_t *topk_idx_opt, int n_threads);
int toploc_oracle_verify(const uint16_t *h, uint64_t n_chunks, uint64_t n, uint32_t k, uint32_t M, const uint8_t *proofs,
                         uint32_t t_exp, uint32_t t_mean, uint32_t t_median, result_rec *results, int n_threads);
int toploc_oracle32_build(const uint32_t *h, uint64_t n_chunks, uint64_t n, uint32_t k, uint64_t M, uint8_t *proofs,
                          uint8_t *status, uint32_t *topk_idx_opt, int n_threads);
int toploc_oracle32_verify(const void *h, int h_dtype, uint64_t n_chunks, uint64_t n, uint32_t k, const uint8_t *proofs,
                           int p_dtype, uint64_t M_proof, uint32_t t_exp, uint32_t t_mean, uint32_t t_median,
                           result_rec *results, int n_threads);
int toploc_oracle_find_injective_modulus_batch(const uint32_t *x, uint64_t n_sets, uint32_t n, uint32_t M, uint32_t *m_out,
                                               uint8_t *status);
int64_t toploc_oracle_mod_inverse(int64_t a, int64_t m, int *err);
int toploc_oracle_interpolate(const int64_t *x, const int64_t *y, uint32_t n, int64_t M, int64_t *c);
int64_t toploc_oracle_horner(const int64_t *c, uint32_t n_coef, int64_t x, int64_t M);

static void die(const char *what) { fprintf(stderr, "oracle_san: %s\n", what); exit(2); }

static void *read_all(const char *path, size_t *size)
{
    FILE *f = fopen(path, "rb");
    if (!f) die("cannot open the request");
    fseek(f, 0, SEEK_END);
    long len = ftell(f);
    fseek(f, 0, SEEK_SET);
    void *buf = malloc((size_t)len + 1);
    if (!buf || fread(buf, 1, (size_t)len, f) != (size_t)len) die("cannot read the request");
    fclose(f);
    *size = (size_t)len;
    return buf;
}

int main(int argc, char **argv)
{
    if (argc != 3) die("usage: oracle_san request result");
    size_t size = 0;
    uint8_t *req = (uint8_t *)read_all(argv[1], &size);
    if (size < 128) die("short request");
    uint64_t w[16];
    memcpy(w, req, sizeof(w));
    if (w[0] != 0x544F504C4F43ull) die("bad magic");
    const uint64_t op = w[1], n_chunks = w[4], n = w[5], M = w[7];
    const int h_dt = (int)w[2], p_dt = (int)w[3], threads = (int)w[11];
    const uint32_t k = (uint32_t)w[6];
    const uint8_t *payload = req + 128;
    const size_t payload_size = size - 128;
    const size_t h_elem = h_dt ? 4 : 2, pb = 2 + (size_t)k * (p_dt ? 4 : 2);
    FILE *out = fopen(argv[2], "wb");
    if (!out) die("cannot open the result");
    int rc = 0;
    if (op == 0) {
        if (payload_size != n_chunks * n * h_elem) die("build: payload size");
        /* exact-size copies, so that a read or write one element past an array is seen */
        void *h = malloc(n_chunks * n * h_elem + 1);
        memcpy(h, payload, n_chunks * n * h_elem);
        uint8_t *proofs = (uint8_t *)malloc(n_chunks * pb + 1), *status = (uint8_t *)malloc(n_chunks + 1);
        uint32_t *idx = (uint32_t *)malloc(n_chunks * k * sizeof(uint32_t) + 4);
        memset(proofs, 0, n_chunks * pb);
        rc = h_dt ? toploc_oracle32_build((const uint32_t *)h, n_chunks, n, k, M, proofs, status, idx, threads)
                  : toploc_oracle_build((const uint16_t *)h, n_chunks, n, k, (uint32_t)M, proofs, status, idx, threads);
        fwrite(&rc, sizeof(rc), 1, out);
        fwrite(proofs, 1, n_chunks * pb, out);
        fwrite(status, 1, n_chunks, out);
        fwrite(idx, sizeof(uint32_t), n_chunks * k, out);
        free(h); free(proofs); free(status); free(idx);
    } else if (op == 1) {
        if (payload_size != n_chunks * n * h_elem + n_chunks * pb) die("verify: payload size");
        void *h = malloc(n_chunks * n * h_elem + 1);
        memcpy(h, payload, n_chunks * n * h_elem);
        uint8_t *proofs = (uint8_t *)malloc(n_chunks * pb + 1);
        memcpy(proofs, payload + n_chunks * n * h_elem, n_chunks * pb);
        result_rec *res = (result_rec *)calloc(n_chunks + 1, sizeof(result_rec));
        if (h_dt == 0 && p_dt == 0 && w[12] == 0)
            rc = toploc_oracle_verify((const uint16_t *)h, n_chunks, n, k, (uint32_t)M, proofs, (uint32_t)w[8], (uint32_t)w[9],
                                      (uint32_t)w[10], res, threads);
        else
            rc = toploc_oracle32_verify(h, h_dt, n_chunks, n, k, proofs, p_dt, M, (uint32_t)w[8], (uint32_t)w[9],
                                        (uint32_t)w[10], res, threads);
        fwrite(&rc, sizeof(rc), 1, out);
        fwrite(res, sizeof(result_rec), n_chunks, out);
        free(h); free(proofs); free(res);
    } else if (op == 2) {
        /* payload: n_chunks index sets of k uint32 each */
        if (payload_size != n_chunks * k * sizeof(uint32_t)) die("subroutines: payload size");
        uint32_t *sets = (uint32_t *)malloc(n_chunks * k * sizeof(uint32_t) + 4);
        memcpy(sets, payload, n_chunks * k * sizeof(uint32_t));
        uint32_t *m_out = (uint32_t *)malloc(n_chunks * sizeof(uint32_t) + 4);
        uint8_t *st = (uint8_t *)malloc(n_chunks + 1);
        rc = toploc_oracle_find_injective_modulus_batch(sets, n_chunks, k, (uint32_t)M, m_out, st);
        fwrite(&rc, sizeof(rc), 1, out);
        fwrite(m_out, sizeof(uint32_t), n_chunks, out);
        fwrite(st, 1, n_chunks, out);
        /* Algorithm 4 over every residue of GF(65497) and its two special exits; Algorithm 3 and 5
         * on the first set's residues as points: P(x_j) must give y_j back */
        int64_t inv_sum = 0;
        int err = 0;
        for (int64_t a = 1; a < 65497; ++a) inv_sum += toploc_oracle_mod_inverse(a, 65497, &err) * a % 65497;
        inv_sum += toploc_oracle_mod_inverse(5, 1, &err);
        (void)toploc_oracle_mod_inverse(6, 9, &err);
        inv_sum += err;
        fwrite(&inv_sum, sizeof(inv_sum), 1, out);
        if (n_chunks && st[0] == 0) {
            int64_t *x = (int64_t *)malloc(sizeof(int64_t) * k), *y = (int64_t *)malloc(sizeof(int64_t) * k);
            int64_t *c = (int64_t *)malloc(sizeof(int64_t) * k);
            for (uint32_t j = 0; j < k; ++j) { x[j] = (sets[j] % m_out[0]) % 65497; y[j] = (sets[j] * 2654435761u >> 16) % 65497; }
            int irc = toploc_oracle_interpolate(x, y, k, 65497, c);
            int64_t bad = irc;
            for (uint32_t j = 0; j < k && irc == 0; ++j) bad += toploc_oracle_horner(c, k, x[j], 65497) != y[j];
            fwrite(&bad, sizeof(bad), 1, out);
            fwrite(c, sizeof(int64_t), k, out);
            free(x); free(y); free(c);
        }
        free(sets); free(m_out); free(st);
    } else {
        die("unknown op");
    }
    fclose(out);
    free(req);
    return 0;
}
