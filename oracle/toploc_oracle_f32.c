/*
 * TopLoc CPU oracle, 32-bit variant -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * Proof generation over fp32 hidden states and proof validation across the two
 * precisions of the paper's precision study (Section 5.7, Table 5; fp32 thresholds
 * in Section 5.2).  Same rules as toploc_oracle.c: plain, slow, step by step, the
 * paper's order and notation (Algorithms 1-6), a full qsort for top-k and for the
 * median, exact integer arithmetic (unsigned 128-bit products where a 64-bit one
 * would overflow).  Shares no code with the GPU path and must never be called from it.
 *
 * Readings (the paper leaves all of this open; each is listed in the design notes):
 *   - an fp32 value enters the polynomial as its 32-bit pattern; the modulus M of
 *     Algorithms 3 and 5 is the prime 4294967291 = 2^32 - 5 (Appendix C bounds M by
 *     2^32 for 32-bit types); the 5 patterns >= M (negative NaNs) are taken mod M.
 *   - top-k ranks by magnitude: key = bits & 0x7FFFFFFF as an unsigned integer, ties
 *     to the lower flat index, output order (magnitude desc, index asc).
 *   - Algorithm 6 to the letter: residues j mod i with i <= 65536 < M are already
 *     field elements, so distinct residues are distinct in the field.
 *   - proof bytes: [0..1] = m mod 65536 little endian (0 stands for 65536), then the k
 *     coefficients c_0..c_{k-1}, 4 bytes each, little endian: 2 + 4k bytes.
 *   - extractBits of a 32-bit pattern: exponent = bits 30..23, mantissa = bits 22..0;
 *     of a 16-bit (bf16) pattern: exponent = bits 14..7, mantissa = bits 6..0.
 *   - validating an fp32 proof with bf16 activations: the proof's mantissa is scaled to
 *     bf16's width, m_p = mantissa23 >> 16, and compared with the bf16 mantissa
 *     (Section 5.7 scales the fp32 mantissa to bf16's width for a bf16 validator).
 *   - validating a bf16 proof with fp32 activations: the proof's value gets 16 zero
 *     bits appended, m_p = mantissa7 << 16, and is compared with the fp32 mantissa
 *     (Section 5.7 pads the bf16 representation with 16 zero bits for an fp32 validator).
 *   - decision rule as in toploc_oracle.c: sum > T_mean * n, lower median, an empty
 *     err_m fails neither mantissa test.
 *
 * Pins (tests/test_oracle_f32_pins.py): round trip P(x_j) = y_j; the interpolation
 * against Lagrange sums in Python integers; small-prime exhaustive cases shared with
 * the 16-bit routine (same M gives the same coefficients); brute-force top-k; the
 * cross-precision identities (a bf16 proof of bf16(x) validated against fp32 x gives
 * |m_p - m_v| = distance to the rounded value); Table 5's qualitative outcome on
 * synthetic data.  Proof bytes are printed nowhere in the paper: parity unpinned for
 * the byte layout itself.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ENOMOD 1
#define ORACLE_ENOINV 2
#define ORACLE_EMALFORMED 3
#define ORACLE_EARG (-1)

#define DTYPE_BF16 0
#define DTYPE_F32 1

typedef unsigned __int128 u128;

typedef struct {
    uint32_t err_exp, n_match, mant_sum, mant_median;
    uint8_t accept, status, pad[2];
} oracle32_verify_result;

/* ------------------------------------------------------------------------- */
/* topk(h, k) by magnitude over 32-bit or 16-bit patterns                      */
/* ------------------------------------------------------------------------- */
typedef struct { uint32_t mag; uint32_t idx; } okey;

static int okey_cmp(const void *pa, const void *pb)
{
    const okey *a = (const okey *)pa, *b = (const okey *)pb;
    if (a->mag != b->mag) return (a->mag > b->mag) ? -1 : 1;
    if (a->idx != b->idx) return (a->idx < b->idx) ? -1 : 1;
    return 0;
}

/* h: n patterns of the given dtype; val_out receives the patterns widened to 32 bit */
int toploc_oracle32_topk(const void *h, int dtype, uint64_t n, uint32_t k, uint32_t *idx_out, uint32_t *val_out)
{
    if (k == 0 || k > n || n > 0xFFFFFFFFull) return ORACLE_EARG;
    okey *keys = (okey *)malloc((size_t)n * sizeof(okey));
    if (!keys) return ORACLE_EARG;
    for (uint64_t i = 0; i < n; ++i) {
        keys[i].mag = dtype == DTYPE_F32 ? (((const uint32_t *)h)[i] & 0x7FFFFFFFu)
                                         : (uint32_t)(((const uint16_t *)h)[i] & 0x7FFFu);
        keys[i].idx = (uint32_t)i;
    }
    qsort(keys, (size_t)n, sizeof(okey), okey_cmp);
    for (uint32_t j = 0; j < k; ++j) {
        idx_out[j] = keys[j].idx;
        val_out[j] = dtype == DTYPE_F32 ? ((const uint32_t *)h)[keys[j].idx] : (uint32_t)((const uint16_t *)h)[keys[j].idx];
    }
    free(keys);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 4 (extended Euclid), operands below 2^33: signed 64 bit suffices  */
/* ------------------------------------------------------------------------- */
static int64_t safe_mod64(int64_t s, int64_t m) { return ((s % m) + m) % m; }

int64_t toploc_oracle32_mod_inverse(int64_t a, int64_t m, int *err)
{
    *err = ORACLE_OK;
    if (m <= 1) return 0;
    int64_t old_r = a, r = m, old_s = 1, s = 0;
    while (r != 0) {
        int64_t q = old_r / r;
        int64_t tmp_r = old_r - q * r; old_r = r; r = tmp_r;
        int64_t tmp_s = old_s - q * s; old_s = s; s = tmp_s;   /* |s| stays below m */
    }
    if (old_r != 1) { *err = ORACLE_ENOINV; return 0; }
    return safe_mod64(old_s, m);
}

static uint64_t mulmod(uint64_t a, uint64_t b, uint64_t M) { return (uint64_t)(((u128)a * b) % M); }

/* ------------------------------------------------------------------------- */
/* Algorithm 3 for a modulus up to 2^32: x, y, c are residues in [0, M)        */
/* ------------------------------------------------------------------------- */
int toploc_oracle32_interpolate(const uint64_t *x, const uint64_t *y, uint32_t n, uint64_t M, uint64_t *c)
{
    if (n == 0 || M <= 1 || M > (1ull << 32)) return ORACLE_EARG;
    uint64_t *dd = (uint64_t *)malloc(sizeof(uint64_t) * n);
    uint64_t *factor = (uint64_t *)malloc(sizeof(uint64_t) * n);
    if (!dd || !factor) { free(dd); free(factor); return ORACLE_EARG; }
    for (uint32_t i = 0; i < n; ++i) dd[i] = y[i] % M;
    for (uint32_t k = 1; k + 1 <= n; ++k) {                      /* divided differences */
        for (uint32_t i = n - 1; i >= k; --i) {
            uint64_t numerator = (dd[i] + M - dd[i - 1]) % M;
            uint64_t denominator = (x[i] % M + M - x[i - k] % M) % M;
            int err;
            int64_t inv = toploc_oracle32_mod_inverse((int64_t)denominator, (int64_t)M, &err);
            if (err) { free(dd); free(factor); return ORACLE_ENOINV; }
            dd[i] = mulmod(numerator, (uint64_t)inv, M);
        }
    }
    for (uint32_t i = 0; i < n; ++i) { c[i] = 0; factor[i] = 0; }   /* Newton form -> standard form */
    factor[0] = 1 % M;
    for (uint32_t i = 0; i < n; ++i) {
        for (uint32_t j = 0; j <= i; ++j) c[j] = (c[j] + mulmod(dd[i], factor[j], M)) % M;
        if (i + 1 < n) {
            uint64_t neg_xi = (M - x[i] % M) % M;
            for (uint32_t d = i + 1; d >= 1; --d) factor[d] = (factor[d - 1] + mulmod(factor[d], neg_xi, M)) % M;
            factor[0] = mulmod(factor[0], neg_xi, M);
        }
    }
    free(dd);
    free(factor);
    return ORACLE_OK;
}

/* Algorithm 5 */
uint64_t toploc_oracle32_horner(const uint64_t *c, uint32_t n_coef, uint64_t x, uint64_t M)
{
    uint64_t result = c[n_coef - 1] % M;
    for (uint32_t i = 1; i < n_coef; ++i) result = (mulmod(result, x % M, M) + c[n_coef - 1 - i]) % M;
    return result;
}

/* Algorithm 6 to the letter */
static int u32_cmp(const void *pa, const void *pb)
{
    uint32_t a = *(const uint32_t *)pa, b = *(const uint32_t *)pb;
    return (a > b) - (a < b);
}

int toploc_oracle32_find_injective_modulus(const uint32_t *x, uint32_t n, uint32_t *m_out)
{
    if (n == 0) return ORACLE_EARG;
    uint32_t *S = (uint32_t *)malloc(sizeof(uint32_t) * n);
    if (!S) return ORACLE_EARG;
    for (uint32_t i = 65536u; i >= 32769u; --i) {
        for (uint32_t t = 0; t < n; ++t) S[t] = x[t] % i;
        qsort(S, n, sizeof(uint32_t), u32_cmp);
        uint32_t distinct = 1;
        for (uint32_t t = 1; t < n; ++t) distinct += (S[t] != S[t - 1]);
        if (distinct == n) { *m_out = i; free(S); return ORACLE_OK; }
    }
    free(S);
    return ORACLE_ENOMOD;
}

/* ------------------------------------------------------------------------- */
/* proof bytes: coefficient width 4 (fp32 proof) or 2 (bf16 proof)             */
/* ------------------------------------------------------------------------- */
static size_t proof_bytes(uint32_t k, int dtype) { return 2 + (size_t)k * (dtype == DTYPE_F32 ? 4 : 2); }

static int decode(const uint8_t *p, uint32_t k, int dtype, uint64_t M, uint32_t *m, uint64_t *c)
{
    uint32_t mf = (uint32_t)p[0] | ((uint32_t)p[1] << 8);
    *m = mf ? mf : 65536u;
    int bad = (*m < 32769u);
    const int w = dtype == DTYPE_F32 ? 4 : 2;
    for (uint32_t j = 0; j < k; ++j) {
        uint64_t v = 0;
        for (int b = 0; b < w; ++b) v |= (uint64_t)p[2 + w * j + b] << (8 * b);
        c[j] = v;
        if (v >= M) bad = 1;
    }
    return bad ? ORACLE_EMALFORMED : ORACLE_OK;
}

/* Algorithm 1 on one chunk of fp32 patterns */
int toploc_oracle32_build_chunk(const uint32_t *h, uint64_t n, uint32_t k, uint64_t M, uint8_t *proof,
                                uint32_t *topk_idx_opt)
{
    uint32_t *i = (uint32_t *)malloc(sizeof(uint32_t) * k);
    uint32_t *v = (uint32_t *)malloc(sizeof(uint32_t) * k);
    uint64_t *i_m = (uint64_t *)malloc(sizeof(uint64_t) * k);
    uint64_t *y = (uint64_t *)malloc(sizeof(uint64_t) * k);
    uint64_t *c = (uint64_t *)malloc(sizeof(uint64_t) * k);
    int rc = ORACLE_EARG;
    if (!i || !v || !i_m || !y || !c) goto done;
    memset(proof, 0, proof_bytes(k, DTYPE_F32));
    rc = toploc_oracle32_topk(h, DTYPE_F32, n, k, i, v);             /* (i, v) <- topk(h, k) */
    if (rc) goto done;
    if (topk_idx_opt) memcpy(topk_idx_opt, i, sizeof(uint32_t) * k);
    uint32_t m;
    rc = toploc_oracle32_find_injective_modulus(i, k, &m);            /* m <- findInjectiveModulus(i) */
    if (rc) goto done;
    for (uint32_t j = 0; j < k; ++j) { i_m[j] = i[j] % m; y[j] = v[j]; }   /* i_m <- i mod m */
    rc = toploc_oracle32_interpolate(i_m, y, k, M, c);                /* P(x) */
    if (rc) goto done;
    uint32_t mf = m % 65536u;                                         /* p <- encode(m, P) */
    proof[0] = (uint8_t)(mf & 0xFF);
    proof[1] = (uint8_t)(mf >> 8);
    for (uint32_t j = 0; j < k; ++j)
        for (int b = 0; b < 4; ++b) proof[2 + 4 * j + b] = (uint8_t)((c[j] >> (8 * b)) & 0xFF);
done:
    free(i); free(v); free(i_m); free(y); free(c);
    return rc;
}

/* extractBits in the validator's precision.  `bits` is a pattern of `from` precision
 * (a proof value or an activation); the pair (e, m) comes out in `to` precision. */
static void extract_bits(uint32_t bits, int from, int to, uint32_t *e, uint32_t *mant)
{
    uint32_t e8, m;
    if (from == DTYPE_F32) { e8 = (bits >> 23) & 0xFFu; m = bits & 0x7FFFFFu; }
    else                   { e8 = (bits >> 7) & 0xFFu;  m = bits & 0x7Fu; }
    if (from == DTYPE_F32 && to == DTYPE_BF16) m >>= 16;        /* fp32 mantissa scaled to bf16's 7 bits */
    if (from == DTYPE_BF16 && to == DTYPE_F32) m <<= 16;        /* 16 zero bits appended                 */
    *e = e8;
    *mant = m;
}

/* Algorithm 2 on one chunk: activations of h_dtype, proof of p_dtype; comparisons in
 * the validator's (h_dtype's) precision. */
int toploc_oracle32_verify_chunk(const void *h, int h_dtype, uint64_t n, uint32_t k, const uint8_t *proof, int p_dtype,
                                 uint64_t M_proof, uint32_t t_exp, uint32_t t_mean, uint32_t t_median,
                                 oracle32_verify_result *res)
{
    memset(res, 0, sizeof(*res));
    uint32_t *i = (uint32_t *)malloc(sizeof(uint32_t) * k);
    uint32_t *v = (uint32_t *)malloc(sizeof(uint32_t) * k);
    uint64_t *c = (uint64_t *)malloc(sizeof(uint64_t) * k);
    uint32_t *err_m = (uint32_t *)malloc(sizeof(uint32_t) * k);
    int rc = ORACLE_EARG;
    if (!i || !v || !c || !err_m) goto done;
    uint32_t m;
    rc = decode(proof, k, p_dtype, M_proof, &m, c);                   /* k, m, P <- decode(p) */
    if (rc == ORACLE_EMALFORMED) { res->status = ORACLE_EMALFORMED; rc = ORACLE_OK; goto done; }
    rc = toploc_oracle32_topk(h, h_dtype, n, k, i, v);                /* (i, v) <- topk(h, k) */
    if (rc) goto done;
    uint32_t err_e = 0, n_m = 0;
    uint64_t sum = 0;
    for (uint32_t j = 0; j < k; ++j) {
        uint64_t i_m = i[j] % m;                                      /* i_m <- i mod m */
        uint32_t P = (uint32_t)toploc_oracle32_horner(c, k, i_m, M_proof);
        uint32_t e_p, m_p, e_v, m_v;
        extract_bits(P, p_dtype, h_dtype, &e_p, &m_p);
        extract_bits(v[j], h_dtype, h_dtype, &e_v, &m_v);
        if (e_p == e_v) { err_m[n_m] = m_p > m_v ? m_p - m_v : m_v - m_p; sum += err_m[n_m]; n_m++; }
        else err_e += 1;
    }
    uint32_t median = 0;
    if (n_m) { qsort(err_m, n_m, sizeof(uint32_t), u32_cmp); median = err_m[(n_m - 1) / 2]; }
    int reject = (err_e > t_exp);
    if (n_m) {
        if (sum > (uint64_t)t_mean * n_m) reject = 1;
        if (median > t_median) reject = 1;
    }
    res->err_exp = err_e;
    res->n_match = n_m;
    res->mant_sum = (uint32_t)sum;      /* k * (2^23 - 1) < 2^32 for k <= 512 */
    res->mant_median = median;
    res->accept = (uint8_t)(!reject);
    rc = ORACLE_OK;
done:
    free(i); free(v); free(c); free(err_m);
    return rc;
}

/* batches: one chunk per task */
int toploc_oracle32_build(const uint32_t *h, uint64_t n_chunks, uint64_t n, uint32_t k, uint64_t M, uint8_t *proofs,
                          uint8_t *status, uint32_t *topk_idx_opt, int n_threads)
{
    if (k == 0 || k > n) return ORACLE_EARG;
    const size_t pb = proof_bytes(k, DTYPE_F32);
    int bad = 0;
    (void)n_threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads > 0 ? n_threads : 1)
#endif
    for (int64_t cidx = 0; cidx < (int64_t)n_chunks; ++cidx) {
        int rc = toploc_oracle32_build_chunk(h + (size_t)cidx * n, n, k, M, proofs + (size_t)cidx * pb,
                                             topk_idx_opt ? topk_idx_opt + (size_t)cidx * k : NULL);
        if (rc < 0) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            bad = 1;
            status[cidx] = 255;
        } else {
            status[cidx] = (uint8_t)rc;
        }
    }
    return bad ? ORACLE_EARG : ORACLE_OK;
}

int toploc_oracle32_verify(const void *h, int h_dtype, uint64_t n_chunks, uint64_t n, uint32_t k, const uint8_t *proofs,
                           int p_dtype, uint64_t M_proof, uint32_t t_exp, uint32_t t_mean, uint32_t t_median,
                           oracle32_verify_result *results, int n_threads)
{
    if (k == 0 || k > n) return ORACLE_EARG;
    const size_t pb = proof_bytes(k, p_dtype);
    const size_t es = h_dtype == DTYPE_F32 ? 4 : 2;
    int bad = 0;
    (void)n_threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads > 0 ? n_threads : 1)
#endif
    for (int64_t cidx = 0; cidx < (int64_t)n_chunks; ++cidx) {
        int rc = toploc_oracle32_verify_chunk((const uint8_t *)h + (size_t)cidx * n * es, h_dtype, n, k,
                                              proofs + (size_t)cidx * pb, p_dtype, M_proof, t_exp, t_mean, t_median,
                                              &results[cidx]);
        if (rc != ORACLE_OK) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            bad = 1;
        }
    }
    return bad ? ORACLE_EARG : ORACLE_OK;
}
