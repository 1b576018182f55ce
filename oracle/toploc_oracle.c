/*
 * TopLoc CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, step-by-step CPU implementation of proof generation and
 * proof validation as the paper states them (Section 4, Algorithms 1 and 2,
 * and the subroutines of Appendix C, Algorithms 3-6).  It exists only so that
 * tests, the smoke check and the benchmark's cpu_baseline leg can compare the
 * GPU library against it.  It shares no code with the GPU path and must never
 * be called from it.
 *
 * Every function follows the paper's steps in the paper's order and notation.
 * Library primitives used as steps: qsort (a full sort for top-k and for the
 * median), nothing else.  All arithmetic is exact integer arithmetic in
 * signed 64 bit; bf16 values are handled as their 16-bit patterns.
 *
 * Readings of points the paper leaves open (each is listed with its reason in
 * the design notes of this repository):
 *   - top-k ranks by magnitude (Section 5.3 speaks of the k elements of largest magnitude):
 *     key = bits & 0x7FFF compared as an unsigned integer; ties go to the
 *     lower flat index; output order is (magnitude desc, index asc).
 *   - the polynomial modulus M of Algorithms 3 and 5 is the prime 65497.
 *   - Algorithm 6 accepts a candidate modulus i when the residues j mod i are
 *     distinct AFTER reduction mod M as well (otherwise Algorithm 3 would meet
 *     a zero denominator).  With M = 0 the routine is Algorithm 6 to the letter.
 *   - proof bytes: [0..1] = m mod 65536 little endian (0 stands for 65536),
 *     then the k coefficients c_0..c_{k-1} (ascending power), 2 bytes each,
 *     little endian: 2 + 2k bytes (Sections 1, 5.8, 7: 258 bytes for k = 128).
 *   - extractBits: exponent = bits 14..7, mantissa = bits 6..0; the sign is not
 *     compared (Algorithm 2 extracts only exponent and mantissa).
 *   - mean(err_m) > T  is tested as  sum > T * n  in integers; median is the
 *     lower median sorted[(n-1)/2]; with err_m empty both tests are false.
 *
 * Pins (tests/test_oracle_pins.py): round trip P(x_j) = y_j; uniqueness against
 * Lagrange / Gaussian elimination written in Python; injectivity and maximality
 * of m; the appendix's distribution of return values against the closed-form birthday product and
 * the paper's printed values; 258-byte size; brute-force top-k on tiny inputs;
 * Algorithm 4 against Fermat's little theorem; verification identities.
 * The actual proof BYTES of a tensor are printed nowhere in the paper, so the
 * byte layout above is a convention of this build: parity unpinned for the
 * layout itself (everything the layout carries is pinned).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ENOMOD 1      /* Algorithm 6: no injective modulus found          */
#define ORACLE_ENOINV 2      /* Algorithm 4: gcd(a, m) != 1                      */
#define ORACLE_EMALFORMED 3  /* decode: modulus or a coefficient out of range    */
#define ORACLE_EARG (-1)

typedef struct {
    uint32_t err_exp;      /* err_e of Algorithm 2                               */
    uint32_t n_match;      /* |err_m|                                            */
    uint32_t mant_sum;     /* sum of err_m                                       */
    uint32_t mant_median;  /* lower median of err_m (0 when empty)               */
    uint8_t accept;        /* the Boolean of Algorithm 2                         */
    uint8_t status;        /* ORACLE_OK or ORACLE_EMALFORMED                     */
    uint8_t pad[2];
} oracle_verify_result;

/* ------------------------------------------------------------------------- */
/* topk(h, k): Algorithm 1 step 1 / Algorithm 2 step 2, by magnitude          */
/* ------------------------------------------------------------------------- */
typedef struct { uint32_t mag; uint32_t idx; } oracle_key;

static int oracle_key_cmp(const void *pa, const void *pb)
{
    const oracle_key *a = (const oracle_key *)pa, *b = (const oracle_key *)pb;
    if (a->mag != b->mag) return (a->mag > b->mag) ? -1 : 1;   /* larger |h| first */
    if (a->idx != b->idx) return (a->idx < b->idx) ? -1 : 1;   /* then lower index */
    return 0;
}

int toploc_oracle_topk(const uint16_t *h, uint64_t n, uint32_t k,
                       uint32_t *idx_out, uint16_t *val_out)
{
    if (k == 0 || k > n || n > 0xFFFFFFFFull) return ORACLE_EARG;
    oracle_key *keys = (oracle_key *)malloc((size_t)n * sizeof(oracle_key));
    if (!keys) return ORACLE_EARG;
    for (uint64_t i = 0; i < n; ++i) {
        keys[i].mag = (uint32_t)(h[i] & 0x7FFFu);
        keys[i].idx = (uint32_t)i;
    }
    qsort(keys, (size_t)n, sizeof(oracle_key), oracle_key_cmp);
    for (uint32_t j = 0; j < k; ++j) {
        idx_out[j] = keys[j].idx;
        val_out[j] = h[keys[j].idx];
    }
    free(keys);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 4: modular inverse by the extended Euclidean algorithm           */
/* ------------------------------------------------------------------------- */
static int64_t oracle_safe_mod(int64_t s, int64_t m)
{
    return ((s % m) + m) % m;
}

int64_t toploc_oracle_mod_inverse(int64_t a, int64_t m, int *err)
{
    *err = ORACLE_OK;
    if (m <= 1) return 0;
    int64_t old_r = a, r = m;
    int64_t old_s = 1, s = 0;
    while (r != 0) {
        int64_t q = old_r / r;          /* operands are non-negative here: floor */
        int64_t tmp_r = old_r - q * r;
        old_r = r;
        r = tmp_r;
        int64_t tmp_s = old_s - q * s;
        old_s = s;
        s = tmp_s;
    }
    if (old_r != 1) { *err = ORACLE_ENOINV; return 0; }
    return oracle_safe_mod(old_s, m);
}

/* ------------------------------------------------------------------------- */
/* Algorithm 3: Newton polynomial congruence interpolation                    */
/* ------------------------------------------------------------------------- */
int toploc_oracle_interpolate(const int64_t *x, const int64_t *y, uint32_t n,
                              int64_t M, int64_t *c)
{
    if (n == 0 || M <= 1) return ORACLE_EARG;
    int64_t *dd = (int64_t *)malloc(sizeof(int64_t) * n);
    int64_t *factor = (int64_t *)malloc(sizeof(int64_t) * n);
    if (!dd || !factor) { free(dd); free(factor); return ORACLE_EARG; }

    for (uint32_t i = 0; i < n; ++i) dd[i] = oracle_safe_mod(y[i], M);

    /* divided differences */
    for (uint32_t k = 1; k + 1 <= n; ++k) {
        for (uint32_t i = n - 1; i >= k; --i) {
            int64_t numerator = oracle_safe_mod(dd[i] - dd[i - 1], M);
            int64_t denominator = oracle_safe_mod(x[i] - x[i - k], M);
            int err;
            int64_t inv = toploc_oracle_mod_inverse(denominator, M, &err);
            if (err) { free(dd); free(factor); return ORACLE_ENOINV; }
            dd[i] = (numerator * inv) % M;
        }
    }

    /* expansion of the Newton form  sum_i dd[i] * prod_{t<i} (X - x[t])  into
     * standard-form coefficients; factor holds the running product */
    for (uint32_t i = 0; i < n; ++i) { c[i] = 0; factor[i] = 0; }
    factor[0] = 1;
    for (uint32_t i = 0; i < n; ++i) {
        for (uint32_t j = 0; j <= i; ++j)
            c[j] = (c[j] + dd[i] * factor[j]) % M;
        if (i + 1 < n) {
            /* factor(X) <- factor(X) * (X - x[i]); degree grows from i to i+1 */
            int64_t neg_xi = oracle_safe_mod(-x[i], M);
            for (uint32_t d = i + 1; d >= 1; --d)
                factor[d] = (factor[d - 1] + factor[d] * neg_xi) % M;
            factor[0] = (factor[0] * neg_xi) % M;
        }
    }
    free(dd);
    free(factor);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 5: Horner evaluation; c has n_coef entries c_0..c_{n_coef-1}     */
/* ------------------------------------------------------------------------- */
int64_t toploc_oracle_horner(const int64_t *c, uint32_t n_coef, int64_t x, int64_t M)
{
    int64_t result = c[n_coef - 1];
    for (uint32_t i = 1; i < n_coef; ++i)
        result = (result * x + c[n_coef - 1 - i]) % M;
    return result % M;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 6: largest i in [2^15+1, 65536] with j mod i injective on x.     */
/* M = 0: to the letter.  M > 0: residues are compared after reduction mod M  */
/* too (the form in which Algorithms 3 and 5 consume them).                   */
/* ------------------------------------------------------------------------- */
static int oracle_u32_cmp(const void *pa, const void *pb)
{
    uint32_t a = *(const uint32_t *)pa, b = *(const uint32_t *)pb;
    return (a > b) - (a < b);
}

int toploc_oracle_find_injective_modulus(const uint32_t *x, uint32_t n, uint32_t M,
                                         uint32_t *m_out)
{
    if (n == 0) return ORACLE_EARG;
    uint32_t *S = (uint32_t *)malloc(sizeof(uint32_t) * n);
    if (!S) return ORACLE_EARG;
    for (uint32_t i = 65536u; i >= 32769u; --i) {
        for (uint32_t t = 0; t < n; ++t) {
            uint32_t r = x[t] % i;
            S[t] = M ? (r % M) : r;
        }
        qsort(S, n, sizeof(uint32_t), oracle_u32_cmp);
        uint32_t distinct = 1;
        for (uint32_t t = 1; t < n; ++t) distinct += (S[t] != S[t - 1]);
        if (distinct == n) { *m_out = i; free(S); return ORACLE_OK; }
    }
    free(S);
    return ORACLE_ENOMOD;
}

/* Many independent sets at once (the experiment behind the appendix's table of return values). */
int toploc_oracle_find_injective_modulus_batch(const uint32_t *x, uint64_t n_sets,
                                               uint32_t n, uint32_t M,
                                               uint32_t *m_out, uint8_t *status)
{
    for (uint64_t s = 0; s < n_sets; ++s) {
        uint32_t m = 0;
        status[s] = (uint8_t)toploc_oracle_find_injective_modulus(x + s * n, n, M, &m);
        m_out[s] = m;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* encode / decode                                                            */
/* ------------------------------------------------------------------------- */
static void oracle_encode(uint32_t m, const int64_t *c, uint32_t k, uint8_t *p)
{
    uint32_t mf = m % 65536u;
    p[0] = (uint8_t)(mf & 0xFF);
    p[1] = (uint8_t)(mf >> 8);
    for (uint32_t j = 0; j < k; ++j) {
        p[2 + 2 * j] = (uint8_t)(c[j] & 0xFF);
        p[3 + 2 * j] = (uint8_t)((c[j] >> 8) & 0xFF);
    }
}

static int oracle_decode(const uint8_t *p, uint32_t k, uint32_t M, uint32_t *m, int64_t *c)
{
    uint32_t mf = (uint32_t)p[0] | ((uint32_t)p[1] << 8);
    *m = mf ? mf : 65536u;
    int bad = (*m < 32769u);
    for (uint32_t j = 0; j < k; ++j) {
        c[j] = (int64_t)((uint32_t)p[2 + 2 * j] | ((uint32_t)p[3 + 2 * j] << 8));
        if (c[j] >= (int64_t)M) bad = 1;
    }
    return bad ? ORACLE_EMALFORMED : ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 on one chunk                                                   */
/* ------------------------------------------------------------------------- */
int toploc_oracle_build_chunk(const uint16_t *h, uint64_t n, uint32_t k, uint32_t M,
                              uint8_t *proof, uint32_t *topk_idx_opt)
{
    uint32_t *i = (uint32_t *)malloc(sizeof(uint32_t) * k);
    uint16_t *v = (uint16_t *)malloc(sizeof(uint16_t) * k);
    int64_t *i_m = (int64_t *)malloc(sizeof(int64_t) * k);
    int64_t *y = (int64_t *)malloc(sizeof(int64_t) * k);
    int64_t *c = (int64_t *)malloc(sizeof(int64_t) * k);
    int rc = ORACLE_EARG;
    if (!i || !v || !i_m || !y || !c) goto done;
    memset(proof, 0, 2 + 2 * (size_t)k);

    rc = toploc_oracle_topk(h, n, k, i, v);                      /* (i, v) <- topk(h, k) */
    if (rc) goto done;
    if (topk_idx_opt) memcpy(topk_idx_opt, i, sizeof(uint32_t) * k);

    uint32_t m;
    rc = toploc_oracle_find_injective_modulus(i, k, M, &m);      /* m <- findInjectiveModulus(i) */
    if (rc) goto done;

    for (uint32_t j = 0; j < k; ++j) {
        i_m[j] = (int64_t)(i[j] % m);                            /* i_m <- i mod m */
        y[j] = (int64_t)v[j];                                    /* the bf16 bit pattern */
    }
    rc = toploc_oracle_interpolate(i_m, y, k, (int64_t)M, c);    /* P(x) */
    if (rc) goto done;
    oracle_encode(m, c, k, proof);                               /* p <- encode(m, P) */
done:
    free(i); free(v); free(i_m); free(y); free(c);
    return rc;
}

/* Decision rule of Algorithm 2 alone, on a caller-supplied err_e and err_m
 * multiset (lets tests pin the thresholds' strictness and the median rule). */
int toploc_oracle_decide(uint32_t err_e, const uint32_t *err_m_in, uint32_t n_m,
                         uint32_t t_exp, uint32_t t_mean, uint32_t t_median,
                         oracle_verify_result *res)
{
    memset(res, 0, sizeof(*res));
    uint32_t *err_m = (uint32_t *)malloc(sizeof(uint32_t) * (n_m ? n_m : 1));
    if (!err_m) return ORACLE_EARG;
    uint64_t sum = 0;
    for (uint32_t t = 0; t < n_m; ++t) { err_m[t] = err_m_in[t]; sum += err_m[t]; }
    uint32_t median = 0;
    if (n_m) {
        qsort(err_m, n_m, sizeof(uint32_t), oracle_u32_cmp);
        median = err_m[(n_m - 1) / 2];
    }
    int reject = (err_e > t_exp);
    if (n_m) {
        if (sum > (uint64_t)t_mean * n_m) reject = 1;
        if (median > t_median) reject = 1;
    }
    res->err_exp = err_e;
    res->n_match = n_m;
    res->mant_sum = (uint32_t)sum;
    res->mant_median = median;
    res->accept = (uint8_t)(!reject);
    free(err_m);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 2 on one chunk                                                   */
/* ------------------------------------------------------------------------- */
static void oracle_extract_bits(uint32_t bits16, uint32_t *e, uint32_t *mant)
{
    *e = (bits16 >> 7) & 0xFFu;
    *mant = bits16 & 0x7Fu;
}

int toploc_oracle_verify_chunk(const uint16_t *h, uint64_t n, uint32_t k, uint32_t M,
                               const uint8_t *proof, uint32_t t_exp, uint32_t t_mean,
                               uint32_t t_median, oracle_verify_result *res)
{
    memset(res, 0, sizeof(*res));
    uint32_t *i = (uint32_t *)malloc(sizeof(uint32_t) * k);
    uint16_t *v = (uint16_t *)malloc(sizeof(uint16_t) * k);
    int64_t *c = (int64_t *)malloc(sizeof(int64_t) * k);
    uint32_t *err_m = (uint32_t *)malloc(sizeof(uint32_t) * k);
    int rc = ORACLE_EARG;
    if (!i || !v || !c || !err_m) goto done;

    uint32_t m;
    rc = oracle_decode(proof, k, M, &m, c);                      /* k, m, P <- decode(p) */
    if (rc == ORACLE_EMALFORMED) { res->status = ORACLE_EMALFORMED; res->accept = 0; rc = ORACLE_OK; goto done; }

    rc = toploc_oracle_topk(h, n, k, i, v);                      /* (i, v) <- topk(h, k) */
    if (rc) goto done;

    uint32_t err_e = 0, n_m = 0;
    for (uint32_t j = 0; j < k; ++j) {
        int64_t i_m = (int64_t)(i[j] % m);                       /* i_m <- i mod m */
        uint32_t P = (uint32_t)toploc_oracle_horner(c, k, i_m, (int64_t)M);
        uint32_t e_p, m_p, e_v, m_v;
        oracle_extract_bits(P, &e_p, &m_p);
        oracle_extract_bits(v[j], &e_v, &m_v);
        if (e_p == e_v) err_m[n_m++] = (m_p > m_v) ? (m_p - m_v) : (m_v - m_p);
        else err_e += 1;
    }

    /* thresholds: err_e > T_exp or mean(err_m) > T_mean or median(err_m) > T_median */
    rc = toploc_oracle_decide(err_e, err_m, n_m, t_exp, t_mean, t_median, res);
    if (rc) goto done;
    rc = ORACLE_OK;
done:
    free(i); free(v); free(c); free(err_m);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Batches: one chunk per task, independent chunks spread over host threads.  */
/* h is [n_chunks][n] bf16 patterns, contiguous.                              */
/* ------------------------------------------------------------------------- */
int toploc_oracle_build(const uint16_t *h, uint64_t n_chunks, uint64_t n, uint32_t k,
                        uint32_t M, uint8_t *proofs, uint8_t *status,
                        uint32_t *topk_idx_opt, int n_threads)
{
    if (k == 0 || k > n) return ORACLE_EARG;
    const size_t pb = 2 + 2 * (size_t)k;
    int bad = 0;
    (void)n_threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads > 0 ? n_threads : 1)
#endif
    for (int64_t cidx = 0; cidx < (int64_t)n_chunks; ++cidx) {
        int rc = toploc_oracle_build_chunk(h + (size_t)cidx * n, n, k, M, proofs + (size_t)cidx * pb,
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

int toploc_oracle_verify(const uint16_t *h, uint64_t n_chunks, uint64_t n, uint32_t k,
                         uint32_t M, const uint8_t *proofs, uint32_t t_exp, uint32_t t_mean,
                         uint32_t t_median, oracle_verify_result *results, int n_threads)
{
    if (k == 0 || k > n) return ORACLE_EARG;
    const size_t pb = 2 + 2 * (size_t)k;
    int bad = 0;
    (void)n_threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads > 0 ? n_threads : 1)
#endif
    for (int64_t cidx = 0; cidx < (int64_t)n_chunks; ++cidx) {
        int rc = toploc_oracle_verify_chunk(h + (size_t)cidx * n, n, k, M, proofs + (size_t)cidx * pb,
                                            t_exp, t_mean, t_median, &results[cidx]);
        if (rc != ORACLE_OK) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            bad = 1;
        }
    }
    return bad ? ORACLE_EARG : ORACLE_OK;
}

int toploc_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
