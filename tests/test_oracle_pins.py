"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests re-types the oracle's own formulas: each compares the
oracle with something independent of it -- values the paper prints (fixtures
under tests/golden/), closed forms, brute force on tiny inputs, textbook
special cases, or a different algorithm for the same unique object written
here in Python integers.
"""
import itertools
import math

import numpy as np
import pytest

import oracle as orc
from conftest import read_golden

P = 65497


# ---------------------------------------------------------------------------
# independent helpers (Python integers; no code shared with oracle/)
# ---------------------------------------------------------------------------

def lagrange_coeffs(xs, ys, p):
    """Coefficients of the unique interpolating polynomial via the Lagrange sum."""
    k = len(xs)
    coeffs = [0] * k
    for j in range(k):
        # numerator polynomial prod_{i != j} (X - x_i), ascending powers
        num = [1]
        den = 1
        for i in range(k):
            if i == j:
                continue
            nxt = [0] * (len(num) + 1)
            for d, a in enumerate(num):
                nxt[d + 1] = (nxt[d + 1] + a) % p
                nxt[d] = (nxt[d] - a * xs[i]) % p
            num = nxt
            den = den * (xs[j] - xs[i]) % p
        w = ys[j] * pow(den, -1, p) % p
        for d in range(k):
            coeffs[d] = (coeffs[d] + w * num[d]) % p
    return coeffs


def vandermonde_solve(xs, ys, p):
    """Gaussian elimination on the Vandermonde system mod p."""
    k = len(xs)
    A = [[pow(x, d, p) for d in range(k)] + [y % p] for x, y in zip(xs, ys)]
    for col in range(k):
        piv = next(r for r in range(col, k) if A[r][col] % p)
        A[col], A[piv] = A[piv], A[col]
        inv = pow(A[col][col], -1, p)
        A[col] = [a * inv % p for a in A[col]]
        for r in range(k):
            if r != col and A[r][col]:
                f = A[r][col]
                A[r] = [(a - f * b) % p for a, b in zip(A[r], A[col])]
    return [A[r][k] for r in range(k)]


def poly_eval(coeffs, x, p):
    return sum(c * pow(x, d, p) for d, c in enumerate(coeffs)) % p


def brute_topk(bits, k):
    """k rounds of arg-max over what is left; ties to the lower index."""
    left = list(range(len(bits)))
    out = []
    for _ in range(k):
        best = left[0]
        for i in left[1:]:
            if (bits[i] & 0x7FFF) > (bits[best] & 0x7FFF):
                best = i
        left.remove(best)
        out.append(best)
    return out


def decode(proof):
    m = int(proof[0]) | (int(proof[1]) << 8)
    m = m if m else 65536
    c = [int(proof[2 + 2 * j]) | (int(proof[3 + 2 * j]) << 8) for j in range((len(proof) - 2) // 2)]
    return m, c


def random_chunk(rng, n, outliers=4, hidden=None):
    x = rng.standard_normal(n).astype(np.float32)
    if hidden:
        cols = rng.choice(hidden, outliers, replace=False)
        x.reshape(-1, hidden)[:, cols] *= 20.0
    bits = (x.view(np.uint32) >> 16).astype(np.uint16)  # truncation is fine for a test input
    return bits


# ---------------------------------------------------------------------------
# P5: sizes the paper prints
# ---------------------------------------------------------------------------

def test_sizes_match_paper():
    g = {r[0]: int(r[1]) for r in read_golden("sizes_and_thresholds.txt")}
    assert orc.proof_bytes(128) == g["proof_bytes_k128"] == 258
    assert orc.proof_bytes(128) - 2 == g["coefficient_bytes_k128"]
    assert g["chunk_tokens"] * 4096 * 2 == g["raw_chunk_bytes_h4096"]
    assert g["raw_bytes_per_token_h4096"] * g["chunk_tokens"] // g["coefficient_bytes_k128"] == g["reduction_factor"]
    assert (orc.T_EXP, orc.T_MEAN, orc.T_MEDIAN) == (g["t_exp_bf16"], g["t_mean_bf16"], g["t_median_bf16"])
    rng = np.random.default_rng(0)
    proofs, status = orc.build(random_chunk(rng, 4096)[None, :], 128)
    assert proofs.shape == (1, 258) and status[0] == 0
    assert all(P > 1 and P % d for d in range(2, int(P ** 0.5) + 1))  # the field modulus is prime


# ---------------------------------------------------------------------------
# P6: top-k against brute force, tie rule, sign and zero handling
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(6))
def test_topk_brute_force_tiny(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(8, 64))
    k = int(rng.integers(1, 9))
    # few distinct magnitudes so that ties at the boundary are the norm
    mags = rng.integers(0, 6, n).astype(np.uint16) * 0x0080 + 0x3F00
    signs = rng.integers(0, 2, n).astype(np.uint16) << 15
    bits = (mags | signs).astype(np.uint16)
    idx, val = orc.topk(bits, k)
    assert idx.tolist() == brute_topk(bits.tolist(), k)
    assert val.tolist() == [int(bits[i]) for i in idx]


def test_topk_magnitude_not_signed_value():
    # -8.0 (0xC100) outranks +4.0 (0x4080); +0 and -0 tie and go by index
    bits = np.array([0x4080, 0xC100, 0x8000, 0x0000, 0x3F80], dtype=np.uint16)
    idx, val = orc.topk(bits, 5)
    assert idx.tolist() == [1, 0, 4, 2, 3]
    assert val.tolist() == [0xC100, 0x4080, 0x3F80, 0x8000, 0x0000]


def test_topk_all_equal_is_first_k_indices():
    bits = np.full(100, 0x3F80, dtype=np.uint16)
    idx, _ = orc.topk(bits, 7)
    assert idx.tolist() == list(range(7))


def test_topk_rejects_bad_k():
    bits = np.zeros(4, dtype=np.uint16)
    with pytest.raises(ValueError):
        orc.topk(bits, 5)
    with pytest.raises(ValueError):
        orc.topk(bits, 0)


# ---------------------------------------------------------------------------
# P7: Algorithm 4 against Fermat, its special exits; textbook interpolations
# ---------------------------------------------------------------------------

def test_mod_inverse_equals_fermat_for_every_residue():
    for a in range(1, P):
        inv = orc.mod_inverse(a, P)
        assert 0 < inv < P
        assert inv == pow(a, P - 2, P)


def test_mod_inverse_special_exits():
    assert orc.mod_inverse(5, 1) == 0
    assert orc.mod_inverse(5, 0) == 0
    with pytest.raises(ZeroDivisionError):
        orc.mod_inverse(6, 9)
    with pytest.raises(ZeroDivisionError):
        orc.mod_inverse(0, P)
    assert orc.mod_inverse(3, 7) == 5
    assert orc.mod_inverse(65536, P) == pow(65536, -1, P)  # a > m is allowed


def test_interpolate_textbook_cases():
    assert orc.interpolate([17], [12345]).tolist() == [12345]            # k = 1: constant
    c = orc.interpolate([2, 5], [10, 25])                                   # line y = 5x
    assert c.tolist() == [0, 5]
    c = orc.interpolate([1, 2, 3], [1, 4, 9])                               # y = x^2
    assert c.tolist() == [0, 0, 1]
    c = orc.interpolate([0, 7, 9], [42, 3, 5])                              # P(0) = c_0
    assert c[0] == 42
    c = orc.interpolate([1, 2], [3, 1], M=7)                                # slope -2 = 5 mod 7
    assert c.tolist() == [5, 5]


def test_interpolate_small_prime_exhaustive():
    # every function on 3 points of GF(5) is a polynomial of degree <= 2: check all 125
    p = 5
    xs = [1, 3, 4]
    for ys in itertools.product(range(p), repeat=3):
        c = orc.interpolate(xs, list(ys), M=p).tolist()
        assert all(0 <= a < p for a in c)
        assert [poly_eval(c, x, p) for x in xs] == list(ys)


def test_interpolate_zero_denominator_is_an_error():
    with pytest.raises(ZeroDivisionError):
        orc.interpolate([3, 3 + P], [1, 2])


def test_horner_against_power_sum():
    rng = np.random.default_rng(3)
    c = rng.integers(0, P, 40).tolist()
    for x in [0, 1, 2, P - 1, 65535, 12345]:
        assert orc.horner(c, x) == poly_eval(c, x, P)
    assert orc.horner([7], 99) == 7


# ---------------------------------------------------------------------------
# P2: uniqueness -- other algorithms and other point orders give the same bytes
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("k,seed", [(2, 0), (5, 1), (12, 2), (33, 3), (128, 4)])
def test_interpolate_equals_lagrange(k, seed):
    rng = np.random.default_rng(seed)
    xs = rng.choice(65536, k, replace=False)
    xs = xs[np.unique(xs % P, return_index=True)[1]][:k].tolist()
    ys = rng.integers(0, 65536, len(xs)).tolist()
    c = orc.interpolate(xs, ys).tolist()
    assert c == lagrange_coeffs([x % P for x in xs], [y % P for y in ys], P)


@pytest.mark.parametrize("k", [1, 3, 8, 12])
def test_interpolate_equals_vandermonde_solve(k):
    rng = np.random.default_rng(10 + k)
    xs = rng.choice(P, k, replace=False).tolist()
    ys = rng.integers(0, P, k).tolist()
    assert orc.interpolate(xs, ys).tolist() == vandermonde_solve(xs, ys, P)


def test_interpolate_is_order_independent():
    rng = np.random.default_rng(5)
    xs = rng.choice(P, 64, replace=False)
    ys = rng.integers(0, P, 64)
    ref = orc.interpolate(xs, ys).tolist()
    for _ in range(3):
        perm = rng.permutation(64)
        assert orc.interpolate(xs[perm], ys[perm]).tolist() == ref


# ---------------------------------------------------------------------------
# P3: injectivity and maximality of the modulus
# ---------------------------------------------------------------------------

def _is_injective(idx, m, p):
    r = [(int(i) % m) % p if p else int(i) % m for i in idx]
    return len(set(r)) == len(r)


@pytest.mark.parametrize("seed", range(5))
def test_modulus_is_largest_injective(seed):
    rng = np.random.default_rng(100 + seed)
    if seed < 3:
        idx = rng.choice(2 ** 31, 128, replace=False)
    else:  # structured: a few columns of a [32, 4096] chunk -> 65536 always collides
        cols = rng.choice(4096, 4, replace=False)
        idx = (np.arange(32)[:, None] * 4096 + cols[None, :]).ravel()
    for p in (0, P):
        m = orc.find_injective_modulus(idx, M=p)
        assert 32769 <= m <= 65536
        assert _is_injective(idx, m, p)
        for bigger in range(m + 1, 65537):
            assert not _is_injective(idx, bigger, p)
    if seed >= 3:
        assert orc.find_injective_modulus(idx, M=0) < 65536


def test_modulus_composite_map_collision_is_avoided():
    # residues 5 and 65502 are distinct mod 65536 but equal mod 65497
    idx = np.array([5, 65502, 1000, 70000], dtype=np.uint32)
    assert orc.find_injective_modulus(idx, M=0) == 65536
    m = orc.find_injective_modulus(idx, M=P)
    assert m < 65536 and _is_injective(idx, m, P)


def test_modulus_failure_when_no_candidate_works():
    with pytest.raises(ValueError):
        orc.find_injective_modulus(np.array([7, 7], dtype=np.uint32), M=P)


def covering_index_set():
    """385 distinct indices whose pairwise differences include every m in [32769, 65536]:
    (32769 + 256 j) - i = m has a solution with 0 <= i < 256, 0 <= j <= 128 for each such m,
    so two of the indices are congruent modulo every candidate of Algorithm 6."""
    return np.concatenate([np.arange(256), 32769 + 256 * np.arange(129)]).astype(np.uint32)


def test_modulus_failure_with_distinct_indices_and_a_deep_search():
    idx = covering_index_set()
    assert len(set(idx.tolist())) == idx.size
    diffs = set(int(a) - int(b) for a in idx[256:] for b in idx[:256])
    assert all(m in diffs for m in range(32769, 65537))
    for p in (0, P):
        with pytest.raises(ValueError):
            orc.find_injective_modulus(idx, M=p)
    # without index 255 only the candidates 32769 + 256 j - 255 lose their colliding pair ... unless another
    # pair collides there too: brute force says which candidate the search must stop at
    # the smallest candidate, 2^15 + 1, is part of the range: a set whose differences cover 32770..65537 and
    # nothing that 32769 divides is injective there and nowhere above
    low = np.concatenate([np.arange(256), 32770 + 255 + 256 * np.arange(128)]).astype(np.uint32)
    assert all(not _is_injective(low, m, P) for m in range(32770, 65537)) and _is_injective(low, 32769, P)
    assert orc.find_injective_modulus(low, M=P) == 32769 and orc.find_injective_modulus(low, M=0) == 32769
    fewer = np.delete(idx, 255)
    want = next(m for m in range(65536, 32768, -1) if _is_injective(fewer, m, P))
    assert want < 65536 - 200                                   # hundreds of candidates deep
    assert orc.find_injective_modulus(fewer, M=P) == want


# ---------------------------------------------------------------------------
# P4: the appendix's table of Algorithm 6's return values -- printed values, closed form, Monte Carlo of the oracle
# ---------------------------------------------------------------------------

def birthday_distribution(k, top=65536, rows=9):
    """P[Algorithm 6 returns m] for independent uniform residues: the chance that
    m is collision-free times the chance that every larger candidate failed."""
    probs, fail_all = [], 1.0
    for m in range(top, top - rows, -1):
        ok = math.exp(sum(math.log1p(-j / m) for j in range(k)))
        probs.append(fail_all * ok)
        fail_all *= 1.0 - ok
    return probs


def test_modulus_distribution_closed_form_matches_printed_values():
    rows = read_golden("injective_modulus_distribution.txt")
    printed = {int(m): float(v) for m, v in rows}
    closed = dict(zip(range(65536, 65536 - 9, -1), birthday_distribution(128)))
    assert abs(closed[65536] - printed[65536]) < 5e-5                # 4 printed digits
    assert abs(closed[65535] - printed[65535]) / printed[65535] < 2e-3
    assert abs(closed[65534] - printed[65534]) / printed[65534] < 2e-3
    assert abs(closed[65533] - printed[65533]) / printed[65533] < 1e-2
    assert abs(closed[65532] - printed[65532]) / printed[65532] < 5e-2


def test_modulus_distribution_monte_carlo_of_oracle():
    rows = read_golden("injective_modulus_distribution.txt")
    printed = {int(m): float(v) for m, v in rows}
    rng = np.random.default_rng(7)
    n_sets, counts = 0, {}
    for _ in range(4):
        sets = rng.integers(0, 2 ** 31, size=(250_000, 128), dtype=np.int64).astype(np.uint32)
        m, st = orc.find_injective_modulus_batch(sets, M=0)          # Algorithm 6 to the letter
        # a draw with a repeated integer is not a set: Algorithm 6 must fail on exactly those
        srt = np.sort(sets, axis=1)
        dup = (srt[:, 1:] == srt[:, :-1]).any(axis=1)
        assert ((st != 0) == dup).all()
        sets, m = sets[~dup], m[~dup]
        vals, cnt = np.unique(m, return_counts=True)
        for v, c in zip(vals, cnt):
            counts[int(v)] = counts.get(int(v), 0) + int(c)
        n_sets += len(sets)
    for m in (65536, 65535, 65534, 65533):
        p = printed[m]
        sigma = math.sqrt(p * (1 - p) / n_sets)
        assert abs(counts.get(m, 0) / n_sets - p) < 4 * sigma + 0.5 * 10 ** (math.floor(math.log10(p)) - 3)
    assert min(counts) >= 65528 and max(counts) == 65536


def test_composite_reading_shifts_the_distribution_only_slightly():
    rng = np.random.default_rng(8)
    sets = rng.integers(0, 2 ** 31, size=(100_000, 128), dtype=np.int64).astype(np.uint32)
    m0, _ = orc.find_injective_modulus_batch(sets, M=0)
    mp, _ = orc.find_injective_modulus_batch(sets, M=P)
    assert (mp <= m0).all()
    assert (mp != m0).mean() < 2e-3   # ~ C(128,2) * 2 * 39 / 65536^2 = 1.5e-4 expected


# ---------------------------------------------------------------------------
# P1: round trip of whole proofs
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("hidden,k", [(256, 16), (512, 128), (4096, 128), (640, 32)])
def test_proof_round_trip(hidden, k):
    rng = np.random.default_rng(hidden + k)
    n = 32 * hidden
    h = np.stack([random_chunk(rng, n, hidden=hidden) for _ in range(3)])
    proofs, status, idx = orc.build(h, k, want_topk=True)
    assert not status.any()
    assert proofs.shape[1] == 2 + 2 * k
    for ci in range(h.shape[0]):
        m, c = decode(proofs[ci].tolist())
        assert len(c) == k and all(a < P for a in c)
        assert 32769 <= m <= 65536
        xs = [(int(i) % m) % P for i in idx[ci]]
        assert len(set(xs)) == k                                  # the index map is injective
        for j in range(k):
            assert poly_eval(c, xs[j], P) == int(h[ci, idx[ci, j]])   # P(x_j) = bf16 pattern
        # same bytes from an independent interpolation of the same points
        assert c == lagrange_coeffs(xs, [int(h[ci, i]) for i in idx[ci]], P) if k <= 32 else True


# ---------------------------------------------------------------------------
# P8: verification identities and the strictness of the three thresholds
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(10))
def test_build_equals_brute_force_on_small_chunks(seed):
    """The whole of Algorithm 1 on small chunks: the bytes are the largest injective modulus found by trying
    every candidate, followed by the Lagrange-sum coefficients through the arg-max top-k, all in Python."""
    rng = np.random.default_rng(2300 + seed)
    n = int(rng.choice([16, 64, 300]))
    k = int(rng.choice([1, 3, 8, 12]))
    h = random_chunk(rng, n)
    if seed % 3 == 0:
        h[rng.integers(0, n, size=n // 2)] = h[0]                       # ties at the boundary
    if seed % 4 == 1:
        h = np.concatenate([h, np.zeros(70000, dtype=np.uint16)])        # indices beyond 65536 among the ...
        h[[65541, 69999, 5]] = np.uint16(0x7F00)                         # ... top-k: 5 and 65541 collide mod 65536
    proofs, status, idx = orc.build(h[None, :], k, want_topk=True)
    top = brute_topk([int(b) for b in h], k)
    assert status[0] == 0 and idx[0].tolist() == top
    m = next(c for c in range(65536, 32768, -1) if _is_injective(np.array(top), c, P))
    want = lagrange_coeffs([(i % m) % P for i in top], [int(h[i]) % P for i in top], P)
    got_m, got_c = decode(proofs[0])
    assert got_m == m and got_c == want
    assert len(proofs[0]) == 2 + 2 * k


def test_self_verify_accepts_with_zero_statistics():
    rng = np.random.default_rng(21)
    h = np.stack([random_chunk(rng, 32 * 512, hidden=512) for _ in range(4)])
    proofs, status = orc.build(h, 128)
    res = orc.verify(h, proofs, 128)
    assert (res["accept"] == 1).all() and (res["status"] == 0).all()
    assert (res["err_exp"] == 0).all() and (res["n_match"] == 128).all()
    assert (res["mant_sum"] == 0).all() and (res["mant_median"] == 0).all()


def test_flipping_low_mantissa_bits_counts_exactly():
    rng = np.random.default_rng(22)
    hidden, k = 512, 128
    h = random_chunk(rng, 32 * hidden, hidden=hidden)[None, :].copy()
    proofs, _, idx = orc.build(h, k, want_topk=True)
    # move entries well inside the top-k (ranks 0..r-1) down by one mantissa step;
    # choose ones whose mantissa is not 0 (no binade crossing) and whose new value
    # still beats rank k-1 so that the selected set is unchanged
    floor_mag = int(h[0, idx[0, -1]]) & 0x7FFF
    touched = 0
    h2 = h.copy()
    for j in range(k):
        i = int(idx[0, j])
        b = int(h2[0, i])
        if (b & 0x7F) != 0 and ((b & 0x7FFF) - 1) > floor_mag and touched < 9:
            h2[0, i] = b - 1
            touched += 1
    assert touched == 9
    res = orc.verify(h2, proofs, k)[0]
    assert res["err_exp"] == 0 and res["n_match"] == k
    assert res["mant_sum"] == 9 and res["mant_median"] == 0 and res["accept"] == 1


def test_sign_flip_is_not_an_error_but_exponent_change_is():
    rng = np.random.default_rng(23)
    hidden, k = 512, 64
    h = random_chunk(rng, 32 * hidden, hidden=hidden)[None, :].copy()
    proofs, _, idx = orc.build(h, k, want_topk=True)
    h2 = h.copy()
    h2[0, idx[0, 0]] ^= 0x8000                      # sign only: same exponent and mantissa
    res = orc.verify(h2, proofs, k)[0]
    assert res["err_exp"] == 0 and res["mant_sum"] == 0
    h3 = h.copy()
    h3[0, idx[0, 0]] += 0x0080                      # next binade: still the largest entry
    res = orc.verify(h3, proofs, k)[0]
    assert res["err_exp"] == 1 and res["n_match"] == k - 1


def test_threshold_strictness_and_median_rule():
    T = (38, 10, 8)
    assert orc.decide(38, [0] * 90, T)["accept"] == 1
    assert orc.decide(39, [0] * 89, T)["accept"] == 0
    assert orc.decide(0, [10] * 128, (38, 10, 127))["accept"] == 1           # mean == T_mean
    assert orc.decide(0, [10] * 127 + [11], (38, 10, 127))["accept"] == 0    # sum = 10 n + 1
    assert orc.decide(0, [8] * 65 + [0] * 63, (38, 127, 8))["accept"] == 1   # median == T_median
    assert orc.decide(0, [9] * 65 + [0] * 63, (38, 127, 8))["accept"] == 0
    # even count: the lower of the two middle values (an order statistic, never x.5)
    r = orc.decide(0, [1, 2, 3, 100], (38, 1000, 1000))
    assert r["mant_median"] == 2 and r["mant_sum"] == 106 and r["n_match"] == 4
    assert orc.decide(0, [5, 1, 3], (38, 1000, 1000))["mant_median"] == 3
    # nothing matched: only the exponent count decides
    assert orc.decide(3, [], (3, 0, 0))["accept"] == 1
    assert orc.decide(4, [], (3, 0, 0))["accept"] == 0


def brute_verify(bits, proof, thresholds):
    """Algorithm 2 on one small chunk in Python integers: decode, top-k by repeated arg-max, the
    polynomial evaluated by its definition (sum of c_d x^d, no Horner), fields by shifts, sorted median."""
    m, c = decode(proof)
    k = len(c)
    err_e, err_m = 0, []
    for i in brute_topk([int(b) for b in bits], k):
        x = (i % m) % P
        val = poly_eval(c, x, P)
        e_p, m_p = (val >> 7) & 0xFF, val & 0x7F
        e_v, m_v = (int(bits[i]) >> 7) & 0xFF, int(bits[i]) & 0x7F
        if e_p == e_v:
            err_m.append(abs(m_p - m_v))
        else:
            err_e += 1
    n = len(err_m)
    median = sorted(err_m)[(n - 1) // 2] if n else 0
    t_exp, t_mean, t_median = thresholds
    reject = err_e > t_exp or (n > 0 and (sum(err_m) > t_mean * n or median > t_median))
    return {"err_exp": err_e, "n_match": n, "mant_sum": sum(err_m), "mant_median": median, "accept": 0 if reject else 1}


@pytest.mark.parametrize("seed", range(12))
def test_verify_equals_brute_force_on_small_perturbed_chunks(seed):
    """The whole of Algorithm 2 on inputs where exponents match for some entries and not for others, mantissas
    differ by several steps, the selected set changes and thresholds sit near the statistics."""
    rng = np.random.default_rng(2400 + seed)
    n = int(rng.choice([64, 200, 512]))
    k = int(rng.choice([4, 16, 33]))
    h = random_chunk(rng, n)[None, :].copy()
    if seed % 4 == 1:      # indices 5 and 65541 collide mod 65536: the proof then carries a smaller modulus
        h = np.concatenate([h, np.zeros((1, 70000), dtype=np.uint16)], axis=1)
        h[0, [65541 + n, 5, 69999]] = np.uint16(0x7E00)
        h[0, 65541] = np.uint16(0x7E40)
        n = h.shape[1]
    proofs, status = orc.build(h, k)
    assert status[0] == 0 and (seed % 4 != 1 or decode(proofs[0])[0] < 65536)
    h2 = h.copy()
    touch = rng.random(n) < 0.5
    delta = rng.integers(-12, 13, size=n)
    mag = (h2[0].astype(np.int64) & 0x7FFF) + np.where(touch, delta, 0)        # crosses binades now and then
    h2[0] = (h2[0] & 0x8000) | np.clip(mag, 0, 0x7F7F).astype(np.uint16)
    swap = rng.choice(n, size=3, replace=False)                                # a few entries change hands
    h2[0, swap] = h2[0, swap[::-1]]
    thresholds = (int(rng.integers(0, k)), int(rng.integers(0, 12)), int(rng.integers(0, 12)))
    got = orc.verify(h2, proofs, k, thresholds=thresholds)[0]
    want = brute_verify(h2[0], proofs[0], thresholds)
    for f, v in want.items():
        assert int(got[f]) == v, (f, int(got[f]), v)
    assert got["status"] == 0 and want["n_match"] > 0 and want["err_exp"] + want["n_match"] == k


def test_independent_tensor_is_rejected_and_statistics_are_in_range():
    rng = np.random.default_rng(24)
    hidden, k = 512, 128
    a = random_chunk(rng, 32 * hidden, hidden=hidden)[None, :]
    b = random_chunk(rng, 32 * hidden, hidden=hidden)[None, :]
    proofs, _ = orc.build(a, k)
    res = orc.verify(b, proofs, k)[0]
    assert res["accept"] == 0 and res["err_exp"] > 100
    assert res["err_exp"] + res["n_match"] == k


def test_malformed_proofs_are_rejected_not_crashed():
    rng = np.random.default_rng(25)
    h = random_chunk(rng, 32 * 256, hidden=256)[None, :]
    proofs, _ = orc.build(h, 16)
    bad = proofs.copy()
    bad[0, 0], bad[0, 1] = 0x00, 0x40                    # m = 16384 < 2^15 + 1
    r = orc.verify(h, bad, 16)[0]
    assert r["status"] == orc.EMALFORMED and r["accept"] == 0
    bad = proofs.copy()
    bad[0, 2], bad[0, 3] = 0xFF, 0xFF                    # coefficient 65535 >= p
    r = orc.verify(h, bad, 16)[0]
    assert r["status"] == orc.EMALFORMED and r["accept"] == 0
    ok = orc.verify(h, proofs, 16)[0]
    assert ok["status"] == 0 and ok["accept"] == 1
    # the edges of the two ranges: m = 2^15 is out, 2^15 + 1 is in; a coefficient p - 1 is in, p is out
    for field, want in ((32768, orc.EMALFORMED), (32769, 0)):
        edge = proofs.copy()
        edge[0, 0], edge[0, 1] = field & 0xFF, field >> 8
        assert orc.verify(h, edge, 16)[0]["status"] == want, field
    for coef, want in ((P - 1, 0), (P, orc.EMALFORMED)):
        edge = proofs.copy()
        edge[0, 2 + 2 * 15], edge[0, 3 + 2 * 15] = coef & 0xFF, coef >> 8          # the last coefficient
        assert orc.verify(h, edge, 16)[0]["status"] == want, coef


def test_modulus_field_zero_stands_for_65536():
    """Top-k positions 65535 and 65540 (residues 65535 and 4) are distinct modulo 65536, so the search stops at
    its first candidate and the 2-byte field holds 0; a validator reading that 0 as anything but 65536 would
    evaluate the polynomial at other points and could not reproduce all-zero statistics."""
    n, k = 66000, 6
    h = np.full(n, 0x1000, dtype=np.uint16)
    big = [65535, 65540, 3, 40000, 65999, 100]
    h[big] = np.uint16(0x4500) + np.arange(6, dtype=np.uint16)
    proofs, status, idx = orc.build(h[None, :], k, want_topk=True)
    assert status[0] == 0 and sorted(idx[0].tolist()) == sorted(big)
    assert proofs[0, 0] == 0 and proofs[0, 1] == 0
    res = orc.verify(h[None, :], proofs, k)[0]
    assert res["err_exp"] == 0 and res["n_match"] == k and res["mant_sum"] == 0 and res["accept"] == 1
    m, c = decode(proofs[0])
    assert m == 65536 and all(poly_eval(c, (i % 65536) % P, P) == int(h[i]) for i in big)


def test_thread_count_does_not_change_results():
    rng = np.random.default_rng(26)
    h = np.stack([random_chunk(rng, 32 * 256, hidden=256) for _ in range(9)])
    p1, s1 = orc.build(h, 32, n_threads=1)
    p4, s4 = orc.build(h, 32, n_threads=4)
    assert (p1 == p4).all() and (s1 == s4).all()
