"""Pins for the 32-bit CPU oracle (oracle/toploc_oracle_f32.c), CPU only.

The paper prints no worked example for fp32 proofs either, so the pins are what the
mathematics fixes: uniqueness of the interpolating polynomial (against Lagrange sums in
Python integers and against the already pinned 16-bit routine on a common modulus),
exhaustive small fields, brute-force top-k, Algorithm 6 against the pinned routine, the
round trip P(x_j) = y_j through the proof bytes, and closed-form outcomes of validation
across precisions (Section 5.7) on inputs built so that the result is known by hand.
"""
import itertools

import numpy as np
import pytest

import oracle as orc

P32 = orc.PRIME32


def lagrange_coeffs(xs, ys, M):
    """Coefficients (ascending) of the interpolating polynomial mod prime M, Python integers."""
    n = len(xs)
    out = [0] * n
    for j in range(n):
        num = [1]                                   # prod_{i != j} (X - x_i)
        den = 1
        for i in range(n):
            if i == j:
                continue
            num = [(a - xs[i] * b) % M for a, b in zip([0] + num, num + [0])]
            den = den * (xs[j] - xs[i]) % M
        scale = ys[j] * pow(den, M - 2, M) % M
        for d in range(n):
            out[d] = (out[d] + scale * num[d]) % M
    return out


def test_prime_and_sizes(golden):
    g = {r[0]: int(r[1]) for r in golden("sizes_and_thresholds.txt")}
    assert orc.F32_THRESHOLDS == (g["t_exp_fp32"], g["t_mean_fp32"], g["t_median_fp32"])
    assert g["mantissa_bits_fp32"] - g["mantissa_bits_bf16"] == 16          # the shift between the two precisions
    assert P32 == 2 ** 32 - 5
    assert all(P32 % q for q in range(2, 65536))     # trial division up to sqrt(2^32)
    assert orc.proof_bytes32(128) == 514 and orc.proof_bytes32(1) == 6
    assert orc.F32_THRESHOLDS == (8, 256, 128)        # Section 5.2, fp32 inference


@pytest.mark.parametrize("n", [1, 2, 3, 7, 24])
def test_interpolation_equals_lagrange_and_round_trips(n):
    rng = np.random.default_rng(100 + n)
    xs = rng.choice(65536, size=n, replace=False).astype(np.uint64)
    ys = rng.integers(0, 2 ** 32, size=n, dtype=np.uint64)
    c = orc.interpolate32(xs, ys)
    want = lagrange_coeffs([int(v) for v in xs], [int(v) % P32 for v in ys], P32)
    assert [int(v) for v in c] == want
    for x, y in zip(xs, ys):
        assert orc.horner32(c, int(x)) == int(y) % P32
    perm = rng.permutation(n)
    assert np.array_equal(orc.interpolate32(xs[perm], ys[perm]), c)      # uniqueness: order is irrelevant


def test_values_at_and_above_the_modulus_reduce():
    xs = np.array([3, 9, 12], dtype=np.uint64)
    ys = np.array([P32, 2 ** 32 - 1, 7], dtype=np.uint64)
    c = orc.interpolate32(xs, ys)
    assert [orc.horner32(c, int(x)) for x in xs] == [0, 4, 7]


def test_same_modulus_same_coefficients_as_the_16_bit_routine():
    rng = np.random.default_rng(7)
    xs = rng.choice(65497, size=16, replace=False)
    ys = rng.integers(0, 65497, size=16)
    assert [int(v) for v in orc.interpolate32(xs, ys, M=65497)] == [int(v) for v in orc.interpolate(xs, ys, M=65497)]
    assert orc.horner32(orc.interpolate32(xs, ys, M=65497), 1234, M=65497) == \
        orc.horner(orc.interpolate(xs, ys, M=65497), 1234, M=65497)


def test_every_function_on_three_points_of_gf5():
    for ys in itertools.product(range(5), repeat=3):
        c = orc.interpolate32([0, 1, 2], list(ys), M=5)
        assert all(int(v) < 5 for v in c)
        for x in range(3):
            assert orc.horner32(c, x, M=5) == ys[x]


def test_zero_denominator_is_reported():
    with pytest.raises(ZeroDivisionError):
        orc.interpolate32([4, 4], [1, 2])


def brute_topk(bits, k, mask):
    mags = [int(b) & mask for b in bits]
    taken = []
    for _ in range(k):
        best = None
        for i, m in enumerate(mags):
            if i in taken:
                continue
            if best is None or m > mags[best]:
                best = i
        taken.append(best)
    return taken


def test_topk_brute_force_both_precisions():
    rng = np.random.default_rng(11)
    for trial in range(20):
        n = int(rng.integers(8, 48))
        k = int(rng.integers(1, 9))
        b32 = rng.integers(0, 2 ** 32, size=n, dtype=np.uint64).astype(np.uint32)
        b32[rng.integers(0, n, size=n // 3)] = b32[0]                    # ties
        b32[rng.integers(0, n)] ^= np.uint32(0x80000000)                 # a sign flip must not change the rank
        idx, val = orc.topk32(b32, k, orc.F32)
        want = brute_topk(b32, k, 0x7FFFFFFF)
        assert idx.tolist() == want and val.tolist() == [int(b32[i]) for i in want]
        b16 = (b32 >> 16).astype(np.uint16)
        idx, val = orc.topk32(b16, k, orc.BF16)
        want = brute_topk(b16, k, 0x7FFF)
        assert idx.tolist() == want and val.tolist() == [int(b16[i]) for i in want]
        i16, v16 = orc.topk(b16, k)                                      # the pinned 16-bit routine agrees
        assert i16.tolist() == want


def test_modulus_equals_the_pinned_algorithm_6():
    rng = np.random.default_rng(12)
    for _ in range(200):
        idx = rng.integers(0, 2 ** 31, size=128, dtype=np.int64).astype(np.uint32)
        assert orc.find_injective_modulus32(idx) == orc.find_injective_modulus(idx, M=0)
    assert orc.find_injective_modulus32(np.array([0, 65536, 5], dtype=np.uint32)) == 65535


def f32_chunks(n_chunks, n, seed, n_big=160):
    """fp32 patterns: small bulk, n_big large well-separated magnitudes per chunk (distinct upper 16 bits)."""
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((n_chunks, n)) * 0.01).astype(np.float32)
    bits = x.view(np.uint32).copy()
    for c in range(n_chunks):
        pos = rng.choice(n, size=n_big, replace=False)
        hi = rng.choice(np.arange(0x4000, 0x4700), size=n_big, replace=False).astype(np.uint32)  # 2.0 .. 8192
        lo = rng.integers(0, 2 ** 16, size=n_big, dtype=np.uint64).astype(np.uint32)
        sign = rng.integers(0, 2, size=n_big, dtype=np.uint64).astype(np.uint32) << 31
        bits[c, pos] = sign | (hi << 16) | lo
    return bits


def decode32(proof, k):
    m = int(proof[0]) | int(proof[1]) << 8
    m = m if m else 65536
    c = np.frombuffer(proof[2:].tobytes(), dtype="<u4").astype(np.uint64)
    assert c.size == k
    return m, c


def test_build_round_trip_through_the_proof_bytes():
    bits = f32_chunks(3, 4096, 21)
    proofs, status, idx = orc.build32(bits, 128, want_topk=True)
    assert proofs.shape == (3, 514) and not status.any()
    for c in range(3):
        m, coef = decode32(proofs[c], 128)
        assert 32769 <= m <= 65536 and (coef < P32).all()
        res = idx[c] % m
        assert len(set(res.tolist())) == 128                              # injective
        for i in idx[c]:
            assert orc.horner32(coef, int(i) % m) == int(bits[c, i]) % P32
        want_idx, _ = orc.topk32(bits[c], 128, orc.F32)
        assert np.array_equal(idx[c], want_idx)


def test_self_validation_and_mantissa_bit_flips():
    bits = f32_chunks(2, 4096, 22)
    proofs, _ = orc.build32(bits, 128)
    res = orc.verify_mixed(bits, orc.F32, proofs, orc.F32, 128)
    assert (res["accept"] == 1).all() and (res["err_exp"] == 0).all() and (res["mant_sum"] == 0).all()
    assert (res["n_match"] == 128).all() and (res["mant_median"] == 0).all()
    idx, _ = orc.topk32(bits[0], 128, orc.F32)
    rec = bits.copy()
    for r, i in enumerate(idx[:40]):
        rec[0, i] ^= np.uint32(1 << 9)                                    # |delta mantissa| = 512 each, rank unchanged
    res = orc.verify_mixed(rec, orc.F32, proofs, orc.F32, 128)
    assert res["mant_sum"][0] == 40 * 512 and res["err_exp"][0] == 0 and res["mant_median"][0] == 0
    assert res["accept"][0] == 1                                          # mean 160 <= 256, median 0
    for i in idx[40:70]:
        rec[0, i] ^= np.uint32(1 << 9)
    res = orc.verify_mixed(rec, orc.F32, proofs, orc.F32, 128)
    assert res["mant_sum"][0] == 70 * 512 and res["mant_median"][0] == 512 and res["accept"][0] == 0   # mean 280 > 256
    rec = bits.copy()
    rec[1, idx[0]] ^= np.uint32(0x80000000)                               # the sign is not compared
    rec[1, orc.topk32(bits[1], 128, orc.F32)[0][5]] ^= np.uint32(1 << 23)  # one binade step: an exponent mismatch
    res = orc.verify_mixed(rec, orc.F32, proofs, orc.F32, 128)
    assert res["err_exp"][1] >= 1 and res["n_match"][1] + res["err_exp"][1] == 128


def round_to_bf16(bits32):
    """Round to nearest even of fp32 patterns to bf16 patterns (no NaN/Inf in the inputs here)."""
    b = bits32.astype(np.uint64)
    lsb = (b >> 16) & 1
    return (((b + 0x7FFF + lsb) >> 16) & 0xFFFF).astype(np.uint16)


def test_validation_across_precisions_closed_forms():
    bits = f32_chunks(2, 4096, 23)
    # keep mantissa carries and rounding ties out of the picture: top 7 mantissa bits never all ones, low half never 0x8000
    big = (bits & 0x7FFFFFFF) > 0x3F800000
    bits[big & ((bits >> 16) & 0x7F == 0x7F)] ^= np.uint32(1 << 16)
    bits[big & ((bits & 0xFFFF) == 0x8000)] ^= np.uint32(1)
    b16 = round_to_bf16(bits)
    k = 128
    p32, _ = orc.build32(bits, k)
    p16, _ = orc.build(b16, k)
    for c in range(2):
        idx, val = orc.topk32(bits[c], k, orc.F32)
        idx16, _ = orc.topk32(b16[c], k, orc.BF16)
        assert set(idx.tolist()) == set(idx16.tolist())                   # distinct upper halves: same top-k set
        low = val & 0xFFFF
        up = low > 0x8000
        # fp32 proof, bf16 validator: the proof mantissa is cut to 7 bits, the validator's was rounded
        res = orc.verify_mixed(b16[c:c + 1], orc.BF16, p32[c:c + 1], orc.F32, k)
        assert res["err_exp"][0] == 0 and res["n_match"][0] == k
        assert res["mant_sum"][0] == int(up.sum()) and res["accept"][0] == 1
        # bf16 proof, fp32 validator: the proof mantissa gets 16 zero bits, the validator's has them all
        res = orc.verify_mixed(bits[c:c + 1], orc.F32, p16[c:c + 1], orc.BF16, k)
        want = np.where(up, 65536 - low.astype(np.int64), low.astype(np.int64))
        assert res["err_exp"][0] == 0 and res["n_match"][0] == k
        assert res["mant_sum"][0] == int(want.sum())
        assert res["mant_median"][0] == int(np.sort(want)[(k - 1) // 2])
        assert res["accept"][0] == 0                                      # fp32 thresholds 256 / 128: always fails (Table 5)
    # values that bf16 holds exactly validate with all-zero statistics in every combination
    exact = bits & np.uint32(0xFFFF0000)
    e16 = (exact >> 16).astype(np.uint16)
    pe32, _ = orc.build32(exact, k)
    pe16, _ = orc.build(e16, k)
    for h, hd, p, pd in ((exact, orc.F32, pe16, orc.BF16), (e16, orc.BF16, pe32, orc.F32), (exact, orc.F32, pe32, orc.F32),
                         (e16, orc.BF16, pe16, orc.BF16)):
        res = orc.verify_mixed(h, hd, p, pd, k)
        assert (res["accept"] == 1).all() and (res["mant_sum"] == 0).all() and (res["err_exp"] == 0).all()
    # the bf16 / bf16 combination is the pinned 16-bit oracle
    a = orc.verify_mixed(b16, orc.BF16, p16, orc.BF16, k)
    b = orc.verify(b16, p16, k)
    for f in ("err_exp", "n_match", "mant_sum", "mant_median", "accept", "status"):
        assert np.array_equal(a[f], b[f])


def test_malformed_proofs():
    bits = f32_chunks(1, 1024, 24)
    p, _ = orc.build32(bits, 16)
    bad = p.copy()
    bad[0, 2:6] = (0xFF, 0xFF, 0xFF, 0xFF)                                 # c_0 = 2^32 - 1 >= M
    res = orc.verify_mixed(bits, orc.F32, bad, orc.F32, 16)
    assert res["status"][0] == orc.EMALFORMED and res["accept"][0] == 0
    bad = p.copy()
    bad[0, 0], bad[0, 1] = 0x00, 0x40                                      # m = 16384
    res = orc.verify_mixed(bits, orc.F32, bad, orc.F32, 16)
    assert res["status"][0] == orc.EMALFORMED and res["accept"][0] == 0
    # the edges: m = 2^15 is out, 2^15 + 1 is in; a coefficient M - 1 is in, M is out
    for field, want in ((32768, orc.EMALFORMED), (32769, 0)):
        edge = p.copy()
        edge[0, 0], edge[0, 1] = field & 0xFF, field >> 8
        assert orc.verify_mixed(bits, orc.F32, edge, orc.F32, 16)["status"][0] == want, field
    for coef, want in ((P32 - 1, 0), (P32, orc.EMALFORMED)):
        edge = p.copy()
        edge[0, 2 + 4 * 15: 6 + 4 * 15] = np.frombuffer(int(coef).to_bytes(4, "little"), dtype=np.uint8)
        assert orc.verify_mixed(bits, orc.F32, edge, orc.F32, 16)["status"][0] == want, coef
    # a field of 0 stands for 65536: positions 65535 and 65540 do not collide there
    n, k = 66000, 6
    b = np.full(n, 0x3C000000, dtype=np.uint32)
    big = [65535, 65540, 3, 40000, 65999, 100]
    b[big] = np.uint32(0x45000000) + np.arange(6, dtype=np.uint32) * np.uint32(0x10001)
    proofs, status = orc.build32(b[None, :], k)
    assert status[0] == 0 and proofs[0, 0] == 0 and proofs[0, 1] == 0
    res = orc.verify_mixed(b[None, :], orc.F32, proofs, orc.F32, k)
    assert res["err_exp"][0] == 0 and res["mant_sum"][0] == 0 and res["n_match"][0] == k


def brute_verify_mixed(bits, h_dtype, proof, p_dtype, thresholds):
    """Algorithm 2 across precisions on one small chunk in Python integers: decode, top-k by repeated
    arg-max, the polynomial by its definition (sum of c_d x^d), fields by shifts, the mantissa brought to
    the validator's width, sorted lower median."""
    width = 4 if p_dtype == orc.F32 else 2
    M = P32 if p_dtype == orc.F32 else 65497
    m = int(proof[0]) | (int(proof[1]) << 8)
    m = m if m else 65536
    k = (len(proof) - 2) // width
    c = [int.from_bytes(bytes(proof[2 + width * j: 2 + width * (j + 1)].tolist()), "little") for j in range(k)]
    mask = 0x7FFFFFFF if h_dtype == orc.F32 else 0x7FFF
    err_e, err_m = 0, []
    for i in brute_topk(bits, k, mask):
        x = (i % m) % M
        val = sum(cd * pow(x, d, M) for d, cd in enumerate(c)) % M
        if p_dtype == orc.F32:
            e_p, m_p = (val >> 23) & 0xFF, val & 0x7FFFFF
        else:
            e_p, m_p = (val >> 7) & 0xFF, val & 0x7F
        v = int(bits[i])
        if h_dtype == orc.F32:
            e_v, m_v = (v >> 23) & 0xFF, v & 0x7FFFFF
        else:
            e_v, m_v = (v >> 7) & 0xFF, v & 0x7F
        if p_dtype == orc.F32 and h_dtype == orc.BF16:
            m_p >>= 16                                   # 23 bits scaled to 7
        if p_dtype == orc.BF16 and h_dtype == orc.F32:
            m_p <<= 16                                   # 16 zero bits appended
        if e_p == e_v:
            err_m.append(abs(m_p - m_v))
        else:
            err_e += 1
    n = len(err_m)
    median = sorted(err_m)[(n - 1) // 2] if n else 0
    t_exp, t_mean, t_median = thresholds
    reject = err_e > t_exp or (n > 0 and (sum(err_m) > t_mean * n or median > t_median))
    return {"err_exp": err_e, "n_match": n, "mant_sum": sum(err_m), "mant_median": median, "accept": 0 if reject else 1}


@pytest.mark.parametrize("seed", range(8))
def test_validation_equals_brute_force_in_all_four_precision_pairs(seed):
    rng = np.random.default_rng(5200 + seed)
    n = int(rng.choice([32, 96, 256]))
    k = int(rng.choice([4, 12, 25]))
    x = (rng.standard_normal(n) * 3.0).astype(np.float32)
    b32 = x.view(np.uint32).copy()
    b16 = (b32 >> 16).astype(np.uint16)
    p32, st32 = orc.build32(b32[None, :], k)
    p16, st16 = orc.build(b16[None, :], k)
    assert st32[0] == 0 and st16[0] == 0
    # a recomputation: low mantissa bits move everywhere, a few exponents step, a few entries change hands
    r32 = b32.copy()
    r32 ^= rng.integers(0, 1 << 19, size=n, dtype=np.uint64).astype(np.uint32) * (rng.random(n) < 0.6)
    step = rng.choice(n, size=max(1, n // 16), replace=False)
    r32[step] += np.uint32(1 << 23)
    swap = rng.choice(n, size=2, replace=False)
    r32[swap] = r32[swap[::-1]]
    r16 = (r32 >> 16).astype(np.uint16)
    for rbits, h_dt in ((r32, orc.F32), (r16, orc.BF16)):
        for proof, p_dt in ((p32[0], orc.F32), (p16[0], orc.BF16)):
            hi = 1 << 18 if h_dt == orc.F32 else 12
            thresholds = (int(rng.integers(0, k)), int(rng.integers(0, hi)), int(rng.integers(0, hi)))
            got = orc.verify_mixed(rbits[None, :], h_dt, proof[None, :], p_dt, k, thresholds=thresholds)[0]
            want = brute_verify_mixed(rbits, h_dt, proof, p_dt, thresholds)
            for f, v in want.items():
                assert int(got[f]) == v, (h_dt, p_dt, f, int(got[f]), v)
            assert got["status"] == 0 and want["err_exp"] + want["n_match"] == k


def test_thresholds_are_strict_and_the_search_reaches_its_last_candidate():
    """Equality with a threshold accepts, one more rejects (Algorithm 2 compares with '>'), for each of the
    three statistics; Algorithm 6's range ends at 2^15 + 1 inclusive."""
    bits = f32_chunks(1, 4096, 31)
    k = 128
    proofs, _ = orc.build32(bits, k)
    idx, _ = orc.topk32(bits[0], k, orc.F32)
    rec = bits.copy()
    for i in idx[:64]:
        rec[0, i] ^= np.uint32(1 << 4)                 # 64 entries differ by 16, 64 by 0: sum = 8 k, lower median 0
    for i in idx[64:67]:
        rec[0, i] ^= np.uint32(1 << 23)                # three binade steps: err_e = 3, their mantissas drop out
    base = orc.verify_mixed(rec, orc.F32, proofs, orc.F32, k, thresholds=(3, 1 << 20, 1 << 20))[0]
    assert base["err_exp"] == 3 and base["n_match"] == k - 3 and base["mant_sum"] == 64 * 16 and base["accept"] == 1
    assert orc.verify_mixed(rec, orc.F32, proofs, orc.F32, k, thresholds=(2, 1 << 20, 1 << 20))[0]["accept"] == 0
    rec = bits.copy()
    for i in idx[:96]:
        rec[0, i] ^= np.uint32(1 << 4)                 # 96 * 16 = 1536 = 12 * 128: mean exactly 12, median 16
    assert orc.verify_mixed(rec, orc.F32, proofs, orc.F32, k, thresholds=(0, 12, 16))[0]["accept"] == 1
    assert orc.verify_mixed(rec, orc.F32, proofs, orc.F32, k, thresholds=(0, 11, 16))[0]["accept"] == 0
    assert orc.verify_mixed(rec, orc.F32, proofs, orc.F32, k, thresholds=(0, 12, 15))[0]["accept"] == 0
    # the smallest candidate: differences cover 32770..65537, nothing that 32769 divides
    low = np.concatenate([np.arange(256), 32770 + 255 + 256 * np.arange(128)]).astype(np.uint32)
    assert orc.find_injective_modulus32(low) == 32769 == orc.find_injective_modulus(low, M=0)
    cover = np.concatenate([np.arange(256), 32769 + 256 * np.arange(129)]).astype(np.uint32)
    with pytest.raises(ValueError):
        orc.find_injective_modulus32(cover)


def test_validation_maps_indices_with_the_proofs_modulus():
    """Top-k positions 5 and 65541 collide modulo 65536, so the proof carries a smaller modulus; a validator
    that mapped indices with anything else would evaluate the polynomial at the wrong points."""
    rng = np.random.default_rng(41)
    n, k = 70000, 8
    b32 = (rng.standard_normal(n) * 0.01).astype(np.float32).view(np.uint32).copy()
    big = [5, 65541, 69999, 40000, 123, 65536 + 123 + 7, 33000, 1]
    b32[big] = (np.float32(100.0) + np.arange(8, dtype=np.float32)).view(np.uint32)
    for bits, dt, build in ((b32, orc.F32, orc.build32), ((b32 >> 16).astype(np.uint16), orc.BF16, orc.build)):
        proofs, status = build(bits[None, :], k)
        m = int(proofs[0, 0]) | (int(proofs[0, 1]) << 8)
        assert status[0] == 0 and 32769 <= m < 65536
        rec = bits.copy()
        rec[big[:4]] ^= rec.dtype.type(1)                                  # four low mantissa bits move
        for h_dt, rbits in ((dt, rec),):
            got = orc.verify_mixed(rbits[None, :], h_dt, proofs, dt, k)[0]
            want = brute_verify_mixed(rbits, h_dt, proofs[0], dt, (8, 256, 128) if h_dt == orc.F32 else (38, 10, 8))
            assert want["err_exp"] == 0 and want["mant_sum"] == 4
            for f, v in want.items():
                assert int(got[f]) == v, (dt, f, int(got[f]), v)
