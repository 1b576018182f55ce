"""Host code under gcc's sanitizers (CPU only).

* tests/host/plan_check: the planning / validation header the HIP library compiles, built for the
  host with -fsanitize=address,undefined, re-runs the C ABI's rejection cases and sweeps the plans'
  invariants.
* tests/host/oracle_san: the CPU oracle's two C files behind a file-driven main, same sanitizers.  It
  gets the same bytes as the ordinary build of the oracle and must return the same bytes, on inputs
  chosen to walk the oracle's edges (k = N, one vector, ties, NaN patterns, a covering index set with no
  modulus, malformed proofs, both precisions and all four validator / proof pairs).
* the oracle's pins once more against a build with the undefined-behaviour sanitizer (a shared object
  with that sanitizer alone can be loaded into an ordinary Python).
"""
import os
import struct
import subprocess
import sys

import numpy as np
import pytest

import oracle as orc
from conftest import ROOT

sys.path.insert(0, os.path.join(ROOT, "tests", "host"))
import build_host  # noqa: E402

MAGIC = 0x544F504C4F43


@pytest.fixture(scope="module")
def programs():
    return build_host.build()


def run_clean(cmd, **kw):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600, **kw)
    assert res.returncode == 0, "%s failed (%d):\n%s\n%s" % (cmd[0], res.returncode, res.stdout[-2000:], res.stderr[-4000:])
    assert "runtime error" not in res.stderr and "Sanitizer" not in res.stderr, res.stderr[-4000:]
    return res


def test_planning_and_validation_header_under_sanitizers(programs):
    res = run_clean([programs[0]])
    assert "plan_check ok" in res.stdout


def request(tmp_path, op, payload, h_dtype=0, p_dtype=0, n_chunks=0, n=0, k=0, M=orc.PRIME, thr=(38, 10, 8), threads=2,
            mixed=0):
    words = [MAGIC, op, h_dtype, p_dtype, n_chunks, n, k, M, thr[0], thr[1], thr[2], threads, mixed, 0, 0, 0]
    req = tmp_path / ("req_%d_%d.bin" % (op, len(list(tmp_path.iterdir()))))
    req.write_bytes(struct.pack("<16Q", *words) + payload)
    return req, tmp_path / (req.name + ".out")


def sanitized_build(programs, tmp_path, bits, k, dtype=0, M=None):
    n_chunks, n = bits.shape
    M = M if M is not None else (orc.PRIME32 if dtype else orc.PRIME)
    req, out = request(tmp_path, 0, bits.tobytes(), h_dtype=dtype, p_dtype=dtype, n_chunks=n_chunks, n=n, k=k, M=M)
    run_clean([programs[1], str(req), str(out)])
    raw = out.read_bytes()
    pb = 2 + k * (4 if dtype else 2)
    rc = struct.unpack_from("<i", raw, 0)[0]
    proofs = np.frombuffer(raw, np.uint8, n_chunks * pb, 4).reshape(n_chunks, pb)
    status = np.frombuffer(raw, np.uint8, n_chunks, 4 + n_chunks * pb)
    idx = np.frombuffer(raw[4 + n_chunks * pb + n_chunks:], np.uint32, n_chunks * k).reshape(n_chunks, k)
    return rc, proofs, status, idx


def sanitized_verify(programs, tmp_path, bits, proofs, k, h_dtype=0, p_dtype=0, thr=(38, 10, 8)):
    n_chunks, n = bits.shape
    M = orc.PRIME32 if p_dtype else orc.PRIME
    req, out = request(tmp_path, 1, bits.tobytes() + np.ascontiguousarray(proofs).tobytes(), h_dtype=h_dtype, p_dtype=p_dtype,
                       n_chunks=n_chunks, n=n, k=k, M=M, thr=thr, mixed=1 if (h_dtype or p_dtype) else 0)
    run_clean([programs[1], str(req), str(out)])
    raw = out.read_bytes()
    return struct.unpack_from("<i", raw, 0)[0], np.frombuffer(raw, orc.RESULT_DTYPE, n_chunks, 4)


def edge_chunks_bf16():
    rng = np.random.default_rng(31)
    cases = []
    normal = (rng.standard_normal((3, 4096)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    normal[0, 17], normal[0, 99], normal[1, 5], normal[1, 6], normal[2, 0] = 0x7F80, 0xFF80, 0x7FC0, 0xFFFF, 0xFFD9
    cases.append((normal, 64))
    cases.append((np.full((2, 512), 0x3F80, dtype=np.uint16), 128))                         # all equal
    cases.append((rng.integers(0, 1 << 16, size=(2, 8)).astype(np.uint16), 8))              # one vector, k = N
    cases.append((rng.integers(0, 1 << 16, size=(4, 64)).astype(np.uint16), 1))             # k = 1
    asc = (np.arange(2048, dtype=np.uint32) * 15).astype(np.uint16).reshape(1, -1)
    cases.append((asc, 512))                                                                # sorted, k = N / 4
    collide = np.full((1, 70016), 0x3C00, dtype=np.uint16)
    for i, b in ((5, 0x4500), (65502, 0x4480), (1000, 0x4400), (70000, 0x4380)):
        collide[0, i] = b                                                                   # 5 and 65502 meet in GF(p)
    cases.append((collide, 4))
    cover = np.concatenate([np.arange(256), 32769 + 256 * np.arange(129)])                  # defeats every modulus
    nomod = (rng.integers(0x3000, 0x3800, size=(1, 32 * 4096)).astype(np.uint16))
    nomod[0, cover] = rng.integers(0x4000, 0x4400, size=cover.size).astype(np.uint16)
    cases.append((nomod, 512))
    return cases


def test_oracle_under_sanitizers_returns_the_same_bytes(programs, tmp_path):
    for bits, k in edge_chunks_bf16():
        want = orc.build(bits, k, want_topk=True)
        rc, proofs, status, idx = sanitized_build(programs, tmp_path, bits, k)
        assert rc == 0 and np.array_equal(proofs, want[0]) and np.array_equal(status, want[1]) and np.array_equal(idx, want[2])
        # verify against a perturbed copy, and against proofs damaged at both ends of the decode ranges
        rec = bits.copy()
        rec[:, ::7] ^= 1
        broken = want[0].copy()
        if broken.shape[0] > 1:
            broken[0, 0], broken[0, 1] = 0x00, 0x40                  # m = 16384
            broken[1, -2], broken[1, -1] = 0xFF, 0xFF                # a coefficient >= p
        for p in (want[0], broken):
            for thr in ((38, 10, 8), (0, 0, 0)):
                rc, res = sanitized_verify(programs, tmp_path, rec, p, k, thr=thr)
                assert rc == 0 and np.array_equal(res, orc.verify(rec, p, k, thresholds=thr))


def test_oracle32_under_sanitizers_returns_the_same_bytes(programs, tmp_path):
    rng = np.random.default_rng(32)
    x = rng.standard_normal((3, 2048)).astype(np.float32)
    x[0, 5], x[1, 7] = np.inf, -np.inf
    b32 = x.view(np.uint32).copy()
    b32[2, 9] = 0xFFFFFFFD                                            # a pattern >= 2^32 - 5
    b16 = (b32 >> 16).astype(np.uint16)
    for k in (1, 16, 128):
        want = orc.build32(b32, k, want_topk=True)
        rc, proofs, status, idx = sanitized_build(programs, tmp_path, b32, k, dtype=1)
        assert rc == 0 and np.array_equal(proofs, want[0]) and np.array_equal(status, want[1]) and np.array_equal(idx, want[2])
        p16 = orc.build(b16, k)[0]
        rec32 = b32.copy()
        rec32[:, ::5] ^= 0x200
        rec16 = (rec32 >> 16).astype(np.uint16)
        for rec, h_dt in ((rec32, orc.F32), (rec16, orc.BF16)):
            for p, p_dt in ((want[0], orc.F32), (p16, orc.BF16)):
                thr = (8, 256, 128) if h_dt == orc.F32 else (38, 10, 8)
                rc, res = sanitized_verify(programs, tmp_path, rec, p, k, h_dtype=h_dt, p_dtype=p_dt, thr=thr)
                assert rc == 0 and np.array_equal(res, orc.verify_mixed(rec, h_dt, p, p_dt, k, thresholds=thr))


def test_oracle_subroutines_under_sanitizers(programs, tmp_path):
    rng = np.random.default_rng(33)
    k = 128
    sets = np.stack([rng.choice(1 << 22, k, replace=False) for _ in range(64)]).astype(np.uint32)
    sets[1, :2] = (5, 65502)                                          # collide in GF(p) at m = 65536
    sets[2, :2] = (9, 9)                                              # a repeated index: no modulus at all
    req, out = request(tmp_path, 2, sets.tobytes(), n_chunks=sets.shape[0], k=k)
    run_clean([programs[1], str(req), str(out)])
    raw = out.read_bytes()
    n = sets.shape[0]
    m = np.frombuffer(raw, np.uint32, n, 4)
    st = np.frombuffer(raw, np.uint8, n, 4 + 4 * n)
    want_m, want_st = orc.find_injective_modulus_batch(sets)
    assert np.array_equal(st, want_st) and np.array_equal(m[st == 0], want_m[want_st == 0]) and st[2] == orc.ENOMOD
    pos = 4 + 5 * n
    inv_sum, bad = struct.unpack_from("<qq", raw, pos)
    # a * a^-1 = 1 for every residue; modulus 1 gives 0; gcd(6, 9) != 1 sets the error code
    assert inv_sum == 65496 + 0 + orc.ENOINV
    assert bad == 0                          # Algorithm 5 on Algorithm 3's output returns every encoded value
    coef = np.frombuffer(raw, np.int64, k, pos + 16)
    x = (sets[0] % m[0]) % orc.PRIME
    y = ((sets[0].astype(np.uint64) * 2654435761 % (1 << 32)) >> 16) % orc.PRIME
    assert np.array_equal(coef, orc.interpolate(x, y))
    # Algorithm 6 to the letter (M = 0): indices 5 and 65502 are then fine at m = 65536
    req, out = request(tmp_path, 2, sets[1:3].tobytes(), n_chunks=2, k=k, M=0)
    run_clean([programs[1], str(req), str(out)])
    raw = out.read_bytes()
    want_m, want_st = orc.find_injective_modulus_batch(sets[1:3], M=0)
    assert np.array_equal(np.frombuffer(raw, np.uint8, 2, 12), want_st) and want_st.tolist() == [0, orc.ENOMOD]
    assert np.frombuffer(raw, np.uint32, 2, 4)[0] == want_m[0]


def test_oracle_pins_against_the_undefined_behaviour_sanitizer_build():
    env = dict(os.environ, TOPLOC_ORACLE_SANITIZE="undefined")
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                          os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_oracle_f32_pins.py")],
                         cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=1200)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "runtime error" not in res.stdout
    assert os.path.exists(os.path.join(ROOT, "oracle", "libtoploc_oracle_undefined.so"))
