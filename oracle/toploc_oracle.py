"""ctypes access to the plain-C TopLoc oracle (oracle/toploc_oracle.c).

Test infrastructure only: argument marshalling between numpy arrays and the C
functions, nothing of the method is computed here.  The C file states which
passage of the paper each function follows (Section 4, Algorithms 1-2;
Appendix C, Algorithms 3-6).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "toploc_oracle.c")
_SRC32 = os.path.join(_HERE, "toploc_oracle_f32.c")
_LIB = os.path.join(_HERE, "libtoploc_oracle.so")

PRIME = 65497
T_EXP, T_MEAN, T_MEDIAN = 38, 10, 8  # bf16 thresholds, Section 5.2

OK, ENOMOD, ENOINV, EMALFORMED = 0, 1, 2, 3

RESULT_DTYPE = np.dtype(
    [
        ("err_exp", "<u4"),
        ("n_match", "<u4"),
        ("mant_sum", "<u4"),
        ("mant_median", "<u4"),
        ("accept", "u1"),
        ("status", "u1"),
        ("pad", "u1", (2,)),
    ]
)
assert RESULT_DTYPE.itemsize == 20


# TOPLOC_ORACLE_SANITIZE=undefined selects a second build of the same two C files with gcc's
# undefined-behaviour sanitizer (every finding aborts), so that the pins can be run against it.
_SANITIZE = os.environ.get("TOPLOC_ORACLE_SANITIZE", "")
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libtoploc_oracle_%s.so" % _SANITIZE.replace(",", "_"))


def build_library(force=False):
    """Compile the oracle with gcc (plain C11, -O2, OpenMP over chunks)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC),
                                                                          os.path.getmtime(_SRC32)):
        flags = ["-O2"]
        if _SANITIZE:
            flags = ["-O1", "-g", "-fsanitize=" + _SANITIZE, "-fno-sanitize-recover=all"]
        subprocess.check_call(
            ["gcc"] + flags + ["-std=gnu11", "-Wall", "-Wextra", "-fopenmp", "-fPIC", "-shared", _SRC, _SRC32, "-o", _LIB]
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build_library()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        P = c.c_void_p
        lib.toploc_oracle_topk.argtypes = [P, c.c_uint64, c.c_uint32, P, P]
        lib.toploc_oracle_mod_inverse.argtypes = [c.c_int64, c.c_int64, c.POINTER(c.c_int)]
        lib.toploc_oracle_mod_inverse.restype = c.c_int64
        lib.toploc_oracle_interpolate.argtypes = [P, P, c.c_uint32, c.c_int64, P]
        lib.toploc_oracle_horner.argtypes = [P, c.c_uint32, c.c_int64, c.c_int64]
        lib.toploc_oracle_horner.restype = c.c_int64
        lib.toploc_oracle_find_injective_modulus.argtypes = [P, c.c_uint32, c.c_uint32, c.POINTER(c.c_uint32)]
        lib.toploc_oracle_find_injective_modulus_batch.argtypes = [P, c.c_uint64, c.c_uint32, c.c_uint32, P, P]
        lib.toploc_oracle_build.argtypes = [P, c.c_uint64, c.c_uint64, c.c_uint32, c.c_uint32, P, P, P, c.c_int]
        lib.toploc_oracle_verify.argtypes = [
            P, c.c_uint64, c.c_uint64, c.c_uint32, c.c_uint32, P, c.c_uint32, c.c_uint32, c.c_uint32, P, c.c_int,
        ]
        lib.toploc_oracle_decide.argtypes = [c.c_uint32, P, c.c_uint32, c.c_uint32, c.c_uint32, c.c_uint32, P]
        lib.toploc_oracle_max_threads.restype = c.c_int
        lib.toploc_oracle32_topk.argtypes = [P, c.c_int, c.c_uint64, c.c_uint32, P, P]
        lib.toploc_oracle32_interpolate.argtypes = [P, P, c.c_uint32, c.c_uint64, P]
        lib.toploc_oracle32_horner.argtypes = [P, c.c_uint32, c.c_uint64, c.c_uint64]
        lib.toploc_oracle32_horner.restype = c.c_uint64
        lib.toploc_oracle32_find_injective_modulus.argtypes = [P, c.c_uint32, c.POINTER(c.c_uint32)]
        lib.toploc_oracle32_build.argtypes = [P, c.c_uint64, c.c_uint64, c.c_uint32, c.c_uint64, P, P, P, c.c_int]
        lib.toploc_oracle32_verify.argtypes = [P, c.c_int, c.c_uint64, c.c_uint64, c.c_uint32, P, c.c_int, c.c_uint64,
                                               c.c_uint32, c.c_uint32, c.c_uint32, P, c.c_int]
        _lib = lib
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def max_threads():
    return int(_load().toploc_oracle_max_threads())


def proof_bytes(k):
    return 2 + 2 * k


def topk(h_bits, k):
    """h_bits: 1-D uint16 array of bf16 patterns. Returns (idx uint32[k], val uint16[k])."""
    h = np.ascontiguousarray(h_bits, dtype=np.uint16).ravel()
    idx = np.empty(k, dtype=np.uint32)
    val = np.empty(k, dtype=np.uint16)
    rc = _load().toploc_oracle_topk(_ptr(h), h.size, k, _ptr(idx), _ptr(val))
    if rc:
        raise ValueError("oracle topk: bad arguments (k=%d, n=%d)" % (k, h.size))
    return idx, val


def mod_inverse(a, m):
    err = ctypes.c_int(0)
    r = _load().toploc_oracle_mod_inverse(int(a), int(m), ctypes.byref(err))
    if err.value:
        raise ZeroDivisionError("no inverse: gcd(%d, %d) != 1" % (a, m))
    return int(r)


def interpolate(x, y, M=PRIME):
    x = np.ascontiguousarray(x, dtype=np.int64)
    y = np.ascontiguousarray(y, dtype=np.int64)
    assert x.shape == y.shape and x.ndim == 1
    c = np.empty(x.size, dtype=np.int64)
    rc = _load().toploc_oracle_interpolate(_ptr(x), _ptr(y), x.size, int(M), _ptr(c))
    if rc == ENOINV:
        raise ZeroDivisionError("interpolate: non-invertible denominator")
    if rc:
        raise ValueError("interpolate: bad arguments")
    return c


def horner(c, x, M=PRIME):
    c = np.ascontiguousarray(c, dtype=np.int64)
    return int(_load().toploc_oracle_horner(_ptr(c), c.size, int(x), int(M)))


def find_injective_modulus(idx, M=PRIME):
    """M=0: Algorithm 6 to the letter; M=p: residues must stay distinct mod p too."""
    idx = np.ascontiguousarray(idx, dtype=np.uint32)
    m = ctypes.c_uint32(0)
    rc = _load().toploc_oracle_find_injective_modulus(_ptr(idx), idx.size, int(M), ctypes.byref(m))
    if rc == ENOMOD:
        raise ValueError("No injective modulus found!")
    if rc:
        raise ValueError("find_injective_modulus: bad arguments")
    return int(m.value)


def find_injective_modulus_batch(sets, M=PRIME):
    sets = np.ascontiguousarray(sets, dtype=np.uint32)
    n_sets, n = sets.shape
    m = np.empty(n_sets, dtype=np.uint32)
    st = np.empty(n_sets, dtype=np.uint8)
    _load().toploc_oracle_find_injective_modulus_batch(_ptr(sets), n_sets, n, int(M), _ptr(m), _ptr(st))
    return m, st


def build(h_bits, k, M=PRIME, want_topk=False, n_threads=0):
    """h_bits: uint16 [n_chunks, N]. Returns (proofs uint8 [n_chunks, 2+2k], status uint8 [n_chunks][, idx])."""
    h = np.ascontiguousarray(h_bits, dtype=np.uint16)
    assert h.ndim == 2
    n_chunks, n = h.shape
    proofs = np.zeros((n_chunks, proof_bytes(k)), dtype=np.uint8)
    status = np.zeros(n_chunks, dtype=np.uint8)
    idx = np.zeros((n_chunks, k), dtype=np.uint32) if want_topk else None
    nt = n_threads if n_threads > 0 else max_threads()
    rc = _load().toploc_oracle_build(
        _ptr(h), n_chunks, n, k, int(M), _ptr(proofs), _ptr(status), _ptr(idx) if want_topk else None, nt
    )
    if rc:
        raise ValueError("oracle build: bad arguments")
    return (proofs, status, idx) if want_topk else (proofs, status)


def verify(h_bits, proofs, k, M=PRIME, thresholds=(T_EXP, T_MEAN, T_MEDIAN), n_threads=0):
    """Returns a structured array (RESULT_DTYPE) with one record per chunk."""
    h = np.ascontiguousarray(h_bits, dtype=np.uint16)
    assert h.ndim == 2
    n_chunks, n = h.shape
    proofs = np.ascontiguousarray(proofs, dtype=np.uint8)
    assert proofs.shape == (n_chunks, proof_bytes(k))
    res = np.zeros(n_chunks, dtype=RESULT_DTYPE)
    nt = n_threads if n_threads > 0 else max_threads()
    rc = _load().toploc_oracle_verify(
        _ptr(h), n_chunks, n, k, int(M), _ptr(proofs), int(thresholds[0]), int(thresholds[1]), int(thresholds[2]),
        _ptr(res), nt,
    )
    if rc:
        raise ValueError("oracle verify: bad arguments")
    return res


def decide(err_e, err_m, thresholds=(T_EXP, T_MEAN, T_MEDIAN)):
    err_m = np.ascontiguousarray(err_m, dtype=np.uint32)
    res = np.zeros(1, dtype=RESULT_DTYPE)
    _load().toploc_oracle_decide(
        int(err_e), _ptr(err_m), err_m.size, int(thresholds[0]), int(thresholds[1]), int(thresholds[2]), _ptr(res)
    )
    return res[0]


# ---------------------------------------------------------------------------
# 32-bit variant (oracle/toploc_oracle_f32.c): fp32 proofs and validation across precisions
# ---------------------------------------------------------------------------
PRIME32 = 4294967291          # 2^32 - 5
BF16, F32 = 0, 1
F32_THRESHOLDS = (8, 256, 128)  # T_exp, T_mean, T_median for fp32 inference, Section 5.2


def proof_bytes32(k):
    return 2 + 4 * k


def _patterns(h, dtype):
    return np.ascontiguousarray(h, dtype=np.uint32 if dtype == F32 else np.uint16)


def topk32(h_bits, k, dtype=F32):
    """1-D patterns (uint32 for F32, uint16 for BF16). Returns (idx uint32[k], val uint32[k])."""
    h = _patterns(h_bits, dtype).ravel()
    idx = np.empty(k, dtype=np.uint32)
    val = np.empty(k, dtype=np.uint32)
    rc = _load().toploc_oracle32_topk(_ptr(h), dtype, h.size, k, _ptr(idx), _ptr(val))
    if rc:
        raise ValueError("oracle topk32: bad arguments")
    return idx, val


def interpolate32(x, y, M=PRIME32):
    x = np.ascontiguousarray(x, dtype=np.uint64)
    y = np.ascontiguousarray(y, dtype=np.uint64)
    assert x.shape == y.shape and x.ndim == 1
    c = np.empty(x.size, dtype=np.uint64)
    rc = _load().toploc_oracle32_interpolate(_ptr(x), _ptr(y), x.size, int(M), _ptr(c))
    if rc == ENOINV:
        raise ZeroDivisionError("interpolate32: non-invertible denominator")
    if rc:
        raise ValueError("interpolate32: bad arguments")
    return c


def horner32(c, x, M=PRIME32):
    c = np.ascontiguousarray(c, dtype=np.uint64)
    return int(_load().toploc_oracle32_horner(_ptr(c), c.size, int(x), int(M)))


def find_injective_modulus32(idx):
    idx = np.ascontiguousarray(idx, dtype=np.uint32)
    m = ctypes.c_uint32(0)
    rc = _load().toploc_oracle32_find_injective_modulus(_ptr(idx), idx.size, ctypes.byref(m))
    if rc:
        raise ValueError("No injective modulus found!")
    return int(m.value)


def build32(h_bits, k, M=PRIME32, want_topk=False, n_threads=0):
    """h_bits: uint32 [n_chunks, N] fp32 patterns. Returns (proofs uint8 [n_chunks, 2+4k], status[, idx])."""
    h = np.ascontiguousarray(h_bits, dtype=np.uint32)
    assert h.ndim == 2
    n_chunks, n = h.shape
    proofs = np.zeros((n_chunks, proof_bytes32(k)), dtype=np.uint8)
    status = np.zeros(n_chunks, dtype=np.uint8)
    idx = np.zeros((n_chunks, k), dtype=np.uint32) if want_topk else None
    nt = n_threads if n_threads > 0 else max_threads()
    rc = _load().toploc_oracle32_build(_ptr(h), n_chunks, n, k, int(M), _ptr(proofs), _ptr(status),
                                       _ptr(idx) if want_topk else None, nt)
    if rc:
        raise ValueError("oracle build32: bad arguments")
    return (proofs, status, idx) if want_topk else (proofs, status)


def verify_mixed(h_bits, h_dtype, proofs, p_dtype, k, thresholds=None, n_threads=0):
    """Algorithm 2 with activations of h_dtype and proofs of p_dtype; comparisons and (by default)
    thresholds are those of the validator's precision h_dtype."""
    h = _patterns(h_bits, h_dtype)
    assert h.ndim == 2
    n_chunks, n = h.shape
    proofs = np.ascontiguousarray(proofs, dtype=np.uint8)
    assert proofs.shape == (n_chunks, proof_bytes32(k) if p_dtype == F32 else proof_bytes(k))
    if thresholds is None:
        thresholds = F32_THRESHOLDS if h_dtype == F32 else (T_EXP, T_MEAN, T_MEDIAN)
    res = np.zeros(n_chunks, dtype=RESULT_DTYPE)
    nt = n_threads if n_threads > 0 else max_threads()
    rc = _load().toploc_oracle32_verify(_ptr(h), h_dtype, n_chunks, n, k, _ptr(proofs), p_dtype,
                                        PRIME32 if p_dtype == F32 else PRIME, int(thresholds[0]), int(thresholds[1]),
                                        int(thresholds[2]), _ptr(res), nt)
    if rc:
        raise ValueError("oracle verify_mixed: bad arguments")
    return res
