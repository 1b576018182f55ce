"""Seeded random differential test: many small random shapes, value distributions and
entry points against the CPU oracle, bit for bit.  Every case is reproducible from its seed."""
import os

import numpy as np
import pytest
import torch

import oracle as orc
from paper_2501_16007_amd import binding as tl
from paper_2501_16007_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
FIELDS = ("err_exp", "n_match", "mant_sum", "mant_median", "accept", "status")


def random_bits16(rng, n_chunks, n):
    """bf16 patterns from one of several laws: gaussian, few distinct values, heavy ties at the
    top, sorted, sparse spikes on zeros, raw random patterns (NaN / Inf included)."""
    law = int(rng.integers(0, 6))
    if law == 0:
        x = rng.standard_normal((n_chunks, n)).astype(np.float32) * float(rng.choice([1e-3, 1.0, 300.0]))
        bits = (x.view(np.uint32) >> 16).astype(np.uint16)
    elif law == 1:
        vals = rng.integers(0, 65536, size=int(rng.integers(1, 6))).astype(np.uint16)
        bits = vals[rng.integers(0, vals.size, size=(n_chunks, n))]
    elif law == 2:
        x = rng.standard_normal((n_chunks, n)).astype(np.float32)
        bits = (x.view(np.uint32) >> 16).astype(np.uint16)
        top = rng.integers(0, n, size=(n_chunks, max(1, n // 3)))
        for c in range(n_chunks):
            bits[c, top[c]] = np.uint16(0x4640 | (int(rng.integers(0, 2)) << 15))     # many equal large magnitudes
    elif law == 3:
        base = np.sort(rng.integers(0, 0x7F80, size=n).astype(np.uint16))
        bits = np.stack([base if c % 2 == 0 else base[::-1] for c in range(n_chunks)]).copy()
    elif law == 4:
        bits = np.zeros((n_chunks, n), dtype=np.uint16)
        for c in range(n_chunks):
            pos = rng.choice(n, size=min(n, int(rng.integers(1, 40))), replace=False)
            bits[c, pos] = rng.integers(0x3000, 0x4800, size=pos.size).astype(np.uint16)
    else:
        bits = rng.integers(0, 65536, size=(n_chunks, n)).astype(np.uint16)
    return np.ascontiguousarray(bits)


def compare(g, o, what):
    for f in FIELDS:
        assert np.array_equal(g[f], o[f]), "%s: %s gpu %s oracle %s" % (what, f, g[f][:4], o[f][:4])


N_CASES = int(os.environ.get("TOPLOC_RANDOM_CASES", "40"))      # more seeds for an occasional longer sweep


@pytest.mark.parametrize("seed", range(N_CASES))
def test_random_case(seed):
    rng = np.random.default_rng(31000 + seed)
    hidden = int(rng.choice([8, 16, 24, 64, 136, 520, 1024, 2048])) * int(rng.choice([1, 1, 2, 3]))
    tokens = int(rng.choice([1, 2, 5, 8, 32]))
    n = hidden * tokens
    k = int(min(n, rng.choice([1, 2, 7, 32, 100, 128, 129, 300, 512])))
    n_chunks = int(rng.integers(1, 7))
    parts = int(rng.choice([0, 0, 1, 2, 3, 9]))
    bits = random_bits16(rng, n_chunks, n)
    what = "seed %d H=%d T=%d k=%d chunks=%d parts=%d" % (seed, hidden, tokens, k, n_chunks, parts)
    print("[case] " + what, flush=True)
    chunks = synth.from_bits(bits, DEV)
    o_proofs, o_status, o_idx = orc.build(bits, k, want_topk=True)
    rec_bits = bits.copy()
    flip = rng.random(bits.shape) < 0.02
    rec_bits[flip] ^= np.uint16(1 << int(rng.integers(0, 9)))
    rec = synth.from_bits(rec_bits, DEV)
    o_res = orc.verify(rec_bits, o_proofs, k)
    try:
        tl.toploc_set_split(parts)
        proofs, status, idx = tl.toploc_build_proofs(chunks, k=k, chunk_tokens=1, want_topk=True)
        res = tl.toploc_verify_proofs(rec, torch.from_numpy(o_proofs).to(DEV), k=k, chunk_tokens=1)
        t_idx, t_val = tl.toploc_topk(chunks, k=k, chunk_tokens=1)
        torch.cuda.synchronize()
    finally:
        tl.toploc_set_split(0)
    assert np.array_equal(idx.cpu().numpy().view(np.uint32), o_idx), what + ": indices"
    assert np.array_equal(t_idx.cpu().numpy().view(np.uint32), o_idx), what + ": topk indices"
    assert np.array_equal(status.cpu().numpy(), o_status), what + ": status"
    assert np.array_equal(proofs.cpu().numpy(), o_proofs), what + ": proof bytes"
    compare(tl.results_numpy(res), o_res, what)
    # the same chunks as rows of one matrix through the segment calls (whole chunks as segments)
    off = np.arange(n_chunks + 1, dtype=np.uint64) * tokens
    mat = chunks.reshape(n_chunks * tokens, hidden)
    p_seg, s_seg = tl.toploc_build_proofs_segments(mat, off, k=k)
    r_seg = tl.toploc_verify_proofs_segments(rec.reshape(n_chunks * tokens, hidden), off, torch.from_numpy(o_proofs).to(DEV), k=k)
    torch.cuda.synchronize()
    assert np.array_equal(p_seg.cpu().numpy(), o_proofs) and np.array_equal(s_seg.cpu().numpy(), o_status), what + ": segments"
    compare(tl.results_numpy(r_seg), o_res, what + " segments")
    # and row by row through the running top-k
    state = tl.toploc_stream_new_state(n_chunks, k, DEV)
    rows = chunks.reshape(n_chunks, tokens, hidden).transpose(0, 1).contiguous()
    for t in rng.permutation(tokens).tolist():
        tl.toploc_stream_append(state, rows[t], t, k=k, chunk_tokens=tokens)
    p_st, s_st = tl.toploc_stream_emit(state, n_chunks, k=k)
    torch.cuda.synchronize()
    assert np.array_equal(p_st.cpu().numpy(), o_proofs) and np.array_equal(s_st.cpu().numpy(), o_status), what + ": stream"
    # the same rows through the indexed calls: slots in a random order, each row at its own token
    state = tl.toploc_stream_new_state(n_chunks + 2, k, DEV)
    slot_of = rng.permutation(n_chunks + 2)[:n_chunks]            # chunk c lives in slot slot_of[c]
    step = max(1, n_chunks // 2)                                   # a few rows per call, distinct slots in each
    for t in range(tokens):
        for c0 in range(0, n_chunks, step):
            cs = list(range(c0, min(n_chunks, c0 + step)))
            tl.toploc_stream_append_rows(state, n_chunks + 2, rows[t][cs].contiguous(), slot_of[cs],
                                         np.full(len(cs), t), k=k, chunk_tokens=tokens)
    p_ix, s_ix = tl.toploc_stream_emit_rows(state, n_chunks + 2, slot_of, k=k)
    torch.cuda.synchronize()
    assert np.array_equal(p_ix.cpu().numpy(), o_proofs) and np.array_equal(s_ix.cpu().numpy(), o_status), what + ": rows"


@pytest.mark.parametrize("seed", range(max(10, N_CASES // 4)))
def test_random_case_in_a_launch_of_several_generations(seed):
    """the same laws in launches of 1300 to 1700 chunks: past 1280 chunks the fused kernels with two rounds of loads in
    flight run instead of the three-round instantiation the small cases above take"""
    rng = np.random.default_rng(33000 + seed)
    hidden = int(rng.choice([8, 16, 24, 64, 136, 520])) * int(rng.choice([1, 1, 2, 3]))
    tokens = int(rng.choice([1, 2, 5, 8, 32]))
    n = hidden * tokens
    k = int(min(n, rng.choice([1, 2, 7, 32, 100, 128])))
    n_chunks = int(rng.integers(1300, 1700))
    bits = random_bits16(rng, n_chunks, n)
    what = "many chunks: seed %d H=%d T=%d k=%d chunks=%d" % (seed, hidden, tokens, k, n_chunks)
    print("[case] " + what, flush=True)
    chunks = synth.from_bits(bits, DEV)
    o_proofs, o_status, o_idx = orc.build(bits, k, want_topk=True)
    rec_bits = bits.copy()
    flip = rng.random(bits.shape) < 0.02
    rec_bits[flip] ^= np.uint16(1 << int(rng.integers(0, 9)))
    o_res = orc.verify(rec_bits, o_proofs, k)
    parts = int(rng.choice([0, 0, 2]))     # 2: the part kernels in a launch of several generations, then the merges
    try:
        tl.toploc_set_split(parts)
        proofs, status, idx = tl.toploc_build_proofs(chunks, k=k, chunk_tokens=1, want_topk=True)
        res = tl.toploc_verify_proofs(synth.from_bits(rec_bits, DEV), torch.from_numpy(o_proofs).to(DEV), k=k, chunk_tokens=1)
        torch.cuda.synchronize()
    finally:
        tl.toploc_set_split(0)
    what += " parts=%d" % parts
    assert np.array_equal(idx.cpu().numpy().view(np.uint32), o_idx), what + ": indices"
    assert np.array_equal(status.cpu().numpy(), o_status), what + ": status"
    assert np.array_equal(proofs.cpu().numpy(), o_proofs), what + ": proof bytes"
    compare(tl.results_numpy(res), o_res, what)


@pytest.mark.parametrize("seed", range(max(12, N_CASES // 3)))
def test_random_case_f32(seed):
    rng = np.random.default_rng(32000 + seed)
    hidden = int(rng.choice([8, 16, 64, 136, 520, 1024]))
    tokens = int(rng.choice([1, 2, 5, 32]))
    n = hidden * tokens
    k = int(min(n, rng.choice([1, 2, 7, 32, 100, 128])))
    n_chunks = int(rng.integers(1, 5))
    law = int(rng.integers(0, 3))
    if law == 0:
        bits = (rng.standard_normal((n_chunks, n)).astype(np.float32) * 50.0).view(np.uint32)
    elif law == 1:
        vals = rng.integers(0, 2 ** 32, size=4, dtype=np.uint64).astype(np.uint32)
        bits = vals[rng.integers(0, 4, size=(n_chunks, n))]
    else:
        bits = rng.integers(0, 2 ** 32, size=(n_chunks, n), dtype=np.uint64).astype(np.uint32)
    bits = np.ascontiguousarray(bits)
    what = "f32 seed %d H=%d T=%d k=%d chunks=%d law=%d" % (seed, hidden, tokens, k, n_chunks, law)
    print("[case] " + what, flush=True)
    chunks = synth.from_bits(bits, DEV)
    o_proofs, o_status, o_idx = orc.build32(bits, k, want_topk=True)
    proofs, status, idx = tl.toploc_build_proofs_f32(chunks, k=k, chunk_tokens=1, want_topk=True)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy().view(np.uint32), o_idx), what + ": indices"
    assert np.array_equal(status.cpu().numpy(), o_status) and np.array_equal(proofs.cpu().numpy(), o_proofs), what
    rec_bits = bits.copy()
    flip = rng.random(bits.shape) < 0.05
    rec_bits[flip] ^= np.uint32(1 << int(rng.integers(0, 25)))
    b16 = (rec_bits >> 16).astype(np.uint16)
    p16, _ = orc.build((bits >> 16).astype(np.uint16), k)
    for h_bits, h_dt, p, p_dt in ((rec_bits, orc.F32, o_proofs, orc.F32), (b16, orc.BF16, o_proofs, orc.F32),
                                  (rec_bits, orc.F32, p16, orc.BF16)):
        o = orc.verify_mixed(h_bits, h_dt, p, p_dt, k)
        g = tl.toploc_verify_proofs_mixed(synth.from_bits(h_bits, DEV), torch.from_numpy(p).to(DEV), p_dt, k=k, chunk_tokens=1)
        torch.cuda.synchronize()
        compare(tl.results_numpy(g), o, what + " validator %d proof %d" % (h_dt, p_dt))
    # whole chunks as segments of one fp32 matrix, cut into a random number of parts
    if hidden % 8 == 0:
        off = np.arange(n_chunks + 1, dtype=np.uint64) * tokens
        parts = int(rng.choice([0, 1, 2, 5]))
        try:
            tl.toploc_set_split(parts)
            p_seg, s_seg = tl.toploc_build_proofs_segments_f32(chunks.reshape(n_chunks * tokens, hidden), off, k=k)
            r_seg = tl.toploc_verify_proofs_segments_mixed(synth.from_bits(rec_bits, DEV).reshape(n_chunks * tokens, hidden),
                                                           off, torch.from_numpy(o_proofs).to(DEV), orc.F32, k=k)
            torch.cuda.synchronize()
        finally:
            tl.toploc_set_split(0)
        assert np.array_equal(p_seg.cpu().numpy(), o_proofs) and np.array_equal(s_seg.cpu().numpy(), o_status), \
            what + ": segments, parts=%d" % parts
        compare(tl.results_numpy(r_seg), orc.verify_mixed(rec_bits, orc.F32, o_proofs, orc.F32, k), what + " segments")
