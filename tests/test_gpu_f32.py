"""fp32 proofs and validation across precisions (Section 5.7): GPU path vs the 32-bit CPU
oracle, bit for bit, through the C ABI.  Inputs are seeded and synthetic."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2501_16007_amd import binding as tl
from paper_2501_16007_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
FIELDS = ("err_exp", "n_match", "mant_sum", "mant_median", "accept", "status")


def say(msg):
    print("[case] " + msg, flush=True)


def f32_chunks(n_chunks, hidden, tokens, seed, n_outlier=8):
    x = synth.activations(n_chunks, tokens, hidden, seed, n_outlier=min(n_outlier, hidden), device=DEV,
                          dtype=torch.float32)
    return x.reshape(n_chunks, tokens * hidden)


def check_build(chunks, k, what):
    say("%s build n_chunks=%d N=%d k=%d" % (what, chunks.shape[0], chunks.shape[1], k))
    bits = synth.bits_numpy(chunks)
    o_proofs, o_status, o_idx = orc.build32(bits, k, want_topk=True)
    proofs, status, idx = tl.toploc_build_proofs_f32(chunks, k=k, chunk_tokens=1, want_topk=True)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy().view(np.uint32), o_idx), what + ": indices"
    assert np.array_equal(status.cpu().numpy(), o_status), what + ": status"
    assert np.array_equal(proofs.cpu().numpy(), o_proofs), what + ": proof bytes"
    return o_proofs


def check_verify(rec, proofs_np, p_dtype, k, what, thresholds=None):
    h_dtype = orc.F32 if rec.dtype == torch.float32 else orc.BF16
    say("%s verify validator=%s proof=%s" % (what, "fp32" if h_dtype else "bf16", "fp32" if p_dtype else "bf16"))
    o = orc.verify_mixed(synth.bits_numpy(rec), h_dtype, proofs_np, p_dtype, k, thresholds=thresholds)
    res = tl.toploc_verify_proofs_mixed(rec, torch.from_numpy(np.ascontiguousarray(proofs_np)).to(DEV), p_dtype, k=k,
                                        chunk_tokens=1, thresholds=thresholds)
    torch.cuda.synchronize()
    g = tl.results_numpy(res)
    for f in FIELDS:
        bad = np.nonzero(g[f] != o[f])[0]
        assert bad.size == 0, "%s: field %s differs at %s: gpu %s oracle %s" % (what, f, bad[:4], g[f][bad[:4]], o[f][bad[:4]])
    return o


@pytest.mark.parametrize("hidden,tokens,k,n_chunks", [
    (8, 1, 1, 3),            # N = 8: two 16-byte vectors
    (8, 1, 8, 2),            # k = N
    (264, 32, 128, 3),       # ragged against the round size
    (1000, 32, 32, 3),
    (4096, 32, 128, 4),      # the 8B shape in fp32: 512 KiB per chunk
    (8192, 32, 128, 2),      # the 70B shape in fp32: 1 MiB per chunk
    (64, 32, 128, 2),        # N = 2048, k = N/16
])
def test_f32_build_and_self_validation(hidden, tokens, k, n_chunks):
    chunks = f32_chunks(n_chunks, hidden, tokens, 9000 + hidden + k)
    proofs = check_build(chunks, k, "shape H=%d T=%d" % (hidden, tokens))
    res = check_verify(chunks, proofs, orc.F32, k, "self")
    assert (res["accept"] == 1).all() and (res["mant_sum"] == 0).all() and (res["err_exp"] == 0).all()


def test_f32_ties_signs_and_special_patterns():
    rng = np.random.default_rng(91)
    n = 32 * 256
    vals = np.array([0x3F800000, 0xBF800000, 0x40000000, 0x00000000, 0x3F800001], dtype=np.uint32)
    bits = vals[rng.integers(0, len(vals), size=(3, n))]
    bits[0, 17] = 0x7F800000       # +Inf
    bits[0, 99] = 0xFF800000       # -Inf
    bits[1, 5] = 0x7FC00000        # quiet NaN
    bits[1, 6] = 0xFFFFFFFF        # negative NaN whose pattern is >= p
    bits[2, 0] = 0xFFFFFFFB        # smallest pattern >= p
    chunks = synth.from_bits(bits, DEV)
    proofs = check_build(chunks, 128, "ties / specials")
    check_verify(chunks, proofs, orc.F32, 128, "ties / specials")
    eq = np.full((1, n), 0x40490FDB, dtype=np.uint32)     # every value equal: the lowest indices win
    check_build(synth.from_bits(eq, DEV), 64, "all equal")


def test_f32_sorted_magnitudes_overflow_the_candidate_buffer():
    """fp32 magnitudes that never decrease along the chunk (random signs), and the same descending: in the ascending
    chunk every value read is a candidate, sweeps over the queue overflow the candidate buffer and the bound is found from
    the queue's own values through all four radix digits of the 31-bit magnitude.  k = 128 and 512."""
    rng = np.random.default_rng(92)
    n = 32 * 2048
    mag = (np.arange(n, dtype=np.uint64) * 0x7F000000 // (n + 64)).astype(np.uint32)      # finite patterns
    asc = mag | (rng.integers(0, 2, size=n, dtype=np.uint32) << 31)
    few = (np.arange(n, dtype=np.uint32) // 512 * 0x00800000 + 0x20000000).astype(np.uint32)   # 128 steps of 512 equal values
    bits = np.stack([asc, asc[::-1].copy(), few])
    chunks = synth.from_bits(bits, DEV)
    for k in (128, 512):
        proofs = check_build(chunks, k, "sorted fp32 k=%d" % k)
        res = check_verify(chunks, proofs, orc.F32, k, "sorted fp32 k=%d" % k)
        assert (res["accept"] == 1).all()


def test_all_four_precision_pairs_match_the_oracle_and_table5_outcomes():
    """Generation in fp32 or bf16, validation in fp32 or bf16, on the 8B shape: the recomputed tensors are
    the original values moved by a small relative perturbation (an fp32-sized one for the fp32 validator)."""
    k, n_chunks, hidden = 128, 6, 4096
    x32 = synth.activations(n_chunks, 32, hidden, 9100, n_outlier=8, device=DEV, dtype=torch.float32)
    x16 = x32.to(torch.bfloat16)                                            # the bf16 model's activations
    c32, c16 = x32.reshape(n_chunks, -1), x16.reshape(n_chunks, -1)
    p32 = check_build(c32, k, "generation fp32")
    p16, _ = orc.build(synth.bits_numpy(c16), k)
    g = torch.Generator(device=DEV)
    g.manual_seed(9101)
    rec32 = (c32 * (1.0 + (torch.rand(c32.shape, generator=g, device=DEV) * 2 - 1) * 2.0 ** -20)).contiguous()
    rec16 = synth.perturb_relative(c16, 2.0 ** -9, 9102)
    out = {}
    out["fp32/fp32"] = check_verify(rec32, p32, orc.F32, k, "gen fp32")
    out["fp32/bf16"] = check_verify(rec16, p32, orc.F32, k, "gen fp32")
    out["bf16/fp32"] = check_verify(rec32, p16, orc.BF16, k, "gen bf16")
    out["bf16/bf16"] = check_verify(rec16, p16, orc.BF16, k, "gen bf16")
    say("accepted of %d: %s" % (n_chunks, {a: int(r["accept"].sum()) for a, r in out.items()}))
    say("mean mantissa difference: %s" % {a: float(r["mant_sum"].sum()) / max(1, int(r["n_match"].sum()))
                                          for a, r in out.items()})
    assert (out["fp32/fp32"]["accept"] == 1).all()       # Table 5: fp32 generation passes with either validator
    assert (out["fp32/bf16"]["accept"] == 1).all()
    assert (out["bf16/bf16"]["accept"] == 1).all()       # bf16 generation passes only with a bf16 validator
    assert (out["bf16/fp32"]["accept"] == 0).all()


def test_thresholds_and_malformed_proofs_in_the_32_bit_field():
    chunks = f32_chunks(3, 512, 32, 9200)
    bits = synth.bits_numpy(chunks)
    proofs, _ = orc.build32(bits, 64)
    rec = (chunks * (1.0 + 2.0 ** -18)).contiguous()
    for thr in ((8, 256, 128), (0, 0, 0), (128, 1 << 22, 1 << 22), (1, 3, 2)):
        check_verify(rec, proofs, orc.F32, 64, "thresholds %s" % (thr,), thresholds=thr)
    bad = proofs.copy()
    bad[0, 0], bad[0, 1] = 0x00, 0x40                     # m = 16384
    bad[1, 6:10] = (0xFB, 0xFF, 0xFF, 0xFF)               # c_1 = p
    o = check_verify(chunks, bad, orc.F32, 64, "malformed")
    assert o["status"].tolist() == [tl.CHUNK_MALFORMED, tl.CHUNK_MALFORMED, tl.CHUNK_OK]


def test_decode_edges_in_the_32_bit_field():
    chunks = f32_chunks(4, 64, 32, 7300)
    bits = synth.bits_numpy(chunks)
    proofs, _ = orc.build32(bits, 16)
    for c, field in ((0, 32768), (1, 32769)):
        proofs[c, 0], proofs[c, 1] = field & 0xFF, field >> 8
    for c, coef in ((2, orc.PRIME32 - 1), (3, orc.PRIME32)):
        proofs[c, 2 + 4 * 15: 6 + 4 * 15] = np.frombuffer(int(coef).to_bytes(4, "little"), dtype=np.uint8)
    o = check_verify(chunks, proofs, orc.F32, 16, "decode edges")
    assert o["status"].tolist() == [tl.CHUNK_MALFORMED, 0, 0, tl.CHUNK_MALFORMED]


def test_f32_arguments_are_checked():
    x = torch.zeros((1, 32 * 64), dtype=torch.float32, device=DEV)
    with pytest.raises(tl.ToplocError):
        tl.toploc_build_proofs_f32(x, k=513, chunk_tokens=32)        # k > TOPLOC_MAX_K_F32
    with pytest.raises(tl.ToplocError):
        tl.toploc_build_proofs_f32(x, k=0, chunk_tokens=32)
    e = torch.empty((0, 2048), dtype=torch.float32, device=DEV)
    proofs, status = tl.toploc_build_proofs_f32(e, k=8, chunk_tokens=32)
    assert proofs.shape == (0, 34)


def test_f32_full_size_sampled():
    """32 x 2048 x 4096 fp32 (1 GiB, 2048 chunks): properties at full size, oracle on a seeded sample."""
    x = synth.activations(32, 2048, 4096, 9300, n_outlier=8, device=DEV, dtype=torch.float32)
    chunks = synth.as_chunks(x)
    n_chunks = chunks.shape[0]
    proofs, status, idx = tl.toploc_build_proofs_f32(chunks, k=128, chunk_tokens=1, want_topk=True)
    res = tl.toploc_verify_proofs_mixed(chunks, proofs, tl.DTYPE_F32, k=128, chunk_tokens=1)
    torch.cuda.synchronize()
    g = tl.results_numpy(res)
    assert int(status.max()) == 0 and (g["accept"] == 1).all() and (g["mant_sum"] == 0).all() and (g["n_match"] == 128).all()
    sel = np.sort(np.random.default_rng(93).choice(n_chunks, 24, replace=False))
    selt = torch.from_numpy(sel).to(DEV)
    o_proofs, o_status, o_idx = orc.build32(synth.bits_numpy(chunks[selt]), 128, want_topk=True)
    assert np.array_equal(proofs[selt].cpu().numpy(), o_proofs)
    assert np.array_equal(idx[selt].cpu().numpy().view(np.uint32), o_idx)


def _to_bf16_model(x32):
    """What a bf16 run of the same model would hold: the fp32 activations rounded to bf16."""
    return x32.to(torch.bfloat16)


@pytest.mark.parametrize("hidden,rows,k,parts", [
    (4096, [100, 32, 32, 7], 128, 0),      # prompt, two full chunks, a ragged last chunk
    (1024, [64, 9, 33, 1], 64, 0),
    (8, [1, 2, 5], 8, 0),                  # the smallest rows: two vectors each
    (4096, [300, 5], 128, 5),              # forced cuts: parts of unequal length, ties across borders by chance
    (5120, [40, 32], 32, 1),
    (4096, [70, 32, 9], 512, 0),           # k above 128: the larger candidate buffer, 512 points in the 32-bit field
    (1024, [33, 64], 256, 3),
])
def test_f32_segments_build_and_the_four_precision_pairs(hidden, rows, k, parts):
    """Segments of unequal length with fp32 activations: proofs, status, indices and the verify records of all
    four validator/proof precision pairs equal the oracle's, which sees every segment as one flat array."""
    total = int(sum(rows))
    say("f32 segments H=%d rows=%s k=%d parts=%d" % (hidden, rows, k, parts))
    x32 = synth.activations(1, total, hidden, 9300 + hidden + k, n_outlier=min(8, hidden), device=DEV,
                            dtype=torch.float32).reshape(total, hidden)
    x16 = _to_bf16_model(x32)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.uint64)
    b32, b16 = synth.bits_numpy(x32), synth.bits_numpy(x16)
    try:
        tl.toploc_set_split(parts)
        proofs32, status32, idx32 = tl.toploc_build_proofs_segments_f32(x32, off, k=k, want_topk=True)
        proofs16, status16 = tl.toploc_build_proofs_segments(x16, off, k=k)
        torch.cuda.synchronize()
        o32 = np.zeros((len(rows), 2 + 4 * k), dtype=np.uint8)
        o16 = np.zeros((len(rows), 2 + 2 * k), dtype=np.uint8)
        for i in range(len(rows)):
            a, b = int(off[i]), int(off[i + 1])
            p, st, ix = orc.build32(b32[a:b].reshape(1, -1), k, want_topk=True)
            assert np.array_equal(idx32[i].cpu().numpy().view(np.uint32), ix[0]), "segment %d indices" % i
            assert int(status32[i]) == int(st[0]) and np.array_equal(proofs32[i].cpu().numpy(), p[0]), "segment %d" % i
            o32[i] = p[0]
            o16[i] = orc.build(b16[a:b].reshape(1, -1), k)[0][0]
        assert np.array_equal(proofs16.cpu().numpy(), o16)
        # a recomputation that differs a little, in both precisions
        r32 = x32 * (1.0 + 2.0 ** -12 * torch.sin(torch.arange(hidden, device=DEV, dtype=torch.float32)))
        r16 = _to_bf16_model(r32)
        for rec, rbits, h_dt in ((r32, synth.bits_numpy(r32), orc.F32), (r16, synth.bits_numpy(r16), orc.BF16)):
            for p_np, p_dt in ((o32, orc.F32), (o16, orc.BF16)):
                res = tl.toploc_verify_proofs_segments_mixed(rec, off, torch.from_numpy(p_np).to(DEV), p_dt, k=k)
                torch.cuda.synchronize()
                g = tl.results_numpy(res)
                for i in range(len(rows)):
                    a, b = int(off[i]), int(off[i + 1])
                    o = orc.verify_mixed(rbits[a:b].reshape(1, -1), h_dt, p_np[i:i + 1], p_dt, k)
                    for f in FIELDS:
                        assert g[f][i] == o[f][0], "validator %d proof %d segment %d field %s: gpu %s oracle %s" % (
                            h_dt, p_dt, i, f, g[f][i], o[f][0])
    finally:
        tl.toploc_set_split(0)


def test_f32_segments_equal_fixed_chunks_and_reject_bad_arguments():
    x = f32_chunks(4, 1024, 32, 9400).reshape(4 * 32, 1024)
    off = np.arange(5, dtype=np.uint64) * 32
    p_seg, s_seg, i_seg = tl.toploc_build_proofs_segments_f32(x, off, k=128, want_topk=True)
    p_fix, s_fix, i_fix = tl.toploc_build_proofs_f32(x.reshape(4, -1), k=128, chunk_tokens=1, want_topk=True)
    torch.cuda.synchronize()
    assert torch.equal(p_seg, p_fix) and torch.equal(s_seg, s_fix) and torch.equal(i_seg, i_fix)
    with pytest.raises(tl.ToplocError):
        tl.toploc_build_proofs_segments_f32(x, off, k=513)                       # k above the fp32 limit
    with pytest.raises(tl.ToplocError):
        tl.toploc_verify_proofs_segments_mixed(x.to(torch.bfloat16), off,
                                               torch.zeros((4, 2 + 4 * 513), dtype=torch.uint8, device=DEV), orc.F32, k=513)
    assert tl.toploc_segments_workspace_bytes_dtype(4, 128, 1024, 128, tl.DTYPE_F32) > \
        tl.toploc_segments_workspace_bytes_dtype(4, 128, 1024, 128, tl.DTYPE_BF16) > 0


# ---------------------------------------------------------------------------
# k above 128 in the 32-bit field (Section 5.7's precision study does not bound k) and the running top-k
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("hidden,tokens,k,n_chunks,parts", [
    (4096, 32, 512, 3, 0),       # the 8B shape, largest k: split launches with the library's cut
    (5120, 32, 256, 2, 0),
    (1024, 32, 129, 4, 1),       # just above the fused limit, one part per chunk
    (4096, 32, 512, 2, 5),       # forced cut into 5 parts
    (64, 32, 512, 2, 0),         # N = 2048, k = N/4
])
def test_f32_large_k_build_and_the_four_precision_pairs(hidden, tokens, k, n_chunks, parts):
    x32 = f32_chunks(n_chunks, hidden, tokens, 9500 + hidden + k)
    x16 = _to_bf16_model(x32)
    try:
        tl.toploc_set_split(parts)
        assert tl.toploc_workspace_bytes_f32(k, 1, x32.shape[1], n_chunks) >= n_chunks * k * 8
        p32 = check_build(x32, k, "large k H=%d parts=%d" % (hidden, parts))
    finally:
        tl.toploc_set_split(0)
    p16, _ = orc.build(synth.bits_numpy(x16), k)
    r32 = (x32 * (1.0 + 2.0 ** -12 * torch.sin(torch.arange(x32.shape[1], device=DEV, dtype=torch.float32)))).contiguous()
    r16 = _to_bf16_model(r32)
    res = check_verify(x32, p32, orc.F32, k, "self")
    assert (res["accept"] == 1).all() and (res["mant_sum"] == 0).all() and (res["n_match"] == k).all()
    for rec in (r32, r16):
        for p, p_dt in ((p32, orc.F32), (p16, orc.BF16)):
            check_verify(rec, p, p_dt, k, "large k")
    with pytest.raises(tl.ToplocError):     # k > 128 needs the workspace
        tl.toploc_build_proofs_f32(x32, k=k, chunk_tokens=1, workspace=torch.empty(16, dtype=torch.uint8, device=DEV))


@pytest.mark.parametrize("hidden,T,k,n_seq", [
    (5120, 32, 128, 5),
    (4096, 32, 512, 3),
    (1000, 7, 32, 3),
    (8, 16, 16, 2),
])
def test_f32_running_topk_matches_the_oracle_on_the_assembled_chunk(hidden, T, k, n_seq):
    """The running top-k over fp32 rows: proofs, status and indices of the emission equal the 32-bit oracle's on
    the chunk assembled from the appended rows; rows arrive in a scrambled order, the state is reused."""
    say("f32 stream H=%d T=%d k=%d n_seq=%d" % (hidden, T, k, n_seq))
    steps = synth.activations(n_seq, 2 * T, hidden, 9600 + hidden + k, n_outlier=min(8, hidden), device=DEV,
                              dtype=torch.float32).transpose(0, 1).contiguous()          # [2T, n_seq, hidden]
    state = tl.toploc_stream_new_state(n_seq, k, DEV, dtype=tl.DTYPE_F32)
    assert state.numel() >= n_seq * (16 + 8 * k)
    order = np.random.default_rng(96).permutation(T)
    for window in range(2):
        for t in order:
            tl.toploc_stream_append(state, steps[window * T + int(t)], int(t), k=k, chunk_tokens=T)
        proofs, status, idx = tl.toploc_stream_emit(state, n_seq, k=k, want_topk=True, dtype=tl.DTYPE_F32)
        torch.cuda.synchronize()
        chunk = steps[window * T:(window + 1) * T].transpose(0, 1).contiguous().reshape(n_seq, T * hidden)
        o_proofs, o_status, o_idx = orc.build32(synth.bits_numpy(chunk), k, want_topk=True)
        assert np.array_equal(idx.cpu().numpy().view(np.uint32), o_idx), "window %d: indices" % window
        assert np.array_equal(status.cpu().numpy(), o_status) and np.array_equal(proofs.cpu().numpy(), o_proofs), window
        g_proofs, _ = tl.toploc_build_proofs_f32(chunk, k=k, chunk_tokens=1)
        torch.cuda.synchronize()
        assert torch.equal(g_proofs, proofs)
    # continuous batching in fp32: rows of a subset of the sequences, each at its own position; a short state
    tl.toploc_stream_append_rows(state, n_seq, steps[0, :2].contiguous(), [1, 0], [3, 0], k=k, chunk_tokens=T)
    proofs, status = tl.toploc_stream_emit_rows(state, n_seq, [0, 1], k=k, dtype=tl.DTYPE_F32)
    torch.cuda.synchronize()
    if hidden >= k:
        # one row as token `tok`: the proof of a chunk that is zero except for that row would rank the zeros by
        # index too, so compare with the oracle on exactly what was appended: a one-row chunk whose flat
        # indices start at tok * hidden (the oracle ranks a flat array; shift its indices accordingly)
        assert status.tolist() == [tl.CHUNK_OK, tl.CHUNK_OK]
        state2 = tl.toploc_stream_new_state(n_seq, k, DEV, dtype=tl.DTYPE_F32)
        tl.toploc_stream_append_rows(state2, n_seq, steps[0, :2].contiguous(), [1, 0], [3, 0], k=k, chunk_tokens=T)
        _, _, idx = tl.toploc_stream_emit_rows(state2, n_seq, [0, 1], k=k, want_topk=True, dtype=tl.DTYPE_F32)
        torch.cuda.synchronize()
        for out_row, (src_row, tok) in enumerate(((1, 0), (0, 3))):
            oi, _ = orc.topk32(synth.bits_numpy(steps[0, src_row]), k)
            assert np.array_equal(idx[out_row].cpu().numpy().view(np.uint32), oi + np.uint32(tok * hidden))
    else:
        assert status.tolist() == [tl.CHUNK_SHORT, tl.CHUNK_SHORT] and not proofs.any()
