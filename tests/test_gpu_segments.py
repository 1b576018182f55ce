"""Split launches and variable-length segments vs the CPU oracle, through the C ABI.

A chunk or a segment may be cut into parts whose candidates a second launch merges;
whatever the cut, top-k indices, proof bytes, status and verify records must equal the
oracle's, which sees every segment as one flat array (Algorithm 1 and 2 on the whole
prompt, Section 5.6, or on a ragged last chunk).
"""
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


@pytest.fixture(autouse=True)
def library_chooses_the_split_again():
    yield
    tl.toploc_set_split(0)


def _fixed_case(chunks, k, parts, what):
    """Fixed chunks with the chunk cut into `parts` parts (0: the library's choice)."""
    say("%s n_chunks=%d N=%d k=%d parts=%d" % (what, chunks.shape[0], chunks.shape[1], k, parts))
    bits = synth.bits_numpy(chunks)
    o_proofs, o_status, o_idx = orc.build(bits, k, want_topk=True)
    o_res = orc.verify(bits, o_proofs, k)
    tl.toploc_set_split(parts)
    proofs, status, idx = tl.toploc_build_proofs(chunks, k=k, chunk_tokens=1, want_topk=True)
    res = tl.toploc_verify_proofs(chunks, torch.from_numpy(o_proofs).to(DEV), k=k, chunk_tokens=1)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy().view(np.uint32), o_idx), what + ": indices"
    assert np.array_equal(status.cpu().numpy(), o_status), what + ": status"
    assert np.array_equal(proofs.cpu().numpy(), o_proofs), what + ": proof bytes"
    g = tl.results_numpy(res)
    for f in FIELDS:
        assert np.array_equal(g[f], o_res[f]), what + ": " + f


@pytest.mark.parametrize("parts", [1, 2, 3, 7, 16])
@pytest.mark.parametrize("k", [128, 512])
def test_fixed_chunks_any_cut_gives_the_same_bytes(parts, k):
    x = synth.activations(5, 32, 4096, 4100 + k, n_outlier=8, device=DEV).reshape(5, 32 * 4096)
    _fixed_case(x, k, parts, "cut")


def test_parts_shorter_than_k_are_padded():
    # N = 2048 values in 16 parts of 128 values, k = 512: every part holds fewer than k
    x = synth.activations(3, 32, 64, 4200, n_outlier=2, device=DEV).reshape(3, 2048)
    _fixed_case(x, 512, 16, "short parts")
    # more parts than vectors: trailing parts are empty
    y = synth.activations(2, 1, 64, 4201, n_outlier=2, device=DEV).reshape(2, 64)
    _fixed_case(y, 16, 12, "empty parts")


def test_ties_across_part_borders():
    rng = np.random.default_rng(43)
    vals = np.array([0x3F80, 0xBF80, 0x4000, 0x0000], dtype=np.uint16)
    bits = vals[rng.integers(0, len(vals), size=(3, 32 * 1024))]
    _fixed_case(synth.from_bits(bits, DEV), 128, 5, "ties")
    _fixed_case(synth.from_bits(bits, DEV), 512, 3, "ties k=512")


def test_small_batch_default_plan_matches():
    x = synth.activations(2, 32, 8192, 4300, n_outlier=16, device=DEV).reshape(2, 32 * 8192)
    assert tl.toploc_workspace_bytes(128, 1, 32 * 8192, 2) > 0      # the library cuts such a batch
    _fixed_case(x, 128, 0, "default plan")


def _segment_case(hidden, rows, k, seed, parts=0, what="segments"):
    """rows: rows per segment.  One [total_rows, hidden] matrix, oracle per segment."""
    total = int(sum(rows))
    say("%s H=%d rows=%s k=%d parts=%d" % (what, hidden, list(rows), k, parts))
    x = synth.activations(1, total, hidden, seed, n_outlier=min(8, hidden), device=DEV).reshape(total, hidden)
    off = np.concatenate([[0], np.cumsum(rows)]).astype(np.uint64)
    bits = synth.bits_numpy(x)
    tl.toploc_set_split(parts)
    proofs, status, idx = tl.toploc_build_proofs_segments(x, off, k=k, want_topk=True)
    torch.cuda.synchronize()
    proofs_np, status_np, idx_np = proofs.cpu().numpy(), status.cpu().numpy(), idx.cpu().numpy().view(np.uint32)
    o_all = np.zeros_like(proofs_np)
    for i in range(len(rows)):
        seg = bits[int(off[i]):int(off[i + 1])].reshape(1, -1)
        o_proofs, o_status, o_idx = orc.build(seg, k, want_topk=True)
        assert np.array_equal(idx_np[i], o_idx[0]), "%s: segment %d indices" % (what, i)
        assert status_np[i] == o_status[0], "%s: segment %d status" % (what, i)
        assert np.array_equal(proofs_np[i], o_proofs[0]), "%s: segment %d proof bytes" % (what, i)
        o_all[i] = o_proofs[0]
    # verify against a perturbed recomputation so that the statistics are not all zero
    rec = synth.perturb_relative(x, 2.0 ** -7, seed + 1)
    res = tl.toploc_verify_proofs_segments(rec, off, torch.from_numpy(o_all).to(DEV), k=k)
    torch.cuda.synchronize()
    g = tl.results_numpy(res)
    rbits = synth.bits_numpy(rec)
    for i in range(len(rows)):
        seg = rbits[int(off[i]):int(off[i + 1])].reshape(1, -1)
        o = orc.verify(seg, o_all[i:i + 1], k)
        for f in FIELDS:
            assert g[f][i] == o[f][0], "%s: segment %d field %s" % (what, i, f)


def test_segments_prompt_plus_ragged_last_chunk():
    # a 100-token prompt as one proof, three full 32-token chunks, a ragged last chunk of 7 tokens
    _segment_case(4096, [100, 32, 32, 32, 7], 128, 5000)


def test_segments_one_row_and_tiny_hidden():
    _segment_case(8, [1, 2, 1, 5], 8, 5001)
    _segment_case(256, [1, 1, 3], 128, 5002)


def test_segments_long_prompt_many_parts():
    # a 2048-token prompt at hidden 4096 is 8 Mi values: cut into many parts by default
    _segment_case(4096, [2048, 32, 5], 128, 5003)


def test_segments_forced_cuts_and_large_k():
    _segment_case(1024, [64, 9, 33], 512, 5004, parts=1)
    _segment_case(1024, [64, 9, 33], 512, 5004, parts=6)
    _segment_case(5120, [40, 32, 1], 32, 5005, parts=3)


def test_segments_equal_fixed_chunks_on_a_regular_layout():
    x = synth.activations(3, 64, 2048, 5100, n_outlier=4, device=DEV)        # 6 chunks of 32 rows
    chunks = synth.as_chunks(x)
    off = np.arange(7, dtype=np.uint64) * 32
    p_seg, s_seg, i_seg = tl.toploc_build_proofs_segments(x.reshape(-1, 2048), off, k=128, want_topk=True)
    p_fix, s_fix, i_fix = tl.toploc_build_proofs(chunks, k=128, chunk_tokens=1, want_topk=True)
    torch.cuda.synchronize()
    assert torch.equal(p_seg, p_fix) and torch.equal(s_seg, s_fix) and torch.equal(i_seg, i_fix)


def test_segments_empty_and_invalid():
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device=DEV)
    proofs, status = tl.toploc_build_proofs_segments(x, np.zeros(1, dtype=np.uint64), k=8)
    assert proofs.shape == (0, 18) and status.shape == (0,)
    with pytest.raises(ValueError):
        tl.toploc_build_proofs_segments(x, np.array([0, 9], dtype=np.uint64), k=8)        # past the tensor
    with pytest.raises(tl.ToplocError):
        tl.toploc_build_proofs_segments(x, np.array([0, 4], dtype=np.uint64), k=513)      # k above the limit


def test_segments_that_cannot_carry_a_proof_are_reported_per_segment():
    """The offsets live on the device, so what is wrong with one segment is that segment's status: too short
    for k, offsets that decrease or leave the matrix.  The other segments get their oracle bytes."""
    hidden, k = 256, 128
    x = synth.activations(1, 40, hidden, 5050, n_outlier=4, device=DEV).reshape(40, hidden)
    bits = synth.bits_numpy(x)
    #        0: fine        1: empty   2: fine     3: decreasing  4: beyond the matrix (41 > 40 rows)
    off = torch.tensor([0, 12, 12, 30, 25, 41], dtype=torch.int64, device=DEV)
    say("segments with bad offsets: %s of %d rows" % (off.tolist(), x.shape[0]))
    proofs, status, idx = tl.toploc_build_proofs_segments(x, off, k=k, want_topk=True)
    res = tl.toploc_verify_proofs_segments(x, off, proofs, k=k)
    torch.cuda.synchronize()
    g = tl.results_numpy(res)
    assert status.tolist() == [tl.CHUNK_OK, tl.CHUNK_SHORT, tl.CHUNK_OK, tl.CHUNK_BAD_SEGMENT, tl.CHUNK_BAD_SEGMENT]
    assert g["status"].tolist() == status.tolist() and g["accept"].tolist() == [1, 0, 1, 0, 0]
    for i, (a, b) in ((0, (0, 12)), (2, (12, 30))):
        o_proofs, o_status, o_idx = orc.build(bits[a:b].reshape(1, -1), k, want_topk=True)
        assert np.array_equal(proofs[i].cpu().numpy(), o_proofs[0]) and np.array_equal(idx[i].cpu().numpy().view(np.uint32), o_idx[0])
    for i in (1, 3, 4):
        assert not proofs[i].any() and (idx[i] == -1).all()
    # one row of 256 values is exactly k = 256: the shortest segment that works; k = 257 does not fit
    one = torch.tensor([7, 8], dtype=torch.int64, device=DEV)
    p256, s256 = tl.toploc_build_proofs_segments(x, one, k=256)
    p257, s257 = tl.toploc_build_proofs_segments(x, one, k=257)
    torch.cuda.synchronize()
    assert s256.tolist() == [tl.CHUNK_OK] and s257.tolist() == [tl.CHUNK_SHORT]
    assert np.array_equal(p256[0].cpu().numpy(), orc.build(bits[7:8].reshape(1, -1), 256)[0][0])


def test_segment_calls_captured_in_a_graph_follow_the_offsets_on_the_device():
    """The segment calls only launch kernels: a captured build + verify pair is replayed with different row
    offsets written into the same device array between replays, program work and synchronisations in between,
    and every replay must give the bytes of an eager call and of the oracle on those offsets."""
    hidden, k, total, n_seg = 2048, 128, 300, 5
    x = synth.activations(1, total, hidden, 5400, n_outlier=4, device=DEV).reshape(total, hidden)
    rec = synth.perturb_relative(x, 2.0 ** -7, 5401)
    bits, rbits = synth.bits_numpy(x), synth.bits_numpy(rec)
    layouts = [[0, 100, 132, 164, 196, 203], [0, 1, 2, 130, 131, 300], [10, 50, 50, 90, 290, 300],
               [0, 100, 132, 164, 196, 203]]
    off = torch.zeros(n_seg + 1, dtype=torch.int64, device=DEV)
    out = (torch.empty((n_seg, 2 + 2 * k), dtype=torch.uint8, device=DEV), torch.empty(n_seg, dtype=torch.uint8, device=DEV),
           torch.empty((n_seg, k), dtype=torch.int32, device=DEV))
    res = torch.empty((n_seg, 20), dtype=torch.uint8, device=DEV)
    ws_b, ws_v = tl.new_segments_workspace(x, n_seg, k), tl.new_segments_workspace(x, n_seg, k)
    off.copy_(torch.tensor(layouts[0], dtype=torch.int64))
    side = torch.cuda.Stream(device=DEV)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # warm-up on the capture stream, then capture
        tl.toploc_build_proofs_segments(x, off, k=k, want_topk=True, workspace=ws_b, out=out)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            tl.toploc_build_proofs_segments(x, off, k=k, want_topk=True, workspace=ws_b, out=out)
            tl.toploc_verify_proofs_segments(rec, off, out[0], k=k, workspace=ws_v, out=res)
    torch.cuda.current_stream().wait_stream(side)
    for rep, lay in enumerate(layouts):
        say("graph replay %d with offsets %s" % (rep, lay))
        off.copy_(torch.tensor(lay, dtype=torch.int64))
        for t in out + (res,):
            t.fill_(0x5A if t.dtype == torch.uint8 else 7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        e_proofs, e_status, e_idx = tl.toploc_build_proofs_segments(x, lay, k=k, want_topk=True)      # eager, fresh buffers
        e_res = tl.toploc_verify_proofs_segments(rec, lay, e_proofs, k=k)
        torch.cuda.synchronize()
        assert torch.equal(out[0], e_proofs) and torch.equal(out[1], e_status) and torch.equal(out[2], e_idx), "replay %d" % rep
        assert torch.equal(res, e_res), "replay %d: verify records" % rep
        g = tl.results_numpy(res)
        for i in range(n_seg):
            a, b = lay[i], lay[i + 1]
            if (b - a) * hidden < k:
                assert int(out[1][i]) == tl.CHUNK_SHORT and g["status"][i] == tl.CHUNK_SHORT
                continue
            o_proofs, o_status = orc.build(bits[a:b].reshape(1, -1), k)
            assert np.array_equal(out[0][i].cpu().numpy(), o_proofs[0]) and int(out[1][i]) == int(o_status[0])
            o = orc.verify(rbits[a:b].reshape(1, -1), o_proofs, k)
            for f in FIELDS:
                assert g[f][i] == o[f][0], "replay %d segment %d field %s" % (rep, i, f)


def test_generation_layout_prefill_plus_decode_segments():
    """One sequence as the paper cuts it: a 75-token prompt, then 70 generated tokens in 32-token segments."""
    hidden, n_prompt, n_total, k = 4096, 75, 145, 128
    x = synth.activations(1, n_total, hidden, 5200, n_outlier=8, device=DEV).reshape(n_total, hidden)
    proofs, status, off = tl.toploc_build_proofs_generation(x, n_prompt, k=k)
    assert off.tolist() == [0, 75, 107, 139, 145]
    res = tl.toploc_verify_proofs_segments(x, off, proofs, k=k)
    torch.cuda.synchronize()
    assert not status.cpu().numpy().any() and (tl.results_numpy(res)["accept"] == 1).all()
    bits = synth.bits_numpy(x)
    for i in range(len(off) - 1):
        o_proofs, _ = orc.build(bits[int(off[i]):int(off[i + 1])].reshape(1, -1), k)
        assert np.array_equal(proofs[i].cpu().numpy(), o_proofs[0]), "segment %d" % i
    assert tl.generation_row_offsets(0, 64).tolist() == [0, 32, 64]
    assert tl.generation_row_offsets(10, 10).tolist() == [0, 10]


def test_host_threads_on_their_own_streams():
    """Four host threads call different entry points at once, each on a stream of its own."""
    import threading
    k = 128
    x_fused = synth.activations(40, 32, 1024, 5300, n_outlier=4, device=DEV).reshape(40, 32 * 1024)
    x_split = synth.activations(2, 32, 8192, 5301, n_outlier=8, device=DEV).reshape(2, 32 * 8192)
    x_seg = synth.activations(1, 77, 2048, 5302, n_outlier=4, device=DEV).reshape(77, 2048)
    off = np.array([0, 40, 72, 77], dtype=np.uint64)
    want = {
        "fused": orc.build(synth.bits_numpy(x_fused), k)[0],
        "split": orc.build(synth.bits_numpy(x_split), k)[0],
        "seg": np.stack([orc.build(synth.bits_numpy(x_seg)[int(off[i]):int(off[i + 1])].reshape(1, -1), k)[0][0]
                         for i in range(3)]),
    }
    want["verify"] = orc.verify(synth.bits_numpy(x_fused), want["fused"], k)
    proofs_dev = torch.from_numpy(want["fused"]).to(DEV)
    torch.cuda.synchronize()
    failures = []

    def worker(name):
        try:
            stream = torch.cuda.Stream(device=DEV)
            with torch.cuda.stream(stream):
                for rep in range(6):
                    if name == "fused":
                        got = tl.toploc_build_proofs(x_fused, k=k, chunk_tokens=1)[0]
                    elif name == "split":
                        got = tl.toploc_build_proofs(x_split, k=k, chunk_tokens=1)[0]
                    elif name == "seg":
                        got = tl.toploc_build_proofs_segments(x_seg, off, k=k)[0]
                    else:
                        got = tl.toploc_verify_proofs(x_fused, proofs_dev, k=k, chunk_tokens=1)
                    stream.synchronize()
                    if name == "verify":
                        g = tl.results_numpy(got)
                        ok = all(np.array_equal(g[f], want["verify"][f]) for f in FIELDS)
                    else:
                        ok = np.array_equal(got.cpu().numpy(), want[name])
                    if not ok:
                        failures.append("%s rep %d" % (name, rep))
        except Exception as e:  # reported by the main thread
            failures.append("%s: %r" % (name, e))

    say("threads fused/split/seg/verify, 6 calls each")
    threads = [threading.Thread(target=worker, args=(n,)) for n in ("fused", "split", "seg", "verify")]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not failures, failures
