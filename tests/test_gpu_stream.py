"""Online path without the ring: the running top-k kept per sequence while rows are
appended must give, at emission, the bytes Algorithm 1 gives for the assembled chunk
(the CPU oracle sees the chunk as one flat array)."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2501_16007_amd import binding as tl
from paper_2501_16007_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


def run_stream(steps, k, T, order=None):
    """steps [T, n_seq, H] -> (proofs, status, idx) after appending the T rows (in `order`) and emitting."""
    n_seq = steps.shape[1]
    state = tl.toploc_stream_new_state(n_seq, k, DEV)
    for t in (range(T) if order is None else order):
        tl.toploc_stream_append(state, steps[t], t, k=k, chunk_tokens=T)
    proofs, status, idx = tl.toploc_stream_emit(state, n_seq, k=k, want_topk=True)
    torch.cuda.synchronize()
    return state, proofs.cpu().numpy(), status.cpu().numpy(), idx.cpu().numpy().view(np.uint32)


def check_against_oracle(steps, k, T, order=None, what=""):
    say("%s n_seq=%d H=%d T=%d k=%d" % (what, steps.shape[1], steps.shape[2], T, k))
    chunk_bits = synth.bits_numpy(steps.transpose(0, 1).contiguous()).reshape(steps.shape[1], -1)
    o_proofs, o_status, o_idx = orc.build(chunk_bits, k, want_topk=True)
    state, proofs, status, idx = run_stream(steps, k, T, order)
    assert np.array_equal(idx, o_idx), what + ": indices"
    assert np.array_equal(status, o_status), what + ": status"
    assert np.array_equal(proofs, o_proofs), what + ": proof bytes"
    return state


@pytest.mark.parametrize("hidden,T,k,n_seq", [
    (5120, 32, 128, 6),     # the online workload's width
    (5120, 32, 32, 3),
    (5120, 32, 512, 3),
    (4096, 32, 128, 4),
    (8192, 32, 128, 2),
    (64, 32, 128, 3),       # a row holds fewer than k values: the state fills over two rows
    (8, 16, 16, 2),         # one vector per row
    (1000, 7, 64, 3),       # ragged sizes
])
def test_stream_matches_oracle_on_the_assembled_chunk(hidden, T, k, n_seq):
    steps = synth.config5_steps(n_seq, hidden, T, seed=7000 + hidden + k, device=DEV)
    check_against_oracle(steps, k, T, what="stream")


def test_stream_rows_in_any_order_and_state_reuse():
    T, k, n_seq, hidden = 32, 128, 4, 2048
    steps = synth.config5_steps(n_seq, hidden, 2 * T, seed=7100, device=DEV)
    order = np.random.default_rng(71).permutation(T).tolist()
    state = check_against_oracle(steps[:T], k, T, order=order, what="shuffled rows")
    # the emission emptied the state: a second chunk through the same memory
    for t in range(T):
        tl.toploc_stream_append(state, steps[T + t], t, k=k, chunk_tokens=T)
    proofs, status = tl.toploc_stream_emit(state, n_seq, k=k)
    torch.cuda.synchronize()
    bits = synth.bits_numpy(steps[T:].transpose(0, 1).contiguous()).reshape(n_seq, -1)
    o_proofs, o_status = orc.build(bits, k)
    assert np.array_equal(proofs.cpu().numpy(), o_proofs) and np.array_equal(status.cpu().numpy(), o_status)


def test_stream_ties_and_equal_rows():
    T, k, n_seq, hidden = 8, 128, 2, 512
    vals = np.array([0x3F80, 0xBF80, 0x4000, 0x0000], dtype=np.uint16)
    bits = vals[np.random.default_rng(72).integers(0, 4, size=(T, n_seq, hidden))]
    bits[:, 1, :] = 0x3F80                      # sequence 1: every value equal, the lowest indices win
    steps = synth.from_bits(bits, DEV)
    check_against_oracle(steps, k, T, what="ties")


@pytest.mark.parametrize("k", [128, 512])
def test_stream_rows_that_grow_step_by_step(k):
    """every row larger than all rows before it (and ascending inside the row): each append finds its whole row above
    the stored threshold, the queue and the candidate buffer overflow, and the bound comes from the queue's own values
    on top of the k seeds the state brought in"""
    T, n_seq, hidden = 32, 3, 8192
    n = T * hidden
    mag = (np.arange(n, dtype=np.uint32) * 0x7F00 // (n + 64)).astype(np.uint16)      # finite bf16 patterns, ascending
    sign = np.random.default_rng(73).integers(0, 2, size=(n_seq, n)).astype(np.uint16) << 15
    bits = (mag[None, :] | sign).reshape(n_seq, T, hidden).transpose(1, 0, 2)         # [T, n_seq, hidden]
    steps = synth.from_bits(np.ascontiguousarray(bits), DEV)
    check_against_oracle(steps, k, T, what="growing rows")


def test_stream_short_chunk_is_reported():
    n_seq, hidden, k = 3, 16, 128
    steps = synth.config5_steps(n_seq, hidden, 4, seed=7200, device=DEV)
    state = tl.toploc_stream_new_state(n_seq, k, DEV)
    for t in range(4):                          # 64 values < k
        tl.toploc_stream_append(state, steps[t], t, k=k, chunk_tokens=32)
    proofs, status, idx = tl.toploc_stream_emit(state, n_seq, k=k, want_topk=True)
    torch.cuda.synchronize()
    assert (status.cpu().numpy() == tl.CHUNK_SHORT).all() and not proofs.cpu().numpy().any()


def test_stream_equals_the_ring_path_at_full_width():
    """1024 sequences x 5120: streamed proofs equal toploc_build_proofs over the ring; oracle on a sample."""
    n_seq, hidden, T = 1024, 5120, 32
    steps = synth.config5_steps(n_seq, hidden, T, device=DEV)
    ring = torch.zeros((n_seq, T, hidden), dtype=torch.bfloat16, device=DEV)
    for t in range(T):
        tl.toploc_ring_append(ring, steps[t], t)
    chunks = ring.reshape(n_seq, T * hidden)
    sel = np.sort(np.random.default_rng(73).choice(n_seq, 8, replace=False))
    sample_bits = synth.bits_numpy(chunks[torch.from_numpy(sel).to(DEV)])
    for k in (32, 128, 512):
        say("full width k=%d" % k)
        _, proofs, status, idx = run_stream(steps, k, T)
        r_proofs, r_status, r_idx = tl.toploc_build_proofs(chunks, k=k, chunk_tokens=1, want_topk=True)
        torch.cuda.synchronize()
        assert np.array_equal(proofs, r_proofs.cpu().numpy()) and np.array_equal(status, r_status.cpu().numpy())
        assert np.array_equal(idx, r_idx.cpu().numpy().view(np.uint32))
        o_proofs, o_status, o_idx = orc.build(sample_bits, k, want_topk=True)
        assert np.array_equal(proofs[sel], o_proofs) and np.array_equal(idx[sel], o_idx)


def test_stream_window_captured_in_a_graph_replays_like_eager():
    """32 appends and the emission captured once (no memset nodes: the library only launches kernels),
    replayed three times on fresh data with eager work and synchronisations in between."""
    n_seq, hidden, T, k = 64, 5120, 32, 128
    steps = synth.config5_steps(n_seq, hidden, 3 * T, seed=7300, device=DEV)
    static = torch.empty((T, n_seq, hidden), dtype=torch.bfloat16, device=DEV)
    state = tl.toploc_stream_new_state(n_seq, k, DEV)
    proofs = torch.empty((n_seq, 2 + 2 * k), dtype=torch.uint8, device=DEV)
    status = torch.empty(n_seq, dtype=torch.uint8, device=DEV)

    def window():
        for t in range(T):
            tl.toploc_stream_append(state, static[t], t, k=k, chunk_tokens=T)
        tl.toploc_stream_emit(state, n_seq, k=k, out=(proofs, status))

    static.copy_(steps[:T])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        window()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        window()
    for rep in range(3):
        static.copy_(steps[rep * T:(rep + 1) * T])
        proofs.zero_()
        graph.replay()
        torch.cuda.synchronize()
        replayed = proofs.clone()
        window()                                   # the same window, eager
        torch.cuda.synchronize()
        assert torch.equal(replayed, proofs) and int(status.max()) == 0, "replay %d differs from eager" % rep
        bits = synth.bits_numpy(static.transpose(0, 1).contiguous()).reshape(n_seq, -1)
        o_proofs, _ = orc.build(bits[:8], k)
        assert np.array_equal(replayed[:8].cpu().numpy(), o_proofs)


def test_continuous_batching_against_the_oracle_per_sequence():
    """Sequences join and leave a running batch at different steps; every proof the prover cuts (full
    32-token chunks, ragged tails, the prompt) equals the oracle's on the rows that went into it."""
    from paper_2501_16007_amd.online import OnlineProver
    hidden, k, n_slots = 1024, 128, 6
    plan = {0: (0, 70), 1: (3, 33), 2: (10, 64), 3: (10, 5), 4: (40, 100), 5: (41, 32)}   # slot: (first step, tokens)
    rows = {s: synth.activations(1, n, hidden, 6100 + s, n_outlier=4, device=DEV).reshape(n, hidden)
            for s, (_, n) in plan.items()}
    say("continuous batching: %d slots, lengths %s" % (n_slots, [n for _, n in plan.values()]))
    prover = OnlineProver(n_slots, hidden, k=k, device=DEV)
    got = {s: [] for s in plan}
    for step in range(150):
        active = [s for s, (t0, n) in plan.items() if t0 <= step < t0 + n]
        if active:
            batch = torch.stack([rows[s][step - plan[s][0]] for s in active])
            out = prover.append(batch, active)
            if out is not None:
                for s, p, st in zip(out[0].tolist(), out[1].cpu().numpy(), out[2].cpu().numpy()):
                    got[s].append((p, int(st)))
        ended = [s for s, (t0, n) in plan.items() if step == t0 + n - 1]
        out = prover.finish(ended) if ended else None
        if out is not None:
            for s, p, st in zip(out[0].tolist(), out[1].cpu().numpy(), out[2].cpu().numpy()):
                got[s].append((p, int(st)))
    assert not prover.rows.any()
    for s, (_, n) in plan.items():
        bits = synth.bits_numpy(rows[s])
        cuts = list(range(0, n, 32)) + [n]
        assert len(got[s]) == len(cuts) - 1, "slot %d: %d proofs" % (s, len(got[s]))
        for c, (p, st) in enumerate(got[s]):
            o_proofs, o_status = orc.build(bits[cuts[c]:cuts[c + 1]].reshape(1, -1), k)
            assert st == int(o_status[0]) and np.array_equal(p, o_proofs[0]), "slot %d chunk %d" % (s, c)
    # the prompt's proof is the segment call on the prompt's rows
    p, st = prover.prefill(rows[4][:75])
    o_proofs, _ = orc.build(synth.bits_numpy(rows[4][:75]).reshape(1, -1), k)
    assert int(st) == 0 and np.array_equal(p.cpu().numpy(), o_proofs[0])


def test_indexed_stream_calls_skip_rows_that_are_out_of_range():
    hidden, k = 256, 16
    state = tl.toploc_stream_new_state(3, k, DEV)
    x = synth.activations(1, 4, hidden, 6200, n_outlier=2, device=DEV).reshape(4, hidden)
    # rows 1 and 3 name a slot / a token that do not exist: they must leave every state alone
    tl.toploc_stream_append_rows(state, 3, x, [2, 7, 0, 1], [0, 0, 5, 32], k=k)
    proofs, status, idx = tl.toploc_stream_emit_rows(state, 3, [0, 1, 2, 9], k=k, want_topk=True)
    torch.cuda.synchronize()
    bits = synth.bits_numpy(x)
    o2, s2, i2 = orc.build(bits[0:1], k, want_topk=True)                   # slot 2: row 0 as token 0
    o0, s0, i0 = orc.build(bits[2:3], k, want_topk=True)                   # slot 0: row 2 as token 5
    assert status.cpu().numpy().tolist() == [0, tl.CHUNK_SHORT, 0, tl.CHUNK_SHORT]
    assert np.array_equal(proofs[2].cpu().numpy(), o2[0]) and np.array_equal(idx[2].cpu().numpy().view(np.uint32), i2[0])
    assert np.array_equal(idx[0].cpu().numpy().view(np.uint32), i0[0] + 5 * hidden)
    assert not proofs[1].any() and not proofs[3].any()
    # emission emptied the states
    _, status = tl.toploc_stream_emit_rows(state, 3, [0, 1, 2], k=k)
    assert status.cpu().numpy().tolist() == [tl.CHUNK_SHORT] * 3
