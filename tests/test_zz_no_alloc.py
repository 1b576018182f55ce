"""toploc_build_proofs_static (the entry point that allocates nothing) against toploc_build_proofs.

Two calls in a row share the library's fixed scratch array, the second with a smaller input, so
stale candidates of the first call lie behind the second call's.  Outputs must be byte for byte
those of the entry point with a caller-provided workspace; a sample is also checked against the
oracle.  No device memory is allocated between the two calls (torch's allocator statistics).
"""
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


def outputs(n_chunks, k):
    return (torch.full((n_chunks, 2 + 2 * k), 0xAB, dtype=torch.uint8, device=DEV),
            torch.full((n_chunks,), 0xCD, dtype=torch.uint8, device=DEV),
            torch.full((n_chunks, k), -1, dtype=torch.int32, device=DEV))


def reference(chunks, k):
    proofs, status, idx = tl.toploc_build_proofs(chunks, k=k, chunk_tokens=1, want_topk=True)
    torch.cuda.synchronize()
    return proofs, status, idx


@pytest.mark.parametrize("first,second", [
    ((48, 32 * 4096, 512), (5, 32 * 4096, 128)),      # split launches both times, k shrinks too
    ((200, 32 * 5120, 128), (3, 32 * 5120, 512)),     # the second call has fewer chunks but larger k
    ((2048, 32 * 1024, 128), (7, 32 * 2040, 32)),      # fused launch (no scratch), then a split one
])
def test_static_scratch_matches_workspace_entry_point(first, second):
    cases = []
    for i, (n_chunks, n, k) in enumerate((first, second)):
        x = synth.activations(n_chunks, 1, n, 8800 + 13 * i + n_chunks, n_outlier=4, device=DEV).reshape(n_chunks, n)
        cases.append((x, k, reference(x, k), outputs(n_chunks, k)))
    # first use on this device (looks the array's address up) happens before the region that must not allocate
    x0, k0, _, (p0, s0, i0) = cases[0]
    need0 = tl.toploc_workspace_bytes(k0, 1, x0.shape[1], x0.shape[0])
    need1 = tl.toploc_workspace_bytes(cases[1][1], 1, cases[1][0].shape[1], cases[1][0].shape[0])
    say("static scratch: %s then %s, workspace sizes %d then %d of %d" % (first, second, need0, need1,
                                                                          tl.STATIC_SCRATCH_BYTES))
    assert need1 > 0 and max(need0, need1) <= tl.STATIC_SCRATCH_BYTES
    allocs_before = torch.cuda.memory_stats(DEV)["allocation.all.allocated"]
    for x, k, _, (p, s, i) in cases:                       # back to back on one stream, no sync between
        tl.toploc_build_proofs_static(x, (p, s), k=k, chunk_tokens=1, topk_out=i)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats(DEV)["allocation.all.allocated"] == allocs_before
    for (x, k, (rp, rs, ri), (p, s, i)), name in zip(cases, ("first", "second")):
        assert torch.equal(p, rp), name + " call: proofs differ from toploc_build_proofs"
        assert torch.equal(s, rs), name + " call: status differs"
        assert torch.equal(i, ri), name + " call: indices differ"
        n_or = min(x.shape[0], 16)
        bits = synth.bits_numpy(x[:n_or])
        o_proofs, o_status, o_idx = orc.build(bits, k, want_topk=True)
        assert np.array_equal(p[:n_or].cpu().numpy(), o_proofs), name + " call: proofs differ from the oracle"
        assert np.array_equal(i[:n_or].cpu().numpy().view(np.uint32), o_idx)
        assert np.array_equal(s[:n_or].cpu().numpy(), o_status)


def test_static_scratch_rejects_what_does_not_fit():
    n_chunks, n, k = 4096, 32 * 512, 512                 # 4096 parts x 512 candidates x 6 bytes = 12 MiB
    x = torch.zeros((n_chunks, n), dtype=torch.bfloat16, device=DEV)
    p, s, i = outputs(n_chunks, k)
    assert tl.toploc_workspace_bytes(k, 1, n, n_chunks) > tl.STATIC_SCRATCH_BYTES
    with pytest.raises(tl.ToplocError) as err:
        tl.toploc_build_proofs_static(x, (p, s), k=k, chunk_tokens=1, topk_out=i)
    assert err.value.code == tl.ESCRATCH
    torch.cuda.synchronize()
    assert int(p.min()) == 0xAB and int(s.min()) == 0xCD  # nothing was enqueued
