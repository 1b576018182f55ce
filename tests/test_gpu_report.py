"""Statistics the paper tabulates, taken from the GPU path's own outputs."""
import numpy as np
import pytest
import torch

import oracle as orc
from paper_2501_16007_amd import binding as tl
from paper_2501_16007_amd import report, synth

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def test_modulus_distribution_on_unstructured_indices_follows_the_birthday_law():
    """Gaussian chunks without outlier channels: the top-k indices are a uniform random k-subset of [0, N).
    With N a multiple of 65536 the probability that Algorithm 6 stops at its first candidate has the closed
    form prod_j (N - j*N/65536) / (N - j); as N grows it tends to Table 7's 0.8833.  The GPU's share of
    m = 65536 must match it within sampling error, and later candidates must thin out fast (Table 7)."""
    k, n_chunks, hidden, tokens = 128, 8192, 8192, 32
    n = hidden * tokens
    x = synth.activations(n_chunks // 8, 8 * tokens, hidden, 8100, n_outlier=0, device=DEV)
    chunks = synth.as_chunks(x, tokens)
    proofs, status = tl.toploc_build_proofs(chunks, k=k, chunk_tokens=1)
    torch.cuda.synchronize()
    assert int(status.max()) == 0
    dist = report.modulus_distribution(proofs)
    per = n // 65536
    p_first = float(np.prod([(n - j * per) / (n - j) for j in range(k)]))
    sigma = (p_first * (1 - p_first) / n_chunks) ** 0.5
    print("[case] m = 65536: measured %.4f, closed form %.4f (Table 7 for unbounded indices: 0.8833)" % (
        dist.get(65536, 0.0), p_first), flush=True)
    assert abs(dist.get(65536, 0.0) - p_first) < 5 * sigma
    assert dist.get(65535, 0.0) < 0.15 and dist.get(65534, 0.0) < 0.03
    assert sum(v for m, v in dist.items() if m < 65530) < 5e-3
    # the oracle agrees on the modulus of a sample (bit-exact parity is tested elsewhere)
    sel = torch.arange(0, n_chunks, n_chunks // 8, device=DEV)
    o_proofs, _ = orc.build(synth.bits_numpy(chunks[sel]), k)
    assert np.array_equal(report.proof_modulus(o_proofs).numpy(), report.proof_modulus(proofs[sel]).cpu().numpy())


def test_summaries_topk_mismatch_and_text_codec():
    x = synth.config2(DEV, n_seq=2, n_tok=256)
    chunks = synth.as_chunks(x)
    proofs, status, idx = tl.toploc_build_proofs(chunks, k=128, chunk_tokens=1, want_topk=True)
    rec = synth.as_chunks(synth.perturb_relative(x, 2.0 ** -7, 8200))
    _, _, idx_rec = tl.toploc_build_proofs(rec, k=128, chunk_tokens=1, want_topk=True)
    res = tl.toploc_verify_proofs(rec, proofs, k=128, chunk_tokens=1)
    torch.cuda.synchronize()
    s = report.summarize_results(res)
    assert s["chunks"] == 16 and s["accepted"] == 16 and s["malformed"] == 0
    assert s["exp_mismatch_max"] <= 38 and s["mant_mean_max"] <= 10 and s["mant_median_max"] <= 8
    miss = report.topk_mismatch(idx, idx_rec).cpu().numpy()
    a, b = idx.cpu().numpy().view(np.uint32), idx_rec.cpu().numpy().view(np.uint32)
    want = [len(set(a[c].tolist()) - set(b[c].tolist())) for c in range(16)]
    assert miss.tolist() == want and max(want) < 20                      # reordering noise moves few entries
    assert report.topk_mismatch(idx, idx).sum().item() == 0
    text = report.proof_to_text(proofs[3])
    assert torch.equal(report.proof_from_text(text, DEV), proofs[3]) and len(text) == 344   # 258 bytes in base64
