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
    form prod_j (N - j*N/65536) / (N - j); as N grows it tends to the 0.8833 the appendix's table of
    Algorithm 6's return values prints.  The GPU's share of
    m = 65536 must match it within sampling error, and later candidates must thin out fast (same table)."""
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
    print("[case] m = 65536: measured %.4f, closed form %.4f (the paper's table, unbounded indices: 0.8833)" % (
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
    hexed = report.proof_to_text(proofs[3], encoding="hex")
    assert len(hexed) == 516 and torch.equal(report.proof_from_text(hexed, DEV, encoding="hex"), proofs[3])


def _exp(bits):
    return ((bits.astype(np.int64) >> 7) & 0xFF)


def _bin(d):
    ad = np.abs(d)
    cols = (d == 0, d == -1, d == 1, d == -2, d == 2, (d <= -3) & (d >= -10), (d >= 3) & (d <= 10),
            (ad > 10) & (ad < 100), ad >= 100)
    return {name: int(c.sum()) for name, c in zip(report.EXPONENT_DEVIATION_COLUMNS, cols)}


@pytest.mark.parametrize("k", [128, 1024])
def test_exponent_deviation_table_and_overlap_against_the_oracles_topk(k):
    """Table 1's counting on a perturbed recomputation, checked against the same counting over the
    oracle's top-k positions."""
    x = synth.activations(4, 32, 2048, 8300, n_outlier=8, device=DEV).reshape(4, -1)
    y = synth.perturb_relative(x, 2.0 ** -5, 8301)          # large enough to move exponents near powers of two
    xb, yb = synth.bits_numpy(x), synth.bits_numpy(y)
    got = report.exponent_deviation_counts(x, y, k)
    got_both = report.exponent_deviation_counts(x, y, k, both_only=True)
    miss = report.topk_mismatch_by_k(x, y, ks=(k,))[k]
    d_all, d_both, shares = [], [], []
    for c in range(4):
        ia, _ = orc.topk(xb[c], k)
        ib, _ = orc.topk(yb[c], k)
        d = _exp(yb[c][ia]) - _exp(xb[c][ia])
        keep = np.isin(ia, ib)
        d_all.append(d)
        d_both.append(np.abs(d[keep]))
        shares.append(keep.mean())
    assert got == _bin(np.concatenate(d_all))
    assert got_both == _bin(np.concatenate(d_both))
    assert sum(got.values()) == 4 * k and got["0"] > 0.8 * 4 * k and got["-1"] + got["+1"] > 0
    assert got_both["-1"] == 0 and got_both["-2"] == 0
    ratios = 1.0 - np.array(shares)
    assert abs(miss["mean"] - ratios.mean()) < 1e-12 and abs(miss["max"] - ratios.max()) < 1e-12
    assert abs(miss["median"] - np.median(ratios)) < 1e-12


def test_threshold_sweep_on_honest_and_tampered_recomputations():
    """One verify pass per recomputation serves every threshold triple: the re-decided accept bits equal the
    kernel's own under the same thresholds, and the paper's triple separates small numeric noise from
    activations of another input (Section 5.2; Tables 2 and 3)."""
    x = synth.config2(DEV, n_seq=2, n_tok=256)
    chunks = synth.as_chunks(x)
    proofs, _ = tl.toploc_build_proofs(chunks, k=128, chunk_tokens=1)
    honest_in = synth.as_chunks(synth.perturb_relative(x, 2.0 ** -7, 8400))
    tampered_in = synth.as_chunks(synth.activations(2, 256, 4096, 8401, n_outlier=8, device=DEV))
    honest = tl.results_numpy(tl.toploc_verify_proofs(honest_in, proofs, k=128, chunk_tokens=1))
    tampered = tl.results_numpy(tl.toploc_verify_proofs(tampered_in, proofs, k=128, chunk_tokens=1))
    for thr in ((38, 10, 8), (0, 0, 0), (5, 2, 1), (128, 127, 127)):
        for inp, rec in ((honest_in, honest), (tampered_in, tampered)):
            kernel = tl.results_numpy(tl.toploc_verify_proofs(inp, proofs, k=128, chunk_tokens=1, thresholds=thr))
            assert np.array_equal(report.decisions_under(rec, thr), kernel["accept"] == 1), thr
    rows = report.threshold_sweep(honest, tampered, [(38, 10, 8), (0, 0, 0), (128, 127, 127)])
    assert rows[0] == ((38, 10, 8), 0.0, 0.0)               # the paper's triple: no false reject, no false accept
    assert rows[1][1] > 0.9 and rows[1][2] == 0.0            # zero tolerance rejects honest noise too
    assert rows[2][1] == 0.0                                 # nothing honest fails the loosest triple
    sep = report.separation(honest, tampered)
    assert sep["exp_mismatch"][0] <= 38 < sep["exp_mismatch"][1]
    assert sep["mant_mean"][0] <= 10 and sep["mant_median"][0] <= 8


def test_error_statistics_row_against_the_oracle():
    """The row of Tables 2-5 for an honest pair (small numeric noise) and for a tampered pair (another
    input), each statistic checked against the same reduction over the oracle's records and top-k."""
    x = synth.activations(8, 32, 2048, 8500, n_outlier=8, device=DEV).reshape(8, -1)
    honest = synth.perturb_relative(x, 2.0 ** -7, 8501)
    other = synth.activations(8, 32, 2048, 8502, n_outlier=8, device=DEV).reshape(8, -1)
    k = 128
    xb = synth.bits_numpy(x)
    o_proofs, _, o_idx = orc.build(xb, k, want_topk=True)
    for val, should_pass in ((honest, True), (other, False)):
        row = report.error_statistics_row(x, val, k=k)
        vb = synth.bits_numpy(val)
        o = orc.verify(vb, o_proofs, k)
        miss = [len(set(o_idx[c].tolist()) - set(orc.topk(vb[c], k)[0].tolist())) for c in range(8)]
        assert row["chunks"] == 8 and row["accepted"] == int(o["accept"].sum()) == (8 if should_pass else 0)
        assert row["topk_mismatch_max"] == max(miss) and row["exp_mismatch_max"] == int(o["err_exp"].max())
        assert row["exp_mismatch_min"] == int(o["err_exp"].min())
        some = o["n_match"] > 0
        if some.any():
            mean = o["mant_sum"][some] / o["n_match"][some]
            assert abs(row["mant_mean_max"] - mean.max()) < 1e-12 and abs(row["mant_mean_min"] - mean.min()) < 1e-12
            assert row["mant_median_max"] == int(o["mant_median"][some].max())
        if should_pass:
            assert row["exp_mismatch_max"] <= 38 and row["mant_mean_max"] <= 10 and row["mant_median_max"] <= 8
        else:
            assert row["exp_mismatch_min"] > 38      # the best case of a wrong input is still far above T_exp


def test_report_command_line_prints_every_table(capsys):
    report.main(["--seqs", "2", "--tokens", "64", "--hidden", "1024", "--ks", "64", "128", "1024"])
    out = capsys.readouterr().out
    for title in ("error statistics per generation", "exponent deviation at the top-k positions",
                  "top-k mismatch ratio by k", "injective modulus of the proofs"):
        assert title in out
    assert "relative noise 2^-7" in out and "   4/4" in out           # small noise: every chunk accepted
