"""Reading aids for proofs and verify records: what the paper tabulates (the modulus
Algorithm 6 returns, the appendix's table of its return values; exponent mismatches and mantissa differences, Tables 2-5;
top-k mismatch, Table 1) taken from the library's outputs.  Nothing here is on the
build / verify path; these are reductions over its results with plain tensor ops."""
import base64

import numpy as np
import torch

from . import binding


def proof_modulus(proofs):
    """uint8 [n, proof_bytes] (device or host) -> int64 tensor [n] of the injective modulus m."""
    p = proofs if isinstance(proofs, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(proofs))
    m = p[:, 0].to(torch.int64) | (p[:, 1].to(torch.int64) << 8)
    return torch.where(m == 0, torch.full_like(m, 65536), m)


def modulus_distribution(proofs):
    """{m: fraction of proofs}, largest modulus first (the shape of the appendix's table of Algorithm 6's return values)."""
    m = proof_modulus(proofs).cpu().numpy()
    vals, counts = np.unique(m, return_counts=True)
    order = np.argsort(-vals)
    return {int(vals[i]): float(counts[i]) / m.size for i in order}


def summarize_results(results):
    """Worst and mean statistics over a batch of verify records (device tensor [n, 20] or the
    structured array of binding.results_numpy): the columns of Tables 2-5."""
    r = binding.results_numpy(results) if isinstance(results, torch.Tensor) else results
    n = max(1, r.size)
    matched = np.maximum(r["n_match"], 1)
    mean = r["mant_sum"] / matched
    return {
        "chunks": int(r.size),
        "accepted": int(r["accept"].sum()),
        "malformed": int((r["status"] != binding.CHUNK_OK).sum()),
        "exp_mismatch_max": int(r["err_exp"].max()) if r.size else 0,
        "exp_mismatch_mean": float(r["err_exp"].sum()) / n,
        "mant_mean_max": float(mean.max()) if r.size else 0.0,
        "mant_mean_mean": float(mean.mean()) if r.size else 0.0,
        "mant_median_max": int(r["mant_median"].max()) if r.size else 0,
    }


def error_statistics_row(chunks_gen, chunks_val, k=128, thresholds=binding.BF16_THRESHOLDS):
    """One row of the paper's error-statistics tables (Tables 2-5): proofs built from `chunks_gen`
    [n_chunks, N] are validated against `chunks_val`.  Worst case over the chunks as Table 2 prints it
    (for a pair that should pass) and best case as Tables 3 and 4 print it (for a pair that should fail)."""
    proofs, status, idx_gen = binding.toploc_build_proofs(chunks_gen, k=k, chunk_tokens=1, want_topk=True)
    idx_val, _ = binding.toploc_topk(chunks_val, k=k, chunk_tokens=1)
    r = binding.results_numpy(binding.toploc_verify_proofs(chunks_val, proofs, k=k, chunk_tokens=1, thresholds=thresholds))
    miss = topk_mismatch(idx_gen, idx_val).cpu().numpy()
    mean = r["mant_sum"] / np.maximum(r["n_match"], 1)
    some = r["n_match"] > 0                           # the paper prints "-" where nothing matched
    return {
        "chunks": int(r.size), "accepted": int(r["accept"].sum()), "unbuilt": int((status != 0).sum().item()),
        "topk_mismatch_max": int(miss.max()), "topk_mismatch_max_pct": 100.0 * float(miss.max()) / k,
        "exp_mismatch_max": int(r["err_exp"].max()), "exp_mismatch_max_pct": 100.0 * float(r["err_exp"].max()) / k,
        "exp_mismatch_min": int(r["err_exp"].min()),
        "mant_mean_max": float(mean[some].max()) if some.any() else None,
        "mant_mean_min": float(mean[some].min()) if some.any() else None,
        "mant_median_max": int(r["mant_median"][some].max()) if some.any() else None,
        "mant_median_min": int(r["mant_median"][some].min()) if some.any() else None,
    }


def topk_mismatch(idx_a, idx_b):
    """Per chunk, how many of the k indices of idx_a are missing from idx_b (Table 1's top-k
    mismatch); both are [n_chunks, k] index tensors as the build calls export them."""
    a = idx_a.to(torch.int64) & 0xFFFFFFFF
    b = idx_b.to(torch.int64) & 0xFFFFFFFF
    bs, _ = torch.sort(b, dim=1)
    pos = torch.searchsorted(bs, a).clamp(max=bs.shape[1] - 1)
    found = torch.gather(bs, 1, pos) == a
    return (~found).sum(dim=1)


def proof_to_text(proof, encoding="base64"):
    """One proof (uint8 tensor or bytes) as base64 or hex text, e.g. to attach to a response."""
    raw = bytes(proof.cpu().numpy().tobytes()) if isinstance(proof, torch.Tensor) else bytes(proof)
    if encoding == "hex":
        return raw.hex()
    if encoding != "base64":
        raise ValueError("encoding is 'base64' or 'hex'")
    return base64.b64encode(raw).decode("ascii")


def proof_from_text(text, device="cpu", encoding="base64"):
    if encoding == "hex":
        raw = bytes.fromhex(text)
    elif encoding == "base64":
        raw = base64.b64decode(text.encode("ascii"), validate=True)
    else:
        raise ValueError("encoding is 'base64' or 'hex'")
    return torch.from_numpy(np.frombuffer(raw, dtype=np.uint8).copy()).to(device)


# Columns of Table 1 (signed deviation d of the 8-bit exponent field) and of its appendix
# twin (|d| only).  The table's ranges share their end points; here 10 belongs to "3..10"
# and 100 to ">=100".
EXPONENT_DEVIATION_COLUMNS = ("0", "-1", "+1", "-2", "+2", "-10..-3", "+3..+10", "10<|d|<100", "|d|>=100")


def _exponent(chunks, idx):
    bits = chunks.view(torch.int16).to(torch.int64) & 0xFFFF
    return (torch.gather(bits, 1, idx.to(torch.int64) & 0xFFFFFFFF) >> 7) & 0xFF


def exponent_deviation_counts(chunks_a, chunks_b, k, both_only=False):
    """Table 1 for one k over [n_chunks, N] bf16 chunks: at the top-k positions of `chunks_a`
    (the library's toploc_topk, so k may reach 4096), d = exponent(chunks_b) - exponent(chunks_a),
    counted per column of EXPONENT_DEVIATION_COLUMNS.  both_only: only positions that are also among
    the top-k of `chunks_b`, |d| in place of d (the appendix table: its negative columns stay empty).
    Returns {column: count}."""
    idx_a, _ = binding.toploc_topk(chunks_a, k=k, chunk_tokens=1)
    d = _exponent(chunks_b, idx_a) - _exponent(chunks_a, idx_a)
    if both_only:
        idx_b, _ = binding.toploc_topk(chunks_b, k=k, chunk_tokens=1)
        a = idx_a.to(torch.int64) & 0xFFFFFFFF
        bs, _ = torch.sort(idx_b.to(torch.int64) & 0xFFFFFFFF, dim=1)
        pos = torch.searchsorted(bs, a).clamp(max=k - 1)
        d = d.abs()[torch.gather(bs, 1, pos) == a]
    d = d.reshape(-1)
    ad = d.abs()
    cols = (d == 0, d == -1, d == 1, d == -2, d == 2, (d <= -3) & (d >= -10), (d >= 3) & (d <= 10),
            (ad > 10) & (ad < 100), ad >= 100)
    return {name: int(c.sum().item()) for name, c in zip(EXPONENT_DEVIATION_COLUMNS, cols)}


def topk_mismatch_by_k(chunks_a, chunks_b, ks=(64, 128, 256, 512, 1024, 2048, 4096)):
    """{k: {"max", "median", "mean"}} of the mismatch ratio per chunk: the share of the top-k positions of
    chunks_a that are not top-k positions of chunks_b, the two index sets compared as sets (the quantity
    Section 5.5 plots over k as maximum and median)."""
    out = {}
    for k in ks:
        ia, _ = binding.toploc_topk(chunks_a, k=k, chunk_tokens=1)
        ib, _ = binding.toploc_topk(chunks_b, k=k, chunk_tokens=1)
        ratio = (topk_mismatch(ia, ib).to(torch.float64) / k).cpu().numpy()
        out[int(k)] = {"max": float(ratio.max()), "median": float(np.median(ratio)), "mean": float(ratio.mean())}
    return out


def decisions_under(results, thresholds):
    """The accept bit every record would get under other thresholds (t_exp, t_mean, t_median): the
    rule of Algorithm 2 applied again to the stored statistics, so that one verify pass serves a
    whole sweep.  Malformed records stay rejected.  Returns a bool array."""
    r = binding.results_numpy(results) if isinstance(results, torch.Tensor) else results
    t_exp, t_mean, t_median = thresholds
    n = r["n_match"].astype(np.int64)
    reject = r["err_exp"].astype(np.int64) > t_exp
    reject |= (n > 0) & (r["mant_sum"].astype(np.int64) > t_mean * n)
    reject |= (n > 0) & (r["mant_median"].astype(np.int64) > t_median)
    reject |= r["status"] != binding.CHUNK_OK
    return ~reject


def threshold_sweep(honest, tampered, grid):
    """For every (t_exp, t_mean, t_median) of `grid`: the share of honest records rejected and of
    tampered records accepted.  Returns a list of (thresholds, false_reject, false_accept)."""
    rows = []
    for thr in grid:
        fr = 1.0 - float(decisions_under(honest, thr).mean()) if len(honest) else 0.0
        fa = float(decisions_under(tampered, thr).mean()) if len(tampered) else 0.0
        rows.append((tuple(thr), fr, fa))
    return rows


def separation(honest, tampered):
    """Per statistic, the worst honest value and the best tampered value (the two numbers the paper
    reads its thresholds from, Section 5.2 with Tables 2-5): a threshold between them separates the
    two sets on that statistic alone.  Returns {statistic: (honest_max, tampered_min)}."""
    def stats(res):
        r = binding.results_numpy(res) if isinstance(res, torch.Tensor) else res
        r = r[r["status"] == binding.CHUNK_OK]
        mean = r["mant_sum"] / np.maximum(r["n_match"], 1)
        return {"exp_mismatch": r["err_exp"].astype(np.float64), "mant_mean": mean.astype(np.float64),
                "mant_median": r["mant_median"].astype(np.float64)}
    h, t = stats(honest), stats(tampered)
    return {name: (float(h[name].max()) if h[name].size else float("nan"),
                   float(t[name].min()) if t[name].size else float("nan")) for name in h}


def main(argv=None):
    """Prints the shape of the paper's statistics tables on seeded synthetic activations and a few kinds of
    recomputation (the paper's own numbers need its models and dataset): python -m paper_2501_16007_amd.report"""
    import argparse

    from . import synth
    ap = argparse.ArgumentParser(description=main.__doc__)
    ap.add_argument("--seqs", type=int, default=8)
    ap.add_argument("--tokens", type=int, default=512)
    ap.add_argument("--hidden", type=int, default=4096)
    ap.add_argument("--k", type=int, default=128)
    ap.add_argument("--ks", type=int, nargs="*", default=[64, 128, 256, 512, 1024, 2048, 4096])
    ap.add_argument("--device", default="cuda:0")
    args = ap.parse_args(argv)
    x = synth.activations(args.seqs, args.tokens, args.hidden, synth.BASE_SEED + 40, n_outlier=8, device=args.device)
    chunks = synth.as_chunks(x)
    pairs = [
        ("relative noise 2^-9", synth.as_chunks(synth.perturb_relative(x, 2.0 ** -9, 41))),
        ("relative noise 2^-7", synth.as_chunks(synth.perturb_relative(x, 2.0 ** -7, 42))),
        ("relative noise 2^-5", synth.as_chunks(synth.perturb_relative(x, 2.0 ** -5, 43))),
        ("fp8 e4m3 round trip", synth.as_chunks(synth.roundtrip_e4m3(x))),
        ("another input", synth.as_chunks(synth.activations(args.seqs, args.tokens, args.hidden, synth.BASE_SEED + 44,
                                                          n_outlier=8, device=args.device))),
    ]
    print("%d chunks of %d values, k = %d" % (chunks.shape[0], chunks.shape[1], args.k))
    print("\nerror statistics per generation / validation pair (worst case; best case in brackets)")
    print("%-22s %9s %14s %14s %14s %14s" % ("validation input", "accepted", "top-k mismatch", "exp mismatch", "mant mean",
                                            "mant median"))
    for name, val in pairs:
        r = error_statistics_row(chunks, val, k=args.k)
        fmt = lambda hi, lo: "-" if hi is None else "%.4g [%.4g]" % (hi, lo)
        print("%-22s %4d/%-4d %14s %14s %14s %14s" % (
            name, r["accepted"], r["chunks"], "%d (%.1f%%)" % (r["topk_mismatch_max"], r["topk_mismatch_max_pct"]),
            "%d [%d]" % (r["exp_mismatch_max"], r["exp_mismatch_min"]), fmt(r["mant_mean_max"], r["mant_mean_min"]),
            fmt(r["mant_median_max"], r["mant_median_min"])))
    val = pairs[1][1]
    ks = [k for k in args.ks if k <= chunks.shape[1]]
    print("\nexponent deviation at the top-k positions, validation input '%s'" % pairs[1][0])
    print("%6s " % "k" + " ".join("%11s" % c for c in EXPONENT_DEVIATION_COLUMNS))
    for k in ks:
        counts = exponent_deviation_counts(chunks, val, k)
        print("%6d " % k + " ".join("%11d" % counts[c] for c in EXPONENT_DEVIATION_COLUMNS))
    print("\ntop-k mismatch ratio by k (max / median over chunks), same pair")
    for k, m in topk_mismatch_by_k(chunks, val, ks=ks).items():
        print("%6d  %.4f / %.4f" % (k, m["max"], m["median"]))
    proofs, _ = binding.toploc_build_proofs(chunks, k=args.k, chunk_tokens=1)
    print("\ninjective modulus of the proofs (share of chunks)")
    for m, share in list(modulus_distribution(proofs).items())[:6]:
        print("%6d  %.4f" % (m, share))


if __name__ == "__main__":
    main()
