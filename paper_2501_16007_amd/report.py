"""Reading aids for proofs and verify records: what the paper tabulates (the modulus
Algorithm 6 returns, Table 7; exponent mismatches and mantissa differences, Tables 2-5;
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
    """{m: fraction of proofs}, largest modulus first (the shape of Table 7)."""
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


def topk_mismatch(idx_a, idx_b):
    """Per chunk, how many of the k indices of idx_a are missing from idx_b (Table 1's top-k
    mismatch); both are [n_chunks, k] index tensors as the build calls export them."""
    a = idx_a.to(torch.int64) & 0xFFFFFFFF
    b = idx_b.to(torch.int64) & 0xFFFFFFFF
    bs, _ = torch.sort(b, dim=1)
    pos = torch.searchsorted(bs, a).clamp(max=bs.shape[1] - 1)
    found = torch.gather(bs, 1, pos) == a
    return (~found).sum(dim=1)


def proof_to_text(proof):
    """One proof (uint8 tensor or bytes) as base64 text, e.g. to attach to a response."""
    raw = bytes(proof.cpu().numpy().tobytes()) if isinstance(proof, torch.Tensor) else bytes(proof)
    return base64.b64encode(raw).decode("ascii")


def proof_from_text(text, device="cpu"):
    raw = base64.b64decode(text.encode("ascii"))
    return torch.from_numpy(np.frombuffer(raw, dtype=np.uint8).copy()).to(device)
