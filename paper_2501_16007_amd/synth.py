"""Seeded synthetic inputs shaped like LLM last-layer hidden states.

This module serves both the CPU oracle's tests and the GPU path.  It holds
none of the method's arithmetic: no top-k, no modular arithmetic, no bit
extraction.  It only draws tensors.

The paper measured on UltraChat prompts run through Llama-3.1-8B/70B,
INTELLECT-1 and Gemma-2-9b (Section 5.1 and the appendix's table of model configurations); neither the dataset nor
any weights are available here, so these tensors stand in for them.  They
take the shapes (hidden 4096 / 8192 / 5120 / 3584, bf16) and the structure
that makes top-k reproducible in real models (Section 3.3): a near-Gaussian
bulk plus a few fixed channels of much larger magnitude.
"""
import numpy as np
import torch

BASE_SEED = 20250116
CHUNK_TOKENS = 32


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def outlier_channels(hidden, n_outlier, seed):
    """The fixed set of high-magnitude channels of the emulated model."""
    g = _gen(seed, "cpu")
    return torch.randperm(hidden, generator=g)[:n_outlier].sort().values


def activations(n_seq, n_tok, hidden, seed, n_outlier=8, outlier_scale=20.0, lognormal_sigma=0.5,
                device="cpu", channel_seed=None, dtype=torch.bfloat16):
    """bf16 (or fp32) tensor [n_seq, n_tok, hidden]: N(0,1) bulk; `n_outlier` fixed channels
    multiplied by outlier_scale * exp(lognormal_sigma * z), z ~ N(0,1) drawn per
    (sequence, channel).  lognormal_sigma = 0 gives the plain x`outlier_scale` case.
    Built one sequence at a time so the fp32 staging stays small."""
    device = torch.device(device)
    ch = outlier_channels(hidden, n_outlier, seed if channel_seed is None else channel_seed).to(device)
    g = _gen(seed + 1, device)
    gs = _gen(seed + 2, "cpu")
    z = torch.randn((n_seq, n_outlier), generator=gs)
    scale = (outlier_scale * torch.exp(lognormal_sigma * z)).to(device)
    out = torch.empty((n_seq, n_tok, hidden), dtype=dtype, device=device)
    for s in range(n_seq):
        x = torch.randn((n_tok, hidden), generator=g, device=device, dtype=torch.float32)
        if n_outlier:
            x[:, ch] *= scale[s][None, :]
        out[s] = x.to(dtype)
    return out


def as_chunks(x, chunk_tokens=CHUNK_TOKENS):
    """View [n_seq, n_tok, hidden] as [n_chunks, chunk_tokens * hidden]: chunks are
    groups of consecutive token rows of one sequence, flat index = t * hidden + c."""
    n_seq, n_tok, hidden = x.shape
    assert n_tok % chunk_tokens == 0
    return x.reshape(n_seq * (n_tok // chunk_tokens), chunk_tokens * hidden)


def bits_numpy(x):
    """bf16 (fp32) tensor -> numpy uint16 (uint32) array of the bit patterns (host copy)."""
    if x.dtype == torch.float32:
        return x.contiguous().view(torch.int32).cpu().numpy().view(np.uint32)
    return x.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def from_bits(bits, device="cpu"):
    """numpy uint16 patterns -> bf16 tensor; uint32 patterns -> fp32 tensor."""
    bits = np.ascontiguousarray(bits)
    if bits.dtype == np.uint32:
        return torch.from_numpy(bits.view(np.int32).copy()).view(torch.float32).to(device)
    t = torch.from_numpy(bits.view(np.int16).copy())
    return t.view(torch.bfloat16).to(device)


def perturb_ulp(x, frac, seed):
    """Copy of x with a fraction `frac` of entries moved by one bf16 ulp: the
    magnitude pattern goes up or down by one (direction by seed), never below
    zero magnitude and never into Inf/NaN."""
    g = _gen(seed, x.device)
    bits = x.contiguous().view(torch.int16).to(torch.int32) & 0xFFFF
    pick = torch.rand(bits.shape, generator=g, device=x.device) < frac
    up = torch.rand(bits.shape, generator=g, device=x.device) < 0.5
    mag = bits & 0x7FFF
    sign = bits & 0x8000
    new_mag = torch.where(up, mag + 1, mag - 1)
    new_mag = torch.where(new_mag < 0, mag + 1, new_mag)
    new_mag = torch.where(new_mag >= 0x7F80, mag - 1, new_mag)
    out = torch.where(pick, sign | new_mag, bits)
    out = torch.where(out >= 0x8000, out - 0x10000, out).to(torch.int16)
    return out.view(torch.bfloat16)


def perturb_relative(x, max_rel, seed):
    """bf16(x * (1 + d)), d ~ U(-max_rel, max_rel) in fp32: emulates the small
    deviations of a reordered computation (Section 5.6, Table 2)."""
    g = _gen(seed, x.device)
    out = torch.empty_like(x)
    flat_in = x.reshape(-1)
    flat_out = out.reshape(-1)
    step = 1 << 26
    for s in range(0, flat_in.numel(), step):
        xs = flat_in[s:s + step].to(torch.float32)
        d = (torch.rand(xs.shape, generator=g, device=x.device) * 2.0 - 1.0) * max_rel
        flat_out[s:s + step] = (xs * (1.0 + d)).to(torch.bfloat16)
    return out


def roundtrip_e4m3(x):
    """bf16 -> fp8 e4m3 (saturating, round to nearest even) -> bf16: emulates
    the output of a reduced-precision computation (Section 6.1)."""
    out = torch.empty_like(x)
    flat_in = x.reshape(-1)
    flat_out = out.reshape(-1)
    step = 1 << 26
    for s in range(0, flat_in.numel(), step):
        xs = flat_in[s:s + step].to(torch.float32).clamp(-448.0, 448.0)
        flat_out[s:s + step] = xs.to(torch.float8_e4m3fn).to(torch.bfloat16)
    return out


# ---------------------------------------------------------------------------
# The workloads (shapes and distributions of the five configurations)
# ---------------------------------------------------------------------------

def config1(device="cpu"):
    """One chunk: 32 tokens x hidden 4096, 8 outlier channels scaled x20."""
    return activations(1, 32, 4096, BASE_SEED + 1, n_outlier=8, outlier_scale=20.0,
                       lognormal_sigma=0.0, device=device)


def config2(device="cpu", n_seq=64, n_tok=2048):
    """Llama-3.1-8B-shaped decode: 64 x 2048 x 4096, 8 outlier channels."""
    return activations(n_seq, n_tok, 4096, BASE_SEED + 2, n_outlier=8, device=device)


def config3(device="cpu", n_seq=128, n_tok=4096):
    """Llama-3.1-70B-shaped prefill+decode: 128 x 4096 x 8192, 16 outlier channels."""
    return activations(n_seq, n_tok, 8192, BASE_SEED + 3, n_outlier=16, device=device)


LAWS = ("outliers", "gaussian", "heavy_tail", "ascending", "all_equal", "few_values")


def law_activations(law, n_seq, n_tok, hidden, seed, n_outlier, device="cpu"):
    """The same shape under six value laws, to show how much the selection's cost depends on the input:
    outliers    the recipe of `activations` (what the workloads use)
    gaussian    N(0,1) everywhere, no outlier channels: the top-k are spread over all channels
    heavy_tail  N(0,1) * exp(N(0,1)) per element: large values everywhere, the threshold keeps rising
    ascending   inside every 32-token chunk the magnitudes never decrease with the flat index (random signs):
                every value read is larger than all before it, the worst case of a streaming selection
    all_equal   one magnitude per sequence (zero padding is the everyday case), random signs: ranking is by index alone
    few_values  seven patterns drawn uniformly (five magnitudes, zero among them): thousands share the k-th magnitude"""
    if law == "outliers":
        return activations(n_seq, n_tok, hidden, seed, n_outlier=n_outlier, device=device)
    if law == "gaussian":
        return activations(n_seq, n_tok, hidden, seed, n_outlier=0, device=device)
    device = torch.device(device)
    g = _gen(seed + 1, device)
    out = torch.empty((n_seq, n_tok, hidden), dtype=torch.bfloat16, device=device)
    if law == "heavy_tail":
        for s in range(n_seq):
            x = torch.randn((n_tok, hidden), generator=g, device=device, dtype=torch.float32)
            x *= torch.exp(torch.randn((n_tok, hidden), generator=g, device=device, dtype=torch.float32))
            out[s] = x.to(torch.bfloat16)
        return out
    if law == "ascending":
        assert n_tok % CHUNK_TOKENS == 0
        n = CHUNK_TOKENS * hidden
        ramp = (torch.arange(n, device=device, dtype=torch.int64) * 0x7F00 // (n + 64)).to(torch.int32)   # finite patterns
        for s in range(n_seq):
            sign = torch.randint(0, 2, (n_tok // CHUNK_TOKENS, n), generator=g, device=device, dtype=torch.int32) << 15
            bits = (ramp[None, :] | sign).to(torch.uint16).view(torch.bfloat16)
            out[s] = bits.reshape(n_tok, hidden)
        return out
    if law == "all_equal":
        for s in range(n_seq):
            sign = torch.randint(0, 2, (n_tok, hidden), generator=g, device=device, dtype=torch.int32) << 15
            out[s] = ((0x3F00 + s % 97) | sign).to(torch.uint16).view(torch.bfloat16)
        return out
    if law == "few_values":
        table = torch.tensor([0x3F80, 0xBF80, 0x4000, 0xC040, 0x0000, 0x8000, 0x3E00], device=device, dtype=torch.int32)
        for s in range(n_seq):
            pick = torch.randint(0, table.numel(), (n_tok, hidden), generator=g, device=device)
            out[s] = table[pick].to(torch.uint16).view(torch.bfloat16)
        return out
    raise ValueError("unknown law %r" % (law,))


def config4_variants(x, device=None):
    """Recomputed tensors for the verification stress test, from the original x:
    (a) relative perturbation <= 2^-7, (b) independent activations (different
    seed and different outlier channels), (c) fp8 e4m3 round trip."""
    device = x.device if device is None else device
    n_seq, n_tok, hidden = x.shape
    a = perturb_relative(x, 2.0 ** -7, BASE_SEED + 41)
    b = activations(n_seq, n_tok, hidden, BASE_SEED + 42, n_outlier=8, device=device)
    c = roundtrip_e4m3(x)
    return a, b, c


def config5_steps(n_seq, hidden, n_steps, seed=BASE_SEED + 5, device="cpu"):
    """Decode-step vectors [n_steps, n_seq, hidden] for the online path:
    the same law as `activations`, laid out step-major."""
    x = activations(n_seq, n_steps, hidden, seed, n_outlier=8, device=device)
    return x.transpose(0, 1).contiguous()
