"""Thin ctypes binding of include/toploc.h: argument marshalling only.

Every step of the path runs in the HIP kernels of libtoploc_hip.so.  PyTorch
is used for device memory and the current HIP stream, nothing else.  There is
no fallback: if the library has not been built, loading raises.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtoploc_hip.so")

PRIME = 65497
MAX_K = 512
OK, EINVAL, EWORKSPACE, EHIP, ESCRATCH = 0, -1, -2, -3, -4
STATIC_SCRATCH_BYTES = 8 << 20
CHUNK_OK, CHUNK_NO_MODULUS, CHUNK_MALFORMED, CHUNK_SHORT, CHUNK_BAD_SEGMENT = 0, 1, 3, 4, 5
(KERNEL_SELECT, KERNEL_PART, KERNEL_BUILD_MERGE, KERNEL_VERIFY_MERGE, KERNEL_BUILD, KERNEL_VERIFY, KERNEL_RING,
 KERNEL_READ, KERNEL_STREAM_APPEND, KERNEL_STREAM_EMIT, KERNEL_PLAN, KERNEL_COUNT) = range(12)
KERNEL_NAMES = ("select_kernel", "part_kernel", "build_merge_kernel", "verify_merge_kernel", "build_kernel",
                "verify_kernel", "ring_kernel", "read_kernel", "stream_append_kernel", "stream_emit_kernel",
                "plan_segments_kernel")
BF16_THRESHOLDS = (38, 10, 8)  # T_exp, T_mean, T_median (Section 5.2 of the paper)
F32_THRESHOLDS = (8, 256, 128)  # the same for fp32 inference
DTYPE_BF16, DTYPE_F32 = 0, 1
PRIME32 = 4294967291
MAX_K_F32 = 512

RESULT_DTYPE = np.dtype(
    [
        ("err_exp", "<u4"),
        ("n_match", "<u4"),
        ("mant_sum", "<u4"),
        ("mant_median", "<u4"),
        ("accept", "u1"),
        ("status", "u1"),
        ("pad", "u1", (2,)),
    ]
)

EXPORTS = (
    "toploc_proof_bytes",
    "toploc_workspace_bytes",
    "toploc_workspace_query",
    "toploc_set_split",
    "toploc_segments_workspace_bytes",
    "toploc_build_proofs_segments",
    "toploc_verify_proofs_segments",
    "toploc_build_proofs",
    "toploc_build_proofs_static",
    "toploc_verify_proofs",
    "toploc_topk",
    "toploc_proof_bytes_dtype",
    "toploc_workspace_bytes_f32",
    "toploc_build_proofs_f32",
    "toploc_verify_proofs_mixed",
    "toploc_segments_workspace_bytes_dtype",
    "toploc_build_proofs_segments_f32",
    "toploc_verify_proofs_segments_mixed",
    "toploc_stream_state_bytes",
    "toploc_stream_reset",
    "toploc_stream_append",
    "toploc_stream_emit",
    "toploc_stream_append_rows",
    "toploc_stream_emit_rows",
    "toploc_stream_state_bytes_dtype",
    "toploc_stream_reset_dtype",
    "toploc_stream_append_dtype",
    "toploc_stream_emit_dtype",
    "toploc_ring_append",
    "toploc_bench_read",
    "toploc_selection_stats",
    "toploc_build_id",
    "toploc_profile_enable",
    "toploc_profile_read",
    "toploc_strerror",
    "toploc_last_hip_error",
)


class Params(ctypes.Structure):
    _fields_ = [("k", ctypes.c_uint32), ("chunk_tokens", ctypes.c_uint32), ("hidden", ctypes.c_uint32),
                ("prime", ctypes.c_uint32)]


class Thresholds(ctypes.Structure):
    _fields_ = [("t_exp", ctypes.c_uint32), ("t_mean", ctypes.c_uint32), ("t_median", ctypes.c_uint32)]


class ToplocError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__("%s: %s (code %d, hip error %d)" % (
            what, lib().toploc_strerror(code).decode(), code, lib().toploc_last_hip_error()))


_lib = None


def lib():
    """Load libtoploc_hip.so (built by paper_2501_16007_amd.build). Raises if missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "libtoploc_hip.so is not built: run `python -m paper_2501_16007_amd.build` (hipcc, gfx950). "
                "There is no CPU fallback.")
        L = ctypes.CDLL(LIB_PATH)
        c = ctypes
        P = c.c_void_p
        L.toploc_proof_bytes.argtypes = [c.c_uint32]
        L.toploc_proof_bytes.restype = c.c_size_t
        L.toploc_workspace_bytes.argtypes = [c.POINTER(Params), c.c_uint64]
        L.toploc_workspace_bytes.restype = c.c_size_t
        L.toploc_workspace_query.argtypes = [c.POINTER(Params), c.c_uint64, c.POINTER(c.c_size_t)]
        L.toploc_build_proofs.argtypes = [P, c.c_uint64, c.POINTER(Params), P, P, P, P, c.c_size_t, P]
        L.toploc_verify_proofs.argtypes = [P, c.c_uint64, c.POINTER(Params), P, c.POINTER(Thresholds), P, P,
                                           c.c_size_t, P]
        L.toploc_build_proofs_static.argtypes = [P, c.c_uint64, c.POINTER(Params), P, P, P, P]
        L.toploc_topk.argtypes = [P, c.c_uint64, c.POINTER(Params), P, P, P]
        L.toploc_set_split.argtypes = [c.c_uint32]
        L.toploc_segments_workspace_bytes.argtypes = [c.c_uint64, c.c_uint64, c.c_uint32, c.c_uint32]
        L.toploc_segments_workspace_bytes.restype = c.c_size_t
        L.toploc_build_proofs_segments.argtypes = [P, c.c_uint64, P, c.c_uint64, c.c_uint32, c.c_uint32, P, P, P, P,
                                                   c.c_size_t, P]
        L.toploc_verify_proofs_segments.argtypes = [P, c.c_uint64, P, c.c_uint64, c.c_uint32, c.c_uint32, P,
                                                    c.POINTER(Thresholds), P, P, c.c_size_t, P]
        L.toploc_ring_append.argtypes = [P, P, c.c_uint32, c.c_uint32, c.c_uint32, c.c_uint32, P]
        L.toploc_proof_bytes_dtype.argtypes = [c.c_uint32, c.c_uint32]
        L.toploc_proof_bytes_dtype.restype = c.c_size_t
        L.toploc_workspace_bytes_f32.argtypes = [c.POINTER(Params), c.c_uint64]
        L.toploc_workspace_bytes_f32.restype = c.c_size_t
        L.toploc_build_proofs_f32.argtypes = [P, c.c_uint64, c.POINTER(Params), P, P, P, P, c.c_size_t, P]
        L.toploc_verify_proofs_mixed.argtypes = [P, c.c_uint32, c.c_uint64, c.POINTER(Params), P, c.c_uint32,
                                                 c.POINTER(Thresholds), P, P]
        L.toploc_segments_workspace_bytes_dtype.argtypes = [c.c_uint64, c.c_uint64, c.c_uint32, c.c_uint32, c.c_uint32]
        L.toploc_segments_workspace_bytes_dtype.restype = c.c_size_t
        L.toploc_build_proofs_segments_f32.argtypes = [P, c.c_uint64, P, c.c_uint64, c.c_uint32, c.c_uint32, P, P, P, P,
                                                       c.c_size_t, P]
        L.toploc_verify_proofs_segments_mixed.argtypes = [P, c.c_uint32, c.c_uint64, P, c.c_uint64, c.c_uint32, c.c_uint32, P,
                                                          c.c_uint32, c.POINTER(Thresholds), P, P, c.c_size_t, P]
        L.toploc_stream_state_bytes.argtypes = [c.c_uint32, c.c_uint32]
        L.toploc_stream_state_bytes.restype = c.c_size_t
        L.toploc_stream_reset.argtypes = [P, c.c_uint32, c.c_uint32, P]
        L.toploc_stream_append.argtypes = [P, P, c.c_uint32, c.c_uint32, c.c_uint32, c.c_uint32, c.c_uint32, P]
        L.toploc_stream_emit.argtypes = [P, c.c_uint32, c.c_uint32, P, P, P, P]
        L.toploc_stream_append_rows.argtypes = [P, c.c_uint32, P, P, P, c.c_uint32, c.c_uint32, c.c_uint32, c.c_uint32, P]
        L.toploc_stream_emit_rows.argtypes = [P, c.c_uint32, P, c.c_uint32, c.c_uint32, P, P, P, P]
        L.toploc_stream_state_bytes_dtype.argtypes = [c.c_uint32, c.c_uint32, c.c_uint32]
        L.toploc_stream_state_bytes_dtype.restype = c.c_size_t
        L.toploc_stream_reset_dtype.argtypes = [P, c.c_uint32, c.c_uint32, c.c_uint32, P]
        L.toploc_stream_append_dtype.argtypes = [P, c.c_uint32, P, c.c_uint32, P, P, c.c_uint32, c.c_uint32, c.c_uint32,
                                                 c.c_uint32, c.c_uint32, P]
        L.toploc_stream_emit_dtype.argtypes = [P, c.c_uint32, c.c_uint32, P, c.c_uint32, c.c_uint32, P, P, P, P]
        L.toploc_bench_read.argtypes = [P, c.c_uint64, c.c_uint64, P, P]
        L.toploc_selection_stats.argtypes = [P, c.c_uint64, c.POINTER(Params), P, P]
        L.toploc_build_id.restype = c.c_char_p
        L.toploc_profile_enable.argtypes = [c.c_int]
        L.toploc_profile_read.argtypes = [c.POINTER(c.c_uint32), c.POINTER(c.c_float)]
        L.toploc_strerror.argtypes = [c.c_int]
        L.toploc_strerror.restype = c.c_char_p
        L.toploc_last_hip_error.restype = c.c_int
        _lib = L
    return _lib


def _stream(t):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _chunks(hidden, chunk_tokens):
    """[n_seq, n_tok, H] or [n_chunks, chunk_tokens*H] bf16 device tensor -> (n_chunks, H or None)."""
    if hidden.dtype != torch.bfloat16 or not hidden.is_cuda or not hidden.is_contiguous():
        raise ValueError("hidden must be a contiguous bf16 tensor on the GPU")
    if hidden.dim() == 3:
        n_seq, n_tok, h = hidden.shape
        if n_tok % chunk_tokens:
            raise ValueError("n_tok must be a multiple of chunk_tokens")
        return n_seq * (n_tok // chunk_tokens), h
    if hidden.dim() == 2:
        n_chunks, n = hidden.shape
        if n % chunk_tokens:
            raise ValueError("chunk length must be a multiple of chunk_tokens")
        return n_chunks, n // chunk_tokens
    raise ValueError("hidden must be [n_seq, n_tok, H] or [n_chunks, chunk_tokens*H]")


def toploc_proof_bytes(k):
    return int(lib().toploc_proof_bytes(k))


def toploc_workspace_bytes(k, chunk_tokens, hidden, n_chunks):
    p = Params(k, chunk_tokens, hidden, PRIME)
    return int(lib().toploc_workspace_bytes(ctypes.byref(p), n_chunks))


def toploc_workspace_query(k, chunk_tokens, hidden, n_chunks):
    """(return code, bytes): tells unusable parameters (EINVAL) from 'no scratch needed' (OK, 0)."""
    p = Params(k, chunk_tokens, hidden, PRIME)
    nbytes = ctypes.c_size_t(0)
    rc = lib().toploc_workspace_query(ctypes.byref(p), n_chunks, ctypes.byref(nbytes))
    return rc, int(nbytes.value)


def new_workspace(k, chunk_tokens, hidden, n_chunks, device):
    nbytes = max(16, toploc_workspace_bytes(k, chunk_tokens, hidden, n_chunks))
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def toploc_build_proofs(hidden, k=128, chunk_tokens=32, want_topk=False, workspace=None, out=None):
    """Algorithm 1 over every chunk. Returns (proofs uint8 [n_chunks, 2+2k], status uint8 [n_chunks][, idx])."""
    n_chunks, h = _chunks(hidden, chunk_tokens)
    dev = hidden.device
    p = Params(k, chunk_tokens, h, PRIME)
    pb = 2 + 2 * k
    if out is None:
        proofs = torch.empty((n_chunks, pb), dtype=torch.uint8, device=dev)
        status = torch.empty(n_chunks, dtype=torch.uint8, device=dev)
    else:
        proofs, status = out
    idx = torch.empty((n_chunks, k), dtype=torch.int32, device=dev) if want_topk else None
    if workspace is None:
        workspace = new_workspace(k, chunk_tokens, h, n_chunks, dev)
    rc = lib().toploc_build_proofs(
        hidden.data_ptr(), n_chunks, ctypes.byref(p), proofs.data_ptr(), status.data_ptr(),
        idx.data_ptr() if want_topk else None, workspace.data_ptr(), workspace.numel(), _stream(hidden))
    if rc != OK:
        raise ToplocError(rc, "toploc_build_proofs")
    return (proofs, status, idx) if want_topk else (proofs, status)


def toploc_build_proofs_static(hidden, out, k=128, chunk_tokens=32, topk_out=None):
    """toploc_build_proofs with the library's own fixed scratch: allocates nothing, so the caller passes
    every output. out = (proofs uint8 [n_chunks, 2+2k], status uint8 [n_chunks]); topk_out int32 [n_chunks, k]."""
    n_chunks, h = _chunks(hidden, chunk_tokens)
    p = Params(k, chunk_tokens, h, PRIME)
    proofs, status = out
    rc = lib().toploc_build_proofs_static(
        hidden.data_ptr(), n_chunks, ctypes.byref(p), proofs.data_ptr(), status.data_ptr(),
        topk_out.data_ptr() if topk_out is not None else None, _stream(hidden))
    if rc != OK:
        raise ToplocError(rc, "toploc_build_proofs_static")


def toploc_verify_proofs(hidden, proofs, k=128, chunk_tokens=32, thresholds=BF16_THRESHOLDS, out=None, workspace=None):
    """Algorithm 2 over every chunk. Returns a uint8 device tensor [n_chunks, 20]; see results_numpy."""
    n_chunks, h = _chunks(hidden, chunk_tokens)
    if proofs.dtype != torch.uint8 or not proofs.is_cuda or not proofs.is_contiguous() or \
            proofs.numel() != n_chunks * (2 + 2 * k):
        raise ValueError("proofs must be a contiguous uint8 device tensor of n_chunks * (2+2k) bytes")
    p = Params(k, chunk_tokens, h, PRIME)
    t = Thresholds(*thresholds)
    res = out if out is not None else torch.empty((n_chunks, RESULT_DTYPE.itemsize), dtype=torch.uint8,
                                                  device=hidden.device)
    if workspace is None:
        workspace = new_workspace(k, chunk_tokens, h, n_chunks, hidden.device)
    rc = lib().toploc_verify_proofs(hidden.data_ptr(), n_chunks, ctypes.byref(p), proofs.data_ptr(), ctypes.byref(t),
                                    res.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(hidden))
    if rc != OK:
        raise ToplocError(rc, "toploc_verify_proofs")
    return res


def results_numpy(res):
    """Device result records -> numpy structured array (host copy, synchronises)."""
    return res.cpu().numpy().reshape(-1).view(RESULT_DTYPE)


def toploc_topk(hidden, k=128, chunk_tokens=32):
    """topk(h, k) per chunk: (idx int32 [n_chunks, k], val int16 [n_chunks, k] bf16 patterns)."""
    n_chunks, h = _chunks(hidden, chunk_tokens)
    p = Params(k, chunk_tokens, h, PRIME)
    idx = torch.empty((n_chunks, k), dtype=torch.int32, device=hidden.device)
    val = torch.empty((n_chunks, k), dtype=torch.int16, device=hidden.device)
    rc = lib().toploc_topk(hidden.data_ptr(), n_chunks, ctypes.byref(p), idx.data_ptr(), val.data_ptr(),
                           _stream(hidden))
    if rc != OK:
        raise ToplocError(rc, "toploc_topk")
    return idx, val


def toploc_set_split(parts_per_chunk):
    """0: the library chooses into how many parts a chunk is cut; n: force n parts (tuning / tests)."""
    rc = lib().toploc_set_split(parts_per_chunk)
    if rc != OK:
        raise ToplocError(rc, "toploc_set_split")


def _segments_any(hidden, row_offsets):
    """[total_rows, H] bf16 or fp32 device tensor and n_segments + 1 row offsets -> (offsets as an int64 device
    tensor, n_segments, H, dtype code).  Offsets given on the host (list, numpy) are checked and uploaded here;
    an int64 device tensor is handed to the library as it is (the library never reads offsets on the host)."""
    if hidden.dtype not in (torch.bfloat16, torch.float32) or not hidden.is_cuda or not hidden.is_contiguous() or \
            hidden.dim() != 2:
        raise ValueError("hidden must be a contiguous [total_rows, H] bf16 or fp32 tensor on the GPU")
    if isinstance(row_offsets, torch.Tensor):
        off = row_offsets
        if off.dtype != torch.int64 or off.dim() != 1 or off.numel() < 1 or not off.is_contiguous() or \
                off.device != hidden.device:
            raise ValueError("row_offsets must be a contiguous 1-D int64 tensor on the device of hidden")
    else:
        host = np.ascontiguousarray(row_offsets, dtype=np.uint64)
        if host.ndim != 1 or host.size < 1 or int(host[-1]) > hidden.shape[0]:
            raise ValueError("row_offsets must be a 1-D array of n_segments + 1 row numbers inside the tensor")
        off = torch.from_numpy(host.view(np.int64)).to(hidden.device)
    return off, off.numel() - 1, hidden.shape[1], (DTYPE_F32 if hidden.dtype == torch.float32 else DTYPE_BF16)


def toploc_segments_workspace_bytes(n_segments, total_rows, hidden_size, k):
    return int(lib().toploc_segments_workspace_bytes(n_segments, total_rows, hidden_size, k))


def toploc_segments_workspace_bytes_dtype(n_segments, total_rows, hidden_size, k, hidden_dtype):
    return int(lib().toploc_segments_workspace_bytes_dtype(n_segments, total_rows, hidden_size, k, hidden_dtype))


def new_segments_workspace(hidden, n_segments, k):
    dt = DTYPE_F32 if hidden.dtype == torch.float32 else DTYPE_BF16
    nbytes = toploc_segments_workspace_bytes_dtype(n_segments, hidden.shape[0], hidden.shape[1], k, dt)
    return torch.empty(max(16, nbytes), dtype=torch.uint8, device=hidden.device)


def _build_segments(hidden, row_offsets, k, want_topk, want_dtype, workspace, out):
    off, n_seg, h, dt = _segments_any(hidden, row_offsets)
    if dt != want_dtype:
        raise ValueError("hidden must be %s" % ("fp32" if want_dtype == DTYPE_F32 else "bf16"))
    dev = hidden.device
    if out is None:
        proofs = torch.empty((n_seg, 2 + (4 if dt == DTYPE_F32 else 2) * k), dtype=torch.uint8, device=dev)
        status = torch.empty(n_seg, dtype=torch.uint8, device=dev)
        idx = torch.empty((n_seg, k), dtype=torch.int32, device=dev) if want_topk else None
    else:
        proofs, status, idx = out
    ws = workspace if workspace is not None else new_segments_workspace(hidden, n_seg, k)
    fn = lib().toploc_build_proofs_segments_f32 if dt == DTYPE_F32 else lib().toploc_build_proofs_segments
    rc = fn(hidden.data_ptr(), hidden.shape[0], off.data_ptr(), n_seg, h, k, proofs.data_ptr(), status.data_ptr(),
            idx.data_ptr() if idx is not None else None, ws.data_ptr(), ws.numel(), _stream(hidden))
    if rc != OK:
        raise ToplocError(rc, "toploc_build_proofs_segments" + ("_f32" if dt == DTYPE_F32 else ""))
    return (proofs, status, idx) if want_topk else (proofs, status)


def toploc_build_proofs_segments(hidden, row_offsets, k=128, want_topk=False, workspace=None, out=None):
    """Algorithm 1 over segments of rows [row_offsets[i], row_offsets[i+1]) of hidden [total_rows, H] bf16.
    row_offsets: host values or an int64 device tensor; out = (proofs, status, idx or None) to reuse buffers."""
    return _build_segments(hidden, row_offsets, k, want_topk, DTYPE_BF16, workspace, out)


def toploc_verify_proofs_segments(hidden, row_offsets, proofs, k=128, thresholds=BF16_THRESHOLDS, workspace=None, out=None):
    """Algorithm 2 over segments. Returns a uint8 device tensor [n_segments, 20]; see results_numpy."""
    if hidden.dtype != torch.bfloat16:
        raise ValueError("hidden must be bf16")
    return toploc_verify_proofs_segments_mixed(hidden, row_offsets, proofs, DTYPE_BF16, k=k, thresholds=thresholds,
                                               workspace=workspace, out=out)


def generation_row_offsets(n_prompt, n_total, chunk_tokens=32):
    """Row ranges of one sequence as the paper cuts it (Section 5.6): the prompt's activations as one
    segment, then one segment per `chunk_tokens` generated tokens, the last one ragged."""
    if not 0 <= n_prompt <= n_total:
        raise ValueError("need 0 <= n_prompt <= n_total")
    cuts = [0] if n_prompt == 0 else [0, n_prompt]
    t = n_prompt
    while t < n_total:
        t = min(t + chunk_tokens, n_total)
        cuts.append(t)
    return np.asarray(cuts, dtype=np.uint64)


def toploc_build_proofs_generation(hidden, n_prompt, k=128, chunk_tokens=32):
    """Proofs of one sequence's [n_total, H] activations: prefill segment, then 32-token decode segments.
    Returns (proofs, status, row_offsets); pass row_offsets to toploc_verify_proofs_segments."""
    off = generation_row_offsets(n_prompt, hidden.shape[0], chunk_tokens)
    proofs, status = toploc_build_proofs_segments(hidden, off, k=k)
    return proofs, status, off


def toploc_ring_append(ring, step_vec, step):
    """ring [n_seq, chunk_tokens, H] <- step_vec [n_seq, H] at row step mod chunk_tokens."""
    n_seq, chunk_tokens, h = ring.shape
    if step_vec.shape != (n_seq, h) or ring.dtype != torch.bfloat16 or step_vec.dtype != torch.bfloat16 or \
            not ring.is_contiguous() or not step_vec.is_contiguous() or not ring.is_cuda or not step_vec.is_cuda:
        raise ValueError("ring [n_seq, T, H] and step_vec [n_seq, H] must be contiguous bf16 device tensors")
    rc = lib().toploc_ring_append(ring.data_ptr(), step_vec.data_ptr(), n_seq, h, chunk_tokens, step, _stream(ring))
    if rc != OK:
        raise ToplocError(rc, "toploc_ring_append")


def toploc_proof_bytes_dtype(k, dtype):
    return int(lib().toploc_proof_bytes_dtype(k, dtype))


def _chunks_any(hidden, chunk_tokens):
    """Like _chunks for a bf16 or fp32 tensor: (n_chunks, H, dtype code)."""
    if hidden.dtype not in (torch.bfloat16, torch.float32) or not hidden.is_cuda or not hidden.is_contiguous():
        raise ValueError("hidden must be a contiguous bf16 or fp32 tensor on the GPU")
    dt = DTYPE_F32 if hidden.dtype == torch.float32 else DTYPE_BF16
    if hidden.dim() == 3:
        n_seq, n_tok, h = hidden.shape
        if n_tok % chunk_tokens:
            raise ValueError("n_tok must be a multiple of chunk_tokens")
        return n_seq * (n_tok // chunk_tokens), h, dt
    if hidden.dim() == 2:
        n_chunks, n = hidden.shape
        if n % chunk_tokens:
            raise ValueError("chunk length must be a multiple of chunk_tokens")
        return n_chunks, n // chunk_tokens, dt
    raise ValueError("hidden must be [n_seq, n_tok, H] or [n_chunks, chunk_tokens*H]")


def toploc_workspace_bytes_f32(k, chunk_tokens, hidden, n_chunks):
    p = Params(k, chunk_tokens, hidden, PRIME32)
    return int(lib().toploc_workspace_bytes_f32(ctypes.byref(p), n_chunks))


def toploc_build_proofs_f32(hidden, k=128, chunk_tokens=32, want_topk=False, workspace=None):
    """Algorithm 1 over fp32 activations. Returns (proofs uint8 [n_chunks, 2+4k], status[, idx])."""
    n_chunks, h, dt = _chunks_any(hidden, chunk_tokens)
    if dt != DTYPE_F32:
        raise ValueError("hidden must be fp32")
    dev = hidden.device
    p = Params(k, chunk_tokens, h, PRIME32)
    proofs = torch.empty((n_chunks, 2 + 4 * k), dtype=torch.uint8, device=dev)
    status = torch.empty(n_chunks, dtype=torch.uint8, device=dev)
    idx = torch.empty((n_chunks, k), dtype=torch.int32, device=dev) if want_topk else None
    if workspace is None:
        workspace = torch.empty(max(16, toploc_workspace_bytes_f32(k, chunk_tokens, h, n_chunks)), dtype=torch.uint8, device=dev)
    rc = lib().toploc_build_proofs_f32(hidden.data_ptr(), n_chunks, ctypes.byref(p), proofs.data_ptr(), status.data_ptr(),
                                       idx.data_ptr() if want_topk else None, workspace.data_ptr(), workspace.numel(),
                                       _stream(hidden))
    if rc != OK:
        raise ToplocError(rc, "toploc_build_proofs_f32")
    return (proofs, status, idx) if want_topk else (proofs, status)


def toploc_verify_proofs_mixed(hidden, proofs, proof_dtype, k=128, chunk_tokens=32, thresholds=None):
    """Algorithm 2 with bf16 or fp32 activations and bf16 or fp32 proofs; thresholds default to the
    paper's for the validator's precision. Returns a uint8 device tensor [n_chunks, 20]."""
    n_chunks, h, dt = _chunks_any(hidden, chunk_tokens)
    pb = 2 + (4 if proof_dtype == DTYPE_F32 else 2) * k
    if proofs.dtype != torch.uint8 or not proofs.is_cuda or not proofs.is_contiguous() or proofs.numel() != n_chunks * pb:
        raise ValueError("proofs must be a contiguous uint8 device tensor of n_chunks proofs of proof_dtype")
    if thresholds is None:
        thresholds = F32_THRESHOLDS if dt == DTYPE_F32 else BF16_THRESHOLDS
    p = Params(k, chunk_tokens, h, PRIME32 if proof_dtype == DTYPE_F32 else PRIME)
    t = Thresholds(*thresholds)
    res = torch.empty((n_chunks, RESULT_DTYPE.itemsize), dtype=torch.uint8, device=hidden.device)
    rc = lib().toploc_verify_proofs_mixed(hidden.data_ptr(), dt, n_chunks, ctypes.byref(p), proofs.data_ptr(), proof_dtype,
                                          ctypes.byref(t), res.data_ptr(), _stream(hidden))
    if rc != OK:
        raise ToplocError(rc, "toploc_verify_proofs_mixed")
    return res


def toploc_build_proofs_segments_f32(hidden, row_offsets, k=128, want_topk=False, workspace=None, out=None):
    """Algorithm 1 over segments of fp32 rows. Returns (proofs uint8 [n_segments, 2+4k], status[, idx])."""
    return _build_segments(hidden, row_offsets, k, want_topk, DTYPE_F32, workspace, out)


def toploc_verify_proofs_segments_mixed(hidden, row_offsets, proofs, proof_dtype, k=128, thresholds=None, workspace=None,
                                        out=None):
    """Algorithm 2 over segments with bf16 or fp32 activations and bf16 or fp32 proofs; thresholds default to
    the paper's for the validator's precision. Returns a uint8 device tensor [n_segments, 20]."""
    off, n_seg, h, dt = _segments_any(hidden, row_offsets)
    pb = 2 + (4 if proof_dtype == DTYPE_F32 else 2) * k
    if proofs.dtype != torch.uint8 or not proofs.is_cuda or not proofs.is_contiguous() or proofs.numel() != n_seg * pb:
        raise ValueError("proofs must be a contiguous uint8 device tensor of n_segments proofs of proof_dtype")
    if thresholds is None:
        thresholds = F32_THRESHOLDS if dt == DTYPE_F32 else BF16_THRESHOLDS
    t = Thresholds(*thresholds)
    res = out if out is not None else torch.empty((n_seg, RESULT_DTYPE.itemsize), dtype=torch.uint8, device=hidden.device)
    ws = workspace if workspace is not None else new_segments_workspace(hidden, n_seg, k)
    rc = lib().toploc_verify_proofs_segments_mixed(
        hidden.data_ptr(), dt, hidden.shape[0], off.data_ptr(), n_seg, h, k, proofs.data_ptr(), proof_dtype,
        ctypes.byref(t), res.data_ptr(), ws.data_ptr(), ws.numel(), _stream(hidden))
    if rc != OK:
        raise ToplocError(rc, "toploc_verify_proofs_segments_mixed")
    return res


def toploc_stream_state_bytes(n_seq, k, dtype=DTYPE_BF16):
    return int(lib().toploc_stream_state_bytes_dtype(n_seq, k, dtype))


def toploc_stream_new_state(n_seq, k, device, dtype=DTYPE_BF16):
    """Device memory for the running top-k of n_seq sequences (bf16 or fp32 rows), emptied."""
    nbytes = toploc_stream_state_bytes(n_seq, k, dtype)
    if nbytes == 0 and n_seq:
        raise ToplocError(EINVAL, "toploc_stream_state_bytes")
    state = torch.empty(max(16, nbytes), dtype=torch.uint8, device=device)
    toploc_stream_reset(state, n_seq, k, dtype)
    return state


def toploc_stream_reset(state, n_seq, k, dtype=DTYPE_BF16):
    rc = lib().toploc_stream_reset_dtype(state.data_ptr(), n_seq, k, dtype, _stream(state))
    if rc != OK:
        raise ToplocError(rc, "toploc_stream_reset")


def _step_dtype(step_vec):
    if step_vec.dtype not in (torch.bfloat16, torch.float32) or not step_vec.is_cuda or not step_vec.is_contiguous() or \
            step_vec.dim() != 2:
        raise ValueError("step_vec must be a contiguous [rows, H] bf16 or fp32 tensor on the GPU")
    return DTYPE_F32 if step_vec.dtype == torch.float32 else DTYPE_BF16


def toploc_stream_append(state, step_vec, token, k=128, chunk_tokens=32):
    """Row `token` of the current chunk for every sequence: step_vec [n_seq, H] bf16 or fp32 (the state's precision)."""
    dt = _step_dtype(step_vec)
    n_seq, h = step_vec.shape
    if state.numel() < toploc_stream_state_bytes(n_seq, k, dt):
        raise ValueError("state too small for n_seq sequences")
    rc = lib().toploc_stream_append_dtype(state.data_ptr(), n_seq, step_vec.data_ptr(), dt, None, None, n_seq, h, chunk_tokens,
                                          token, k, _stream(step_vec))
    if rc != OK:
        raise ToplocError(rc, "toploc_stream_append")


def toploc_stream_emit(state, n_seq, k=128, want_topk=False, out=None, dtype=DTYPE_BF16):
    """Proofs of the chunks appended since the last emission; empties the states."""
    dev = state.device
    if out is None:
        proofs = torch.empty((n_seq, 2 + (4 if dtype == DTYPE_F32 else 2) * k), dtype=torch.uint8, device=dev)
        status = torch.empty(n_seq, dtype=torch.uint8, device=dev)
    else:
        proofs, status = out
    idx = torch.empty((n_seq, k), dtype=torch.int32, device=dev) if want_topk else None
    rc = lib().toploc_stream_emit_dtype(state.data_ptr(), n_seq, dtype, None, n_seq, k, proofs.data_ptr(), status.data_ptr(),
                                        idx.data_ptr() if want_topk else None, _stream(state))
    if rc != OK:
        raise ToplocError(rc, "toploc_stream_emit")
    return (proofs, status, idx) if want_topk else (proofs, status)


def _u32_device(values, device, what):
    """A list, numpy array or tensor of non-negative integers as a contiguous int32 device tensor (uint32 bits)."""
    if isinstance(values, torch.Tensor):
        t = values.to(device=device, dtype=torch.int32)
    else:
        t = torch.from_numpy(np.ascontiguousarray(values, dtype=np.uint32).view(np.int32)).to(device)
    if t.dim() != 1:
        raise ValueError(what + " must be one-dimensional")
    return t.contiguous()


def toploc_stream_append_rows(state, n_slots, step_vec, slots, tokens, k=128, chunk_tokens=32):
    """Continuous batching: row r of step_vec [n_rows, H] (bf16 or fp32) is token tokens[r] of sequence slots[r]."""
    dt = _step_dtype(step_vec)
    n_rows, h = step_vec.shape
    slots = _u32_device(slots, step_vec.device, "slots")
    tokens = _u32_device(tokens, step_vec.device, "tokens")
    if slots.numel() != n_rows or tokens.numel() != n_rows:
        raise ValueError("one slot and one token per row")
    if state.numel() < toploc_stream_state_bytes(n_slots, k, dt):
        raise ValueError("state too small for n_slots sequences")
    rc = lib().toploc_stream_append_dtype(state.data_ptr(), n_slots, step_vec.data_ptr(), dt, slots.data_ptr(),
                                          tokens.data_ptr(), n_rows, h, chunk_tokens, 0, k, _stream(step_vec))
    if rc != OK:
        raise ToplocError(rc, "toploc_stream_append_rows")


def toploc_stream_emit_rows(state, n_slots, slots, k=128, want_topk=False, dtype=DTYPE_BF16):
    """Proofs of the sequences `slots` (output row r belongs to slots[r]); empties their states."""
    dev = state.device
    slots = _u32_device(slots, dev, "slots")
    n_rows = slots.numel()
    proofs = torch.empty((n_rows, 2 + (4 if dtype == DTYPE_F32 else 2) * k), dtype=torch.uint8, device=dev)
    status = torch.empty(n_rows, dtype=torch.uint8, device=dev)
    idx = torch.empty((n_rows, k), dtype=torch.int32, device=dev) if want_topk else None
    if state.numel() < toploc_stream_state_bytes(n_slots, k, dtype):
        raise ValueError("state too small for n_slots sequences")
    if n_rows == 0:
        return (proofs, status, idx) if want_topk else (proofs, status)
    rc = lib().toploc_stream_emit_dtype(state.data_ptr(), n_slots, dtype, slots.data_ptr(), n_rows, k, proofs.data_ptr(),
                                        status.data_ptr(), idx.data_ptr() if want_topk else None, _stream(state))
    if rc != OK:
        raise ToplocError(rc, "toploc_stream_emit_rows")
    return (proofs, status, idx) if want_topk else (proofs, status)


def toploc_bench_read(hidden, out=None):
    """Pure read of [n_chunks, N] with the selection kernel's access pattern (measurement aid)."""
    n_chunks, n = hidden.shape
    if out is None:
        out = torch.zeros(max(1, n_chunks), dtype=torch.int32, device=hidden.device)
    rc = lib().toploc_bench_read(hidden.data_ptr(), n_chunks, n, out.data_ptr(), _stream(hidden))
    if rc != OK:
        raise ToplocError(rc, "toploc_bench_read")
    return out


def toploc_selection_stats(hidden, k=128, chunk_tokens=32):
    """Per chunk: drains, prunes, queued vectors, appended candidates of the selection (int32 [n_chunks, 4])."""
    n_chunks, h = _chunks(hidden, chunk_tokens)
    p = Params(k, chunk_tokens, h, PRIME)
    stats = torch.zeros((n_chunks, 4), dtype=torch.int32, device=hidden.device)
    rc = lib().toploc_selection_stats(hidden.data_ptr(), n_chunks, ctypes.byref(p), stats.data_ptr(), _stream(hidden))
    if rc != OK:
        raise ToplocError(rc, "toploc_selection_stats")
    return stats


def toploc_build_id():
    """Hash of the sources and flags the loaded library was built from."""
    return lib().toploc_build_id().decode()


def toploc_profile_enable(on):
    lib().toploc_profile_enable(1 if on else 0)


def toploc_profile_read():
    """{kernel name: (launches, total ms)} since the last read; synchronises the recorded events."""
    n = (ctypes.c_uint32 * KERNEL_COUNT)()
    ms = (ctypes.c_float * KERNEL_COUNT)()
    rc = lib().toploc_profile_read(n, ms)
    if rc != OK:
        raise ToplocError(rc, "toploc_profile_read")
    return {KERNEL_NAMES[i]: (int(n[i]), float(ms[i])) for i in range(KERNEL_COUNT)}
