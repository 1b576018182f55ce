"""CPU-side checks of the C-ABI library: it loads, exports every symbol the
header declares, and its host-only entry points and argument validation work
without a GPU (no kernel is launched here)."""
import ctypes
import os
import re

import pytest

from conftest import ROOT

binding = pytest.importorskip("paper_2501_16007_amd.binding")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "toploc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(toploc_[a-z_0-9]+)\s*\(", text)))


def test_library_is_built_and_exports_every_declared_symbol():
    assert os.path.exists(binding.LIB_PATH), "run python -m paper_2501_16007_amd.build"
    L = binding.lib()
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_proof_size_matches_paper(golden):
    g = {r[0]: int(r[1]) for r in golden("sizes_and_thresholds.txt")}
    assert binding.toploc_proof_bytes(128) == g["proof_bytes_k128"]
    assert binding.toploc_proof_bytes(32) == 66 and binding.toploc_proof_bytes(512) == 1026
    assert binding.BF16_THRESHOLDS == (g["t_exp_bf16"], g["t_mean_bf16"], g["t_median_bf16"])


def test_workspace_bytes_and_parameter_validation():
    assert binding.toploc_workspace_bytes(128, 32, 8192, 16384) == 0   # large batch: one fused kernel, no scratch
    assert binding.toploc_workspace_bytes(128, 32, 4096, 10) >= 10 * 2 * 128 * 6   # small batch: chunks are cut
    assert binding.toploc_workspace_bytes(512, 32, 8192, 16384) >= 16384 * 512 * 6  # k > 128 always hands pairs on
    assert binding.toploc_workspace_bytes(0, 32, 4096, 10) == 0        # k = 0
    assert binding.toploc_workspace_bytes(513, 32, 4096, 10) == 0      # k > TOPLOC_MAX_K
    assert binding.toploc_workspace_bytes(128, 32, 3, 10) == 0         # N = 96 < k
    assert binding.toploc_workspace_bytes(8, 3, 5, 10) == 0            # N not a multiple of 8
    L = binding.lib()
    bad = binding.Params(128, 32, 4096, 65521)                         # wrong prime
    assert L.toploc_workspace_bytes(ctypes.byref(bad), 1) == 0
    # the query tells the two meanings of 0 apart
    assert binding.toploc_workspace_query(128, 32, 8192, 16384) == (binding.OK, 0)
    assert binding.toploc_workspace_query(0, 32, 4096, 10) == (binding.EINVAL, 0)
    assert binding.toploc_workspace_query(128, 32, 4096, 10) == (binding.OK, binding.toploc_workspace_bytes(128, 32, 4096, 10))
    assert binding.toploc_workspace_query(128, 32, 4096, 0) == (binding.OK, 0)
    assert L.toploc_workspace_query(ctypes.byref(bad), 1, None) == binding.EINVAL


def test_calls_are_rejected_before_any_launch():
    L = binding.lib()
    ok = binding.Params(128, 32, 4096, binding.PRIME)
    bad = binding.Params(0, 32, 4096, binding.PRIME)
    thr = binding.Thresholds(38, 10, 8)
    fake = ctypes.c_void_p(0x1000)  # never dereferenced: every call below is refused or empty
    assert L.toploc_build_proofs(fake, 1, ctypes.byref(bad), fake, fake, None, fake, 1 << 20, None) == binding.EINVAL
    assert L.toploc_build_proofs(None, 1, ctypes.byref(ok), fake, fake, None, fake, 1 << 20, None) == binding.EINVAL
    assert L.toploc_build_proofs(ctypes.c_void_p(0x1008), 1, ctypes.byref(ok), fake, fake, None, fake, 1 << 20,
                                 None) == binding.EINVAL               # misaligned input
    big = binding.Params(512, 32, 4096, binding.PRIME)
    assert L.toploc_build_proofs(fake, 1, ctypes.byref(big), fake, fake, None, fake, 16, None) == binding.EWORKSPACE
    assert L.toploc_build_proofs(fake, 1, ctypes.byref(big), fake, fake, None, None, 1 << 20, None) == binding.EINVAL
    # segment calls: the row offsets are device memory the host never reads, the plan comes from sizes alone
    assert L.toploc_segments_workspace_bytes(2, 9, 4096, 128) > 0
    assert L.toploc_segments_workspace_bytes(2, 9, 4100, 128) == 0           # hidden % 8 != 0
    assert L.toploc_segments_workspace_bytes(2, 9, 4096, 513) == 0           # k > TOPLOC_MAX_K
    assert L.toploc_segments_workspace_bytes(0, 9, 4096, 128) == 0           # nothing to do
    assert L.toploc_segments_workspace_bytes(1 << 31, 9, 4096, 128) == 0     # too many segments
    assert L.toploc_segments_workspace_bytes(2, 1 << 60, 4096, 128) == 0     # value count leaves 64 bits
    assert L.toploc_build_proofs_segments(fake, 9, fake, 2, 4096, 128, fake, fake, None, fake, 16, None) == binding.EWORKSPACE
    assert L.toploc_build_proofs_segments(fake, 9, None, 2, 4096, 128, fake, fake, None, fake, 1 << 30, None) == binding.EINVAL
    assert L.toploc_build_proofs_segments(fake, 9, ctypes.c_void_p(0x1004), 2, 4096, 128, fake, fake, None, fake, 1 << 30,
                                          None) == binding.EINVAL            # misaligned offsets
    assert L.toploc_build_proofs_segments(fake, 9, fake, 2, 4096, 0, fake, fake, None, fake, 1 << 30, None) == binding.EINVAL
    assert L.toploc_verify_proofs_segments(fake, 9, fake, 0, 4096, 128, fake, ctypes.byref(thr), fake, fake, 0, None) == binding.OK
    assert L.toploc_verify_proofs_segments(fake, 9, fake, 2, 4096, 128, fake, None, fake, fake, 1 << 30, None) == binding.EINVAL
    assert L.toploc_set_split(5000) == binding.EINVAL and L.toploc_set_split(0) == binding.OK
    assert L.toploc_build_proofs(fake, 0, ctypes.byref(ok), fake, fake, None, fake, 0, None) == binding.OK
    assert L.toploc_verify_proofs(fake, 1, ctypes.byref(ok), fake, None, fake, None, 0, None) == binding.EINVAL
    assert L.toploc_verify_proofs(fake, 0, ctypes.byref(ok), fake, ctypes.byref(thr), fake, None, 0, None) == binding.OK
    assert L.toploc_topk(fake, 1, ctypes.byref(bad), fake, fake, None) == binding.EINVAL
    assert L.toploc_ring_append(fake, fake, 4, 12, 32, 0, None) == binding.EINVAL   # hidden % 8 != 0
    assert L.toploc_ring_append(fake, fake, 0, 16, 32, 0, None) == binding.OK
    for code in (0, -1, -2, -3, -99):
        assert L.toploc_strerror(code)


def test_stream_state_size_and_argument_checks():
    L = binding.lib()
    fake = ctypes.c_void_p(1 << 40)  # never dereferenced: every call below is refused or empty
    assert binding.toploc_stream_state_bytes(1, 128) == 16 + 512 + 256       # header, k indices, k patterns
    assert binding.toploc_stream_state_bytes(1024, 32) == 1024 * (16 + 128 + 64)
    assert binding.toploc_stream_state_bytes(3, 5) == 3 * (16 + 32 + 16)     # parts rounded up to 16 bytes
    assert binding.toploc_stream_state_bytes(4, 0) == 0 and binding.toploc_stream_state_bytes(4, 513) == 0
    assert L.toploc_stream_append(fake, fake, 4, 4096, 32, 32, 128, None) == binding.EINVAL   # token >= chunk_tokens
    assert L.toploc_stream_append(fake, fake, 4, 4100, 32, 0, 128, None) == binding.EINVAL    # hidden % 8 != 0
    assert L.toploc_stream_append(fake, fake, 4, 1 << 20, 1 << 12, 0, 128, None) == binding.EINVAL  # chunk >= 2^32 values
    assert L.toploc_stream_append(None, fake, 4, 4096, 32, 0, 128, None) == binding.EINVAL
    assert L.toploc_stream_append(fake, fake, 0, 4096, 32, 0, 128, None) == binding.OK
    assert L.toploc_stream_emit(fake, 0, 128, fake, fake, None, None) == binding.OK
    assert L.toploc_stream_emit(fake, 1, 0, fake, fake, None, None) == binding.EINVAL
    assert L.toploc_stream_reset(fake, 0, 128, None) == binding.OK
    assert L.toploc_stream_reset(None, 3, 128, None) == binding.EINVAL


def test_newer_entry_points_check_their_arguments_before_any_launch():
    L = binding.lib()
    fake = ctypes.c_void_p(1 << 40)  # never dereferenced: every call below is refused or empty
    thr = binding.Thresholds(8, 256, 128)
    # the selection alone reaches k = 4096, the proof calls stop at 512
    wide = binding.Params(4096, 32, 4096, binding.PRIME)
    too_wide = binding.Params(4097, 32, 4096, binding.PRIME)
    assert L.toploc_topk(None, 1, ctypes.byref(wide), fake, fake, None) == binding.EINVAL        # only the null pointer is wrong
    assert L.toploc_topk(fake, 0, ctypes.byref(wide), fake, fake, None) == binding.OK
    assert L.toploc_topk(fake, 0, ctypes.byref(too_wide), fake, fake, None) == binding.EINVAL
    assert L.toploc_build_proofs(fake, 0, ctypes.byref(wide), fake, fake, None, fake, 0, None) == binding.EINVAL
    # continuous batching
    assert L.toploc_stream_append_rows(fake, 8, fake, fake, fake, 0, 4096, 32, 128, None) == binding.OK
    assert L.toploc_stream_append_rows(fake, 0, fake, fake, fake, 3, 4096, 32, 128, None) == binding.EINVAL   # no slots
    assert L.toploc_stream_append_rows(fake, 8, fake, None, fake, 3, 4096, 32, 128, None) == binding.EINVAL
    assert L.toploc_stream_append_rows(fake, 8, fake, ctypes.c_void_p((1 << 40) + 2), fake, 3, 4096, 32, 128,
                                       None) == binding.EINVAL                                          # misaligned slots
    assert L.toploc_stream_append_rows(fake, 8, fake, fake, fake, 3, 4100, 32, 128, None) == binding.EINVAL
    assert L.toploc_stream_emit_rows(fake, 8, fake, 0, 128, fake, fake, None, None) == binding.OK
    assert L.toploc_stream_emit_rows(fake, 8, None, 2, 128, fake, fake, None, None) == binding.EINVAL
    assert L.toploc_stream_emit_rows(fake, 8, fake, 2, 513, fake, fake, None, None) == binding.EINVAL
    # fp32 segments: k stops at 128, candidates are wider
    b16 = L.toploc_segments_workspace_bytes_dtype(2, 9, 4096, 128, binding.DTYPE_BF16)
    b32 = L.toploc_segments_workspace_bytes_dtype(2, 9, 4096, 128, binding.DTYPE_F32)
    assert b16 == L.toploc_segments_workspace_bytes(2, 9, 4096, 128) and b32 > b16 > 0
    assert L.toploc_segments_workspace_bytes_dtype(2, 9, 4096, 513, binding.DTYPE_F32) == 0
    assert L.toploc_segments_workspace_bytes_dtype(2, 9, 4096, 128, 7) == 0                           # unknown dtype
    assert L.toploc_build_proofs_segments_f32(fake, 9, fake, 2, 4096, 513, fake, fake, None, fake, 1 << 30, None) == binding.EINVAL
    assert L.toploc_build_proofs_segments_f32(fake, 9, fake, 2, 4096, 128, fake, fake, None, fake, 16, None) == binding.EWORKSPACE
    assert L.toploc_verify_proofs_segments_mixed(fake, binding.DTYPE_BF16, 9, fake, 2, 4096, 513, fake, binding.DTYPE_F32,
                                                 ctypes.byref(thr), fake, fake, 1 << 30, None) == binding.EINVAL
    # fp32 fixed chunks: k up to 512 with a workspace, refused without one
    p32 = binding.Params(512, 32, 4096, binding.PRIME32)
    assert binding.toploc_workspace_bytes_f32(512, 32, 4096, 16) >= 16 * 512 * 8
    assert binding.toploc_workspace_bytes_f32(513, 32, 4096, 16) == 0
    assert L.toploc_build_proofs_f32(fake, 16, ctypes.byref(p32), fake, fake, None, None, 0, None) == binding.EINVAL
    assert L.toploc_build_proofs_f32(fake, 16, ctypes.byref(p32), fake, fake, None, fake, 16, None) == binding.EWORKSPACE
    # the running top-k with the element type as an argument
    assert L.toploc_stream_state_bytes_dtype(1, 128, binding.DTYPE_F32) == 16 + 512 + 512
    assert L.toploc_stream_state_bytes_dtype(1, 128, binding.DTYPE_BF16) == binding.toploc_stream_state_bytes(1, 128)
    assert L.toploc_stream_state_bytes_dtype(1, 128, 2) == 0 and L.toploc_stream_state_bytes_dtype(1, 513, binding.DTYPE_F32) == 0
    assert L.toploc_stream_reset_dtype(fake, 0, 128, binding.DTYPE_F32, None) == binding.OK
    assert L.toploc_stream_reset_dtype(fake, 1, 128, 3, None) == binding.EINVAL
    assert L.toploc_stream_append_dtype(fake, 4, fake, binding.DTYPE_F32, None, None, 0, 4096, 32, 0, 128, None) == binding.OK
    assert L.toploc_stream_append_dtype(fake, 4, fake, binding.DTYPE_F32, None, None, 4, 4096, 32, 32, 128, None) == binding.EINVAL
    assert L.toploc_stream_append_dtype(fake, 4, fake, binding.DTYPE_F32, fake, None, 4, 4096, 32, 0, 128, None) == binding.EINVAL
    assert L.toploc_stream_append_dtype(fake, 4, fake, 9, None, None, 4, 4096, 32, 0, 128, None) == binding.EINVAL
    assert L.toploc_stream_emit_dtype(fake, 4, binding.DTYPE_F32, None, 0, 128, fake, fake, None, None) == binding.OK
    assert L.toploc_stream_emit_dtype(fake, 4, binding.DTYPE_F32, None, 4, 513, fake, fake, None, None) == binding.EINVAL
    assert L.toploc_verify_proofs_segments_mixed(fake, binding.DTYPE_F32, 9, fake, 0, 4096, 128, fake, binding.DTYPE_F32,
                                                 ctypes.byref(thr), fake, fake, 0, None) == binding.OK

def test_static_scratch_entry_point_rejects_before_any_launch():
    L = binding.lib()
    fake = ctypes.c_void_p(1 << 40)  # never dereferenced: every call below is refused or empty
    ok = binding.Params(128, 32, 4096, binding.PRIME)
    bad = binding.Params(0, 32, 4096, binding.PRIME)
    assert L.toploc_build_proofs_static(fake, 1, ctypes.byref(bad), fake, fake, None, None) == binding.EINVAL
    assert L.toploc_build_proofs_static(None, 1, ctypes.byref(ok), fake, fake, None, None) == binding.EINVAL
    assert L.toploc_build_proofs_static(ctypes.c_void_p((1 << 40) + 8), 1, ctypes.byref(ok), fake, fake, None,
                                        None) == binding.EINVAL                 # misaligned input
    assert L.toploc_build_proofs_static(fake, 0, ctypes.byref(ok), fake, fake, None, None) == binding.OK
    # 16384 chunks at k = 512 hand 16384 x 512 candidates of 6 bytes on: far beyond the fixed array
    big = binding.Params(512, 32, 8192, binding.PRIME)
    assert binding.toploc_workspace_bytes(512, 32, 8192, 16384) > binding.STATIC_SCRATCH_BYTES
    assert L.toploc_build_proofs_static(fake, 16384, ctypes.byref(big), fake, fake, None, None) == binding.ESCRATCH
    assert b"TOPLOC_STATIC_SCRATCH_BYTES" in L.toploc_strerror(binding.ESCRATCH)
    hdr = open(os.path.join(ROOT, "include", "toploc.h")).read()
    assert re.search(r"#define TOPLOC_STATIC_SCRATCH_BYTES \(8u << 20\)", hdr) and binding.STATIC_SCRATCH_BYTES == 8 << 20
