"""Host-side checks that need no GPU: the library loads, exports every declared symbol,
and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2205_14135_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2205_14135_amd import build
        build.build()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "attn.h")).read()
    declared = set(re.findall(r"\b(attn_[a-z_0-9]+)\s*\(", header))
    assert declared == set(binding.SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_version_and_strerror(lib):
    assert binding.version() >= 100
    assert binding.strerror(0) == "ok"
    texts = {binding.strerror(-i) for i in range(1, 10)}
    assert len(texts) == 9 and "unknown status" not in texts
    assert binding.strerror(-99) == "unknown status"
    assert "16, 32, 64 or 128" in binding.strerror(-4)


def _params(**kw):
    p = binding.AttnParams()
    p.B, p.H, p.N, p.d = 1, 1, 128, 64
    p.dtype = binding.ATTN_BF16
    p.softmax_scale = 0.125
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def _fwd(lib, p, ptr=0x1000):
    v = ctypes.c_void_p(ptr)
    return lib.attn_fwd(ctypes.byref(p), v, v, v, v, v)


def test_struct_layout_matches_c():
    # int32 x5, pad, int64 x3, float, int32, float, pad, uint64 x2, int32, pad, pointer
    assert ctypes.sizeof(binding.AttnParams) == 104
    assert binding.AttnParams.stride_b.offset == 24
    assert binding.AttnParams.seed.offset == 64
    assert binding.AttnParams.stream.offset == 88
    assert binding.AttnParams.key_lengths.offset == 96


@pytest.mark.parametrize("kw,code", [
    (dict(dtype=2), -3),
    (dict(d=96), -4),
    (dict(d=8), -4),
    (dict(d=48), -4),
    (dict(N=0), -2),
    (dict(N=-128), -2),
    (dict(B=0), -2),
    (dict(stride_b=8192, stride_h=8192, stride_n=60), -2),
    (dict(stride_b=8192, stride_h=8192, stride_n=68), -2),
    (dict(stride_b=1 << 40, stride_h=1 << 36, stride_n=(1 << 23) + 8), -2),   # rows too far apart for the tile copies
    (dict(dropout_p=1.0), -5),
    (dict(dropout_p=-0.1), -5),
    (dict(dropout_p=float("nan")), -5),
    (dict(softmax_scale=0.0), -6),
    (dict(softmax_scale=-1.0), -6),
    (dict(softmax_scale=float("inf")), -6),
    (dict(softmax_scale=float("nan")), -6),
])
def test_bad_params_are_rejected_before_launch(lib, kw, code):
    assert _fwd(lib, _params(**kw)) == code


def test_null_pointers_and_workspace(lib):
    p = _params()
    assert lib.attn_fwd(None, None, None, None, None, None) == -1
    assert _fwd(lib, p, ptr=0) == -1
    v, z = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    need = lib.attn_bwd_workspace_bytes(ctypes.byref(p))
    assert need == 1024 and need % 256 == 0
    args = [v] * 9
    assert lib.attn_bwd(ctypes.byref(p), *args, z, need) == -7                      # NULL workspace
    assert lib.attn_bwd(ctypes.byref(p), *args, ctypes.c_void_p(0x1010), need) == -7  # misaligned
    assert lib.attn_bwd(ctypes.byref(p), *args, v, need - 1) == -7                  # too small
    assert lib.attn_bwd(ctypes.byref(p), *([v] * 8 + [z]), v, need) == -1
    assert lib.attn_bwd_workspace_bytes(ctypes.byref(_params(d=7))) == 0
    sparse_need = lib.attn_blocksparse_bwd_workspace_bytes(ctypes.byref(p))
    assert sparse_need == 1024 + 512 + 2 * 128 * 64 * 4         # D, L | segment list + column counts | fp32 dK, dV
    assert lib.attn_blocksparse_bwd_workspace_bytes(ctypes.byref(_params(N=100))) == 0
    args_m = [v, 128, 0] + [v] * 9
    assert lib.attn_blocksparse_bwd(ctypes.byref(p), *args_m, v, need) == -7     # dense size is too small


def test_tensor_alignment_and_overlapping_strides(lib):
    p = _params()
    v, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1008)
    for slot in range(4):   # Q, K, V, O: every tensor is accessed in 16-byte pieces
        args = [v] * 5
        args[slot] = odd
        assert lib.attn_fwd(ctypes.byref(p), *args) == -2
    need = lib.attn_bwd_workspace_bytes(ctypes.byref(p))
    for slot in (0, 4, 6, 7, 8):   # Q, dO, dQ, dK, dV
        args = [v] * 9
        args[slot] = odd
        assert lib.attn_bwd(ctypes.byref(p), *args, v, need) == -2
    ok = lambda **kw: lib.attn_bwd_workspace_bytes(ctypes.byref(_params(**kw))) != 0
    # head-major with padded rows, token-major view of [B,N,H,d], single-head / single-batch axes
    assert ok(B=2, H=3, N=128, stride_b=3 * 128 * 72, stride_h=128 * 72, stride_n=72)
    assert ok(B=2, H=3, N=128, stride_b=128 * 3 * 64, stride_h=64, stride_n=3 * 64)
    assert ok(B=1, H=1, N=128, stride_b=0, stride_h=0, stride_n=64)
    # aliasing layouts: a zero or too short stride on an axis of size > 1
    assert not ok(B=2, H=1, N=128, stride_b=0, stride_h=128 * 64, stride_n=64)
    assert not ok(B=1, H=2, N=128, stride_b=2 * 128 * 64, stride_h=0, stride_n=64)
    assert not ok(B=1, H=2, N=128, stride_b=2 * 128 * 64, stride_h=64 * 64, stride_n=64)   # heads overlap by half
    assert not ok(B=2, H=2, N=128, stride_b=128 * 64, stride_h=128 * 64, stride_n=64)      # batch 1 = head 1


def test_variant_override_arguments(lib):
    assert lib.attn_debug_set_variant(3, 0) == -2
    assert lib.attn_debug_set_variant(0, 4) == -2
    assert lib.attn_debug_set_variant(0, -2) == -2
    assert lib.attn_debug_set_variant(2, 1) == 0
    assert lib.attn_debug_set_variant(-1, -1) == 0
    assert lib.attn_debug_set_variant(0, 0) == 0
    binding.attn_debug_set_variant(fwd="base", dkv="rs")
    binding.attn_debug_set_variant(fwd="auto", dkv="auto")


def test_static_scratch_entry_point_rejects_large_problems(lib):
    # 2^20 rows over all heads fill the built-in scratch exactly; one block more per head is refused
    v = ctypes.c_void_p(0x1000)
    big = _params(B=64, H=16, N=1024 + 128)
    assert lib.attn_bwd_workspace_bytes(ctypes.byref(big)) > binding.STATIC_SCRATCH_BYTES
    assert lib.attn_bwd_static(ctypes.byref(big), *([v] * 9)) == -7
    assert "built-in scratch" in binding.strerror(-7)
    fits = _params(B=64, H=16, N=1024)
    assert lib.attn_bwd_workspace_bytes(ctypes.byref(fits)) == binding.STATIC_SCRATCH_BYTES
    assert lib.attn_bwd_static(ctypes.byref(fits), *([v] * 8), ctypes.c_void_p(0)) == -1   # NULL dV: nothing launched
    assert lib.attn_bwd_static(ctypes.byref(_params(d=7)), *([v] * 9)) == -4


def test_mfma_rate_probe_arguments(lib):
    v, z = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    assert lib.attn_debug_mfma_rate(binding.ATTN_BF16, 10, 1, z, z, None) == -1
    assert lib.attn_debug_mfma_rate(7, 10, 1, v, z, None) == -3
    assert lib.attn_debug_mfma_rate(binding.ATTN_BF16, 0, 4, v, z, None) == -2
    assert lib.attn_debug_mfma_rate(binding.ATTN_FP16, (1 << 20) + 1, 1, v, z, None) == -2
    assert lib.attn_debug_mfma_rate(binding.ATTN_FP16, 10, 3, v, z, None) == -2


def test_kernel_choice_query(lib):
    """The choice the launchers make, asked for without launching (host only)."""
    binding.attn_debug_set_variant(fwd="auto", dkv="auto")
    choice = lambda sparse=False, **kw: binding.attn_debug_kernel_choice(_params(**kw), sparse)
    assert choice(B=4, H=16, N=4096, d=128) == ("fwd_pp_kernel", "dkv_w64_kernel")
    assert choice(B=4, H=16, N=4096, d=128, causal=1) == ("fwd_pp_kernel", "dkv_fr128_kernel")
    assert choice(B=4, H=16, N=4096, d=128, dropout_p=0.1) == ("fwd_kernel", "dkv_fr128_kernel")
    assert choice(B=8, H=8, N=1024, d=128, causal=1, dropout_p=0.1) == ("fwd_kernel", "dkv_rs_kernel")   # 128 work items only
    assert choice(B=4, H=16, N=4096, d=128, dropout_p=0.003) == ("fwd_pp_kernel", "dkv_w64_kernel")       # rounds down to no dropout
    assert choice(B=16, H=16, N=512, d=64, dropout_p=0.1) == ("fwd_kernel", "dkv_fr_kernel")
    assert choice(B=1, H=8, N=16384, d=64, sparse=True) == ("fwd_kernel", "dkv_fr_kernel")
    assert choice(B=4, H=16, N=4096, d=128, sparse=True) == ("fwd_kernel", "dkv_rs_kernel")
    assert choice(B=4, H=16, N=4010, d=128) == ("fwd_pp_kernel", "dkv_fr128_kernel")      # not whole 32-query tiles
    binding.attn_debug_set_variant(dkv="w64")
    assert choice(B=4, H=16, N=1024, d=128, causal=1)[1] == "dkv_w64_kernel"
    binding.attn_debug_set_variant(dkv="auto")
    f, k = ctypes.c_int32(), ctypes.c_int32()
    assert lib.attn_debug_kernel_choice(ctypes.byref(_params(d=7)), 0, ctypes.byref(f), ctypes.byref(k)) == -4
    assert lib.attn_debug_kernel_choice(ctypes.byref(_params(N=200)), 1, ctypes.byref(f), ctypes.byref(k)) == -2
    assert lib.attn_debug_kernel_choice(ctypes.byref(_params()), 0, None, None) == -1


def test_mask_arguments(lib):
    p = _params(N=256)
    v, z = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    assert lib.attn_blocksparse_fwd(ctypes.byref(p), z, 128, 0, v, v, v, v, v) == -1
    assert lib.attn_blocksparse_fwd(ctypes.byref(p), v, 64, 0, v, v, v, v, v) == -8
    assert lib.attn_blocksparse_fwd(ctypes.byref(p), v, 128, 3, v, v, v, v, v) == -8
    assert lib.attn_blocksparse_fwd(ctypes.byref(p), v, 128, -4, v, v, v, v, v) == -8
    assert lib.attn_debug_dropout_mask(ctypes.byref(p), z) == -1
    # a ragged last block is fine for the dense entry points but not under a 128 x 128 block mask
    ragged = _params(N=200)
    assert lib.attn_blocksparse_fwd(ctypes.byref(ragged), v, 128, 0, v, v, v, v, v) == -2
    assert lib.attn_blocksparse_bwd(ctypes.byref(ragged), v, 128, 0, *([v] * 9), v, 1 << 20) == -2
    assert lib.attn_blocksparse_bwd_workspace_bytes(ctypes.byref(ragged)) == 0
    # dense backward scratch: two floats per row, rows padded to whole blocks of 128 per head
    assert lib.attn_bwd_workspace_bytes(ctypes.byref(ragged)) == 2 * 256 * 4
    assert lib.attn_bwd_workspace_bytes(ctypes.byref(_params(N=1))) == 2 * 128 * 4


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        binding.load()
