"""Sequence lengths that are not a multiple of the 128-token block (nor of the 64-token tile):
every dense kernel path through the C ABI against the oracle.

All [B,H,N,d] tensors are views of buffers with extra guard rows behind the N real rows of every
head.  Input guards hold NaN (a kernel that used a row beyond N would poison its result), output
guards hold a sentinel that must survive (a kernel that wrote a row beyond N would change it)."""
import math

import numpy as np
import pytest
import torch

from oracle import attention_oracle as orc
from tests import helpers as hp
from paper_2205_14135_amd import binding, inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _both_kernels(fwd_variant, dkv_variant):
    """Every test of this module runs with the library's own choice of forward and of dK/dV kernel
    and with the other kernel forced (four combinations)."""


GUARD_ROWS = 130
SENTINEL = 512.0


def _guarded_input(x_np, dtype):
    """[B,H,N,d] numpy -> view [:, :, :N] of a [B,H,N+G,d] device buffer whose guard rows are NaN."""
    B, H, N, d = x_np.shape
    buf = torch.full((B, H, N + GUARD_ROWS, d), float("nan"),
                     dtype=torch.float16 if dtype == "fp16" else torch.bfloat16, device="cuda")
    view = buf[:, :, :N, :]
    view.copy_(inputs.to_torch(x_np, dtype, "cuda"))
    return buf, view


def _guarded_output(like_view, torch_dtype):
    B, H, N, d = like_view.shape
    buf = torch.full((B, H, N + GUARD_ROWS, d), SENTINEL, dtype=torch_dtype, device="cuda")
    return buf, buf[:, :, :N, :]


def _guard_intact(buf, N):
    return bool((buf[:, :, N:, :].float() == SENTINEL).all())


def _run(B, H, N, d, dtype, *, causal=False, p=0.0, lengths=None, o_fp32=False, seed_shift=0):
    t = inputs.gaussian_tensors(B, H, N, d, dtype, inputs.BASE_SEED + 900 + N + d + seed_shift)
    tau = 1 / math.sqrt(d)
    dev = {k: _guarded_input(v, dtype) for k, v in t.items()}
    Q, K, V, dO = (dev[k][1] for k in ("Q", "K", "V", "dO"))
    kw = dict(softmax_scale=tau, causal=causal, dropout_p=p, seed=inputs.BASE_DROPOUT_SEED + 9, offset=3,
              o_fp32=o_fp32, key_lengths=None if lengths is None else
              torch.tensor(lengths, dtype=torch.int32, device="cuda"))
    o_buf, O = _guarded_output(Q, torch.float32 if o_fp32 else Q.dtype)
    lse_buf = torch.full((B * H * N + 256,), SENTINEL, dtype=torch.float32, device="cuda")
    L = lse_buf[:B * H * N].view(B, H, N)
    binding.attn_fwd(Q, K, V, out=O, lse=L, **kw)
    g_bufs = [_guarded_output(Q, Q.dtype) for _ in range(3)]
    binding.attn_bwd(Q, K, V, O, dO, L, grads=tuple(g[1] for g in g_bufs), **kw)
    torch.cuda.synchronize()
    # nothing beyond the N rows of a head, or beyond the end of the statistic, was written
    assert _guard_intact(o_buf, N), "O guard rows"
    assert bool((lse_buf[B * H * N:] == SENTINEL).all()), "LSE guard"
    for name, (buf, _) in zip(("dQ", "dK", "dV"), g_bufs):
        assert _guard_intact(buf, N), name + " guard rows"
    On, Ln = hp.to_np(O), hp.to_np(L)
    grads = [hp.to_np(g[1]) for g in g_bufs]
    worst = dict(o=0.0, lse=0.0, dQ=0.0, dK=0.0, dV=0.0)
    for b in range(B):
        for h in range(H):
            keep = orc.dropout_keep_mask(b, h, H, N, p, kw["seed"], kw["offset"]) if p > 0 else None
            klen = None if lengths is None else lengths[b]
            Oo, Lo = orc.forward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], tau, causal=causal,
                                      p_drop=p, keep=keep, key_length=klen)
            err = np.abs(On[b, h] - Oo)
            assert np.isfinite(On[b, h]).all()
            excess = err if o_fp32 else err - hp.ulp_half(Oo, dtype)
            worst["o"] = max(worst["o"], float(excess.max()))
            fin = np.isfinite(Lo)
            assert (np.isfinite(Ln[b, h]) == fin).all()
            if fin.any():
                worst["lse"] = max(worst["lse"], float(np.abs(Ln[b, h][fin] - Lo[fin]).max()))
            ref = orc.backward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], t["dO"][b, h], tau,
                                    causal=causal, p_drop=p, keep=keep, key_length=klen)
            bounds = None
            for name, got, want in zip(("dQ", "dK", "dV"), grads, ref):
                assert np.isfinite(got[b, h]).all(), name
                # at most one visible key: the exact dQ, dK vanish, the round-off is bounded instead
                if np.sqrt((want ** 2).sum()) < 1e-9:
                    if bounds is None:
                        bounds = hp.vanishing_gradient_bounds(
                            t["Q"][b, h], t["K"][b, h], t["V"][b, h], t["dO"][b, h], Oo, tau,
                            hp.alive_entries(N, causal=causal, key_length=klen, keep=keep),
                            o_round=None if o_fp32 else dtype,
                            keep_scale=1.0 / (1.0 - orc.dropout_effective_p(p)) if p > 0 else 1.0)
                    hp.check_vanishing(name, got[b, h], 0.0, bounds)
                    continue
                worst[name] = max(worst[name], hp.rel_l2(got[b, h], want))
    assert worst["o"] <= hp.FWD_ATOL, worst
    assert worst["lse"] <= hp.LSE_ATOL, worst
    for name in ("dQ", "dK", "dV"):
        assert worst[name] <= hp.GRAD_REL_L2, worst
    return worst


@pytest.mark.parametrize("N", [1, 37, 64, 65, 100, 129, 200, 333])
@pytest.mark.parametrize("causal", [False, True])
def test_ragged_d64(N, causal):
    """d = 64: free-running forward, paired causal items, dQ and both dK/dV kernels."""
    print(_run(2, 2, N, 64, "bf16", causal=causal))


@pytest.mark.parametrize("N,causal", [(100, False), (257, True), (333, False), (449, True)])
def test_ragged_d128_short(N, causal):
    """d = 128 below N = 512: base forward kernel; dQ without pairing."""
    print(_run(2, 2, N, 128, "fp16", causal=causal))


@pytest.mark.parametrize("N,causal", [(520, False), (777, True), (1000, False), (1025, True)])
def test_ragged_d128_two_group_forward(N, causal):
    """d = 128 from N = 512: the two-group forward kernel (256-row workgroups: the last one may hold
    wavefronts with no row at all), causal pairs of row blocks."""
    print(_run(1, 3, N, 128, "bf16", causal=causal))


@pytest.mark.parametrize("N,d,causal", [(100, 128, False), (300, 128, True), (200, 64, True), (77, 64, False),
                                         (203, 32, False)])
def test_ragged_with_dropout(N, d, causal):
    """Dropout draws cover eight keys each: the last group of a row is partial when N % 8 != 0."""
    print(_run(2, 2, N, d, "bf16", causal=causal, p=0.15))


@pytest.mark.parametrize("N,causal", [(77, False), (200, True), (321, False)])
def test_ragged_d32(N, causal):
    print(_run(2, 2, N, 32, "fp16", causal=causal))


def test_ragged_fp32_output():
    print(_run(2, 2, 150, 64, "bf16", o_fp32=True))
    print(_run(1, 2, 600, 128, "bf16", o_fp32=True, causal=True))


@pytest.mark.parametrize("causal", [False, True])
def test_ragged_with_key_padding(causal):
    """Both at once: N = 200 is ragged and the sequences of the batch are shorter still."""
    print(_run(4, 2, 200, 64, "bf16", causal=causal, lengths=[200, 150, 1, 0]))
    print(_run(3, 1, 700, 128, "bf16", causal=causal, lengths=[700, 641, 64]))


@pytest.mark.parametrize("N", [37, 100, 136])
def test_dropout_mask_bit_exact_ragged(N):
    B, H, p, seed, offset = 2, 3, 0.3, inputs.BASE_DROPOUT_SEED + 5, 11
    keep = binding.attn_debug_dropout_mask(B, H, N, p, seed, offset)
    torch.cuda.synchronize()
    keep = keep.cpu().numpy().astype(bool)
    for b in range(B):
        for h in range(H):
            want = orc.dropout_keep_mask(b, h, H, N, p, seed, offset)
            assert (keep[b, h] == want).all()
