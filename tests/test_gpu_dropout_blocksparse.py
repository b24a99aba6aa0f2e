"""Dropout mask bit-exactness, dropout forward parity, and the block-sparse variant."""
import math

import numpy as np
import pytest
import torch

from oracle import attention_oracle as orc
from tests import helpers as hp
from paper_2205_14135_amd import binding, inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,H,N,p,seed,offset", [
    (2, 3, 256, 0.1, inputs.BASE_DROPOUT_SEED + 1, 0),
    (1, 2, 384, 0.5, 0xFEDCBA9876543210, 0x1_0000_0005),
    (1, 1, 128, 0.9, 1, 0xFFFFFFFF),
])
def test_dropout_mask_is_bit_exact(B, H, N, p, seed, offset):
    keep = binding.attn_debug_dropout_mask(B, H, N, p, seed, offset).cpu().numpy().astype(bool)
    for b in range(B):
        for h in range(H):
            want = orc.dropout_keep_mask(b, h, H, N, p, seed, offset)
            assert (keep[b, h] == want).all()


@pytest.mark.parametrize("dtype,d,causal", [("fp16", 64, False), ("bf16", 64, True), ("bf16", 128, True)])
def test_forward_with_dropout(dtype, d, causal):
    t, dev = hp.make_case(2, 2, 384, d, dtype, 400 + d)
    res = hp.check_forward(t, dev, dtype, 1 / math.sqrt(d), causal=causal, p=0.1,
                           seed=inputs.BASE_DROPOUT_SEED + 2, offset=9)
    print("dropout fwd", dtype, d, causal, res)
    hp.assert_forward_ok(res)


@pytest.mark.parametrize("name", ["C2", "C3", "C3_d128"])
def test_dropout_mask_every_bit_at_benchmark_shapes(name):
    """The whole [B, H, N, N] keep mask of the dropout benchmark shapes (seed and offset as bench.py
    uses them), every bit against the oracle."""
    c = inputs.CONFIGS[name]
    B, H, N, p = c["B"], c["H"], c["N"], c["p_drop"]
    seed, offset = inputs.BASE_DROPOUT_SEED, 0
    keep = binding.attn_debug_dropout_mask(B, H, N, p, seed, offset)
    kept = 0
    for b in range(B):
        got = keep[b].cpu().numpy().astype(bool)
        for h in range(H):
            want = orc.dropout_keep_mask(b, h, H, N, p, seed, offset)
            assert (got[h] == want).all(), (b, h)
            kept += int(want.sum())
    frac = kept / (B * H * N * N)
    assert abs(frac - (1 - orc.dropout_effective_p(p))) < 1e-3, frac


def _want_masks(H, N, p, seed, offset, causal):
    want = np.stack([orc.dropout_keep_mask(0, h, H, N, p, seed, offset) for h in range(H)])
    return want & np.tril(np.ones((N, N), dtype=bool)) if causal else want


@pytest.mark.parametrize("d,N,causal,variant", [
    (64, 128, False, "auto"), (64, 256, True, "pp"), (128, 512, False, "pp"), (128, 512, True, "pp"),
    (128, 384, True, "auto"), (32, 128, False, "auto"), (16, 128, True, "auto"),
])
def test_forward_kernels_apply_exactly_the_oracle_mask(d, N, causal, variant):
    """Q = K = 0 makes P uniform over the visible keys, so O_i = (scale / n_i) * sum_{j kept} V_j: with
    V the N x N identity split over d-wide column slabs, O read back slab by slab IS the mask the
    kernel applied (kept and visible entries are positive, all others exactly zero)."""
    B, H, p = 1, 2, 0.3
    seed, offset = 77, 5
    binding.attn_debug_set_variant(fwd=variant)
    try:
        Q = torch.zeros((B, H, N, d), dtype=torch.float16, device="cuda")
        K = torch.zeros_like(Q)
        got = np.zeros((H, N, N), dtype=bool)
        idx = torch.arange(d, device="cuda")
        for slab in range(N // d):
            V = torch.zeros((B, H, N, d), dtype=torch.float16, device="cuda")
            V[:, :, slab * d + idx, idx] = 1.0
            O, _ = binding.attn_fwd(Q, K, V, softmax_scale=1.0, causal=causal, dropout_p=p, seed=seed,
                                    offset=offset, o_fp32=True)
            assert (O >= 0).all()
            got[:, :, slab * d:(slab + 1) * d] = (O[0] > 0).cpu().numpy()
    finally:
        binding.attn_debug_set_variant(fwd="auto")
    assert (got == _want_masks(H, N, p, seed, offset, causal)).all()


@pytest.mark.parametrize("variant", ["auto", "rs", "fr"])
@pytest.mark.parametrize("d,N,causal", [(64, 512, False), (64, 576, True), (128, 512, False), (128, 640, True),
                                        (32, 256, True)])
def test_backward_kernels_apply_exactly_the_oracle_mask(d, N, causal, variant):
    """The same read-back for the dK/dV kernels: with Q = K = 0 and dO the N x N identity split over
    d-wide column slabs, dV_j = sum_i Z_ij P_ij dO_i has dV[j, c] = Z_ij scale / n_i for query
    i = slab * d + c, so dV read back slab by slab is the (transposed) mask the kernel regenerated
    (Appendix B.4, observation 1: the backward pass redraws the forward's mask from the saved state).
    dQ and dK must come out as exact zeros (K = 0 and Q = 0)."""
    B, H, p = 1, 2, 0.3
    seed, offset = 1234567, 0x2_0000_0001
    kw = dict(softmax_scale=1.0, causal=causal, dropout_p=p, seed=seed, offset=offset)
    binding.attn_debug_set_variant(dkv=variant)
    try:
        Q = torch.zeros((B, H, N, d), dtype=torch.bfloat16, device="cuda")
        K, V = torch.zeros_like(Q), torch.zeros_like(Q)
        O, L = binding.attn_fwd(Q, K, V, **kw)
        got = np.zeros((H, N, N), dtype=bool)
        idx = torch.arange(d, device="cuda")
        for slab in range(N // d):
            dO = torch.zeros_like(Q)
            dO[:, :, slab * d + idx, idx] = 1.0
            dQ, dK, dV = binding.attn_bwd(Q, K, V, O, dO, L, **kw)
            assert (dV >= 0).all() and not dQ.any() and not dK.any()
            got[:, slab * d:(slab + 1) * d, :] = (dV[0] > 0).cpu().numpy().transpose(0, 2, 1)
    finally:
        binding.attn_debug_set_variant(dkv="auto")
    assert (got == _want_masks(H, N, p, seed, offset, causal)).all()


def test_dispatcher_takes_the_two_group_forward_with_causal_mask_and_dropout():
    """d = 128 with at least 256 paired work items: the library's own choice is the two-group forward,
    here with the causal mask and dropout at a full-size shape (B=4, H=16, N=2048), against the oracle
    on whole heads and through the V-identity read-back of the applied mask for one head."""
    B, H, N, d, p = 4, 16, 2048, 128, 0.1
    seed = inputs.BASE_DROPOUT_SEED + 5
    t, dev = hp.make_case(B, H, N, d, "bf16", 470)
    prm = binding.make_params(dev["Q"], 1 / math.sqrt(d), causal=True, dropout_p=p, seed=seed)
    assert binding.attn_debug_kernel_choice(prm, sparse=False)[0] == "fwd_pp_kernel"
    heads = [(0, 0), (3, 15)]
    res = hp.check_forward(t, dev, "bf16", 1 / math.sqrt(d), causal=True, p=p, seed=seed, heads=heads)
    print("pp by dispatcher fwd", res)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "bf16", 1 / math.sqrt(d), causal=True, p=p, seed=seed, heads=heads)
    print("pp by dispatcher bwd", resb)
    hp.assert_backward_ok(resb)
    Q = torch.zeros((B, H, N, d), dtype=torch.bfloat16, device="cuda")
    got = np.zeros((N, N), dtype=bool)
    idx = torch.arange(d, device="cuda")
    for slab in range(N // d):
        V = torch.zeros_like(Q)
        V[:, :, slab * d + idx, idx] = 1.0
        O, _ = binding.attn_fwd(Q, Q, V, softmax_scale=1.0, causal=True, dropout_p=p, seed=seed, o_fp32=True)
        got[:, slab * d:(slab + 1) * d] = (O[2, 7] > 0).cpu().numpy()
    want = orc.dropout_keep_mask(2, 7, H, N, p, seed, 0) & np.tril(np.ones((N, N), dtype=bool))
    assert (got == want).all()


def _random_block_mask(T, seed, density=0.4):
    rng = np.random.default_rng(seed)
    m = (rng.random((T, T)) < density).astype(np.uint8)
    m[np.arange(T), np.arange(T)] = 1
    return m


@pytest.mark.parametrize("d", [64, 128])
def test_blocksparse_butterfly_small(d):
    T = 8
    N = 128 * T
    t, dev = hp.make_case(1, 2, N, d, "bf16", 500 + d)
    bm = inputs.butterfly_block_mask(T)
    res = hp.check_forward(t, dev, "bf16", 1 / math.sqrt(d), block_mask=bm)
    print("butterfly fwd", d, res)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "bf16", 1 / math.sqrt(d), block_mask=bm)
    print("butterfly bwd", d, resb)
    hp.assert_backward_ok(resb)


@pytest.mark.parametrize("causal,p", [(False, 0.0), (True, 0.1)])
def test_blocksparse_heavy_column_is_split(causal, p):
    """T = 32: mask column 0 keeps all 32 blocks, which the dK/dV kernel splits over several
    workgroups (fp32 atomics); the other columns take the direct path."""
    T = 32
    N = 128 * T
    t, dev = hp.make_case(1, 2, N, 64, "bf16", 650)
    bm = inputs.butterfly_block_mask(T)
    assert int(bm[:, 0].sum()) == 32 and int(bm[:, 5].sum()) < 12
    kw = dict(causal=causal, p=p, seed=21, offset=2, block_mask=bm)
    res = hp.check_forward(t, dev, "bf16", 0.125, heads=[(0, 1)], **kw)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "bf16", 0.125, heads=[(0, 0), (0, 1)], **kw)
    print("heavy column bwd", causal, p, resb)
    hp.assert_backward_ok(resb)


def test_blocksparse_random_per_head_mask_causal_dropout_and_empty_rows():
    T = 5
    N = 128 * T
    H = 2
    t, dev = hp.make_case(1, H, N, 64, "fp16", 600)
    bm = np.stack([_random_block_mask(T, 1), _random_block_mask(T, 2)])
    bm[1, 3, :] = 0          # a query block that sees nothing: O = 0, LSE = -inf, zero gradients
    kw = dict(causal=True, p=0.2, seed=9, offset=1, block_mask=bm)
    res = hp.check_forward(t, dev, "fp16", 0.125, **kw)
    print("sparse fwd", res)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "fp16", 0.125, **kw)
    print("sparse bwd", resb)
    hp.assert_backward_ok(resb)


def test_blocksparse_all_ones_equals_dense():
    """An all-ones block mask is the dense problem.  The dense call may take a different kernel
    (other summation order, other roundings of P and dS to 16 bits), so O is compared to one output ulp
    and the gradients by relative L2 distance: each is within 2.6e-3 of the exact gradient (the oracle
    tests), so the two are within 5e-3 of each other."""
    T = 3
    t, dev = hp.make_case(1, 2, 128 * T, 128, "bf16", 700)
    kw = dict(softmax_scale=0.09, causal=True, dropout_p=0.1, seed=4)
    ones = torch.ones((T, T), dtype=torch.uint8, device="cuda")
    O, L = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
    Os, Ls = binding.attn_blocksparse_fwd(dev["Q"], dev["K"], dev["V"], ones, **kw)
    g = binding.attn_bwd(dev["Q"], dev["K"], dev["V"], O, dev["dO"], L, **kw)
    gs = binding.attn_blocksparse_bwd(dev["Q"], dev["K"], dev["V"], Os, dev["dO"], Ls, ones, **kw)
    torch.cuda.synchronize()
    assert (L - Ls).abs().max().item() <= 1e-5
    assert ((O.float() - Os.float()).abs() <= 2.0 ** -7 * O.float().abs().clamp_min(2.0 ** -7)).all()
    for a, b in zip(g, gs):
        assert float((a.float() - b.float()).norm() / b.float().norm()) <= 5e-3
