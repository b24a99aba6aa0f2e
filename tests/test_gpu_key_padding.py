"""Key-padding mask (the MASK example of Appendix B.3) through the C ABI against the oracle:
batches of sequences of different true lengths padded to one N, in every kernel variant."""
import math

import numpy as np
import pytest
import torch

from tests import helpers as hp
from paper_2205_14135_amd import binding, inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _both_kernels(fwd_variant, dkv_variant):
    """Every test of this module runs with the library's own choice of forward and of dK/dV kernel
    and with the other kernel forced (four combinations)."""



def _case(B, H, N, d, dtype, lengths, **kw):
    t, dev = hp.make_case(B, H, N, d, dtype, inputs.BASE_SEED + 700 + N + d)
    tau = 1 / math.sqrt(d)
    res = hp.check_forward(t, dev, dtype, tau, key_lengths=lengths, **kw)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, dtype, tau, key_lengths=lengths, **kw)
    hp.assert_backward_ok(resb)
    return res, resb


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("causal", [False, True])
def test_ragged_batch(d, causal):
    """Lengths cover: full, one short of a tile, mid-tile, a single token, an empty sequence, a
    multiple of the tile, one more than a tile."""
    lengths = [384, 383, 200, 1, 0, 128, 65]
    print(_case(len(lengths), 2, 384, d, "bf16", lengths, causal=causal))


@pytest.mark.parametrize("causal", [False, True])
def test_ragged_batch_with_dropout(causal):
    lengths = [256, 97, 130, 31]
    print(_case(4, 3, 256, 64, "fp16", lengths, causal=causal, p=0.17, seed=inputs.BASE_DROPOUT_SEED + 70, offset=5))


@pytest.mark.parametrize("d,causal", [(128, False), (128, True), (64, False)])
def test_ragged_batch_two_group_forward(d, causal):
    """N large enough that the dispatcher picks the two-group forward kernel; lengths leave whole
    256-row workgroups empty, end inside the first 64-key tile, and end one key into a tile."""
    N = 4096 if causal else 2048
    lengths = [N, N - 300, 40, 1025] if not causal else [N, 1500]
    B = len(lengths)
    t, dev = hp.make_case(B, 2, N, d, "bf16", inputs.BASE_SEED + 710 + d)
    tau = 1 / math.sqrt(d)
    heads = [(b, 1) for b in range(B)]
    res = hp.check_forward(t, dev, "bf16", tau, causal=causal, key_lengths=lengths, heads=heads)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "bf16", tau, causal=causal, key_lengths=lengths, heads=heads)
    hp.assert_backward_ok(resb)
    print(res, resb)


def test_ragged_batch_two_group_forward_dropout():
    lengths = [512, 300, 65]
    print(_case(3, 2, 512, 128, "bf16", lengths, p=0.1, seed=inputs.BASE_DROPOUT_SEED + 71))


@pytest.mark.parametrize("causal", [False, True])
def test_ragged_batch_blocksparse(causal):
    N, T = 1024, 8
    bm = inputs.butterfly_block_mask(T)
    lengths = [1024, 700, 129, 0]
    print(_case(4, 2, N, 64, "bf16", lengths, causal=causal, block_mask=bm))


def test_ragged_batch_blocksparse_heavy_columns():
    """All-ones mask with T = 32 > the split threshold: every column is cut into segments that
    accumulate through fp32 atomics; the padded lengths shorten the columns differently per batch."""
    N, T = 4096, 32
    bm = np.ones((T, T), dtype=np.uint8)
    lengths = [4096, 3333, 128 * 25 + 1]
    t, dev = hp.make_case(3, 1, N, 64, "bf16", inputs.BASE_SEED + 720)
    tau = 1 / 8
    resb = hp.check_backward(t, dev, "bf16", tau, block_mask=bm, key_lengths=lengths)
    hp.assert_backward_ok(resb)
    print(resb)


def test_full_lengths_are_bitwise_the_unmasked_result():
    t, dev = hp.make_case(2, 2, 512, 128, "bf16", inputs.BASE_SEED + 730)
    tau = 1 / math.sqrt(128)
    kl = torch.full((2,), 512, dtype=torch.int32, device="cuda")
    O0, L0 = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], softmax_scale=tau, causal=True)
    O1, L1 = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], softmax_scale=tau, causal=True, key_lengths=kl)
    g0 = binding.attn_bwd(dev["Q"], dev["K"], dev["V"], O0, dev["dO"], L0, softmax_scale=tau, causal=True)
    g1 = binding.attn_bwd(dev["Q"], dev["K"], dev["V"], O1, dev["dO"], L1, softmax_scale=tau, causal=True, key_lengths=kl)
    torch.cuda.synchronize()
    assert torch.equal(O0, O1) and torch.equal(L0, L1)
    for a, b in zip(g0, g1):
        assert torch.equal(a, b)


def test_padding_content_is_ignored():
    """Whatever finite values sit in the padded region of Q, K, V, dO, no output changes by a bit.
    (Finite junk, not NaN: a NaN logit times a zero probability is NaN in any implementation.)"""
    B, H, N, d = 2, 2, 256, 64
    lengths = [100, 192]
    t, dev = hp.make_case(B, H, N, d, "bf16", inputs.BASE_SEED + 740)
    tau = 1 / 8
    kl = torch.tensor(lengths, dtype=torch.int32, device="cuda")
    kw = dict(softmax_scale=tau, key_lengths=kl)
    O0, L0 = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
    g0 = binding.attn_bwd(dev["Q"], dev["K"], dev["V"], O0, dev["dO"], L0, **kw)
    dirty = {k: v.clone() for k, v in dev.items()}
    for b, n in enumerate(lengths):
        for k in dirty:
            dirty[k][b, :, n:] = 1e4
    O1, L1 = binding.attn_fwd(dirty["Q"], dirty["K"], dirty["V"], **kw)
    g1 = binding.attn_bwd(dirty["Q"], dirty["K"], dirty["V"], O1, dirty["dO"], L1, **kw)
    torch.cuda.synchronize()
    assert torch.equal(O0, O1) and torch.equal(L0, L1)
    for a, b in zip(g0, g1):
        assert torch.equal(a, b)
