"""Head dimension 16 (the smallest the paper's kernels cover, Appendix E.1): every kernel path
against the oracle.  The tensors' rows hold 16 elements; the kernels are the head-dimension-32 ones
with the upper half of every tile held at zero on chip, so the tests also check that nothing beyond
a row's 16 elements is read (NaN guards between the rows) or written (sentinel guards)."""
import math

import numpy as np
import pytest
import torch

from oracle import attention_oracle as orc
from tests import helpers as hp
from paper_2205_14135_amd import binding, inputs

pytestmark = pytest.mark.gpu
D = 16


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("causal", [False, True])
def test_dense(dtype, causal):
    t, dev = hp.make_case(2, 3, 640, D, dtype, inputs.BASE_SEED + 1600 + causal)
    tau = 1 / math.sqrt(D)
    res = hp.check_forward(t, dev, dtype, tau, causal=causal)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, dtype, tau, causal=causal)
    hp.assert_backward_ok(resb)
    print("d16 dense", dtype, causal, res, resb)


@pytest.mark.parametrize("causal", [False, True])
def test_dropout_key_padding_and_a_ragged_length(causal):
    lengths = [333, 200, 65]
    t, dev = hp.make_case(3, 2, 333, D, "bf16", inputs.BASE_SEED + 1610 + causal)
    tau = 1 / math.sqrt(D)
    kw = dict(causal=causal, p=0.2, seed=inputs.BASE_DROPOUT_SEED + 16, offset=1, key_lengths=lengths)
    res = hp.check_forward(t, dev, "bf16", tau, **kw)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "bf16", tau, **kw)
    hp.assert_backward_ok(resb)
    print("d16 dropout + lengths", causal, res, resb)


def test_blocksparse_with_a_heavy_column():
    """Butterfly mask at T = 64: column 0 keeps all 64 blocks and is split into segments."""
    N, T = 8192, 64
    bm = inputs.butterfly_block_mask(T)
    t, dev = hp.make_case(1, 2, N, D, "bf16", inputs.BASE_SEED + 1620)
    tau = 1 / math.sqrt(D)
    heads = [(0, 1)]
    rows = np.unique(np.concatenate([[0, 1, 127, 128, N - 1], np.random.default_rng(5).integers(0, N, 40)]))
    res = hp.check_forward(t, dev, "bf16", tau, block_mask=bm, heads=heads, rows=rows)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "bf16", tau, block_mask=bm, heads=heads)
    hp.assert_backward_ok(resb)
    print("d16 block-sparse", res, resb)


@pytest.mark.parametrize("causal,o_fp32", [(False, False), (True, True)])
def test_rows_in_a_wider_buffer_with_guards(causal, o_fp32):
    """The [B,H,N,16] tensors are views of [B,H,N,24] buffers (row stride 24 elements): the eight
    elements behind every input row hold NaN, those behind every output row a sentinel."""
    B, H, N, dtype, sentinel = 2, 2, 200, "bf16", 512.0
    t = inputs.gaussian_tensors(B, H, N, D, dtype, inputs.BASE_SEED + 1630 + causal)
    tau = 1 / math.sqrt(D)
    tdt = torch.bfloat16

    def guarded_in(x):
        buf = torch.full((B, H, N, 24), float("nan"), dtype=tdt, device="cuda")
        buf[..., :D].copy_(inputs.to_torch(x, dtype, "cuda"))
        return buf, buf[..., :D]

    def guarded_out(torch_dtype):
        buf = torch.full((B, H, N, 24), sentinel, dtype=torch_dtype, device="cuda")
        return buf, buf[..., :D]

    ins = {k: guarded_in(v) for k, v in t.items()}
    Q, K, V, dO = (ins[k][1] for k in ("Q", "K", "V", "dO"))
    kw = dict(softmax_scale=tau, causal=causal, o_fp32=o_fp32)
    o_buf, O = guarded_out(torch.float32 if o_fp32 else tdt)
    L = torch.empty(B, H, N, dtype=torch.float32, device="cuda")
    binding.attn_fwd(Q, K, V, out=O, lse=L, **kw)
    g_bufs = [guarded_out(tdt) for _ in range(3)]
    binding.attn_bwd(Q, K, V, O, dO, L, grads=tuple(g[1] for g in g_bufs), **kw)
    torch.cuda.synchronize()
    assert bool((o_buf[..., D:].float() == sentinel).all()), "O guard columns"
    for name, (buf, _) in zip(("dQ", "dK", "dV"), g_bufs):
        assert bool((buf[..., D:].float() == sentinel).all()), name + " guard columns"
    On = hp.to_np(O)
    grads = [hp.to_np(g[1]) for g in g_bufs]
    for b in range(B):
        for h in range(H):
            Oo, Lo = orc.forward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], tau, causal=causal)
            err = np.abs(On[b, h] - Oo)
            excess = err if o_fp32 else err - hp.ulp_half(Oo, dtype)
            assert float(excess.max()) <= hp.FWD_ATOL
            assert float(np.abs(hp.to_np(L)[b, h] - Lo).max()) <= hp.LSE_ATOL
            ref = orc.backward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], t["dO"][b, h], tau, causal=causal)
            for name, got, want in zip(("dQ", "dK", "dV"), grads, ref):
                assert np.isfinite(got[b, h]).all(), name
                assert hp.rel_l2(got[b, h], want) <= hp.GRAD_REL_L2, name
