"""Forward parity: HIP library (through the C ABI) vs the fp64 oracle, element by element."""
import math

import numpy as np
import pytest
import torch

from tests import helpers as hp
from paper_2205_14135_amd import binding, inputs


@pytest.fixture(autouse=True)
def _both_kernels(fwd_variant):
    """Every test of this module runs with the library's own kernel choice and with the other kernel forced."""

pytestmark = pytest.mark.gpu


def test_c1_tiny_dense():
    """B=1,H=1,N=128,d=64 fp16, tau=1/sqrt(d), no mask, no dropout."""
    t, dev = hp.make_case(1, 1, 128, 64, "fp16", inputs.BASE_SEED + 0)
    res = hp.check_forward(t, dev, "fp16", 1 / math.sqrt(64))
    print("C1 fwd", res)
    hp.assert_forward_ok(res)
    assert res["o"] <= hp.FWD_ATOL


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("causal", [False, True])
def test_multi_tile_dense(dtype, d, causal):
    """Several Q tiles and K/V tiles, two heads, two batches."""
    t, dev = hp.make_case(2, 2, 384, d, dtype, 100 + d + causal)
    res = hp.check_forward(t, dev, dtype, 1 / math.sqrt(d), causal=causal)
    print("multi-tile fwd", dtype, d, causal, res)
    hp.assert_forward_ok(res)


@pytest.mark.parametrize("scale_mult", [1.0, 4.0])
def test_peaky_softmax(scale_mult):
    t, dev = hp.make_case(1, 2, 512, 128, "bf16", 7)
    res = hp.check_forward(t, dev, "bf16", scale_mult / math.sqrt(128), causal=True)
    print("peaky fwd", scale_mult, res)
    hp.assert_forward_ok(res)


def test_strided_layout_matches_packed():
    """[B,N,H,d] storage viewed as [B,H,N,d] gives the same result as the packed layout."""
    t, dev = hp.make_case(2, 3, 256, 64, "bf16", 11)
    kw = dict(softmax_scale=0.125, causal=True)
    O, L = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
    s = {k: v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for k, v in dev.items()}
    assert s["Q"].stride() != dev["Q"].stride()
    Os, Ls = binding.attn_fwd(s["Q"], s["K"], s["V"], **kw)
    torch.cuda.synchronize()
    assert torch.equal(O, Os) and torch.equal(L, Ls)


def test_forward_is_bitwise_reproducible():
    t, dev = hp.make_case(1, 4, 512, 128, "bf16", 13)
    kw = dict(softmax_scale=0.09, causal=False, dropout_p=0.1, seed=5, offset=1)
    O1, L1 = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
    O2, L2 = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(L1, L2)


def test_closed_forms_on_gpu():
    """Constant V gives O = V; causal row 0 equals V[0]; identical keys give the mean of V."""
    B, H, N, d = 1, 2, 256, 64
    t, dev = hp.make_case(B, H, N, d, "fp16", 17)
    Vc = dev["V"][:, :, :1, :].expand(B, H, N, d).contiguous()
    O, _ = binding.attn_fwd(dev["Q"], dev["K"], Vc, softmax_scale=0.125, o_fp32=True)
    assert (O - Vc.float()).abs().max().item() < 2e-3
    O, L = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], softmax_scale=0.125, causal=True, o_fp32=True)
    assert torch.equal(O[:, :, 0], dev["V"][:, :, 0].float())
    Kc = dev["K"][:, :, :1, :].expand(B, H, N, d).contiguous()
    O, L = binding.attn_fwd(dev["Q"], Kc, dev["V"], softmax_scale=0.125, o_fp32=True)
    mean = dev["V"].float().mean(dim=2, keepdim=True).expand(B, H, N, d)
    assert (O - mean).abs().max().item() < 2e-3


def test_prefix_property():
    """State after j K/V tiles equals attention over the first j tiles (Theorem 1's induction):
    attention over a key prefix, run as its own problem, matches the oracle on that prefix."""
    t, dev = hp.make_case(1, 1, 512, 64, "bf16", 19)
    for n in (128, 256, 384):
        sub_t = {k: v[:, :, :n] for k, v in t.items()}
        sub_d = {k: v[:, :, :n].contiguous() for k, v in dev.items()}
        res = hp.check_forward(sub_t, sub_d, "bf16", 0.125)
        hp.assert_forward_ok(res)


@pytest.mark.parametrize("N,d", [(640, 128), (1152, 64), (1280, 128)])
def test_causal_paired_row_blocks_odd_count(N, d):
    """Causal problems in the two-group kernel, where a work item is a pair of 256-row blocks: an odd
    number of blocks (the middle one stands alone) and a last block of only 128 valid rows."""
    t, dev = hp.make_case(1, 3, N, d, "bf16", 900 + N + d)
    res = hp.check_forward(t, dev, "bf16", 1 / math.sqrt(d), causal=True)
    print("causal pairs fwd", N, d, res)
    hp.assert_forward_ok(res)


@pytest.mark.gpu
def test_mfma_rate_probe_runs_and_reports_its_flops():
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    for dtype in ("fp16", "bf16"):
        for sets in (1, 4):
            flops = binding.attn_debug_mfma_rate(dtype, 100, sink, operand_sets=sets)
            assert flops == 2.0 * 32 * 32 * 16 * 4 * 100 * 4 * 2048
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0      # the sink is never written


@pytest.mark.gpu
@pytest.mark.parametrize("d,dtype", [(64, "bf16"), (128, "bf16"), (128, "fp16")])
@pytest.mark.parametrize("step", [0.02, 0.4, 3.0])
def test_logits_that_grow_along_the_keys(d, dtype, step):
    """The row maximum moves on every key tile: by a little (the softmax reference of the kernels then
    lags behind it for many tiles), by about its rescale threshold per tile, or by far more (a rescale
    on every tile).  Keys are a fixed direction scaled by the key index plus noise, so S_ij rises by
    about `step` per key (in units of the scaled logit).  Forward only: the backward kernels take the
    saved statistic L, checked here, and never see the reference."""
    B, H, N = 1, 2, 1024
    rng = np.random.default_rng(inputs.BASE_SEED + 1400 + d)
    u = rng.standard_normal(d)
    u /= np.linalg.norm(u)
    tau = 1 / math.sqrt(d)
    q = np.tile(u, (B, H, N, 1)) * 4.0 + 0.3 * rng.standard_normal((B, H, N, d))
    ramp = (np.arange(N) * step / (4.0 * tau))[None, None, :, None]
    k = u[None, None, None, :] * ramp + 0.3 * rng.standard_normal((B, H, N, d))
    v = rng.standard_normal((B, H, N, d))
    t = {n: inputs.round_to(x.astype(np.float32), dtype) for n, x in (("Q", q), ("K", k), ("V", v))}
    dev = {n: inputs.to_torch(x, dtype, "cuda") for n, x in t.items()}
    for causal in (False, True):
        res = hp.check_forward(t, dev, dtype, tau, causal=causal)
        print(d, dtype, step, causal, res)
        hp.assert_forward_ok(res)
