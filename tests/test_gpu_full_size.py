"""Parity at the benchmark configurations' full sizes, in the launch configuration bench.py times.

The oracle cannot materialise every head at these sizes in seconds, so each case checks whole
heads where that is cheap (N <= 2048) and otherwise sampled query rows (O, L, dQ depend on their
own row only) plus complete dK/dV for one head computed by the oracle in row chunks (the sum over
row chunks of the per-chunk contributions is the definition's sum over rows).
"""
import math

import numpy as np
import pytest
import torch

from oracle import attention_oracle as orc
from tests import helpers as hp
from paper_2205_14135_amd import binding, inputs

pytestmark = pytest.mark.gpu


def _run(dev, tau, cfg, bm=None):
    kw = dict(softmax_scale=tau, causal=cfg["causal"], dropout_p=cfg["p"], seed=cfg["seed"], offset=cfg["offset"])
    if bm is None:
        O, L = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
        g = binding.attn_bwd(dev["Q"], dev["K"], dev["V"], O, dev["dO"], L, **kw)
    else:
        O, L = binding.attn_blocksparse_fwd(dev["Q"], dev["K"], dev["V"], bm, **kw)
        g = binding.attn_blocksparse_bwd(dev["Q"], dev["K"], dev["V"], O, dev["dO"], L, bm, **kw)
    torch.cuda.synchronize()
    return O, L, g


def _check_rows(t, O, L, dQ, b, h, H, rows, tau, cfg, dtype, bm_np=None):
    N = t["Q"].shape[2]
    rows = np.asarray(rows)
    keep = orc.dropout_keep_mask(b, h, H, N, cfg["p"], cfg["seed"], cfg["offset"], rows=rows) if cfg["p"] > 0 else None
    kw = dict(causal=cfg["causal"], p_drop=cfg["p"], keep=keep, block_mask=bm_np, rows=rows)
    Oo, Lo = orc.forward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], tau, **kw)
    dQo, _, _ = orc.backward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], t["dO"][b, h], tau, **kw)
    idx = torch.from_numpy(rows).cuda()
    Og = hp.to_np(O[b, h].index_select(0, idx))
    Lg = hp.to_np(L[b, h].index_select(0, idx))
    dQg = hp.to_np(dQ[b, h].index_select(0, idx))
    err = np.abs(Og - Oo)
    assert (err - hp.ulp_half(Oo, dtype)).max() <= hp.FWD_ATOL, float(err.max())
    assert np.abs(Lg - Lo).max() <= hp.LSE_ATOL
    rel = hp.rel_l2(dQg, dQo)
    assert rel <= hp.GRAD_REL_L2, rel
    return float(err.max()), rel


def _check_dkv_chunked(t, g, b, h, H, tau, cfg, bm_np=None, chunk=2048):
    N, d = t["Q"].shape[2:]
    dK = np.zeros((N, d)); dV = np.zeros((N, d))
    for r0 in range(0, N, chunk):
        rows = np.arange(r0, min(N, r0 + chunk))
        keep = orc.dropout_keep_mask(b, h, H, N, cfg["p"], cfg["seed"], cfg["offset"], rows=rows) if cfg["p"] > 0 else None
        _, k, v = orc.backward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], t["dO"][b, h], tau,
                                    causal=cfg["causal"], p_drop=cfg["p"], keep=keep, block_mask=bm_np, rows=rows)
        dK += k; dV += v
    rk, rv = hp.rel_l2(hp.to_np(g[1][b, h]), dK), hp.rel_l2(hp.to_np(g[2][b, h]), dV)
    assert rk <= hp.GRAD_REL_L2 and rv <= hp.GRAD_REL_L2, (rk, rv)
    return rk, rv


def _sample_rows(N, seed, n=48):
    rng = np.random.default_rng(seed)
    fixed = [0, 1, 31, 32, 63, 64, 127, 128, N // 2 - 1, N // 2, N - 129, N - 128, N - 1]
    return np.unique(np.concatenate([fixed, rng.integers(0, N, n)]))


def test_c2_bert_large_shape():
    """B=16, H=16, N=512, d=64, fp16, non-causal, p=0.1."""
    cfg = dict(causal=False, p=0.1, seed=inputs.BASE_DROPOUT_SEED + 1, offset=0)
    t, dev = hp.make_case(16, 16, 512, 64, "fp16", inputs.BASE_SEED + 1)
    tau = 1 / math.sqrt(64)
    heads = [(0, 0), (7, 9), (15, 15)]
    res = hp.check_forward(t, dev, "fp16", tau, causal=False, p=0.1, seed=cfg["seed"], heads=heads)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "fp16", tau, causal=False, p=0.1, seed=cfg["seed"], heads=heads)
    hp.assert_backward_ok(resb)
    print("C2", res, resb)


@pytest.mark.parametrize("H,d", [(16, 64), (8, 128)])
def test_c3_gpt2_medium_shape(H, d):
    """B=8, N=1024, bf16, causal, p=0.1; d=64/H=16 and the d=128/H=8 variant."""
    seed = inputs.BASE_DROPOUT_SEED + 2
    t, dev = hp.make_case(8, H, 1024, d, "bf16", inputs.BASE_SEED + 2)
    tau = 1 / math.sqrt(d)
    heads = [(0, 0), (3, H // 2), (7, H - 1)]
    res = hp.check_forward(t, dev, "bf16", tau, causal=True, p=0.1, seed=seed, heads=heads)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "bf16", tau, causal=True, p=0.1, seed=seed, heads=heads)
    hp.assert_backward_ok(resb)
    print("C3", H, d, res, resb)


_grid_case = {}


def _grid_tensors(N, d):
    """One set of seeded tensors per (N, d) of the sweep, shared by its four (mask, scale) points
    (the parametrisation below keeps them adjacent, so one set is alive at a time)."""
    if _grid_case.get("key") != (N, d):
        _grid_case.clear()
        _grid_case["key"] = (N, d)
        _grid_case["val"] = hp.make_case(16384 // N, 16, N, d, "bf16", inputs.BASE_SEED + 3 + N + d)
    return _grid_case["val"]


def _check_whole_head(t, O, L, g, b, h, tau, cfg, dtype):
    Oo, Lo = orc.forward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], tau, causal=cfg["causal"])
    ref = orc.backward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], t["dO"][b, h], tau, causal=cfg["causal"])
    err = np.abs(hp.to_np(O[b, h]) - Oo)
    assert (err - hp.ulp_half(Oo, dtype)).max() <= hp.FWD_ATOL, float(err.max())
    assert np.abs(hp.to_np(L[b, h]) - Lo).max() <= hp.LSE_ATOL
    rels = [hp.rel_l2(hp.to_np(x[b, h]), w) for x, w in zip(g, ref)]
    assert max(rels) <= hp.GRAD_REL_L2, rels
    return float(err.max()), rels


def _check_gradient_identities(dev, g, causal):
    """Two consequences of the definitions that hold at any size, for every head at once.
    Rows of P sum to one, so the keys' dV = P^T dO add up to the queries' dO: sum_j dV_j = sum_i dO_i.
    dQ = tau dS K and dK = tau dS^T Q share dS, so trace(dQ Q^T) = trace(dK K^T) = tau sum_ij dS_ij s_ij.
    The 16-bit gradients carry independent relative errors of about 2^-9 (bf16 roundings of P, dS and of
    the outputs), which add up like a random walk to about 2^-9 of the root-sum-square of the summed
    terms; both identities are held to 2^-5 of it (ten such deviations; the maximum is over 32768
    sums).  A dropped or doubled tile of keys moves either sum by many times that."""
    dQ, dK, dV = (x.double() for x in g)
    Q, K, dO = (dev[n].double() for n in ("Q", "K", "dO"))
    lhs, rhs = dV.sum(dim=2), dO.sum(dim=2)                       # [B, H, d]
    unit = dV.pow(2).sum(dim=2).sqrt()                            # root-sum-square of the rounded terms
    worst_v = float(((lhs - rhs).abs() / unit).max())
    assert worst_v <= 2.0 ** -5, worst_v
    tq, tk = (dQ * Q).sum(dim=3), (dK * K).sum(dim=3)             # [B, H, N] per-token terms
    unit = (tq.pow(2).sum(dim=2) + tk.pow(2).sum(dim=2)).sqrt()
    worst_t = float(((tq.sum(dim=2) - tk.sum(dim=2)).abs() / unit).max())
    assert worst_t <= 2.0 ** -5, worst_t
    return worst_v, worst_t


C4_LENGTHS = (128, 256, 512, 1024, 2048, 4096, 8192, 16384)


@pytest.mark.parametrize("mult", [1.0, 4.0])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("N", C4_LENGTHS)
def test_c4_sweep_every_point(N, d, causal, mult):
    """All 64 sweep points (B*N = 16384, H = 16, bf16; with and without the causal mask; flat (x1) and
    peaky (x4) logits) in the launch configuration the sweep is timed in.  Up to N = 2048 two whole heads
    are compared with the oracle; beyond, sampled query rows of two heads (O, L, dQ depend on their own
    row only), and dK, dV through two identities over all heads (the complete dK/dV of one head at
    four long points is the next test's)."""
    B = 16384 // N
    cfg = dict(causal=causal, p=0.0, seed=0, offset=0)
    t, dev = _grid_tensors(N, d)
    tau = mult / math.sqrt(d)
    O, L, g = _run(dev, tau, cfg)
    for x in g:
        assert torch.isfinite(x.float()).all()
    ident = _check_gradient_identities(dev, g, causal)
    for (b, h) in [(0, 0), (B - 1, 15)]:
        if N <= 2048:
            out = _check_whole_head(t, O, L, g, b, h, tau, cfg, "bf16")
        else:
            out = _check_rows(t, O, L, g[0], b, h, 16, _sample_rows(N, N + h, n=16), tau, cfg, "bf16")
        print("C4", N, d, causal, mult, (b, h), out, ident)


@pytest.mark.parametrize("N,d,causal,mult", [
    (4096, 128, False, 1.0), (8192, 64, True, 1.0), (16384, 128, True, 4.0), (16384, 64, False, 1.0),
])
def test_c4_sweep_long_sequences(N, d, causal, mult):
    """Long sweep points: sampled rows of two heads for O, L, dQ; complete dK, dV of one head."""
    B = 16384 // N
    cfg = dict(causal=causal, p=0.0, seed=0, offset=0)
    t, dev = _grid_tensors(N, d)
    tau = mult / math.sqrt(d)
    O, L, g = _run(dev, tau, cfg)
    for (b, h) in [(0, 3), (B - 1, 15)]:
        e, r = _check_rows(t, O, L, g[0], b, h, 16, _sample_rows(N, N + h), tau, cfg, "bf16")
        print("C4 long rows", N, d, causal, mult, (b, h), e, r)
    rk, rv = _check_dkv_chunked(t, g, B - 1, 15, 16, tau, cfg)
    print("C4 long dK/dV", N, d, rk, rv)
    for x in g:
        assert torch.isfinite(x.float()).all()


def test_c5_blocksparse_16k():
    """B=1, H=8, d=64, bf16, N=16384, butterfly 128-block mask (1270 of 16384 blocks kept);
    the oracle applies the same mask densely."""
    N, H, d = 16384, 8, 64
    bm_np = inputs.butterfly_block_mask(N // 128)
    assert int(bm_np.sum()) == 1270
    cfg = dict(causal=False, p=0.0, seed=0, offset=0)
    t, dev = hp.make_case(1, H, N, d, "bf16", inputs.BASE_SEED + 4)
    tau = 1 / math.sqrt(d)
    O, L, g = _run(dev, tau, cfg, torch.from_numpy(bm_np).cuda())
    for h in (0, 7):
        e, r = _check_rows(t, O, L, g[0], 0, h, H, _sample_rows(N, h), tau, cfg, "bf16", bm_np)
        print("C5 16k rows", h, e, r)
    rk, rv = _check_dkv_chunked(t, g, 0, 5, H, tau, cfg, bm_np)
    print("C5 16k dK/dV", rk, rv)


def test_c5_blocksparse_64k():
    """N=65536 (6132 of 262144 blocks kept).  A query block only interacts with the key blocks its
    mask row keeps (all other entries are masked to exactly zero probability), so the oracle is run
    per query block on the gathered visible keys, without a mask, and its dK/dV contributions are
    scattered back: every output of one head is checked, plus sampled rows of another."""
    N, H, d = 65536, 8, 64
    T = N // 128
    bm_np = inputs.butterfly_block_mask(T)
    assert int(bm_np.sum()) == 6132
    cfg = dict(causal=False, p=0.0, seed=0, offset=0)
    t, dev = hp.make_case(1, H, N, d, "bf16", inputs.BASE_SEED + 5)
    tau = 1 / math.sqrt(d)
    O, L, g = _run(dev, tau, cfg, torch.from_numpy(bm_np).cuda())
    h = 6
    Q, K, V, dO = (t[n][0, h].astype(np.float64) for n in ("Q", "K", "V", "dO"))
    Oo = np.zeros((N, d)); Lo = np.zeros(N); dQo = np.zeros((N, d)); dKo = np.zeros((N, d)); dVo = np.zeros((N, d))
    for I in range(T):
        cols = np.flatnonzero(bm_np[I])
        kidx = (cols[:, None] * 128 + np.arange(128)[None, :]).reshape(-1)
        rs = slice(I * 128, (I + 1) * 128)
        r128 = np.arange(128)
        o, l = orc.forward_head(Q[rs], K[kidx], V[kidx], tau, rows=r128)
        dq, dk, dv = orc.backward_head(Q[rs], K[kidx], V[kidx], dO[rs], tau, rows=r128)
        Oo[rs], Lo[rs], dQo[rs] = o, l, dq
        np.add.at(dKo, kidx, dk)
        np.add.at(dVo, kidx, dv)
    err = np.abs(hp.to_np(O[0, h]) - Oo)
    assert (err - hp.ulp_half(Oo, "bf16")).max() <= hp.FWD_ATOL
    assert np.abs(hp.to_np(L[0, h]) - Lo).max() <= hp.LSE_ATOL
    rels = [hp.rel_l2(hp.to_np(x[0, h]), w) for x, w in zip(g, (dQo, dKo, dVo))]
    print("C5 64k head", h, float(err.max()), rels)
    assert max(rels) <= hp.GRAD_REL_L2
    # the dense-mask oracle on sampled rows of another head (cross-checks the gathered shortcut)
    rows = _sample_rows(N, 1, n=16)
    e, r = _check_rows(t, O, L, g[0], 0, 1, H, rows, tau, cfg, "bf16", bm_np)
    print("C5 64k rows", e, r)
