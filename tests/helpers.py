"""Shared plumbing for the GPU parity tests: seeded inputs -> (HIP library, fp64 oracle)."""
from __future__ import annotations

import math

import numpy as np
import torch

from oracle import attention_oracle as orc
from paper_2205_14135_amd import binding, inputs

FWD_ATOL = 1e-2       # forward max-abs bar (fp16/bf16 inputs, fp32 accumulation)
GRAD_REL_L2 = 2e-2    # dQ/dK/dV relative-L2 bar
LSE_ATOL = 2e-3


def ulp_half(x: np.ndarray, dtype: str) -> np.ndarray:
    """Half a unit in the last place of the 16-bit output type at magnitude |x|."""
    mant = {"bf16": 8, "fp16": 11}[dtype]
    e = np.floor(np.log2(np.maximum(np.abs(x), 2.0 ** -14)))
    return 2.0 ** (e - mant)


def make_case(B, H, N, d, dtype, seed):
    t = inputs.gaussian_tensors(B, H, N, d, dtype, seed)
    dev = {k: inputs.to_torch(v, dtype, "cuda") for k, v in t.items()}
    return t, dev


def rel_l2(a: np.ndarray, b: np.ndarray) -> float:
    den = float(np.sqrt((b.astype(np.float64) ** 2).sum()))
    return float(np.sqrt(((a.astype(np.float64) - b) ** 2).sum())) / max(den, 1e-30)


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """x rounded to the nearest value of the 16-bit type (fp64 in, fp64 out)."""
    tdt = {"bf16": torch.bfloat16, "fp16": torch.float16}[dtype]
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float64)).to(tdt).double().numpy()


def vanishing_gradient_bounds(Qh, Kh, Vh, dOh, Oo, tau, alive, *, o_round=None, keep_scale=1.0):
    """Element-wise bounds on |dQ|, |dK|, |dV| of one head whose exact gradient is zero.

    alive: boolean [N, N], the entries that are visible (all masks) and, under dropout, kept.
    Where every row has at most one alive key, dS = P (dP - D) vanishes because the two length-d dot
    products dP_ij = dO_i . v_j (scaled by keep_scale under dropout) and D_i = dO_i . O_i are equal;
    a kernel computes both in fp32 (unit roundoff u = 2^-24) from exact products of 16-bit values, so
    by the standard bound for a recursive sum each is off by at most d u sum_k |dO_ik v_jk| (taken
    twice over for the keep_scale product and a different summation order).  When O was stored in a
    16-bit type (o_round), D also carries sum_k |dO_ik| |O_ik - round(O_ik)|.  P <= 1 (1.001 covers its
    own rounding), so |dS_ij| <= e_ij on the alive entries and the bounds are |dQ_i| <= tau sum_j e_ij
    |k_j| and |dK_j| <= tau sum_i e_ij |q_i|.  Without any alive entry every gradient, dV included,
    must be exactly zero (O = 0, hence D = 0 and dS = P (0 - 0)); with one, dV does not vanish (None)."""
    N, d = Qh.shape
    u = 2.0 ** -24
    aQ, aK, aV, adO = (np.abs(x.astype(np.float64)) for x in (Qh, Kh, Vh, dOh))
    alive = np.asarray(alive, dtype=bool)
    if not alive.any():
        return np.zeros((N, d)), np.zeros((N, d)), np.zeros((N, d))
    e = 4.0 * d * u * keep_scale * (adO @ aV.T)                             # [N, N]
    if o_round is not None:
        e = e + (adO * np.abs(Oo - round_to(Oo, o_round))).sum(axis=1, keepdims=True)
    e = 1.001 * e * alive
    bQ = tau * (e @ aK)
    # dK_j sums one term per query row; the rows' round-offs are independent, so beyond a few rows the
    # sum of absolute terms is replaced by six times their root-sum-square
    bK = tau * np.minimum(e.T @ aQ, 6.0 * np.sqrt((e.T ** 2) @ (aQ ** 2)))
    return bQ, bK, None


def alive_entries(N, *, causal=False, block_mask=None, key_length=None, keep=None):
    """Visible entries of a head (causal, block and key-padding masks) that dropout kept."""
    vis = orc.visible_mask(N, causal=causal, block_mask=block_mask, key_length=key_length)
    return vis if keep is None else vis & np.asarray(keep, dtype=bool)


def check_vanishing(name, got, want_norm, bounds):
    """True when the oracle's gradient `name` is zero; then `got` must stay within the round-off bound above."""
    if want_norm >= 1e-9:
        return False
    b = bounds[("dQ", "dK", "dV").index(name)]
    assert b is not None, name + ": the exact gradient vanishes where it should not"
    assert (np.abs(got) <= b).all(), (name, float(np.abs(got).max()), float(b.max()))
    return True


def _lengths_arg(key_lengths):
    return None if key_lengths is None else torch.tensor(list(key_lengths), dtype=torch.int32, device="cuda")


def check_forward(t, dev, dtype, tau, *, causal=False, p=0.0, seed=0, offset=0, block_mask=None,
                  heads=None, rows=None, key_lengths=None):
    """Runs fwd through the C ABI twice (dtype O and fp32 O) and compares with the oracle.

    heads: (b, h) pairs the oracle checks (default all); rows: query rows checked (default all).
    Returns a dict of error figures.
    """
    B, H, N, d = t["Q"].shape
    kw = dict(softmax_scale=tau, causal=causal, dropout_p=p, seed=seed, offset=offset,
              key_lengths=_lengths_arg(key_lengths))
    if block_mask is None:
        O, L = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
        O32, L32 = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], o_fp32=True, **kw)
    else:
        bm = torch.from_numpy(block_mask).cuda()
        O, L = binding.attn_blocksparse_fwd(dev["Q"], dev["K"], dev["V"], bm, **kw)
        O32, L32 = binding.attn_blocksparse_fwd(dev["Q"], dev["K"], dev["V"], bm, o_fp32=True, **kw)
    torch.cuda.synchronize()
    assert torch.equal(L, L32)
    O, O32, L = to_np(O), to_np(O32), to_np(L)
    heads = heads or [(b, h) for b in range(B) for h in range(H)]
    res = dict(o32=0.0, o=0.0, o_excess=0.0, lse=0.0)
    for b, h in heads:
        rr = np.arange(N) if rows is None else np.asarray(rows)
        keep = orc.dropout_keep_mask(b, h, H, N, p, seed, offset, rows=rr) if p > 0 else None
        bm_h = None if block_mask is None else (block_mask if block_mask.ndim == 2 else block_mask[h])
        Oo, Lo = orc.forward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], tau, causal=causal,
                                  p_drop=p, keep=keep, block_mask=bm_h, rows=rr,
                                  key_length=None if key_lengths is None else key_lengths[b])
        res["o32"] = max(res["o32"], float(np.abs(O32[b, h][rr] - Oo).max()))
        err = np.abs(O[b, h][rr] - Oo)
        res["o"] = max(res["o"], float(err.max()))
        res["o_excess"] = max(res["o_excess"], float((err - ulp_half(Oo, dtype)).max()))
        fin = np.isfinite(Lo)
        assert (np.isfinite(L[b, h][rr]) == fin).all()
        if fin.any():
            res["lse"] = max(res["lse"], float(np.abs(L[b, h][rr][fin] - Lo[fin]).max()))
        if (~fin).any():
            assert (O[b, h][rr][~fin] == 0).all()
    return res


def assert_forward_ok(res):
    # computed value (before the 16-bit output rounding) meets the bar outright
    assert res["o32"] <= FWD_ATOL, res
    # the 16-bit O meets it up to half a unit in the last place of the output type
    assert res["o_excess"] <= FWD_ATOL, res
    assert res["lse"] <= LSE_ATOL, res


def check_backward(t, dev, dtype, tau, *, causal=False, p=0.0, seed=0, offset=0, block_mask=None,
                   heads=None, o_fp32=False, key_lengths=None):
    """fwd + bwd through the C ABI; dQ, dK, dV compared per head with the oracle (relative L2)."""
    B, H, N, d = t["Q"].shape
    kw = dict(softmax_scale=tau, causal=causal, dropout_p=p, seed=seed, offset=offset, o_fp32=o_fp32,
              key_lengths=_lengths_arg(key_lengths))
    if block_mask is None:
        O, L = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
        g = binding.attn_bwd(dev["Q"], dev["K"], dev["V"], O, dev["dO"], L, **kw)
    else:
        bm = torch.from_numpy(block_mask).cuda()
        O, L = binding.attn_blocksparse_fwd(dev["Q"], dev["K"], dev["V"], bm, **kw)
        g = binding.attn_blocksparse_bwd(dev["Q"], dev["K"], dev["V"], O, dev["dO"], L, bm, **kw)
    torch.cuda.synchronize()
    g = [to_np(x) for x in g]
    heads = heads or [(b, h) for b in range(B) for h in range(H)]
    res = dict(dQ=0.0, dK=0.0, dV=0.0)
    for b, h in heads:
        keep = orc.dropout_keep_mask(b, h, H, N, p, seed, offset) if p > 0 else None
        bm_h = None if block_mask is None else (block_mask if block_mask.ndim == 2 else block_mask[h])
        klen = None if key_lengths is None else key_lengths[b]
        ref = orc.backward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], t["dO"][b, h], tau,
                                causal=causal, p_drop=p, keep=keep, block_mask=bm_h, key_length=klen)
        bounds = None
        for name, got, want in zip(("dQ", "dK", "dV"), g, ref):
            assert np.isfinite(got[b, h]).all(), name
            norm = float(np.sqrt((want ** 2).sum()))
            if norm < 1e-9:
                # the exact gradient vanishes (an empty sequence; a single visible key, where
                # dS = P (dP - D) = 0): a relative error is undefined, bound the round-off instead
                if bounds is None:
                    Oo, _ = orc.forward_head(t["Q"][b, h], t["K"][b, h], t["V"][b, h], tau, causal=causal,
                                             p_drop=p, keep=keep, block_mask=bm_h, key_length=klen)
                    bounds = vanishing_gradient_bounds(
                        t["Q"][b, h], t["K"][b, h], t["V"][b, h], t["dO"][b, h], Oo, tau,
                        alive_entries(N, causal=causal, block_mask=bm_h, key_length=klen, keep=keep),
                        o_round=None if o_fp32 else dtype,
                        keep_scale=1.0 / (1.0 - orc.dropout_effective_p(p)) if p > 0 else 1.0)
                check_vanishing(name, got[b, h], norm, bounds)
                continue
            res[name] = max(res[name], rel_l2(got[b, h], want))
    return res


def assert_backward_ok(res):
    for name in ("dQ", "dK", "dV"):
        assert res[name] <= GRAD_REL_L2, res
