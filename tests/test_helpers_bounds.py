"""The round-off bound that the GPU tests apply where the exact gradient vanishes (a single visible key:
dS = P (dP - D) = 0), checked on the CPU against a float32 emulation of what a kernel computes."""
import numpy as np
import pytest

from oracle import attention_oracle as orc
from tests import helpers as hp
from paper_2205_14135_amd import inputs


def _dot32(a, b, order):
    """Length-d dot product accumulated in float32 in the given order of terms (products exact in fp32
    for 16-bit operands, as in the matrix instruction)."""
    acc = np.float32(0.0)
    for k in order:
        acc = np.float32(acc + np.float32(np.float32(a[k]) * np.float32(b[k])))
    return acc


def _emulate_single_key(t, tau, dtype, keep_scale, o_factor=1.0):
    """dQ, dK of a head whose only visible key is key 0 (P = 1 in every row), the way a kernel does it:
    dP and D as float32 dot products in different orders, O read back from its 16-bit rounding."""
    Q, K, V, dO = (t[n][0, 0] for n in ("Q", "K", "V", "dO"))
    N, d = Q.shape
    O16 = hp.round_to(V[0].astype(np.float64) * keep_scale, dtype) * o_factor     # every row's output is v_0 * scale
    dQ = np.zeros((N, d)); dK = np.zeros((N, d))
    fwd, rev = list(range(d)), list(range(d - 1, -1, -1))
    for i in range(N):
        dp = np.float32(_dot32(dO[i], V[0], fwd) * np.float32(keep_scale))
        D = _dot32(dO[i], O16.astype(np.float32), rev)
        ds = float(np.float32(dp - D))
        dQ[i] = tau * ds * K[0].astype(np.float64)
        dK[0] += tau * ds * Q[i].astype(np.float64)
    return dQ, dK


@pytest.mark.parametrize("dtype,d,p", [("bf16", 64, 0.0), ("fp16", 128, 0.0), ("bf16", 128, 0.1), ("fp16", 64, 0.3)])
def test_bound_holds_for_a_float32_kernel_and_catches_a_wrong_row_term(dtype, d, p):
    N, tau = 96, 1.0 / np.sqrt(d)
    t = inputs.gaussian_tensors(1, 1, N, d, dtype, 4242 + d)
    scale = 1.0 / (1.0 - orc.dropout_effective_p(p)) if p > 0 else 1.0
    Q, K, V, dO = (t[n][0, 0] for n in ("Q", "K", "V", "dO"))
    Oo = np.tile(V[0].astype(np.float64) * scale, (N, 1))          # exact output of every row (all keys kept)
    alive = hp.alive_entries(N, key_length=None) & (np.arange(N)[None, :] == 0)      # key 0 only
    bQ, bK, bV = hp.vanishing_gradient_bounds(Q, K, V, dO, Oo, tau, alive, o_round=dtype, keep_scale=scale)
    assert bV is None                                              # dV does not vanish with a visible key
    dQ, dK = _emulate_single_key(t, tau, dtype, scale)
    assert (np.abs(dQ) <= bQ).all() and (np.abs(dK) <= bK).all()
    assert (bK[1:] == 0).all()                                     # invisible keys: exact zeros required
    # the bound is data dependent: of float32 round-off size when O = v_0 is exact in 16 bits (no dropout),
    # larger when the stored O = round16(scale v_0) differs from the exact one (Eq. (4) then carries that
    # rounding into D)
    if p == 0:
        assert bQ.max() < 2e-3
    # a row term computed from an O that is off by 2^-4 (a wrong scale, a stale buffer) breaks it
    dQ_bad, dK_bad = _emulate_single_key(t, tau, dtype, scale, o_factor=1.0 + 2.0 ** -4)
    assert (np.abs(dQ_bad) > bQ).any() and (np.abs(dK_bad) > bK).any()


def test_no_visible_key_means_exact_zeros():
    t = inputs.gaussian_tensors(1, 1, 8, 32, "bf16", 7)
    Q, K, V, dO = (t[n][0, 0] for n in ("Q", "K", "V", "dO"))
    bounds = hp.vanishing_gradient_bounds(Q, K, V, dO, np.zeros((8, 32)), 0.2, hp.alive_entries(8, key_length=0))
    assert all((b == 0).all() for b in bounds)
    assert hp.check_vanishing("dV", np.zeros((8, 32)), 0.0, bounds)
    with pytest.raises(AssertionError):
        hp.check_vanishing("dK", np.full((8, 32), 1e-9), 0.0, bounds)
