"""fp64 CPU oracle for exact attention with scale, mask, dropout and a block mask.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP kernels are checked against.  It may be imported from tests/, from
__graft_entry__.smoke() and from bench.py's cpu_baseline leg, and from nowhere
else; it shares no code with the GPU path and imports nothing from the
package.  Every function here is pinned by the CPU tests (closed forms, brute
force, finite differences, published Philox known-answer vectors); nothing in
this file is "parity unpinned".

What is computed (per (batch, head) problem, everything in float64):

  forward   S = tau * Q K^T, masked entries set to -inf, P = softmax(S) row
            by row, P_dropped = P o Z, O = P_dropped V, and the per-row
            logsumexp L_i = m_i + ln(l_i) of the scaled, masked logits
            (paper: Section 2.2 / Algorithm 0 for the plain definition,
            Appendix B.3 for tau, MASK and dropout).
  backward  dV = P_dropped^T dO, dP_dropped = dO V^T, dP = dP_dropped o Z,
            dS_ij = P_ij (dP_ij - sum_l P_il dP_il), dQ = tau dS K,
            dK = tau dS^T Q (paper: Algorithm 3 "standard attention backward",
            with the dropout handling of Algorithm 4).  The row term is the
            plain sum over P o dP, not the dO.O shortcut of Eq. (4) in
            Appendix B.2, so the kernels' shortcut is cross-checked.

Readings of points the paper leaves open (each also listed in the design
notes of the repository):
  * batch and heads: B*H independent N x d problems, layout [B, H, N, d];
  * causal mask: key j is visible to query i iff j <= i;
  * block mask: entry (i, j) is visible iff block_mask[i // blk, j // blk] != 0
    (Section 3.3), and it is ANDed with the causal mask when both are given;
  * a row with no visible key yields O = 0, L = -inf and zero gradients;
  * key-padding mask: per-batch length; tokens at positions >= length neither attend nor are
    attended to (their O is 0, L is -inf, and every gradient at those positions is 0);
  * the saved statistic is one number per row, L = m + ln(l); P = exp(S - L)
    equals diag(l)^-1 exp(S - m) of Algorithm 4;
  * the dropout generator is Philox-4x32-10 (Salmon et al., SC'11), see
    dropout_keep_mask() for the exact keying.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "philox4x32_10",
    "dropout_threshold",
    "dropout_effective_p",
    "dropout_keep_mask",
    "visible_mask",
    "forward_head",
    "backward_head",
    "attention_forward",
    "attention_backward",
]

# ---------------------------------------------------------------------------
# Philox-4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
# as 1, 2, 3", SC'11).  Multipliers and Weyl key increments are the published
# constants.
# ---------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)
_SHIFT32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten rounds of Philox-4x32 on arrays of 32-bit counter words.

    c0..c3 are broadcastable integer arrays (the 128-bit counter, word 0
    first), k0/k1 Python ints (the 64-bit key, low word first).  Returns the
    four output words as uint32 arrays.
    """
    c0 = np.asarray(c0).astype(np.uint64) & _MASK32
    c1 = np.asarray(c1).astype(np.uint64) & _MASK32
    c2 = np.asarray(c2).astype(np.uint64) & _MASK32
    c3 = np.asarray(c3).astype(np.uint64) & _MASK32
    c0, c1, c2, c3 = np.broadcast_arrays(c0, c1, c2, c3)
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _PHILOX_M0 * c0          # 64-bit product of word 0
        p1 = _PHILOX_M1 * c2          # 64-bit product of word 2
        n0 = (p1 >> _SHIFT32) ^ c1 ^ np.uint64(k0)
        n1 = p1 & _MASK32
        n2 = (p0 >> _SHIFT32) ^ c3 ^ np.uint64(k1)
        n3 = p0 & _MASK32
        c0, c1, c2, c3 = n0, n1, n2, n3
        k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
        k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return (c0.astype(np.uint32), c1.astype(np.uint32),
            c2.astype(np.uint32), c3.astype(np.uint32))


def dropout_threshold(p_drop) -> int:
    """Integer threshold: an element is KEPT iff its 8-bit field >= threshold.

    The probability travels through the C interface as a float32, so the
    threshold is floor(double(float32(p)) * 2^8); the dropout actually applied
    has P(drop) = threshold / 2^8: p rounded down to a multiple of 1/256
    (dropout_effective_p), and kept entries are scaled by the reciprocal of the
    matching keep probability, so that E[Z] = 1 exactly.
    """
    p = float(np.float32(p_drop))
    if not (0.0 <= p < 1.0):
        raise ValueError("dropout probability must be in [0, 1)")
    return int(np.floor(p * 256.0))


def dropout_effective_p(p_drop) -> float:
    """The drop probability that is really applied: dropout_threshold / 256."""
    return dropout_threshold(p_drop) / 256.0


def dropout_keep_mask(b, h, H, N, p_drop, seed, offset, rows=None):
    """Boolean keep mask Z != 0 for head (b, h): shape [len(rows), N].

    Keying (a reading; the paper only says the generator state is saved and
    the mask regenerated, Appendix B.4 observation 1):
      key     = (seed & 0xffffffff, seed >> 32)
      counter = (j // 16, i, b * H + h, offset & 0xffffffff)
      element (i, j) uses the 8-bit field j % 16 of the 128-bit output: field f
      is byte f % 4 (bits [8 (f % 4), 8 (f % 4) + 7]) of output word f // 4;
      keep iff field >= threshold.
    One generator call therefore decides sixteen consecutive keys of a query.
    i is the query row and j the key column inside the head.  The mask depends
    on indices only: not on tiling, loop order, pass, or other masks.
    """
    if rows is None:
        rows = np.arange(N)
    rows = np.asarray(rows, dtype=np.int64)
    thr = dropout_threshold(p_drop)
    if thr == 0:
        return np.ones((rows.size, N), dtype=bool)
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    k0, k1 = seed & 0xFFFFFFFF, seed >> 32
    ngrp = (N + 15) // 16
    jg = np.arange(ngrp, dtype=np.int64)[None, :]
    ii = rows[:, None]
    w = philox4x32_10(jg, ii, b * H + h, int(offset) & 0xFFFFFFFF, k0, k1)
    words = np.stack(w, axis=-1).astype(np.uint32)                       # [rows, ngrp, 4]
    fields = np.stack([(words >> np.uint32(8 * k)) & np.uint32(0xFF) for k in range(4)], axis=-1)   # [rows, ngrp, 4, 4]
    fields = fields.reshape(rows.size, ngrp * 16)[:, :N]
    return fields >= np.uint32(thr)


def visible_mask(N, causal=False, block_mask=None, mask_block=128, rows=None, key_length=None):
    """Boolean [len(rows), N]: True where key j may be attended by query i.

    key_length (the key-padding mask named as the example of MASK in Appendix B.3): tokens at
    positions >= key_length are padding; they are neither attended to nor do they attend."""
    if rows is None:
        rows = np.arange(N)
    rows = np.asarray(rows, dtype=np.int64)
    vis = np.ones((rows.size, N), dtype=bool)
    j = np.arange(N, dtype=np.int64)[None, :]
    if key_length is not None:
        vis &= (j < int(key_length)) & (rows[:, None] < int(key_length))
    if causal:
        vis &= j <= rows[:, None]
    if block_mask is not None:
        bm = np.asarray(block_mask) != 0
        vis &= bm[(rows // mask_block)[:, None], j // mask_block]
    return vis


def _probabilities(Q, K, tau, vis):
    """S, row max, row sum and P = softmax(masked S); rows with no visible key give P = 0."""
    S = tau * (Q @ K.T)
    S = np.where(vis, S, -np.inf)
    m = S.max(axis=1)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    E = np.exp(S - m_safe[:, None])          # exp(-inf) = 0 at masked entries
    l = E.sum(axis=1)
    with np.errstate(divide="ignore", invalid="ignore"):
        P = np.where(l[:, None] > 0, E / l[:, None], 0.0)
        L = np.where(l > 0, m_safe + np.log(l), -np.inf)
    return P, L


def _dropout_factor(p_drop, keep, shape):
    """Z of Algorithm 4: 1/(1-p) where kept, 0 where dropped, with p the drop probability that
    is really applied (dropout_effective_p); all ones when that is 0."""
    p_eff = dropout_effective_p(p_drop)
    if p_eff > 0.0:
        if keep is None:
            raise ValueError("keep mask required when p_drop > 0")
        return np.where(keep, 1.0 / (1.0 - p_eff), 0.0)
    return np.ones(shape)


def forward_head(Q, K, V, tau, *, causal=False, p_drop=0.0, keep=None,
                 block_mask=None, mask_block=128, rows=None, return_p=False, key_length=None):
    """Forward for one head.  Q, K, V: [N, d].  keep: bool [len(rows), N] or None.

    rows: optional query indices; only those rows of O and L are computed and
    returned (each output row depends on its own query row only).
    Returns (O [R, d], L [R]) and, if return_p, also (P, Z), each [R, N].
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    N = K.shape[0]
    if rows is None:
        rows = np.arange(N)
    rows = np.asarray(rows, dtype=np.int64)
    vis = visible_mask(N, causal, block_mask, mask_block, rows, key_length)
    P, L = _probabilities(Q[rows], K, float(tau), vis)
    Z = _dropout_factor(p_drop, keep, P.shape)
    O = (P * Z) @ V
    if return_p:
        return O, L, P, Z
    return O, L


def backward_head(Q, K, V, dO, tau, *, causal=False, p_drop=0.0, keep=None,
                  block_mask=None, mask_block=128, rows=None, key_length=None):
    """Backward for one head: returns dQ [R, d], dK [N, d], dV [N, d].

    rows: optional query indices.  dQ is returned for those rows only, and dK,
    dV are then the contributions of those query rows alone (the full dK, dV
    are the sums over all rows); with rows=None everything is complete.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    tau = float(tau)
    N = K.shape[0]
    if rows is None:
        rows = np.arange(N)
    rows = np.asarray(rows, dtype=np.int64)
    vis = visible_mask(N, causal, block_mask, mask_block, rows, key_length)
    P, _ = _probabilities(Q[rows], K, tau, vis)
    Z = _dropout_factor(p_drop, keep, P.shape)
    dV = (P * Z).T @ dO[rows]
    dP = (dO[rows] @ V.T) * Z
    D = (P * dP).sum(axis=1)
    dS = P * (dP - D[:, None])
    dQ = tau * (dS @ K)
    dK = tau * (dS.T @ Q[rows])
    return dQ, dK, dV


def _head_block_mask(block_mask, b, h, H):
    if block_mask is None:
        return None
    bm = np.asarray(block_mask)
    if bm.ndim == 2:
        return bm
    if bm.ndim == 3:          # [H, T, T]
        return bm[h]
    raise ValueError("block_mask must be [T, T] or [H, T, T]")


def attention_forward(Q, K, V, tau, *, causal=False, p_drop=0.0, seed=0, offset=0,
                      block_mask=None, mask_block=128, heads=None, key_lengths=None):
    """Batched forward.  Q, K, V: [B, H, N, d] (any float dtype; widened exactly).

    heads: optional list of (b, h) pairs to compute; other heads are left NaN.
    Returns O [B, H, N, d] float64 and L [B, H, N] float64.
    """
    B, H, N, d = Q.shape
    O = np.full((B, H, N, d), np.nan)
    L = np.full((B, H, N), np.nan)
    todo = heads if heads is not None else [(b, h) for b in range(B) for h in range(H)]
    for b, h in todo:
        keep = dropout_keep_mask(b, h, H, N, p_drop, seed, offset) if p_drop > 0 else None
        O[b, h], L[b, h] = forward_head(
            Q[b, h], K[b, h], V[b, h], tau, causal=causal, p_drop=p_drop, keep=keep,
            block_mask=_head_block_mask(block_mask, b, h, H), mask_block=mask_block,
            key_length=None if key_lengths is None else key_lengths[b])
    return O, L


def attention_backward(Q, K, V, dO, tau, *, causal=False, p_drop=0.0, seed=0, offset=0,
                       block_mask=None, mask_block=128, heads=None, key_lengths=None):
    """Batched backward: returns dQ, dK, dV as float64 [B, H, N, d]."""
    B, H, N, d = Q.shape
    dQ = np.full((B, H, N, d), np.nan)
    dK = np.full((B, H, N, d), np.nan)
    dV = np.full((B, H, N, d), np.nan)
    todo = heads if heads is not None else [(b, h) for b in range(B) for h in range(H)]
    for b, h in todo:
        keep = dropout_keep_mask(b, h, H, N, p_drop, seed, offset) if p_drop > 0 else None
        dQ[b, h], dK[b, h], dV[b, h] = backward_head(
            Q[b, h], K[b, h], V[b, h], dO[b, h], tau, causal=causal, p_drop=p_drop, keep=keep,
            block_mask=_head_block_mask(block_mask, b, h, H), mask_block=mask_block,
            key_length=None if key_lengths is None else key_lengths[b])
    return dQ, dK, dV
