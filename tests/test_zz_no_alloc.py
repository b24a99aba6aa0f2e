"""attn_bwd_static (the backward entry point that allocates nothing) against attn_bwd.

Two calls in a row on the same stream, the second on a smaller problem: the built-in scratch is
shared by every call on a GPU and keeps the last call's contents, so the second call must not
read anything the first one left there.  Both are compared with attn_bwd on a caller-supplied
workspace bit for bit (the dense backward is deterministic), and the first also with the oracle."""
import ctypes
import math

import numpy as np
import pytest
import torch

from paper_2205_14135_amd import binding, inputs
from tests import helpers

pytestmark = pytest.mark.gpu


def _run_both(B, H, N, d, dtype, seed, causal, p):
    t, dev = helpers.make_case(B, H, N, d, dtype, seed)
    tau = 1 / math.sqrt(d)
    kw = dict(softmax_scale=tau, causal=causal, dropout_p=p, seed=inputs.BASE_DROPOUT_SEED + 3, offset=5)
    O, L = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
    want = binding.attn_bwd(dev["Q"], dev["K"], dev["V"], O, dev["dO"], L, **kw)
    # outputs are the caller's; poisoned so that rows the call skipped would show
    got = tuple(torch.full_like(dev["Q"], float("nan")) for _ in range(3))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    binding.attn_bwd_static(dev["Q"], dev["K"], dev["V"], O, dev["dO"], L, got, **kw)
    assert torch.cuda.memory_allocated() == before      # torch's allocator was not asked for anything
    torch.cuda.synchronize()
    for name, a, b in zip(("dQ", "dK", "dV"), got, want):
        assert torch.equal(a, b), name
    return t, dev, tau, kw, got


def test_static_scratch_backward_twice_second_smaller():
    # first call: several heads, ragged length (rows padded to whole blocks in the scratch), dropout
    t, dev, tau, kw, got = _run_both(2, 3, 600, 64, "bf16", inputs.BASE_SEED + 71, True, 0.1)
    res = helpers.check_backward(t, dev, "bf16", tau, causal=True, p=0.1, seed=kw["seed"], offset=kw["offset"],
                                 heads=[(0, 0), (1, 2)])
    helpers.assert_backward_ok(res)
    # second call, smaller and of another shape: lands on the stale contents of the first
    _run_both(1, 2, 200, 128, "fp16", inputs.BASE_SEED + 72, False, 0.0)
    # and a third at the first size again, after the small one
    _run_both(2, 3, 600, 64, "bf16", inputs.BASE_SEED + 71, True, 0.1)


def test_static_scratch_limit_is_enforced():
    lib = binding.load()
    p = binding.AttnParams()
    p.B, p.H, p.N, p.d = 64, 16, 1024 + 128, 64          # (2^20 + 2^17) rows: 9 MiB of row vectors
    p.dtype = binding.ATTN_BF16
    p.softmax_scale = 0.125
    assert lib.attn_bwd_workspace_bytes(ctypes.byref(p)) > binding.STATIC_SCRATCH_BYTES
    v = ctypes.c_void_p(0x1000)
    assert lib.attn_bwd_static(ctypes.byref(p), *([v] * 9)) == -7
    p.N = 1024                                           # exactly 8 MiB: accepted by the size check
    assert lib.attn_bwd_workspace_bytes(ctypes.byref(p)) == binding.STATIC_SCRATCH_BYTES
    assert lib.attn_bwd_static(ctypes.byref(p), *([v] * 8), ctypes.c_void_p(0)) == -1   # NULL dV, nothing launched
