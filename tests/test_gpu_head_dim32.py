"""Head dimension 32 (the paper's kernels cover 16 to 128, Appendix E.1): every kernel path against
the oracle."""
import math

import numpy as np
import pytest

from tests import helpers as hp
from paper_2205_14135_amd import inputs

pytestmark = pytest.mark.gpu
D = 32


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("causal", [False, True])
def test_dense(dtype, causal):
    t, dev = hp.make_case(2, 3, 640, D, dtype, inputs.BASE_SEED + 3200 + causal)
    tau = 1 / math.sqrt(D)
    res = hp.check_forward(t, dev, dtype, tau, causal=causal)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, dtype, tau, causal=causal)
    hp.assert_backward_ok(resb)
    print("d32 dense", dtype, causal, res, resb)


@pytest.mark.parametrize("causal", [False, True])
def test_dropout_and_key_padding(causal):
    lengths = [384, 200, 65]
    t, dev = hp.make_case(3, 2, 384, D, "bf16", inputs.BASE_SEED + 3210 + causal)
    tau = 1 / math.sqrt(D)
    kw = dict(causal=causal, p=0.2, seed=inputs.BASE_DROPOUT_SEED + 32, offset=1, key_lengths=lengths)
    res = hp.check_forward(t, dev, "bf16", tau, **kw)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "bf16", tau, **kw)
    hp.assert_backward_ok(resb)
    print("d32 dropout + lengths", causal, res, resb)


def test_blocksparse_with_a_heavy_column():
    """Butterfly mask at T = 64: column 0 keeps all 64 blocks and is split into segments."""
    N, T = 8192, 64
    bm = inputs.butterfly_block_mask(T)
    t, dev = hp.make_case(1, 2, N, D, "bf16", inputs.BASE_SEED + 3220)
    tau = 1 / math.sqrt(D)
    heads = [(0, 1)]
    rows = np.unique(np.concatenate([[0, 1, 127, 128, N - 1], np.random.default_rng(5).integers(0, N, 40)]))
    res = hp.check_forward(t, dev, "bf16", tau, block_mask=bm, heads=heads, rows=rows)
    hp.assert_forward_ok(res)
    resb = hp.check_backward(t, dev, "bf16", tau, block_mask=bm, heads=heads)
    hp.assert_backward_ok(resb)
    print("d32 block-sparse", res, resb)
