"""Backward parity: dQ, dK, dV from the HIP library vs the fp64 oracle (relative L2 <= 2e-2)."""
import math

import numpy as np
import pytest
import torch

from tests import helpers as hp
from paper_2205_14135_amd import binding, inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _both_kernels(dkv_variant):
    """Every test of this module runs with the library's own kernel choice and with the other kernel forced."""


def test_c1_tiny_dense():
    t, dev = hp.make_case(1, 1, 128, 64, "fp16", inputs.BASE_SEED + 0)
    res = hp.check_backward(t, dev, "fp16", 1 / math.sqrt(64))
    print("C1 bwd", res)
    hp.assert_backward_ok(res)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("causal", [False, True])
def test_multi_tile_dense(dtype, d, causal):
    t, dev = hp.make_case(2, 2, 384, d, dtype, 200 + d + causal)
    res = hp.check_backward(t, dev, dtype, 1 / math.sqrt(d), causal=causal)
    print("multi-tile bwd", dtype, d, causal, res)
    hp.assert_backward_ok(res)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("causal", [False, True])
def test_dropout(d, causal):
    t, dev = hp.make_case(1, 3, 256, d, "bf16", 300 + d + causal)
    res = hp.check_backward(t, dev, "bf16", 1 / math.sqrt(d), causal=causal, p=0.1,
                            seed=inputs.BASE_DROPOUT_SEED + 7, offset=3)
    print("dropout bwd", d, causal, res)
    hp.assert_backward_ok(res)


def test_peaky_softmax_and_fp32_o():
    t, dev = hp.make_case(1, 2, 512, 128, "bf16", 31)
    res = hp.check_backward(t, dev, "bf16", 4 / math.sqrt(128), causal=True, o_fp32=True)
    print("peaky bwd", res)
    hp.assert_backward_ok(res)


def test_backward_is_bitwise_reproducible():
    t, dev = hp.make_case(1, 2, 512, 64, "bf16", 37)
    kw = dict(softmax_scale=0.125, causal=True, dropout_p=0.1, seed=3)
    O, L = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
    g1 = binding.attn_bwd(dev["Q"], dev["K"], dev["V"], O, dev["dO"], L, **kw)
    g2 = binding.attn_bwd(dev["Q"], dev["K"], dev["V"], O, dev["dO"], L, **kw)
    torch.cuda.synchronize()
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)


def test_workspace_is_linear_in_n():
    sizes = []
    for N in (128, 1024, 8192):
        q = torch.empty((2, 4, N, 64), dtype=torch.bfloat16, device="cuda")
        sizes.append(binding.attn_bwd_workspace_bytes(binding.make_params(q, 0.125)))
    assert sizes[1] == 8 * sizes[0] and sizes[2] == 8 * sizes[1]
    assert sizes[0] <= 2 * 4 * 128 * 64 * 2


@pytest.mark.parametrize("N,d", [(640, 128), (1152, 64), (896, 64)])
def test_causal_paired_blocks_odd_count(N, d):
    """Causal backward where work items pair a light and a heavy block (key blocks in the dK/dV
    kernel, row blocks in the dQ kernel at d = 64), with an odd number of 128-token blocks."""
    t, dev = hp.make_case(1, 3, N, d, "bf16", 950 + N + d)
    res = hp.check_backward(t, dev, "bf16", 1 / math.sqrt(d), causal=True)
    print("causal pairs bwd", N, d, res)
    hp.assert_backward_ok(res)


@pytest.mark.parametrize("N,causal,dtype", [(768, False, "bf16"), (1120, False, "fp16"), (1120, True, "bf16"),
                                            (2048, False, "bf16"), (544, True, "fp16")])
def test_d128_blocks_of_256_keys(N, causal, dtype):
    """Lengths that are whole 32-query tiles (the 64-keys-per-wavefront dK/dV kernel takes them when it
    is chosen or forced): whole and ragged 256-key blocks, tile counts that are and are not multiples
    of the three-buffer ring, the causal diagonal inside a wavefront's 64 keys."""
    t, dev = hp.make_case(1, 2, N, 128, dtype, 4100 + N + causal)
    res = hp.check_backward(t, dev, dtype, 1 / math.sqrt(128), causal=causal)
    print("256-key blocks bwd", N, causal, dtype, res)
    hp.assert_backward_ok(res)


@pytest.mark.parametrize("causal", [False, True])
def test_d128_blocks_of_256_keys_with_key_padding(causal):
    """Key padding on top: padded keys inside a wavefront's 64 keys, a key block that is all padding,
    an empty sequence."""
    t, dev = hp.make_case(4, 1, 1024, 128, "bf16", 4300 + causal)
    res = hp.check_backward(t, dev, "bf16", 1 / math.sqrt(128), causal=causal, key_lengths=[1024, 700, 130, 0])
    print("256-key blocks bwd, key padding", causal, res)
    hp.assert_backward_ok(res)
