import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C ABI)")


def pytest_collection_modifyitems(config, items):
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


def pytest_generate_tests(metafunc):
    # Which kernel a call takes depends on the problem (head dimension, length, number of heads):
    # the small problems of the parity tests would never reach some kernels.  Test modules that ask
    # for these fixtures run every test twice: with the library's own choice, and with the other
    # kernel forced through the library's override hook.
    if "fwd_variant" in metafunc.fixturenames:
        metafunc.parametrize("fwd_variant", ["auto", "two_group"], indirect=True)
    if "dkv_variant" in metafunc.fixturenames:
        metafunc.parametrize("dkv_variant", ["auto", "role_split", "one_wave_32_keys", "one_wave_64_keys"], indirect=True)


@pytest.fixture
def fwd_variant(request):
    from paper_2205_14135_amd import binding
    binding.attn_debug_set_variant(fwd="pp" if request.param == "two_group" else "auto")   # ignored at d = 32 and for block-sparse calls
    yield request.param
    binding.attn_debug_set_variant(fwd="auto")


@pytest.fixture
def dkv_variant(request):
    from paper_2205_14135_amd import binding
    # ("fr" keeps the 64-keys-per-wavefront kernel of d = 128 out and takes the 32-key one also with
    # the causal mask and dropout together, which "auto" leaves to the role-split kernel; "w64" brings
    # the 64-key kernel in wherever it exists, so that both one-wavefront kernels are reached at every
    # length and under the causal mask)
    binding.attn_debug_set_variant(dkv={"role_split": "rs", "one_wave_32_keys": "fr", "one_wave_64_keys": "w64"}.get(request.param, "auto"))
    yield request.param
    binding.attn_debug_set_variant(dkv="auto")
