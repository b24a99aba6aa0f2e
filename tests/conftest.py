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
    # kernel forced through the environment variables the launchers read on every call.
    if "fwd_variant" in metafunc.fixturenames:
        metafunc.parametrize("fwd_variant", ["auto", "two_group"], indirect=True)
    if "dkv_variant" in metafunc.fixturenames:
        metafunc.parametrize("dkv_variant", ["auto", "role_split"], indirect=True)


@pytest.fixture
def fwd_variant(request, monkeypatch):
    if request.param == "two_group":
        monkeypatch.setenv("ATTN_FWD_VARIANT", "pp")      # ignored at d = 32 and for block-sparse calls
    else:
        monkeypatch.delenv("ATTN_FWD_VARIANT", raising=False)
    return request.param


@pytest.fixture
def dkv_variant(request, monkeypatch):
    if request.param == "role_split":
        monkeypatch.setenv("ATTN_DKV_VARIANT", "rs")      # d = 128 takes that kernel anyway
    else:
        monkeypatch.delenv("ATTN_DKV_VARIANT", raising=False)
    return request.param
