"""The torch.autograd front end: same numbers as the C-ABI calls it wraps, gradients that agree
with PyTorch's own autograd on a materialise-S attention (fp32), strided [B,N,H,d] views."""
import math

import pytest
import torch

from tests import helpers as hp
from paper_2205_14135_amd import binding, inputs
from paper_2205_14135_amd.autograd import flash_attention

pytestmark = pytest.mark.gpu


def _reference(q, k, v, tau, causal, keep=None, p=0.0):
    """Algorithm 0 of the paper in fp32 PyTorch ops (S and P materialised), differentiable."""
    q, k, v = (x.float() for x in (q, k, v))
    s = torch.matmul(q, k.transpose(-1, -2)) * tau
    if causal:
        n = s.shape[-1]
        s = s.masked_fill(torch.ones(n, n, dtype=torch.bool, device=s.device).triu(1), float("-inf"))
    pr = torch.softmax(s, dim=-1)
    if keep is not None:
        pr = pr * keep.float() / (1.0 - p)
    return torch.matmul(pr, v)


def _rel(a, b):
    return float((a.float() - b.float()).norm() / b.float().norm())


@pytest.mark.parametrize("causal,p,d", [(False, 0.0, 64), (True, 0.0, 64), (True, 0.2, 64), (True, 0.2, 16), (False, 0.0, 128)])
def test_gradients_match_pytorch_autograd(causal, p, d):
    B, H, N = 2, 3, 200     # N is not a multiple of the tile on purpose
    t = inputs.gaussian_tensors(B, H, N, d, "bf16", inputs.BASE_SEED + 1200)
    tau = 1 / math.sqrt(d)
    seed, offset = inputs.BASE_DROPOUT_SEED + 12, 7
    leaves = [inputs.to_torch(t[n], "bf16", "cuda").requires_grad_(True) for n in ("Q", "K", "V")]
    w = inputs.to_torch(t["dO"], "bf16", "cuda")
    out = flash_attention(*leaves, causal=causal, dropout_p=p, seed=seed, offset=offset)
    (out.float() * w.float()).sum().backward()
    got = [x.grad.clone() for x in leaves]
    keep = binding.attn_debug_dropout_mask(B, H, N, p, seed, offset).bool() if p > 0 else None
    ref_leaves = [x.detach().clone().requires_grad_(True) for x in leaves]
    ref = _reference(*ref_leaves, tau, causal, keep, p)
    (ref * w.float()).sum().backward()
    assert float((out.detach().float() - ref.detach()).abs().max()) <= hp.FWD_ATOL + 2.0 ** -8 * float(ref.detach().abs().max())
    for g, r in zip(got, ref_leaves):
        assert _rel(g, r.grad) <= hp.GRAD_REL_L2


def test_same_bits_as_the_c_abi_calls():
    B, H, N, d = 2, 2, 384, 128
    t = inputs.gaussian_tensors(B, H, N, d, "fp16", inputs.BASE_SEED + 1201)
    dev = {n: inputs.to_torch(t[n], "fp16", "cuda") for n in t}
    kw = dict(softmax_scale=0.09, causal=True, dropout_p=0.1, seed=99, offset=5)
    O, L = binding.attn_fwd(dev["Q"], dev["K"], dev["V"], **kw)
    want = binding.attn_bwd(dev["Q"], dev["K"], dev["V"], O, dev["dO"], L, **kw)
    leaves = [dev[n].clone().requires_grad_(True) for n in ("Q", "K", "V")]
    out = flash_attention(*leaves, **kw)
    out.backward(dev["dO"])
    assert torch.equal(out, O)
    for x, wnt in zip(leaves, want):
        assert torch.equal(x.grad, wnt)


def test_strided_views_of_a_token_major_tensor():
    """Models usually hold [B,N,H,d]; the [B,H,N,d] views of it (row stride H*d) are taken as they are."""
    B, H, N, d = 2, 4, 256, 64
    t = inputs.gaussian_tensors(B, H, N, d, "bf16", inputs.BASE_SEED + 1202)
    packed = {n: inputs.to_torch(t[n], "bf16", "cuda") for n in t}
    token_major = {n: packed[n].transpose(1, 2).contiguous() for n in packed}       # [B,N,H,d]
    views = [token_major[n].transpose(1, 2).requires_grad_(True) for n in ("Q", "K", "V")]
    assert views[0].stride() == (N * H * d, d, H * d, 1)
    out = flash_attention(*views, causal=True)
    out.backward(packed["dO"])          # a packed dO: the wrapper re-lays it out like q
    dense = [packed[n].clone().requires_grad_(True) for n in ("Q", "K", "V")]
    out2 = flash_attention(*dense, causal=True)
    out2.backward(packed["dO"])
    assert torch.equal(out, out2)
    for a, b in zip(views, dense):
        assert torch.equal(a.grad, b.grad)


def test_default_seed_follows_torch_manual_seed_and_block_mask_path():
    B, H, N, d = 1, 2, 512, 64
    t = inputs.gaussian_tensors(B, H, N, d, "bf16", inputs.BASE_SEED + 1203)
    q, k, v = (inputs.to_torch(t[n], "bf16", "cuda") for n in ("Q", "K", "V"))
    torch.manual_seed(1234)
    a = flash_attention(q, k, v, dropout_p=0.3)
    torch.manual_seed(1234)
    b = flash_attention(q, k, v, dropout_p=0.3)
    c = flash_attention(q, k, v, dropout_p=0.3)
    assert torch.equal(a, b) and not torch.equal(a, c)
    bm = torch.from_numpy(inputs.butterfly_block_mask(N // 128)).cuda()
    leaves = [x.clone().requires_grad_(True) for x in (q, k, v)]
    out = flash_attention(*leaves, block_mask=bm)
    out.sum().backward()
    O, L = binding.attn_blocksparse_fwd(q, k, v, bm, softmax_scale=1 / math.sqrt(d))
    assert torch.equal(out, O)
    assert all(torch.isfinite(x.grad.float()).all() for x in leaves)


def test_cpu_tensors_are_refused():
    x = torch.zeros(1, 1, 128, 64, dtype=torch.bfloat16)
    with pytest.raises(RuntimeError):
        flash_attention(x, x, x)
