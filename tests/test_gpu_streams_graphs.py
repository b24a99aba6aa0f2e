"""The library allocates nothing and never synchronises: its calls can be captured into a HIP
graph and replayed, and issued from several host threads on streams of their own."""
import math
import threading

import pytest
import torch

from paper_2205_14135_amd import binding, inputs

pytestmark = pytest.mark.gpu


def _tensors(B, H, N, d, seed):
    t = inputs.gaussian_tensors(B, H, N, d, "bf16", seed)
    return {n: inputs.to_torch(t[n], "bf16", "cuda") for n in t}


def _eager(x, kw):
    O, L = binding.attn_fwd(x["Q"], x["K"], x["V"], **kw)
    g = binding.attn_bwd(x["Q"], x["K"], x["V"], O, x["dO"], L, **kw)
    torch.cuda.synchronize()
    return [O.clone(), L.clone()] + [y.clone() for y in g]


@pytest.mark.parametrize("p", [0.0, 0.1])
def test_forward_backward_replays_from_a_graph(p):
    B, H, N, d = 2, 4, 384, 64
    kw = dict(softmax_scale=1 / math.sqrt(d), causal=True, dropout_p=p, seed=41, offset=2)
    static = _tensors(B, H, N, d, inputs.BASE_SEED + 1300)
    O = torch.empty_like(static["Q"])
    L = torch.empty((B, H, N), dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty_like(static["Q"]) for _ in range(3))
    ws = torch.empty(binding.attn_bwd_workspace_bytes(binding.make_params(static["Q"], 1.0)), dtype=torch.uint8,
                     device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):     # the binding launches on torch's current stream: the capture stream
        binding.attn_fwd(static["Q"], static["K"], static["V"], out=O, lse=L, **kw)
        binding.attn_bwd(static["Q"], static["K"], static["V"], O, static["dO"], L, grads=grads, workspace=ws, **kw)
    for rep in range(3):              # new inputs before every replay, eager work in between
        fresh = _tensors(B, H, N, d, inputs.BASE_SEED + 1301 + rep)
        want = _eager(fresh, kw)
        for n in static:
            static[n].copy_(fresh[n])
        graph.replay()
        torch.cuda.synchronize()
        for got, w in zip([O, L, *grads], want):
            assert torch.equal(got, w), rep


def test_two_host_threads_on_their_own_streams():
    B, H, N, d = 2, 4, 512, 128
    kw = dict(softmax_scale=1 / math.sqrt(d), causal=False, dropout_p=0.0)
    cases = [_tensors(B, H, N, d, inputs.BASE_SEED + 1310 + i) for i in range(2)]
    want = [_eager(x, kw) for x in cases]
    got = [None, None]
    errors = []

    def worker(i):
        try:
            stream = torch.cuda.Stream()          # default priority
            with torch.cuda.stream(stream):
                out = None
                for _ in range(5):
                    x = cases[i]
                    O, L = binding.attn_fwd(x["Q"], x["K"], x["V"], **kw)
                    g = binding.attn_bwd(x["Q"], x["K"], x["V"], O, x["dO"], L, **kw)
                    out = [O, L, *g]
                stream.synchronize()
                got[i] = out
        except Exception as e:                    # surfaced in the main thread
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors
    torch.cuda.synchronize()
    for i in range(2):
        for a, b in zip(got[i], want[i]):
            assert torch.equal(a, b)
