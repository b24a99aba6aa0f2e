#!/usr/bin/env python3
"""Benchmark of the attention hot path on one MI355X.

A "step" is one forward + one backward pass (attn_fwd, then attn_bwd) over one batch of the
workload.  Default workload: the d=128, N=4096 point of the sequence-length sweep (B*N = 16384
tokens, H=16, bf16, non-causal, no dropout).  Prints ONE JSON line:

  value     fwd+bwd TFLOP/s with FLOPs counted as 4*B*H*N^2*d (forward) + 2.5x that (backward),
            halved under a causal mask, kept blocks only for the block-sparse workloads;
  roofline  the dominant kernel of the step against the MI355X dense bf16/fp16 MFMA peak,
            its duration measured with HIP events recorded on the launch stream;
  cpu_baseline  the fp64 oracle timed on this machine's host cores on a bounded sample.

Other workloads (--workload) exist for profiling and for the sweep table (--sweep).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "fp16": 2500.0}   # MI355X dense MFMA peak
PEAK_HBM_GBPS = 8000.0
ROTATING_SETS = 4      # separate copies of all tensors for the cache-cold timing (>= 1 GiB in total)


def workloads():
    w = {}
    for n in (128, 256, 512, 1024, 2048, 4096, 8192, 16384):
        for d in (64, 128):
            for causal in (False, True):
                name = f"sweep_N{n}_d{d}" + ("_causal" if causal else "")
                w[name] = dict(B=16384 // n, H=16, N=n, d=d, dtype="bf16", causal=causal, p=0.0, sparse=False)
    w["bert_large"] = dict(B=16, H=16, N=512, d=64, dtype="fp16", causal=False, p=0.1, sparse=False)
    w["gpt2_medium"] = dict(B=8, H=16, N=1024, d=64, dtype="bf16", causal=True, p=0.1, sparse=False)
    w["gpt2_medium_d128"] = dict(B=8, H=8, N=1024, d=128, dtype="bf16", causal=True, p=0.1, sparse=False)
    w["blocksparse_N16384"] = dict(B=1, H=8, N=16384, d=64, dtype="bf16", causal=False, p=0.0, sparse=True)
    w["blocksparse_N65536"] = dict(B=1, H=8, N=65536, d=64, dtype="bf16", causal=False, p=0.0, sparse=True)
    return w


DEFAULT_WORKLOAD = "sweep_N4096_d128"


class HipEvents:
    """hipEvent_t handles through the HIP runtime's C API (timing on the launch stream)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.all = []

    def new(self) -> int:
        e = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(e))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        self.all.append(e.value)
        return e.value

    def record(self, ev: int, stream: int):
        rc = self.hip.hipEventRecord(ctypes.c_void_p(ev), ctypes.c_void_p(stream))
        if rc != 0:
            raise RuntimeError(f"hipEventRecord failed: {rc}")

    def elapsed_ms(self, a: int, b: int) -> float:
        self.hip.hipEventSynchronize(ctypes.c_void_p(b))
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), ctypes.c_void_p(a), ctypes.c_void_p(b))
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(ms.value)

    def close(self):
        for e in self.all:
            self.hip.hipEventDestroy(ctypes.c_void_p(e))
        self.all = []


def flops_fwd(cfg, nnz_blocks=None):
    if cfg["sparse"]:
        return 4.0 * cfg["B"] * cfg["H"] * nnz_blocks * 128 * 128 * cfg["d"]
    f = 4.0 * cfg["B"] * cfg["H"] * cfg["N"] ** 2 * cfg["d"]
    return f * (0.5 if cfg["causal"] else 1.0)


def io_bytes(cfg):
    """Minimum HBM bytes of the forward and of the backward pass: every input read once, every
    output written once (forward: Q, K, V in, O and the row statistic out; backward: Q, K, V, O, dO
    and the row statistic in, dQ, dK, dV out)."""
    rows = cfg["B"] * cfg["H"] * cfg["N"]
    elem = rows * cfg["d"] * 2
    return 4 * elem + 4 * rows, 8 * elem + 4 * rows


def run_gpu(cfg, steps, warmup, seed, mask_override=None, nsets=1):
    """Times `steps` forward+backward passes.  nsets > 1 rotates over that many separate copies of
    all inputs and outputs, so that no step finds its tensors in the 256 MB last-level cache."""
    import numpy as np
    import torch
    from paper_2205_14135_amd import binding, inputs

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    B, H, N, d = cfg["B"], cfg["H"], cfg["N"], cfg["d"]
    t = inputs.gaussian_tensors(B, H, N, d, cfg["dtype"], seed)
    g0 = {k: inputs.to_torch(v, cfg["dtype"], dev) for k, v in t.items()}
    tau = 1.0 / math.sqrt(d)
    kw = dict(softmax_scale=tau, causal=cfg["causal"], dropout_p=cfg["p"],
              seed=inputs.BASE_DROPOUT_SEED, offset=0)
    bm = bm_np = None
    nnz = None
    if cfg["sparse"]:
        bm_np = inputs.butterfly_block_mask(N // 128) if mask_override is None else mask_override
        bm = torch.from_numpy(bm_np).to(dev)
        nnz = int(bm_np.sum())
    sets = []
    for i in range(nsets):
        g = g0 if i == 0 else {k: v.clone() for k, v in g0.items()}
        sets.append(dict(g=g, O=torch.empty_like(g["Q"]),
                         L=torch.empty((B, H, N), dtype=torch.float32, device=dev),
                         grads=tuple(torch.empty_like(g["Q"]) for _ in range(3))))
    pp = binding.make_params(g0["Q"], tau)
    ws_bytes = binding.attn_blocksparse_bwd_workspace_bytes(pp) if cfg["sparse"] else binding.attn_bwd_workspace_bytes(pp)
    ws = torch.empty(max(256, ws_bytes), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    hev = HipEvents()

    def fwd(z):
        g = z["g"]
        if bm is None:
            binding.attn_fwd(g["Q"], g["K"], g["V"], out=z["O"], lse=z["L"], **kw)
        else:
            binding.attn_blocksparse_fwd(g["Q"], g["K"], g["V"], bm, out=z["O"], lse=z["L"], **kw)

    def bwd(z):      # the product call
        g = z["g"]
        if bm is None:
            binding.attn_bwd(g["Q"], g["K"], g["V"], z["O"], g["dO"], z["L"], grads=z["grads"], workspace=ws, **kw)
        else:
            binding.attn_blocksparse_bwd(g["Q"], g["K"], g["V"], z["O"], g["dO"], z["L"], bm, grads=z["grads"],
                                         workspace=ws, **kw)

    def bwd_timed(z, events):      # the same launches with events between them, for the per-kernel figures
        g = z["g"]
        binding.attn_bwd_timed(g["Q"], g["K"], g["V"], z["O"], g["dO"], z["L"], events, block_mask=bm,
                               grads=z["grads"], workspace=ws, **kw)

    for i in range(max(warmup, nsets)):     # every set needs its O and row statistic before a backward
        fwd(sets[i % nsets])
        bwd(sets[i % nsets])
    torch.cuda.synchronize()
    # ---- the timed region: `steps` forward + backward passes through attn_fwd / attn_bwd; the only
    # extra work on the stream is one event record before and after each pass
    evs = [[hev.new() for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        e = evs[s]
        z = sets[s % nsets]
        hev.record(e[0], stream)
        fwd(z)
        hev.record(e[1], stream)
        bwd(z)
        hev.record(e[2], stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    fwd_steps = np.array([hev.elapsed_ms(e[0], e[1]) for e in evs])
    bwd_steps = np.array([hev.elapsed_ms(e[1], e[2]) for e in evs])
    stats = dict(fwd_mean=float(fwd_steps.mean()), fwd_median=float(np.median(fwd_steps)), fwd_min=float(fwd_steps.min()),
                 bwd_mean=float(bwd_steps.mean()), bwd_median=float(np.median(bwd_steps)), bwd_min=float(bwd_steps.min()))
    # ---- a second pass for the per-kernel durations (attn_bwd_timed records events between the
    # launches of the backward pass); the kernels are named by the library's own choice
    pk = binding.make_params(g0["Q"], tau, cfg["causal"], cfg["p"], inputs.BASE_DROPOUT_SEED, 0)
    n_fwd, n_dkv = binding.attn_debug_kernel_choice(pk, cfg["sparse"])
    names = [n_fwd, "dq_kernel", n_dkv]
    kevs = [[hev.new() for _ in range(5)] for _ in range(steps)]   # f0, f1=b0, b1, b2, b3
    for s in range(steps):
        e = kevs[s]
        z = sets[s % nsets]
        hev.record(e[0], stream)
        fwd(z)
        bwd_timed(z, e[1:5])
    torch.cuda.synchronize()
    # events: e[0] before the forward, e[1] = e[2] before the backward, e[3] after dQ, e[4] after dK/dV
    spans = [(0, 1), (1, 3), (3, 4)]
    dur = {n: sum(hev.elapsed_ms(e[i0], e[i1]) for e in kevs) / steps for (i0, i1), n in zip(spans, names)}
    hev.close()
    peak_bytes = torch.cuda.max_memory_allocated(dev)
    return dict(ms_per_step=wall_ms / steps, kernel_ms=dur, names=names, nnz=nnz, tensors=t, block_mask=bm_np, tau=tau,
                peak_bytes=peak_bytes, stats=stats)


def measured_mfma_rate(dtype, operand_sets=1):
    """TFLOP/s of a kernel that only issues matrix instructions on register operands: what this
    GPU sustains at the clock it holds under that load (the published peak assumes 2.4 GHz).
    operand_sets = 1: the same two registers every time; 4: four pseudo-random operand pairs in
    turn (more bits change per instruction, the clock the GPU holds is lower)."""
    import torch
    from paper_2205_14135_amd import binding
    dev = torch.device("cuda:0")
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    hev = HipEvents()
    binding.attn_debug_mfma_rate(dtype, 2000, sink, operand_sets)
    torch.cuda.synchronize()
    e = [hev.new() for _ in range(4)]
    flops = 0.0
    for i in range(3):
        hev.record(e[i], stream)
        flops = binding.attn_debug_mfma_rate(dtype, 20000, sink, operand_sets)
    hev.record(e[3], stream)
    torch.cuda.synchronize()
    ms = hev.elapsed_ms(e[0], e[3]) / 3
    hev.close()
    return flops / ms * 1e-9


def sparsity_sweep(steps):
    """Runtime of the block-sparse path against the fraction of kept 128x128 blocks (the shape
    of Fig. 2, right: N = 4096; here B=4, H=16, d=128, bf16), random masks that keep the diagonal,
    next to the dense kernels on the same inputs.  One JSON line per density on stderr."""
    import numpy as np
    from paper_2205_14135_amd import inputs
    base = dict(B=4, H=16, N=4096, d=128, dtype="bf16", causal=False, p=0.0)
    T = base["N"] // 128
    dense = run_gpu(dict(base, sparse=False), steps, 2, inputs.BASE_SEED + 3)
    dk = [dense["kernel_ms"][n] for n in dense["names"]]
    print(json.dumps(dict(density=None, kernel="dense", fwd_ms=round(dk[0], 4), bwd_ms=round(sum(dk[1:]), 4))),
          file=sys.stderr, flush=True)
    rng = np.random.default_rng(inputs.BASE_SEED + 77)
    for dens in (0.05, 0.1, 0.2, 0.4, 0.6, 0.8, 1.0):
        m = (rng.random((T, T)) < dens).astype(np.uint8)
        np.fill_diagonal(m, 1)
        r = run_gpu(dict(base, sparse=True), steps, 2, inputs.BASE_SEED + 3, mask_override=m)
        k = [r["kernel_ms"][n] for n in r["names"]]
        frac = float(m.mean())
        print(json.dumps(dict(density=round(frac, 4), kept_blocks=int(m.sum()), fwd_ms=round(k[0], 4),
                              bwd_ms=round(sum(k[1:]), 4),
                              fwd_ms_per_density=round(k[0] / frac, 4), bwd_ms_per_density=round(sum(k[1:]) / frac, 4))),
              file=sys.stderr, flush=True)


def dropout_cost(wl, steps, warmup):
    """Each dropout workload with its dropout and with p = 0 at the same shape: per-kernel times and their
    ratios (Appendix E.6 of the paper tabulates the same pair of settings)."""
    from paper_2205_14135_amd import inputs
    for name in ("bert_large", "gpt2_medium", "gpt2_medium_d128"):
        c = wl[name]
        with_p = run_gpu(c, steps, warmup, inputs.BASE_SEED + 3)
        without = run_gpu(dict(c, p=0.0), steps, warmup, inputs.BASE_SEED + 3)
        k1 = [with_p["kernel_ms"][n] for n in with_p["names"]]
        k0 = [without["kernel_ms"][n] for n in without["names"]]
        line = dict(workload=name, p=c["p"], kernels=with_p["names"], kernels_without=without["names"],
                    ms=[round(x, 4) for x in k1], ms_without=[round(x, 4) for x in k0],
                    ratio=[round(a / b, 3) for a, b in zip(k1, k0)],
                    fwd_ratio=round(k1[0] / k0[0], 3), bwd_ratio=round(sum(k1[1:]) / sum(k0[1:]), 3),
                    step_ratio=round(sum(k1) / sum(k0), 3),
                    ms_per_step=round(with_p["ms_per_step"], 4), ms_per_step_without=round(without["ms_per_step"], 4),
                    wall_ratio=round(with_p["ms_per_step"] / without["ms_per_step"], 3))
        print(json.dumps(line), file=sys.stderr, flush=True)


def memory_and_naive(steps):
    """Device memory and time of this library against a plain materialise-S attention written with
    PyTorch ops (Algorithm 0 of the paper: S = QK^T, P = softmax(S), O = PV, autograd backward),
    H=16, d=128, bf16, B*N = 16384 tokens.  PyTorch is used here as the comparison system only.
    One JSON line per N on stderr."""
    import torch
    from paper_2205_14135_amd import inputs
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    torch.zeros(1, device=dev)      # initialises the allocator before its statistics are reset
    for n in (512, 1024, 2048, 4096, 8192):
        cfg = dict(B=16384 // n, H=16, N=n, d=128, dtype="bf16", causal=False, p=0.0, sparse=False)
        torch.cuda.empty_cache()
        torch.cuda.reset_peak_memory_stats(dev)
        base_alloc = torch.cuda.memory_allocated(dev)
        r = run_gpu(cfg, steps, 2, inputs.BASE_SEED + 3)
        ours_peak = r["peak_bytes"] - base_alloc
        ours_ms = sum(r["kernel_ms"].values())
        io_bytes = 8 * cfg["B"] * cfg["H"] * n * 128 * 2          # Q K V dO O dQ dK dV
        del r
        torch.cuda.empty_cache()
        g = {k: torch.randn(cfg["B"], 16, n, 128, device=dev, dtype=torch.bfloat16, requires_grad=(k != "dO"))
             for k in ("Q", "K", "V", "dO")}
        tau = 1.0 / math.sqrt(128)

        def naive():
            S = torch.matmul(g["Q"], g["K"].transpose(-1, -2)) * tau
            P = torch.softmax(S, dim=-1)
            O = torch.matmul(P, g["V"])
            O.backward(g["dO"])
            for k in ("Q", "K", "V"):
                g[k].grad = None
        naive()
        torch.cuda.synchronize()
        torch.cuda.reset_peak_memory_stats(dev)
        before = torch.cuda.memory_allocated(dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            naive()
        e1.record()
        torch.cuda.synchronize()
        naive_ms = e0.elapsed_time(e1) / steps
        naive_extra = torch.cuda.max_memory_allocated(dev) - before
        print(json.dumps(dict(N=n, B=cfg["B"], tensors_MiB=round(io_bytes / 2**20, 1),
                              ours_extra_MiB=round((ours_peak - io_bytes) / 2**20, 1),
                              naive_extra_MiB=round(naive_extra / 2**20, 1),
                              ours_fwd_bwd_ms=round(ours_ms, 4), naive_fwd_bwd_ms=round(naive_ms, 4),
                              speedup=round(naive_ms / ours_ms, 2))), file=sys.stderr, flush=True)
        del g


def naive_steps(cfg, steps):
    """Algorithm 0 of the paper with PyTorch ops (S and P written to and read from HBM), forward and
    autograd backward, at the shape of a dense workload: run under rocprofv3 to count its HBM bytes."""
    import torch
    dev = torch.device("cuda:0")
    dt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float16
    shape = (cfg["B"], cfg["H"], cfg["N"], cfg["d"])
    torch.manual_seed(0)
    g = {k: torch.randn(shape, device=dev, dtype=dt, requires_grad=(k != "dO")) for k in ("Q", "K", "V", "dO")}
    tau = 1.0 / math.sqrt(cfg["d"])
    causal = None
    if cfg["causal"]:
        causal = torch.ones(cfg["N"], cfg["N"], dtype=torch.bool, device=dev).triu(1)
    for _ in range(steps):
        S = torch.matmul(g["Q"], g["K"].transpose(-1, -2)) * tau
        if causal is not None:
            S = S.masked_fill(causal, float("-inf"))
        P = torch.softmax(S, dim=-1)
        if cfg["p"] > 0:
            P = torch.nn.functional.dropout(P, cfg["p"])
        O = torch.matmul(P, g["V"])
        O.backward(g["dO"])
        for k in ("Q", "K", "V"):
            g[k].grad = None
    torch.cuda.synchronize()
    print(json.dumps({"naive_steps": steps, "shape": list(shape), "dtype": cfg["dtype"]}))


def cpu_baseline(cfg, run, budget_s=12.0, max_s=30.0):
    """Times the fp64 oracle (forward + backward of whole heads) on the host cores."""
    import numpy as np
    from oracle import attention_oracle as orc
    from paper_2205_14135_amd import inputs
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    t, tau = run["tensors"], run["tau"]
    B, H, N, d = cfg["B"], cfg["H"], cfg["N"], cfg["d"]
    chunk = 2048 if N > 8192 else N      # row chunks keep the N x N temporaries in memory
    heads_done, partial = 0, 0.0
    t0 = time.perf_counter()
    for b, h in [(b, h) for b in range(B) for h in range(H)]:
        q, k, v, do = (t[n][b, h].astype(np.float64) for n in ("Q", "K", "V", "dO"))
        aborted = False
        for r0 in range(0, N, chunk):
            rows = np.arange(r0, min(N, r0 + chunk))
            keep = (orc.dropout_keep_mask(b, h, H, N, cfg["p"], inputs.BASE_DROPOUT_SEED, 0, rows=rows)
                    if cfg["p"] > 0 else None)
            kws = dict(causal=cfg["causal"], p_drop=cfg["p"], keep=keep, block_mask=run["block_mask"], rows=rows)
            orc.forward_head(q, k, v, tau, **kws)
            orc.backward_head(q, k, v, do, tau, **kws)
            partial = min(1.0, (r0 + chunk) / N)
            if time.perf_counter() - t0 > max_s and partial < 1.0:
                aborted = True
                break
        if aborted:
            break
        heads_done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    el = time.perf_counter() - t0
    if heads_done == 0:
        per_head = el / partial
        sample = f"{partial:.3f} of head (0,0) in row chunks of {chunk}, extrapolated to one head"
    else:
        per_head = el / heads_done
        sample = f"{heads_done} of {B * H} heads, forward+backward each"
    nnz = run["nnz"]
    fl_head = 3.5 * flops_fwd(cfg, nnz) / (B * H)
    return dict(value=fl_head / per_head * 1e-12, unit="TFLOP/s", cores=int(threads), kind="oracle",
                sample=sample, seconds=round(el, 2))


def load_traffic(workload, kernel):
    """HBM bytes per launch of this kernel on this workload from the committed rocprofv3 counter
    runs (profiles/hbm_traffic.json, written from the FETCH_SIZE / WRITE_SIZE runs whose summary is
    profiles/<workload>_hbm_counters.txt): None unless that kernel was recorded for that workload."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    try:
        with open(path) as f:
            tab = json.load(f)
        return tab.get(workload, {}).get(kernel)
    except Exception:
        return None


def kernel_bytes(cfg):
    """Minimum HBM bytes per launch of the three kernels: forward reads Q, K, V and writes O and the
    row statistic; the dQ kernel reads Q, K, V, O, dO and the statistic and writes dQ and the two row
    vectors; the dK/dV kernel reads Q, K, V, dO and the row vectors and writes dK, dV."""
    rows = cfg["B"] * cfg["H"] * cfg["N"]
    elem = rows * cfg["d"] * 2
    return [4 * elem + 4 * rows, 6 * elem + 12 * rows, 6 * elem + 8 * rows]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true", help="also time every sweep point (extra JSON lines on stderr)")
    ap.add_argument("--sparsity-sweep", action="store_true",
                    help="only: block-sparse runtime against mask density at N=4096 (JSON lines on stderr)")
    ap.add_argument("--memory-table", action="store_true",
                    help="only: memory and time against a materialise-S attention in PyTorch ops (JSON lines on stderr)")
    ap.add_argument("--naive-steps", type=int, default=0,
                    help="only: run this many forward+backward steps of a materialise-S attention in PyTorch ops at the "
                         "workload's shape (comparison system for the HBM byte counters)")
    ap.add_argument("--dropout-p", type=float, default=None,
                    help="override the workload's dropout probability (0 switches dropout off at the same shape)")
    ap.add_argument("--dropout-cost", action="store_true",
                    help="only: the three dropout workloads timed with their dropout and with none (JSON lines on stderr)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a 1 GiB elementwise copy kernel (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; every (batch, head) problem is independent, so N GPUs "
              "would each take B*H/N heads with no communication. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    wl = workloads()
    if args.workload not in wl:
        print("unknown workload; choose from: " + ", ".join(sorted(wl)), file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")     # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)     # an ordinary elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4, "launches": 3}))
        return
    if args.naive_steps > 0:
        cfg = wl[args.workload]
        naive_steps(cfg, args.naive_steps)
        return
    from paper_2205_14135_amd import binding, inputs
    binding.load()
    if args.dropout_p is not None:
        for c in wl.values():
            c["p"] = args.dropout_p
    if args.sparsity_sweep:
        sparsity_sweep(max(3, args.steps // 3))
        return
    if args.dropout_cost:
        dropout_cost(wl, args.steps, args.warmup)
        return
    if args.memory_table:
        memory_and_naive(max(3, args.steps // 3))
        return

    if args.sweep:
        sweep_steps = max(3, args.steps // 3)
        for name in sorted(wl):
            c = wl[name]
            r = run_gpu(c, sweep_steps, 2, inputs.BASE_SEED + 3)
            f = flops_fwd(c, r["nnz"])
            nnz_blocks = r["nnz"]
            k = [r["kernel_ms"][n] for n in r["names"]]
            fwd_ms, bwd_ms = k[0], sum(k[1:])
            by_f, by_b = io_bytes(c)
            st = r["stats"]
            del r
            cold = run_gpu(c, sweep_steps, 2, inputs.BASE_SEED + 3, nsets=ROTATING_SETS)
            ck = [cold["kernel_ms"][n] for n in cold["names"]]
            del cold
            line = dict(workload=name, fwd_ms=round(fwd_ms, 4), bwd_ms=round(bwd_ms, 4),
                        fwd_tflops=round(f / fwd_ms * 1e-9, 1),
                        bwd_tflops=round(2.5 * f / bwd_ms * 1e-9, 1),
                        fwd_bwd_tflops=round(3.5 * f / (fwd_ms + bwd_ms) * 1e-9, 1),
                        fwd_median_ms=round(st["fwd_median"], 4), fwd_min_ms=round(st["fwd_min"], 4),
                        bwd_median_ms=round(st["bwd_median"], 4), bwd_min_ms=round(st["bwd_min"], 4),
                        fwd_ms_rotating=round(ck[0], 4), bwd_ms_rotating=round(sum(ck[1:]), 4),
                        fwd_min_GBps=round(by_f / fwd_ms * 1e-6, 1), bwd_min_GBps=round(by_b / bwd_ms * 1e-6, 1),
                        fwd_hbm_frac=round(by_f / fwd_ms * 1e-6 / PEAK_HBM_GBPS, 4),
                        bwd_hbm_frac=round(by_b / bwd_ms * 1e-6 / PEAK_HBM_GBPS, 4))
            if c["sparse"]:
                # the dense kernels on the same tensors: the paper's claim is a runtime that falls in
                # proportion to the fraction of kept blocks (Section 3.3, Proposition 4)
                dn = run_gpu(dict(c, sparse=False), 3, 1, inputs.BASE_SEED + 3)
                dk = [dn["kernel_ms"][n] for n in dn["names"]]
                del dn
                T = c["N"] // 128
                line.update(kept_fraction=round(nnz_blocks / (T * T), 5),
                            dense_fwd_ms=round(dk[0], 4), dense_bwd_ms=round(sum(dk[1:]), 4),
                            speedup_fwd=round(dk[0] / fwd_ms, 1), speedup_bwd=round(sum(dk[1:]) / bwd_ms, 1))
            print(json.dumps(line), file=sys.stderr, flush=True)

    cfg = wl[args.workload]
    run = run_gpu(cfg, args.steps, args.warmup, inputs.BASE_SEED + 3)
    f_fwd = flops_fwd(cfg, run["nnz"])
    total = 3.5 * f_fwd
    value = total / run["ms_per_step"] * 1e-9
    rot = run_gpu(cfg, args.steps, args.warmup, inputs.BASE_SEED + 3, nsets=ROTATING_SETS)
    rot_ms = rot["ms_per_step"]
    del rot
    mfma_rate = measured_mfma_rate(cfg["dtype"], 1)
    mfma_rate_varied = measured_mfma_rate(cfg["dtype"], 4)
    kms = run["kernel_ms"]
    st = run["stats"]
    peak = PEAK_TFLOPS[cfg["dtype"]]
    # Tile products per launch (Algorithm 4 has five in the backward pass; one tile product over the
    # whole problem is 2 B H N^2 d FLOPs = f_fwd / 2).  Algorithmic: forward S, PV; dK/dV kernel
    # S, dP, dV, dK; dQ kernel dQ.  Executed: the dQ kernel recomputes S and dP as well.
    n_fwd, n_dq, n_dkv = run["names"]
    products = {n_fwd: (2, 2), n_dq: (1, 3), n_dkv: (4, 4)}
    algo = {n: products[n][0] * 0.5 * f_fwd for n in run["names"]}
    executed = {n: products[n][1] * 0.5 * f_fwd for n in run["names"]}
    kbytes = dict(zip(run["names"], kernel_bytes(cfg)))
    dominant = max(kms, key=lambda n: kms[n])
    # which roofline bounds the dominant kernel: the longer of its algorithmic FLOPs at the matrix
    # peak and its minimum bytes at the HBM peak
    t_mfma = algo[dominant] / (peak * 1e9)            # ms
    t_hbm = kbytes[dominant] / (PEAK_HBM_GBPS * 1e6)  # ms
    if t_mfma >= t_hbm:
        roof = {"bound": "mfma", "kernel": dominant, "achieved": round(algo[dominant] / kms[dominant] * 1e-9, 2),
                "peak": peak, "unit": "TFLOP/s", "frac": round(algo[dominant] / kms[dominant] * 1e-9 / peak, 4)}
    else:
        gbps = kbytes[dominant] / kms[dominant] * 1e-6
        roof = {"bound": "hbm", "kernel": dominant, "achieved": round(gbps, 1), "peak": PEAK_HBM_GBPS,
                "unit": "GB/s", "frac": round(gbps / PEAK_HBM_GBPS, 4)}
    roof["traffic"] = load_traffic(args.workload, dominant)
    roof["traffic_source"] = ("profiles/hbm_traffic.json (rocprofv3 FETCH_SIZE + WRITE_SIZE per launch of this kernel "
                              "on this workload)" if roof["traffic"] is not None else None)
    roof["algorithmic_bytes"] = kbytes[dominant]
    roof["avg_ms"] = round(kms[dominant], 4)
    f_bwd = 2.5 * f_fwd
    passes = {
        "fwd": {"ms": round(st["fwd_mean"], 4), "tflops": round(f_fwd / st["fwd_mean"] * 1e-9, 1)},
        "bwd": {"ms": round(st["bwd_mean"], 4), "tflops": round(f_bwd / st["bwd_mean"] * 1e-9, 1)},
    }
    out = {
        "metric": "attention fwd+bwd TFLOP/s",
        "value": round(value, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(run["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg["dtype"],
        "data": "synthetic",
        "config": {"workload": args.workload, **{k: cfg[k] for k in ("B", "H", "N", "d", "causal", "p", "sparse")}},
        "frac_of_mfma_peak": round(value / peak, 4),
        # whole passes against the published matrix peak, FLOPs as the metric counts them (forward
        # 4 B H N^2 d, backward 2.5 x), timed through attn_fwd / attn_bwd inside the timed region
        "fwd_frac": round(f_fwd / st["fwd_mean"] * 1e-9 / peak, 4),
        "bwd_frac": round(f_bwd / st["bwd_mean"] * 1e-9 / peak, 4),
        "step_frac": round(value / peak, 4),
        "passes": passes,
        "cache": "one set of tensors, reused every step (the value above)",
        "rotating_buffers": {"sets": ROTATING_SETS, "ms_per_step": round(rot_ms, 4),
                             "value": round(total / rot_ms * 1e-9, 2)},
        "measured_mfma_rate": {
            "tflops": round(mfma_rate, 1), "frac_of_it": round(value / mfma_rate, 4),
            "what": "register-operand 32x32x16 MFMA loop on this GPU, same dtype, the same two operand registers every time",
            "varied_operands_tflops": round(mfma_rate_varied, 1),
            "frac_of_varied": round(value / mfma_rate_varied, 4),
            "varied_what": "the same loop over four pseudo-random operand pairs in turn: the clock this GPU holds "
                           "when operand bits change as in a real product"},
        "step_stats_ms": {k: round(v, 4) for k, v in st.items()},
        "roofline": roof,
        "kernels": {n: {"avg_ms": round(v, 4),
                        "tile_products_algorithmic": products[n][0], "tile_products_executed": products[n][1],
                        "algorithmic_tflops": round(algo[n] / v * 1e-9, 1),
                        "executed_tflops": round(executed[n] / v * 1e-9, 1),
                        "executed_frac_of_peak": round(executed[n] / v * 1e-9 / peak, 4)}
                    for n, v in kms.items()},
        "kernels_note": "per-kernel durations from a second pass of the same steps through attn_bwd_timed "
                        "(events between the launches); backward: 5 tile products counted, 7 executed",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, run)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
