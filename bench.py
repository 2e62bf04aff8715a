#!/usr/bin/env python3
"""Benchmark of the quantized-LoRA linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--M TOKENS] [--no-extra]

A "step" is one pass of the whole hot path over one batch of synthetic tokens:
modulora_fwd + modulora_bwd_input + modulora_bwd_lora of one layer, inputs already
resident in HBM.  The headline workload is the largest single-GPU configuration of the
benchmark: the LLaMA-65B up projection (8192 -> 22016, 3-bit, group 128, r = 8) at
M = 4096 tokens; `--workload` / `--M` pick another one.  The timed region replays the K
steps from one HIP graph (no host launch overhead), REPEATS times, and the median replay
is reported; weights rotate over enough distinct copies (>= 512 MB) that no step finds its
packed weights in the last-level cache.  Prints ONE JSON line, which also carries the
second half of the metric -- the packed-weight GB/s of the M <= 16 streaming passes
(`packed_weight_GBps`) -- the roofline of the dominant kernel and of the whole layer, the
CPU oracle timed on a bounded sample, and the other benchmark configurations (`extra`).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, vendor peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, vendor peak
ROTATE_BYTES = 512 << 20        # distinct packed weights touched before one is reused
COPY_CAL_BYTES = 1 << 30        # size of the copy that calibrates the rocprofv3 byte counters
REPEATS = 5                     # timed replays of the K steps; the median is reported
HEADLINE = ("c5_65b_up", 4096)  # the largest single-GPU configuration
ORACLE_ROWS = 768               # token rows the CPU oracle computes where a full step would take minutes


def parse_args():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=50)
    p.add_argument("--warmup", type=int, default=10)
    p.add_argument("--workload", default=None, help="a name from synth.CONFIGS (default: %s at M = %d)" % HEADLINE)
    p.add_argument("--M", type=int, default=None, help="override the token count of the workload")
    p.add_argument("--variant", choices=("bf16", "f16"), default="bf16",
                   help="f16: the layer in the paper's own storage convention (float zero point, binary16, bias)")
    p.add_argument("--no-extra", action="store_true", help="skip the additional workloads")
    p.add_argument("--no-small", action="store_true", help="skip the M <= 16 packed-weight block")
    p.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    p.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    p.add_argument("--no-traffic", action="store_true",
                   help="skip the two rocprofv3 --pmc child runs that measure the HBM traffic of the dominant kernel")
    p.add_argument("--pmc-child", action="store_true",
                   help="(internal) run a few eager steps and a plain copy of known size, print nothing")
    return p.parse_args()


class Workload:
    """Device buffers and prebuilt C-ABI argument lists for one layer configuration."""

    def __init__(self, cfg, host_layer=None, seed=0):
        import numpy as np
        import torch
        from paper_2309_16119_amd import binding as b
        from paper_2309_16119_amd import synth as synth_mod

        self.cfg, self.b, self.torch = cfg, b, torch
        K, N, M, r, bits, g = cfg.K, cfg.N, cfg.M, cfg.r, cfg.bits, cfg.group
        G = K // g
        n_copies = max(1, math.ceil(ROTATE_BYTES / cfg.packed_weight_bytes))
        self.n_copies = n_copies
        self.weights = []
        first = None
        for i in range(n_copies):
            if i == 0 and host_layer is not None:
                w = b.QWeight.from_numpy(host_layer["qweight"], host_layer["scales"], host_layer["zeros"],
                                         K, N, bits, g)
            else:
                # the same distributions, drawn on the device (uniform words = uniform codes)
                T = synth_mod.make_layer_torch(cfg, "cuda", seed=seed + 1000 + i)
                first = first or T
                w = b.QWeight(T["qweight"], T["scales"], T["zeros"], K, N, bits, g)
            self.weights.append(w)
        if host_layer is not None:
            def dev16(a):
                return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
            self.X, self.dY = dev16(host_layer["X"]), dev16(host_layer["dY"])
            self.A, self.B = torch.from_numpy(host_layer["A"]).cuda(), torch.from_numpy(host_layer["B"]).cuda()
        else:
            self.X, self.dY, self.A, self.B = first["X"], first["dY"], first["A"], first["B"]
        self.Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        self.dX = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
        self.XA = torch.empty((M, r), dtype=torch.float32, device="cuda")
        self.dYBt = torch.empty((M, r), dtype=torch.float32, device="cuda")
        self.dA = torch.empty((K, r), dtype=torch.float32, device="cuda")
        self.dB = torch.empty((r, N), dtype=torch.float32, device="cuda")
        nbytes = b.modulora_workspace_bytes(self.weights[0], M, r)
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        self.ws_bytes = nbytes
        self.structs = [w.c_struct() for w in self.weights]

    def step(self, i: int, calls=("fwd", "bwd_input", "bwd_lora")):
        b, cfg = self.b, self.cfg
        st = ctypes.byref(self.structs[i % self.n_copies])
        stream = ctypes.c_void_p(self.torch.cuda.current_stream().cuda_stream)
        p = lambda t: ctypes.c_void_p(t.data_ptr())
        s = float(cfg.lora_scale)
        rc = 0
        if "fwd" in calls:
            rc |= b.lib.modulora_fwd(st, p(self.X), cfg.M, p(self.A), p(self.B), cfg.r, s, p(self.Y), p(self.XA),
                                     p(self.ws), self.ws_bytes, stream)
        if "bwd_input" in calls:
            rc |= b.lib.modulora_bwd_input(st, p(self.dY), cfg.M, p(self.A), p(self.B), cfg.r, s, p(self.dX),
                                           p(self.dYBt), p(self.ws), self.ws_bytes, stream)
        if "bwd_lora" in calls:
            rc |= b.lib.modulora_bwd_lora(cfg.K, cfg.N, cfg.M, cfg.r, s, p(self.X), p(self.dY), p(self.A), p(self.B),
                                          p(self.XA), p(self.dYBt), p(self.dA), p(self.dB), 0, p(self.ws),
                                          self.ws_bytes, stream)
        if rc != 0:
            raise RuntimeError("library call failed with status %d" % rc)


class WorkloadF16:
    """One layer in the paper's own storage convention (float zero point that is added, binary16
    everywhere, bias): device-drawn inputs with the distributions of synth.make_layer_f16."""

    def __init__(self, cfg, host_layer=None, seed=0):
        import numpy as np
        import torch
        from paper_2309_16119_amd import binding as b

        self.cfg, self.b, self.torch = cfg, b, torch
        K, N, M, r, bits, g = cfg.K, cfg.N, cfg.M, cfg.r, cfg.bits, cfg.group
        G = K // g
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed + 77)
        self.n_copies = max(1, math.ceil(ROTATE_BYTES / cfg.packed_weight_bytes))
        self.weights = []
        span = ((1 << bits) - 1) * cfg.scale_hi
        for _ in range(self.n_copies):
            q = torch.randint(-2 ** 31, 2 ** 31 - 1, (K * bits // 32, N), dtype=torch.int32, device="cuda", generator=gen)
            sc = (torch.rand((G, N), device="cuda", generator=gen) * (cfg.scale_hi - cfg.scale_lo) + cfg.scale_lo).to(torch.float16)
            z = (-torch.rand((G, N), device="cuda", generator=gen) * span).to(torch.float16)
            bias = (0.1 * torch.randn((N,), device="cuda", generator=gen)).to(torch.float16)
            self.weights.append(b.QWeightF16(q, sc, z, bias, K, N, bits, g))
        self.X = torch.randn((M, K), device="cuda", generator=gen).to(torch.float16)
        self.dY = torch.randn((M, N), device="cuda", generator=gen).to(torch.float16)
        self.A = 0.02 * torch.randn((K, r), device="cuda", generator=gen)
        self.B = 0.02 * torch.randn((r, N), device="cuda", generator=gen)
        self.host_layer = host_layer
        if host_layer is not None:      # weight copy 0 and the activations are the host layer's (parity against the oracle)
            L = host_layer
            self.weights[0] = b.QWeightF16.from_numpy(L["qweight"], L["scales"], L["zeros_f16"], L["bias"], K, N, bits, g)
            h16 = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
            self.X, self.dY = h16(L["X"]), h16(L["dY"])
            self.A, self.B = torch.from_numpy(L["A"]).cuda(), torch.from_numpy(L["B"]).cuda()
        self.Y = torch.empty((M, N), dtype=torch.float16, device="cuda")
        self.dX = torch.empty((M, K), dtype=torch.float16, device="cuda")
        self.XA = torch.empty((M, r), dtype=torch.float32, device="cuda")
        self.dYBt = torch.empty((M, r), dtype=torch.float32, device="cuda")
        self.dA = torch.empty((K, r), dtype=torch.float32, device="cuda")
        self.dB = torch.empty((r, N), dtype=torch.float32, device="cuda")
        self.ws_bytes = b.modulora_f16_workspace_bytes(self.weights[0], M, r)
        self.ws = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device="cuda")
        self.structs = [w.c_struct() for w in self.weights]

    def step(self, i: int, calls=("fwd", "bwd_input", "bwd_lora")):
        b, cfg = self.b, self.cfg
        st = ctypes.byref(self.structs[i % self.n_copies])
        stream = ctypes.c_void_p(self.torch.cuda.current_stream().cuda_stream)
        p = lambda t: ctypes.c_void_p(t.data_ptr())
        s = float(cfg.lora_scale)
        rc = 0
        if "fwd" in calls:
            rc |= b.lib.modulora_f16_fwd(st, p(self.X), cfg.M, p(self.A), p(self.B), cfg.r, s, p(self.Y), p(self.XA),
                                         p(self.ws), self.ws_bytes, stream)
        if "bwd_input" in calls:
            rc |= b.lib.modulora_f16_bwd_input(st, p(self.dY), cfg.M, p(self.A), p(self.B), cfg.r, s, p(self.dX),
                                               p(self.dYBt), p(self.ws), self.ws_bytes, stream)
        if "bwd_lora" in calls:
            rc |= b.lib.modulora_f16_bwd_lora(cfg.K, cfg.N, cfg.M, cfg.r, s, p(self.X), p(self.dY), p(self.A), p(self.B),
                                              p(self.XA), p(self.dYBt), p(self.dA), p(self.dB), 0, p(self.ws),
                                              self.ws_bytes, stream)
        if rc != 0:
            raise RuntimeError("library call failed with status %d" % rc)


class DecoderLayerWorkload:
    """The seven quantized-LoRA linears of one LLaMA-65B decoder layer (q, k, v, o 8192 x 8192;
    gate, up 8192 -> 22016; down 22016 -> 8192; 3-bit, group 128, r = 8) run forward in order,
    backward in reverse order (modulora_bwd_input + modulora_bwd_lora each), then ONE fused AdamW
    launch over all fourteen adapter factors, which live back to back in one buffer (so do their
    gradients, which modulora_bwd_lora writes in place).  Attention, norms and activation
    functions are not part of the method and not run; every linear gets its own activations of
    the right shape.  Packed weights: 0.30 GB per layer, more than the last-level cache."""

    SHAPES = [("q", 8192, 8192), ("k", 8192, 8192), ("v", 8192, 8192), ("o", 8192, 8192),
              ("gate", 8192, 22016), ("up", 8192, 22016), ("down", 22016, 8192)]

    def __init__(self, M: int, bits: int = 3, group: int = 128, r: int = 8):
        import torch
        from paper_2309_16119_amd import binding as b
        from paper_2309_16119_amd import synth as synth_mod

        self.b, self.torch, self.M, self.r = b, torch, M, r
        self.cfgs = [synth_mod.LayerConfig("dec_" + n, K, N, bits, group, M, r) for n, K, N in self.SHAPES]
        n_flat = sum((K + N) * r for _, K, N in self.SHAPES)
        self.flat = torch.empty(n_flat, dtype=torch.float32, device="cuda")
        self.flat_grad = torch.zeros_like(self.flat)
        self.exp_avg = torch.zeros_like(self.flat)
        self.exp_avg_sq = torch.zeros_like(self.flat)
        acts = {}
        self.layers = []
        off = 0
        ws_bytes = 0
        for i, cfg in enumerate(self.cfgs):
            L = synth_mod.make_layer_torch(cfg, "cuda", seed=100 + i)
            w = b.QWeight(L["qweight"], L["scales"], L["zeros"], cfg.K, cfg.N, cfg.bits, cfg.group)
            for dim, key in ((cfg.K, "X"), (cfg.N, "dY")):
                acts.setdefault((key, dim), L[key])
            nA, nB = cfg.K * r, r * cfg.N
            A, dA = self.flat[off:off + nA].view(cfg.K, r), self.flat_grad[off:off + nA].view(cfg.K, r)
            B, dB = self.flat[off + nA:off + nA + nB].view(r, cfg.N), self.flat_grad[off + nA:off + nA + nB].view(r, cfg.N)
            off += nA + nB
            A.copy_(L["A"])
            B.copy_(L["B"])
            ws_bytes = max(ws_bytes, b.modulora_workspace_bytes(w, M, r))
            self.layers.append(dict(cfg=cfg, w=w, st=w.c_struct(), X=acts[("X", cfg.K)], dY=acts[("dY", cfg.N)],
                                    A=A, B=B, dA=dA, dB=dB,
                                    Y=torch.empty((M, cfg.N), dtype=torch.bfloat16, device="cuda"),
                                    dX=torch.empty((M, cfg.K), dtype=torch.bfloat16, device="cuda"),
                                    XA=torch.empty((M, r), dtype=torch.float32, device="cuda"),
                                    dYBt=torch.empty((M, r), dtype=torch.float32, device="cuda")))
        self.ws = torch.empty(max(ws_bytes, 256), dtype=torch.uint8, device="cuda")
        self.ws_bytes = ws_bytes
        self.flops = sum(c.flops_fwd_bwd for c in self.cfgs)
        self.opt_steps = 0

    def step(self, i: int):
        b, M, r = self.b, self.M, self.r
        stream = ctypes.c_void_p(self.torch.cuda.current_stream().cuda_stream)
        p = lambda t: ctypes.c_void_p(t.data_ptr())
        rc = 0
        for l in self.layers:
            rc |= b.lib.modulora_fwd(ctypes.byref(l["st"]), p(l["X"]), M, p(l["A"]), p(l["B"]), r, 2.0, p(l["Y"]),
                                     p(l["XA"]), p(self.ws), self.ws_bytes, stream)
        for l in reversed(self.layers):
            c = l["cfg"]
            rc |= b.lib.modulora_bwd_input(ctypes.byref(l["st"]), p(l["dY"]), M, p(l["A"]), p(l["B"]), r, 2.0,
                                           p(l["dX"]), p(l["dYBt"]), p(self.ws), self.ws_bytes, stream)
            rc |= b.lib.modulora_bwd_lora(c.K, c.N, M, r, 2.0, p(l["X"]), p(l["dY"]), p(l["A"]), p(l["B"]),
                                          p(l["XA"]), p(l["dYBt"]), p(l["dA"]), p(l["dB"]), 0, p(self.ws),
                                          self.ws_bytes, stream)
        self.opt_steps += 1
        rc |= b.lib.modulora_adamw(p(self.flat), p(self.flat_grad), p(self.exp_avg), p(self.exp_avg_sq),
                                   self.flat.numel(), 1e-4, 0.9, 0.999, 1e-8, 0.0, self.opt_steps, stream)
        if rc != 0:
            raise RuntimeError("library call failed with status %d" % rc)


def time_steps(wl, steps: int, warmup: int, use_graph: bool, calls=None, repeats: int = REPEATS):
    """(median, all) milliseconds per step over `repeats` timed runs of exactly `steps` steps each
    (after `warmup` untimed steps).  `calls` restricts a step to some of the three library calls."""
    torch = wl.torch
    if calls is not None:
        full_step = wl.step
        wl = type("OneCall", (), {"torch": torch, "step": staticmethod(lambda i: full_step(i, calls))})
    for i in range(warmup):
        wl.step(i)
    torch.cuda.synchronize()
    runs = []
    if use_graph:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for i in range(steps):
                    wl.step(i)
        torch.cuda.synchronize()
        graph.replay()          # untimed: uploads the graph
        torch.cuda.synchronize()
        for _ in range(repeats):
            t0 = time.perf_counter()
            graph.replay()
            torch.cuda.synchronize()
            runs.append((time.perf_counter() - t0) * 1e3 / steps)
    else:
        for _ in range(repeats):
            t0 = time.perf_counter()
            for i in range(steps):
                wl.step(i)
            torch.cuda.synchronize()
            runs.append((time.perf_counter() - t0) * 1e3 / steps)
    return statistics.median(runs), runs


def kernel_profile(wl, steps: int, calls=None) -> dict:
    """{kernel: (launches, total_ms)} over `steps` eager steps, from HIP events that the library
    attaches to each of its kernel dispatches (on the stream they are launched on)."""
    b, torch = wl.b, wl.torch
    for i in range(2):              # untimed: the clocks have settled under this load when the events start
        if calls is None:
            wl.step(i)
        else:
            wl.step(i, calls)
    torch.cuda.synchronize()
    b.modulora_profile_begin()
    for i in range(steps):
        if calls is None:
            wl.step(i)
        else:
            wl.step(i, calls)
    prof = b.modulora_profile_end(capacity=64)
    torch.cuda.synchronize()
    return prof


def gemm_flops(cfg, name: str) -> float:
    """Algorithmic flop of one launch of a product kernel with the frozen weight: the product
    plus the rank-r up-projection it carries in its contraction."""
    cout = cfg.N if "fwd" in name else cfg.K
    return 2.0 * cfg.M * cfg.K * cfg.N + 2.0 * cfg.M * cfg.r * cout


def is_product_kernel(name: str) -> bool:
    return name.startswith(("gemm_fwd", "gemm_bwd", "f16_gemm")) and "fixup" not in name


def roofline_of(cfg, prof: dict) -> dict:
    """Roofline entry for the kernel that takes the most time in `prof`."""
    name, (launches, total_ms) = max(prof.items(), key=lambda kv: kv[1][1])
    avg_s = total_ms / launches * 1e-3
    K, N, M, r = cfg.K, cfg.N, cfg.M, cfg.r
    if is_product_kernel(name) and M > 16:
        ach = gemm_flops(cfg, name) / avg_s / 1e12
        return {"kernel": name, "bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                "avg_kernel_us": round(avg_s * 1e6, 2), "launches": launches}
    if name.startswith("gemm_") or name in ("stream_fwd", "stream_bwd", "f16_stream_fwd", "f16_stream_bwd"):
        nbytes = float(cfg.packed_weight_bytes)            # one pass over codes + scales + zeros
    elif "stream_" in name:
        nbytes = 2.0 * M * max(K, N)
    else:
        nbytes = 2.0 * M * (K if ("down" in name) else max(K, N))   # adapter kernels stream the activations once
    ach = nbytes / avg_s / 1e9
    return {"kernel": name, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None, "avg_kernel_us": round(avg_s * 1e6, 2),
            "launches": launches}


def product_kernels(cfg, prof: dict) -> dict:
    """Per product kernel (forward, backward): average duration, TFLOP/s and fraction of the MFMA peak,
    alone and with the second launch (`*_fixup`) that a split last round of tiles needs."""
    out = {}
    for name, (launches, total_ms) in prof.items():
        if not is_product_kernel(name):
            continue
        us = total_ms / launches * 1e3
        fix = [v for k, v in prof.items() if "fixup" in k and ("fwd" in k) == ("fwd" in name)]
        fix_us = sum(t / n * 1e3 for n, t in fix)
        fl = gemm_flops(cfg, name)
        e = {"avg_us": round(us, 2), "TFLOPs": round(fl / us / 1e6, 1), "frac": round(fl / us / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)}
        if fix_us:
            e["fixup_us"] = round(fix_us, 2)
            e["frac_with_fixup"] = round(fl / (us + fix_us) / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4)
        out[name] = e
    return out


def layer_roofline(cfg, ms: float) -> dict:
    """The whole fwd+bwd layer against the MFMA peak: 4MKN + 6Mr(K+N) flop over the step time."""
    ach = cfg.flops_fwd_bwd / (ms * 1e-3) / 1e12
    return {"flops": cfg.flops_fwd_bwd, "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4)}


def per_call_ms(prof: dict) -> dict:
    out = {}
    for name, (launches, total_ms) in prof.items():
        out[name] = round(total_ms / launches * 1e3, 2)   # microseconds per launch
    return out


def host16(t):
    """A device tensor of 16-bit floats as host bit patterns."""
    import numpy as np
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, wl):
    """The oracle, as it stands, timed on the host cores on the workload's own inputs (weight copy
    0 and the activations, copied to the host), and the parity of the GPU outputs against it.
    Where a full step is cheap (4MKN <= 1e11) the oracle computes all of it; otherwise it computes
    Y and dX for ORACLE_ROWS sampled token rows and dA, dB in full (they need only rank-r
    products), and the full-step time is extrapolated: rows' seconds x M / rows + adapter seconds
    (the oracle's cost is linear in the token count)."""
    import numpy as np
    import oracle

    torch = wl.torch
    if isinstance(wl, WorkloadF16):
        return cpu_baseline_f16(cfg, wl)
    K, N, M, r, s = cfg.K, cfg.N, cfg.M, cfg.r, float(cfg.lora_scale)
    w0 = wl.weights[0]
    args = (w0.qweight.cpu().numpy().view(np.uint32), host16(w0.scales), w0.zeros.cpu().numpy(), K, N, cfg.bits, cfg.group)
    Xh, dYh = host16(wl.X), host16(wl.dY)
    Ah, Bh = wl.A.cpu().numpy(), wl.B.cpu().numpy()
    full = 4.0 * M * K * N <= 1e11 or M <= ORACLE_ROWS
    rows = np.arange(M) if full else np.sort(np.random.default_rng(0).choice(M, ORACLE_ROWS, replace=False))
    Xs, dYs = np.ascontiguousarray(Xh[rows]), np.ascontiguousarray(dYh[rows])
    t0 = time.perf_counter()
    Yr, _ = oracle.fwd(*args, Xs, Ah, Bh, s)
    dXr, _ = oracle.bwd_input(*args, dYs, Ah, Bh, s)
    t_rows = time.perf_counter() - t0
    t0 = time.perf_counter()
    dAr, dBr = oracle.bwd_lora(K, N, Xh, dYh, Ah, Bh, s)
    t_lora = time.perf_counter() - t0
    seconds = t_rows * (M / len(rows)) + t_lora
    base = {"value": round(cfg.flops_fwd_bwd / seconds / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "cpu_model": cpu_model(), "kind": "oracle", "seconds_measured": round(t_rows + t_lora, 3), "seconds_full_step": round(seconds, 3),
            "extrapolated": not full,
            "sample": ("one full step (fwd + bwd_input + bwd_lora) of %s, all %d tokens" % (cfg.name, M)) if full else
                      ("%s: Y and dX of %d sampled token rows (%.2f s) + dA, dB in full (%.2f s); full-step time "
                       "extrapolated as rows' seconds x %d/%d + adapter seconds" % (cfg.name, len(rows), t_rows, t_lora, M, len(rows)))}
    wl.step(0)                      # weight copy 0
    torch.cuda.synchronize()
    rows_t = torch.from_numpy(rows).cuda()
    rel = lambda got, ref: float("%.3g" % (np.max(np.abs(got.double().cpu().numpy() - ref)) / np.max(np.abs(ref))))
    What = host16(wl.b.modulora_dequant(w0))
    parity = {"rel_max_err": {"Y": rel(wl.Y[rows_t], Yr), "dX": rel(wl.dX[rows_t], dXr), "dA": rel(wl.dA, dAr), "dB": rel(wl.dB, dBr)},
              "rows_checked": int(len(rows)), "bar": 2e-2,
              "dequant_bit_exact": bool(np.array_equal(What, oracle.dequant_bf16(*args)))}
    return base, parity


def cpu_baseline_f16(cfg, wl):
    """The paper-literal oracle (numpy float64) timed on one full step, and the GPU outputs against it."""
    import numpy as np
    from oracle import paper_literal as pl

    L = wl.host_layer
    args = (L["qweight"], L["scales"], L["zeros_f16"], L["K"], L["N"], L["bits"], L["group"])
    t0 = time.perf_counter()
    Yr, _ = pl.fwd(*args, L["X"], L["A"], L["B"], L["lora_scale"], L["bias"])
    dXr, _ = pl.bwd_input(*args, L["dY"], L["A"], L["B"], L["lora_scale"])
    dAr, dBr = pl.bwd_lora(L["X"], L["dY"], L["A"], L["B"], L["lora_scale"])
    dt = time.perf_counter() - t0
    base = {"value": round(cfg.flops_fwd_bwd / dt / 1e12, 6), "unit": "TFLOP/s", "cores": os.cpu_count(),
            "kind": "oracle", "seconds_measured": round(dt, 3), "seconds_full_step": round(dt, 3), "extrapolated": False,
            "sample": "one full step (fwd + bwd_input + bwd_lora) of %s, all %d tokens, numpy float64" % (cfg.name, cfg.M)}
    wl.step(0)
    wl.torch.cuda.synchronize()
    rel = lambda got, ref: float("%.3g" % (np.max(np.abs(got.double().cpu().numpy() - ref)) / np.max(np.abs(ref))))
    What = wl.b.modulora_f16_dequant(wl.weights[0]).cpu().view(wl.torch.int16).numpy().view(np.uint16)
    parity = {"rel_max_err": {"Y": rel(wl.Y, Yr), "dX": rel(wl.dX, dXr), "dA": rel(wl.dA, dAr), "dB": rel(wl.dB, dBr)},
              "bar": 2e-2, "dequant_bit_exact": bool(np.array_equal(What, pl.dequant_f16(*args)))}
    return base, parity


def read_rate(b, torch, nbytes: int, use_graph: bool) -> dict:
    """GB/s of the library's plain hand-written streaming read (modulora_bench_read) over `nbytes`
    bytes: the kernel alone (HIP events on its dispatch) and as a launch of its own replayed from
    a HIP graph like the layer's calls.  The buffer rotates over >= 512 MB so that no read finds its
    data in the last-level cache."""
    n_copies = max(2, math.ceil(ROTATE_BYTES / nbytes))
    bufs = [torch.randint(0, 1 << 30, (nbytes // 4,), dtype=torch.int32, device="cuda") for _ in range(n_copies)]
    sink = torch.empty(b.BENCH_READ_SINK_WORDS, dtype=torch.int32, device="cuda")

    class W:
        pass
    w = W()
    w.torch, w.b = torch, b
    w.step = lambda i, calls=None: b.modulora_bench_read(bufs[i % n_copies], sink)
    ms, _ = time_steps(w, 20, 3, use_graph)
    prof = kernel_profile(w, 20)
    k_us = prof["bench_read"][1] / prof["bench_read"][0] * 1e3
    return {"bytes": nbytes, "kernel_us": round(k_us, 2), "kernel_GBps": round(nbytes / k_us / 1e3, 1),
            "call_us": round(ms * 1e3, 2), "call_GBps": round(nbytes / ms / 1e6, 1)}


def small_m_block(synth, torch, use_graph: bool) -> dict:
    """The second half of the metric: packed-weight HBM GB/s of the M <= 16 passes.  Per workload
    and pass (fwd, bwd_input): the whole library call as replayed from a HIP graph (every launch
    of the pass), the streaming kernel alone (HIP events on its dispatch), both as GB/s of the
    packed weight (codes + scales + zeros, one pass) and as a fraction of the 8 TB/s peak, beside
    the plain hand-written read of the same number of bytes measured the same two ways."""
    from paper_2309_16119_amd import binding as b
    rows = []
    for name, M in (("c5_65b_up", 16), ("c5_65b_down", 16), ("c5_65b_attn", 16), ("c5_65b_up", 1), ("c5_65b_attn", 1)):
        cfg = synth.CONFIGS[name].with_M(M)
        wl = Workload(cfg)
        W = float(cfg.packed_weight_bytes)
        entry = {"workload": cfg.name, "packed_weight_bytes": int(W)}
        for call, stream_kernel in (("fwd", "stream_fwd"), ("bwd_input", "stream_bwd")):
            ms, _ = time_steps(wl, 20, 3, use_graph, calls=(call,))
            prof = kernel_profile(wl, 20, calls=(call,))
            us = {k: round(v[1] / v[0] * 1e3, 2) for k, v in prof.items()}
            e = {"call_us": round(ms * 1e3, 2), "call_GBps": round(W / ms / 1e6, 1),
                 "call_frac_of_peak": round(W / ms / 1e6 / HBM_PEAK_GBPS, 4), "kernels_us": us}
            if stream_kernel in us:
                e["stream_kernel_GBps"] = round(W / us[stream_kernel] / 1e3, 1)
                e["stream_kernel_frac_of_peak"] = round(W / us[stream_kernel] / 1e3 / HBM_PEAK_GBPS, 4)
            entry[call] = e
        entry["plain_read_same_bytes"] = read_rate(b, torch, int(W) // 16 * 16, use_graph)
        rows.append(entry)
        del wl
        torch.cuda.empty_cache()
    return {"peak_GBps": HBM_PEAK_GBPS, "unit": "GB/s", "target_frac": 0.70, "workloads": rows,
            "plain_read_2GiB": read_rate(b, torch, 1 << 31, use_graph)}


def measured_context(cfg, torch) -> dict:
    """Context measured on this machine (not a target): a dense bfloat16 torch.matmul of the workload's
    M x K x N (resident bf16 weight, no dequantization, one product)."""
    out = {}
    a = torch.randn((cfg.M, cfg.K), device="cuda").to(torch.bfloat16)
    w = torch.randn((cfg.N, cfg.K), device="cuda").to(torch.bfloat16)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        torch.matmul(a, w.t())
    torch.cuda.synchronize()
    e0.record()
    for _ in range(10):
        torch.matmul(a, w.t())
    e1.record(); torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 10
    out["dense_bf16_matmul_us"] = round(ms * 1e3, 2)
    out["dense_bf16_matmul_TFLOPs"] = round(2.0 * cfg.M * cfg.K * cfg.N / (ms * 1e-3) / 1e12, 1)
    out["dense_bf16_matmul_note"] = "torch.matmul [M,K] x [K,N] on a resident bf16 weight, same M, K, N (one product)"
    return out


def rocprof_kernel_pattern(lib_name: str) -> str:
    """Substring of the rocprofv3 kernel name that belongs to a library profile name."""
    if lib_name.startswith(("gemm_fwd_256x256", "gemm_fwd_128x256")):
        return "gemm_big_kernel<%d, false"
    if lib_name.startswith(("gemm_bwd_256x256", "gemm_bwd_128x256")):
        return "gemm_big_kernel<%d, true"
    if lib_name.startswith("gemm_fwd_128x64s"):
        return "gemm_mid_kernel<%d, false"
    if lib_name.startswith("gemm_bwd_128x64s"):
        return "gemm_mid_kernel<%d, true"
    if lib_name.startswith("gemm_fwd"):
        return "gemm_tile_kernel<%d, false"
    if lib_name.startswith("gemm_bwd"):
        return "gemm_tile_kernel<%d, true"
    return {"stream_fwd": "smallm_fwd_kernel<%d", "stream_bwd": "smallm_bwd_kernel<%d",
            "stream_fwd_finish": "smallm_fwd_finish_kernel", "stream_bwd_finish": "smallm_bwd_finish_kernel",
            "f16_stream_fwd": "smallm_fwd_kernel<%d", "f16_stream_bwd": "smallm_bwd_kernel<%d",
            "f16_stream_fwd_finish": "smallm_fwd_finish_kernel", "f16_stream_bwd_finish": "smallm_bwd_finish_kernel",
            "lora_down_finish": "lora_down_finish_kernel", "adamw": "adamw_kernel",
            "lora_down": "lora_down_kernel", "lora_grad": "lora_grad_partial_kernel",
            "lora_grad_reduce": "lora_grad_reduce_kernel"}.get(lib_name, lib_name)


def pmc_child_run(counter: str, workload_args: list) -> dict:
    """Run `rocprofv3 --pmc <counter>` on a child `bench.py --pmc-child` and return
    {kernel name: mean counter value per dispatch}.  The child is started before this process
    touches the GPU.  Any failure returns {}."""
    import csv
    import glob
    import shutil
    import subprocess
    import tempfile

    exe = shutil.which("rocprofv3")
    if exe is None:
        return {}
    # never nest profilers: when this process already runs under one, report no traffic
    if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ) or "rocprof" in os.environ.get("LD_PRELOAD", ""):
        return {}
    out = tempfile.mkdtemp(prefix="modulora_pmc_", dir="/tmp")
    env = dict(os.environ, TMPDIR="/tmp")
    cmd = [exe, "--pmc", counter, "--output-format", "csv", "-d", out, "-o", "pmc", "--", sys.executable,
           os.path.abspath(__file__), "--pmc-child", "--steps", "4", "--warmup", "2"] + workload_args
    try:
        subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=240)
        files = glob.glob(os.path.join(out, "**", "*counter_collection.csv"), recursive=True)
        acc = {}
        for f in files:
            with open(f) as fh:
                for row in csv.DictReader(fh):
                    if row.get("Counter_Name") != counter:
                        continue
                    acc.setdefault(row["Kernel_Name"], []).append(float(row["Counter_Value"]))
        return {k: sum(v) / len(v) for k, v in acc.items()}
    except Exception:
        return {}
    finally:
        shutil.rmtree(out, ignore_errors=True)


def traffic_of(kernel_pattern: str, fetch: dict, write: dict):
    """HBM bytes per launch of the kernel matching `kernel_pattern`: FETCH_SIZE + WRITE_SIZE, each
    scaled by the reading of the plain copy kernel (COPY_CAL_BYTES read, COPY_CAL_BYTES written)."""
    def pick(d, pat):
        hits = [v for k, v in d.items() if pat in k]
        return max(hits) if hits else None
    cal_f, cal_w = pick(fetch, "CUDAFunctorOnSelf_add"), pick(write, "CUDAFunctorOnSelf_add")
    if cal_f is None or cal_w is None:     # name of the torch.add kernel, else the largest elementwise one
        cal_f = cal_f or pick(fetch, "elementwise")
        cal_w = cal_w or pick(write, "elementwise")
    f, w = pick(fetch, kernel_pattern), pick(write, kernel_pattern)
    if not cal_f or not cal_w or f is None or w is None:
        return None
    return {"read_bytes": round(f * COPY_CAL_BYTES / cal_f), "write_bytes": round(w * COPY_CAL_BYTES / cal_w),
            "bytes": round(f * COPY_CAL_BYTES / cal_f + w * COPY_CAL_BYTES / cal_w),
            "copy_kernel_scale": {"FETCH_SIZE_per_GiB": round(cal_f, 1), "WRITE_SIZE_per_GiB": round(cal_w, 1)}}


def workload_entry(cfg, wl, steps: int, use_graph: bool, torch, dense: bool = True) -> dict:
    """One extra workload: median step time, layer-level and per-kernel roofline figures."""
    ms, runs = time_steps(wl, steps, 3, use_graph)
    prof = kernel_profile(wl, steps)
    entry = {"workload": cfg.name, "shape": "d_in=%d d_out=%d %d-bit group %d M=%d r=%d" % (cfg.K, cfg.N, cfg.bits, cfg.group, cfg.M, cfg.r),
             "ms_per_step": round(ms, 5), "tflops": round(cfg.flops_fwd_bwd / (ms * 1e-3) / 1e12, 3),
             "roofline": roofline_of(cfg, prof), "kernel_us": per_call_ms(prof)}
    if cfg.M > 16:
        entry["layer_roofline"] = layer_roofline(cfg, ms)
        entry["product_kernels"] = product_kernels(cfg, prof)
        if dense:
            entry["dense_bf16_matmul_TFLOPs"] = measured_context(cfg, torch)["dense_bf16_matmul_TFLOPs"]   # context only
    return entry


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding). "
              "Run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)
    if args.workload is None:
        if args.variant == "f16":       # its oracle is numpy: a shape it finishes in seconds
            args.workload = "c2_7b_attn"
        else:
            args.workload = HEADLINE[0]
            if args.M is None:
                args.M = HEADLINE[1]
    fetch = write = {}
    if args.variant == "f16":
        args.no_traffic = True          # the counter child runs replay the default variant
    if not (args.no_traffic or args.pmc_child):
        # before this process touches the GPU: two counter runs in child processes
        wargs = ["--workload", args.workload] + (["--M", str(args.M)] if args.M is not None else [])
        fetch = pmc_child_run("FETCH_SIZE", wargs)
        write = pmc_child_run("WRITE_SIZE", wargs) if fetch else {}
    import torch

    from paper_2309_16119_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[args.workload]
    if args.M is not None:
        cfg = cfg.with_M(args.M)
    use_graph = not args.no_graph

    if args.pmc_child:
        # a plain elementwise copy of known size: its FETCH_SIZE / WRITE_SIZE readings turn the
        # counters of the other kernels into bytes
        src = torch.ones(COPY_CAL_BYTES // 4, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
        wl = Workload(cfg)
        for i in range(args.warmup + args.steps):
            wl.step(i)
        torch.cuda.synchronize()
        return

    f16 = args.variant == "f16"
    wl = WorkloadF16(cfg, synth.make_layer_f16(cfg)) if f16 else Workload(cfg)
    ms, runs = time_steps(wl, args.steps, args.warmup, use_graph)
    prof = kernel_profile(wl, args.steps)
    tflops = cfg.flops_fwd_bwd / (ms * 1e-3) / 1e12

    line = {
        "metric": "fwd+bwd TFLOP/s per quantized LoRA layer; packed-weight HBM GB/s at M<=16",
        "value": round(tflops, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if f16 else "bf16", "data": "synthetic",
        "config": {"workload": "%s%s: d_in=%d d_out=%d %d-bit group %d, M=%d tokens, r=%d, lora_scale=%g" % (
            cfg.name, " (paper-literal f16 variant: float zero point, bias)" if f16 else "", cfg.K, cfg.N, cfg.bits, cfg.group,
            cfg.M, cfg.r, cfg.lora_scale),
            "weight_copies_rotated": wl.n_copies, "hip_graph": use_graph,
            "timing": "median of %d replays of %d steps each" % (REPEATS, args.steps)},
        "ms_per_step_replays": [round(x, 5) for x in runs],
        "roofline": roofline_of(cfg, prof),
        "kernel_us": per_call_ms(prof),
    }
    if cfg.M > 16:
        line["roofline"]["layer"] = layer_roofline(cfg, ms)
        line["roofline"]["product_kernels"] = product_kernels(cfg, prof)
    if fetch and write:
        pat = rocprof_kernel_pattern(line["roofline"]["kernel"])
        line["roofline"]["traffic"] = traffic_of(pat % cfg.bits if "%d" in pat else pat, fetch, write)
    line["per_call_us"] = {c: round(time_steps(wl, args.steps, 2, use_graph, calls=(c,))[0] * 1e3, 2)
                           for c in ("fwd", "bwd_input", "bwd_lora")}
    if cfg.M > 16:
        line["measured_context"] = measured_context(cfg, torch)
    if not args.no_cpu:
        line["cpu_baseline"], line["parity_vs_oracle"] = cpu_baseline(cfg, wl)
    del wl
    torch.cuda.empty_cache()

    if f16:
        args.no_extra = args.no_small = True     # those blocks belong to the default variant's line
    if not args.no_small:
        line["packed_weight_GBps"] = small_m_block(synth, torch, use_graph)
    if not args.no_extra:
        extra = []
        steps_x = max(5, min(args.steps, 20))
        # the other benchmark configurations, each at its own token count
        others = [synth.CONFIGS["c2_7b_attn"], synth.CONFIGS["c3_7b_gate_up"], synth.CONFIGS["c3_7b_down"],
                  synth.CONFIGS["c4_30b_attn"], synth.CONFIGS["c4_30b_up"], synth.CONFIGS["c4_30b_down"],
                  synth.CONFIGS["c5_65b_up"].with_M(4096)]
        for ocfg in others:
            if ocfg.name == cfg.name:
                continue
            w2 = Workload(ocfg)
            extra.append(workload_entry(ocfg, w2, steps_x, use_graph, torch))
            del w2
            torch.cuda.empty_cache()
        # config 5 as a sweep: the three distinct matrices of a LLaMA-65B decoder layer at four
        # token counts; per call and summed, and the per-decoder-layer sum (4 x attn + 2 x up + down)
        sweep = []
        for M5 in (1, 16, 256, 4096):
            row = {"M": M5}
            layer_ms = 0.0
            for name, mult in (("c5_65b_attn", 4), ("c5_65b_up", 2), ("c5_65b_down", 1)):
                c5 = synth.CONFIGS[name].with_M(M5)
                w5 = Workload(c5)
                steps = 10 if M5 >= 256 else 20
                ms5, _ = time_steps(w5, steps, 3, use_graph)
                calls = {c: round(time_steps(w5, steps, 2, use_graph, calls=(c,), repeats=3)[0] * 1e3, 2)
                         for c in ("fwd", "bwd_input", "bwd_lora")}
                e5 = {"step_us": round(ms5 * 1e3, 2), "calls_us": calls,
                      "tflops": round(c5.flops_fwd_bwd / (ms5 * 1e-3) / 1e12, 2)}
                if M5 >= 256:
                    e5["layer_frac_of_mfma_peak"] = layer_roofline(c5, ms5)["frac"]
                    e5["product_kernels"] = product_kernels(c5, kernel_profile(w5, steps))
                row[name.replace("c5_65b_", "")] = e5
                layer_ms += mult * ms5
                del w5
                torch.cuda.empty_cache()
            row["decoder_layer_sum_ms"] = round(layer_ms, 4)
            sweep.append(row)
        extra.append({"workload": "c5 sweep: 8192x8192 (x4), 8192->22016 (x2), 22016->8192 (x1), 3-bit group 128 r=8",
                      "rows": sweep})
        # NEXT step of the method: the seven linears of a decoder layer back to back + fused AdamW
        for M_dec in (2048, 128):
            dl = DecoderLayerWorkload(M_dec)
            steps = 5
            ms3, _ = time_steps(dl, steps, 2, use_graph)
            prof3 = kernel_profile(dl, steps)
            by_family = {}
            for name, (launches, total_ms) in prof3.items():
                by_family[name] = round(total_ms / steps * 1e3, 1)       # microseconds per step, all launches
            extra.append({"workload": "decoder_layer_65b_M%d: 7 linears fwd+bwd + fused AdamW, 3-bit group 128 r=8" % M_dec,
                          "ms_per_step": round(ms3, 5), "tflops": round(dl.flops / (ms3 * 1e-3) / 1e12, 3),
                          "layer_frac_of_mfma_peak": round(dl.flops / (ms3 * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                          "tokens_per_s": round(M_dec / (ms3 * 1e-3), 1), "us_per_step_by_kernel": by_family})
            del dl
            torch.cuda.empty_cache()
        # the paper-literal variant (float zero point, binary16, bias) on a mid-size and a large shape
        for cfg_h in (synth.CONFIGS["c2_7b_attn"], synth.CONFIGS["c5_65b_attn"].with_M(4096)):
            wh = WorkloadF16(cfg_h)
            e = workload_entry(cfg_h, wh, steps_x, use_graph, torch, dense=False)
            e["workload"] = "paper-literal f16 variant, %s" % cfg_h.name
            extra.append(e)
            del wh
            torch.cuda.empty_cache()
        # ... and its M <= 16 streaming passes on the largest matrix
        cfg_s = synth.CONFIGS["c5_65b_up"].with_M(16)
        ws_ = WorkloadF16(cfg_s)
        e = workload_entry(cfg_s, ws_, steps_x, use_graph, torch, dense=False)
        e["workload"] = "paper-literal f16 variant, %s" % cfg_s.name
        e["packed_weight_GBps"] = {k: round(cfg_s.packed_weight_bytes / (v * 1e-6) / 1e9, 1)
                                   for k, v in e["kernel_us"].items() if k in ("f16_stream_fwd", "f16_stream_bwd")}
        extra.append(e)
        del ws_
        torch.cuda.empty_cache()
        # the round-to-nearest quantizer + packer on the largest layer shape
        Wq = torch.randn((22016, 8192), device="cuda") * 0.02
        b_mod = __import__("paper_2309_16119_amd.binding", fromlist=["binding"])
        b_mod.modulora_quantize_rtn(Wq, 3, 128)
        torch.cuda.synchronize()
        b_mod.modulora_profile_begin()
        for _ in range(5):
            b_mod.modulora_quantize_rtn(Wq, 3, 128)
        profq = b_mod.modulora_profile_end()
        us = {k: round(v[1] / v[0] * 1e3, 1) for k, v in profq.items()}
        extra.append({"workload": "rtn_quantize 22016 x 8192 fp32 -> 3-bit group 128", "kernel_us": us,
                      "GBps_of_fp32_weight_read": {k: round(Wq.numel() * 4 / (v * 1e-6) / 1e9, 1) for k, v in us.items()}})
        del Wq
        torch.cuda.empty_cache()
        line["extra"] = extra
    print(json.dumps(line))


if __name__ == "__main__":
    main()
