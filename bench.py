#!/usr/bin/env python3
"""Benchmark of the partial-sync tensor-parallel MLP block (forward + backward) on ONE MI355X.

One "step" = caat_block_fwd + caat_block_bwd over one batch of the 1.1B-scale GPT MLP configuration
(h=2048, ffn=8192, GELU, LayerNorm, T=4 emulated ranks, 8192 tokens), synthetic seeded inputs resident in HBM.
Prints ONE JSON line: whole-step TFLOP/s (algorithmic FLOPs: 6*tokens*h*ffn*k, k=2 GELU / 3 SwiGLU), the
roofline of the dominant kernel (measured live with HIP events around every launch), the sync kernels' GB/s
versus p, synced bytes per token versus p, and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.md")


def pmc_traffic_bytes(config: str, p: float, kernel: str):
    """HBM bytes per launch of a kernel family as the rocprofv3 --pmc runs of this same command measured them
    (FETCH_SIZE and WRITE_SIZE, each scaled by what the counter reads for a plain copy of known size): read from the
    tracked table profiles/hbm_traffic_per_launch.md (rows `| config | p | kernel family | read MB | write MB |`).
    None if the table has no row for this configuration, p and kernel."""
    try:
        rows = open(TRAFFIC_TABLE).read().splitlines()
    except OSError:
        return None
    for line in rows:
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) < 5 or cells[0] != config or cells[2].strip("`") != kernel:
            continue
        try:
            if abs(float(cells[1]) - p) < 1e-9:
                return (float(cells[3]) + float(cells[4])) * 1e6
        except ValueError:
            continue
    return None


def hs_of(cfg) -> int:
    """Shared channels of a configuration as the library counts them (caat_shared_channels, Eq. A3)."""
    from paper_2506_19645_amd import binding as B
    return B.shared_channels(cfg.h, float(cfg.p))


def flops_per_launch(name: str, cfg, which: int = 0) -> float:
    """Algorithmic FLOPs of one launch (all T ranks) of a kernel family of the MLP block."""
    n, h, f = cfg.tokens, cfg.h, cfg.ffn
    k1 = 2 if cfg.kind == 1 else 1            # SwiGLU: gate and up projections
    table = {
        "gemm_nt_gelu_fwd": 2.0 * n * h * f, "gemm_nt_swiglu_fwd": 2.0 * n * h * f * 2,
        "gemm_nt_rowpar": 2.0 * n * f * h,
        "gemm_nn_gelu_bwd": 2.0 * n * h * f, "gemm_nn_swiglu_bwd": 2.0 * n * h * f,
        "gemm_nn_dgrad": 2.0 * n * f * h * k1,
        "gemm_tn_wgrad": (2.0 * n * f * h + 2.0 * n * f * h * k1) / 2.0,   # two launches per step: dB and dA
    }
    return table.get(name, 0.0)


def sync_bytes(name: str, cfg, hs: int) -> float:
    """Algorithmic HBM bytes of one launch of a streaming kernel."""
    T, n, h = cfg.T, cfg.tokens, cfg.h
    if name == "partial_sync_fwd":       # read T partials + T residual slices, write T outputs, shared channels only
        return 3.0 * T * n * hs * 2
    if name == "partial_sync_bwd":       # in place: read T, write T, shared channels only
        return 2.0 * T * n * hs * 2
    if name == "partial_sync_norm_fwd":  # one launch: T partials + T residual slices + the private channels read, R' shared
        return (3.0 * T * n * hs + T * n * (h - hs) + T * n * h) * 2 + T * n * 8   # channels and the normalised copy written
    if name == "norm_fwd":
        return 2.0 * T * n * h * 2 + T * n * 8
    if name == "norm_bwd_sync":          # one launch: read dy, dres, x; write g and the reduced / scaled copy
        return 5.0 * T * n * h * 2 + T * n * 8
    if name == "norm_bwd":               # read dy, dres, x; write g and scaled g (whose shared channels the reduce writes)
        return 5.0 * T * n * h * 2 - (T * n * hs * 2 if hs % 8 == 0 else 0) + T * n * 8
    return 0.0


def gemm_power_check(torch, B, bench, cfg, iters=40):
    """The dominant GEMM family's shape class (TN, M = N = h, K = tokens, all T ranks) timed stand-alone twice: on the
    step's own N(0,1) operands and on all-zero operands.  The instruction stream is identical; on zeros the
    matrix units toggle almost nothing, so the gap shows how far the chip's power management (not the kernel's
    schedule) holds the clock down on real data."""
    T, n, h = cfg.T, cfg.tokens, cfg.h
    c = torch.empty(T, h, h, dtype=torch.bfloat16, device="cuda")
    out = {}
    for name, a, b in (("random", bench.x, bench.dxo), ("zeros", torch.zeros_like(bench.x), torch.zeros_like(bench.dxo))):
        run = lambda: B.gemm_bf16(a, b, c, B.GEMM_TN, T, h, h, n, h, h, h, n * h, n * h, h * h)
        for _ in range(15):
            run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        out[name + "_operands_TFLOP/s"] = round(2.0 * T * h * h * n / ms / 1e9, 1)
    out["shape"] = "TN G=%d M=N=%d K=%d, plain epilogue, stand-alone" % (T, h, n)
    return out


class MlpBench:
    def __init__(self, cfg, seed=0):
        import numpy as np
        import torch
        from paper_2506_19645_amd import binding as B
        from paper_2506_19645_amd import inputs as I
        self.B, self.torch, self.cfg = B, torch, cfg
        t0 = time.time()
        d = I.make_inputs(cfg, seed=seed, hs_struct=cfg.h // 2)
        self.host = d
        swi = cfg.kind == I.KIND_MLP_SWIGLU
        ln = cfg.norm == I.NORM_LAYERNORM
        self.w0 = B.to_device(np.concatenate([d["Wg"], d["Wu"]], axis=1) if swi else d["A"])
        self.w1 = B.to_device(d["B"])
        self.gamma = B.to_device(d["gamma"])
        self.beta = B.to_device(d["beta"]) if ln else None
        self.x, self.r = B.to_device(d["X"]), B.to_device(d["R"])
        self.dxo, self.dro = B.to_device(d["dXo"]), B.to_device(d["dRo"])
        self.r_out, self.x_out = torch.empty_like(self.x), torch.empty_like(self.x)
        self.dx, self.dr = torch.empty_like(self.x), torch.empty_like(self.x)
        self.dw0, self.dw1 = torch.empty_like(self.w0), torch.empty_like(self.w1)
        self.dgamma = torch.empty(cfg.h, dtype=torch.float32, device="cuda")
        self.dbeta = torch.empty(cfg.h, dtype=torch.float32, device="cuda") if ln else None
        desc = B.make_desc(cfg)
        self.ws = torch.empty(B.workspace_bytes(desc), dtype=torch.uint8, device="cuda")
        self.weights = [self.w0, self.w1, self.gamma, self.beta]
        self.setup_s = time.time() - t0

    def step(self, desc):
        B = self.B
        B.block_fwd(desc, self.weights, self.x, self.r, self.r_out, self.x_out, self.ws)
        B.block_bwd(desc, self.weights, self.x, self.r_out, self.ws, self.dxo, self.dro, self.dx, self.dr,
                    [self.dw0, self.dw1], self.dgamma, self.dbeta)

    use_graph = False   # --graph: one step is recorded into a HIP graph and the timed region replays it

    def time_steps(self, desc, steps, warmup):
        torch = self.torch
        run = lambda: self.step(desc)
        if self.use_graph:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                self.step(desc)
                torch.cuda.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    self.step(desc)
            torch.cuda.current_stream().wait_stream(side)
            run = graph.replay
        for _ in range(warmup):
            run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            run()
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        return e0.elapsed_time(e1) / steps, wall_ms / steps

    def profile_steps(self, desc, steps):
        """Per-launch durations (HIP events on the launch stream around every kernel) averaged per kernel family."""
        B = self.B
        B.profile_reset()
        B.profile_enable(True)
        for _ in range(steps):
            self.step(desc)
        self.torch.cuda.synchronize()
        B.profile_enable(False)
        acc = {}
        for name, ms in B.profile_records():
            tot, cnt = acc.get(name, (0.0, 0))
            acc[name] = (tot + ms, cnt + 1)
        B.profile_reset()
        return {k: {"avg_ms": v[0] / v[1], "launches_per_step": v[1] / steps} for k, v in acc.items()}


_SYNC_HOST = {}


def standalone_sync(torch, B, cfg, hs, iters=20, nsets=8, compact=False):
    """caat_partial_sync in place on the shared channels, rotating over buffer sets (> 1 GB) so that the
    last-level cache cannot hold the working set: the HBM-bound figure.  Seeded N(0,1) partial sums from the input
    module (one host draw, copied into every set: the rotation is about addresses, not values).
    compact: the shared channels alone as [T, n, hs] buffers (rows of hs channels, all of them shared) -- the layout
    of a communication buffer, where the synced bytes lie contiguously instead of as the first hs channels of rows of h."""
    if hs == 0:
        return 0.0, 0.0
    from paper_2506_19645_amd import inputs as I
    T, n, h = cfg.T, cfg.tokens, (hs if compact else cfg.h)
    # enough sets that the bytes the launches TOUCH (2 T n hs per set) exceed the 256 MB memory-side cache several times
    nsets = max(nsets, int(1.2e9 / (2.0 * T * n * hs)) + 1)
    iters = max(iters, nsets)
    key = (T, n, h)
    if key not in _SYNC_HOST:
        _SYNC_HOST.clear()
        _SYNC_HOST[key] = B.to_device(I.make_sync_inputs(T, n, h, seed=0)["Zt"])
    bufs = [_SYNC_HOST[key].clone() for _ in range(nsets)]
    for b in bufs:
        B.partial_sync(b, None, b, T, n, h, hs, 1.0)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        b = bufs[i % nsets]
        B.partial_sync(b, None, b, T, n, h, hs, 1.0)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / iters
    return ms, 4.0 * T * n * hs / ms / 1e6     # GB/s, algorithmic 4*T*hs bytes per token


def copy_ceiling(torch, B, nbytes=1 << 30, iters=10):
    """What a plain device copy (equal read and write volumes, like the reduce and norm kernels) reaches on this machine:
    the library's streaming probe, contiguous piece per workgroup, with and without the non-temporal hint."""
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    out = {}
    for mode, name in ((3, "copy_GB/s"), (4, "copy_nontemporal_GB/s"), (1, "read_nontemporal_GB/s")):
        for _ in range(3):
            B.hbm_probe(src, dst, nbytes, mode)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            B.hbm_probe(src, dst, nbytes, mode)
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(nbytes * (2 if mode >= 3 else 1) / (e0.elapsed_time(e1) / iters) / 1e6, 1)
    out["note"] = "1 GiB buffers, 16-byte accesses; bytes moved = read + written"
    return out


def cpu_baseline(cfg, host, sample_tokens):
    """The numpy oracle (as it stands: float64) on the first `sample_tokens` tokens of every rank, fwd + bwd; the same
    run in the oracle's float32 variant beside it (the precision the benchmark definition names for the CPU reference)."""
    import numpy as np
    from oracle import caat_oracle as O
    n = min(sample_tokens, cfg.tokens)
    sub = {k: (v[:, :n] if k in ("X", "R", "dXo", "dRo") else v) for k, v in host.items()}
    swi = cfg.kind == 1
    norm = O.LAYERNORM if cfg.norm == 0 else O.RMSNORM
    kw = dict(swiglu=swi, norm=norm, hs=O.shared_channels(cfg.h, cfg.p), eps=cfg.eps, private_scale=cfg.private_scale)
    flops = 6.0 * n * cfg.h * cfg.ffn * (3 if swi else 2)
    res = {}
    for name, dt in (("fp64", np.float64), ("fp32", np.float32)):
        w = {k: O.widen_bf16(v, dt) for k, v in sub.items()}
        t0 = time.perf_counter()
        fwd = O.mlp_block_fwd(w["X"], w["R"], w, w["gamma"], w.get("beta"), **kw)
        O.mlp_block_bwd(w["X"], fwd, w, w["gamma"], w["dXo"], w["dRo"], **kw)
        res[name] = time.perf_counter() - t0
        del w, fwd
    sec = res["fp64"]
    return {"value": flops / sec / 1e12, "unit": "TFLOP/s", "cores": _blas_threads(), "kind": "oracle",
            "sample": "numpy fp64 oracle, fwd+bwd, first %d of %d tokens of each of the %d ranks (%.1f s)"
                      % (n, cfg.tokens, cfg.T, sec), "seconds": sec,
            "fp32_variant": {"value": flops / res["fp32"] / 1e12, "unit": "TFLOP/s", "seconds": res["fp32"],
                             "sample": "the same oracle and sample in float32"}}


def _blas_threads():
    threads = len(os.sched_getaffinity(0))
    try:
        from threadpoolctl import threadpool_info
        blas = [i["num_threads"] for i in threadpool_info() if i.get("user_api") == "blas"]
        if blas:
            threads = max(blas)
    except Exception:
        pass
    return threads


def cpu_baseline_other_kinds(name, cfg, bwd):
    """The numpy fp64 oracle (as it stands) on a bounded sample of the attention / layer workloads: the same layer
    dimensions, T and p, fewer or shorter sequences (fresh seeded inputs of that smaller shape)."""
    from oracle import caat_oracle as O
    from paper_2506_19645_amd import inputs as I
    T, h = cfg.T, cfg.h
    hpr, kvpr = cfg.n_heads // T, cfg.kv_heads // T
    if name == "C5":
        small = cfg                       # the whole decode batch: the oracle needs only seconds for it
    else:
        small = cfg.with_(batch=1, seq=min(cfg.seq, 1024 if h <= 4096 else 512))
    d = I.make_inputs(small, seed=0, with_grads=bwd, hs_struct=cfg.h // 2)
    w = {k: O.widen_bf16(v) for k, v in d.items()}
    n, s = small.tokens, small.seq
    kw = dict(heads_per_rank=hpr, head_dim=cfg.head_dim, hs=O.shared_channels(cfg.h, cfg.p), eps=cfg.eps, private_scale=cfg.private_scale,
              rope_base=cfg.rope_base, kv_heads_per_rank=kvpr)
    t0 = time.perf_counter()
    if name == "C4":
        fwd = O.attn_block_fwd(w["X"], w["R"], w["Wqkv"], w["Wo"], w["gamma"], None, batch=1, seq=s, norm=O.RMSNORM, **kw)
        if bwd:
            O.attn_block_bwd(w["X"], fwd, w["Wqkv"], w["Wo"], w["gamma"], w["dXo"], w["dRo"], batch=1, seq=s,
                             norm=O.RMSNORM, **kw)
        work = (24.0 if bwd else 8.0) * n * h * h + (7.0 if bwd else 2.0) * s * s * h
        unit, scale = "TFLOP/s", 1e12
    elif name == "C5":
        O.decode_layer_fwd(w["R"], w, w["Kc"], w["Vc"], kv_len=cfg.kv_len, **kw)
        fr, hd = cfg.f_r, cfg.hd_r
        work = (2.0 * T * small.batch * kvpr * (cfg.kv_len + 1) * cfg.head_dim * 2 +
                2.0 * T * (cfg.qkv_r * h + h * hd + 2 * fr * h + h * fr))        # KV cache of the sample + all weights
        unit, scale = "GB/s", 1e9
    else:
        O.prefill_layer_fwd(w["R"], w, batch=1, seq=s, **kw)
        work = n * (2.0 * h * T * cfg.qkv_r + 2.0 * h * h + 6.0 * h * cfg.ffn) + 2.0 * s * s * h
        unit, scale = "TFLOP/s", 1e12
    sec = time.perf_counter() - t0
    return {"value": work / sec / scale, "unit": unit, "cores": _blas_threads(), "kind": "oracle",
            "sample": "numpy fp64 oracle, %s, %d sequence(s) of %d token(s) per rank instead of %d x %d, same layer "
                      "dimensions, T and p (%.1f s)" % ("fwd+bwd" if bwd else "fwd", small.batch, s, cfg.batch, cfg.seq, sec),
            "seconds": sec}


class AttnBench(MlpBench):
    """Attention sub-block (C4): forward = QKV GEMM, RoPE, causal attention, o_proj + partial sync, norm; backward =
    norm backward, partial sync, o_proj gradients, attention-core gradient, inverse RoPE, QKV gradients."""

    def __init__(self, cfg, seed=0, backward=True):
        import torch
        from paper_2506_19645_amd import binding as B
        from paper_2506_19645_amd import inputs as I
        self.B, self.torch, self.cfg, self.backward = B, torch, cfg, backward
        d = I.make_inputs(cfg, seed=seed, hs_struct=cfg.h // 2, with_grads=backward)
        self.host = d
        self.weights = [B.to_device(d["Wqkv"]), B.to_device(d["Wo"]), B.to_device(d["gamma"]), None]
        self.x, self.r = B.to_device(d["X"]), B.to_device(d["R"])
        self.r_out, self.x_out = torch.empty_like(self.x), torch.empty_like(self.x)
        self.ws = torch.empty(B.workspace_bytes(B.make_desc(cfg)), dtype=torch.uint8, device="cuda")
        if backward:
            self.dxo, self.dro = B.to_device(d["dXo"]), B.to_device(d["dRo"])
            self.dx, self.dr = torch.empty_like(self.x), torch.empty_like(self.x)
            self.dw = [torch.empty_like(self.weights[0]), torch.empty_like(self.weights[1])]
            self.dgamma = torch.empty(cfg.h, dtype=torch.float32, device="cuda")

    def step(self, desc):
        self.B.block_fwd(desc, self.weights, self.x, self.r, self.r_out, self.x_out, self.ws)
        if self.backward:
            self.B.block_bwd(desc, self.weights, self.x, self.r_out, self.ws, self.dxo, self.dro, self.dx, self.dr,
                             self.dw, self.dgamma, None)


class DecodeBench(MlpBench):
    """Decode layer (C5): one new token per sequence over a KV cache of kv_len positions."""

    def __init__(self, cfg, seed=0):
        import numpy as np
        import torch
        from paper_2506_19645_amd import binding as B
        from paper_2506_19645_amd import inputs as I
        self.B, self.torch, self.cfg = B, torch, cfg
        d = I.make_inputs(cfg, seed=seed, hs_struct=cfg.h // 2)
        self.host = d
        self.weights = [B.to_device(d["gamma_attn"]), B.to_device(d["Wqkv"]), B.to_device(d["Wo"]), B.to_device(d["gamma"]),
                        B.to_device(np.concatenate([d["Wg"], d["Wu"]], axis=1)), B.to_device(d["B"])]
        self.r = B.to_device(d["R"])
        self.kc, self.vc = B.to_device(d["Kc"]), B.to_device(d["Vc"])
        self.r_out = torch.empty_like(self.r)
        self.ws = torch.empty(B.workspace_bytes(B.make_desc(cfg)), dtype=torch.uint8, device="cuda")

    def step(self, desc):
        self.B.block_fwd(desc, self.weights, None, self.r, self.r_out, None, self.ws, kv_k=self.kc, kv_v=self.vc)


class PrefillBench(MlpBench):
    """Prefill decoder layer (C6): a batch of whole prompts through attention + SwiGLU MLP, KV cache filled."""

    def __init__(self, cfg, seed=0, dedup=False):
        import numpy as np
        import torch
        from paper_2506_19645_amd import binding as B
        from paper_2506_19645_amd import inputs as I
        self.B, self.torch, self.cfg = B, torch, cfg
        d = I.make_inputs(cfg, seed=seed, hs_struct=hs_of(cfg) if dedup else cfg.h // 2)
        self.weights = [B.to_device(d["gamma_attn"]), B.to_device(d["Wqkv"]), B.to_device(d["Wo"]), B.to_device(d["gamma"]),
                        B.to_device(np.concatenate([d["Wg"], d["Wu"]], axis=1)), B.to_device(d["B"])]
        if dedup:   # shared channels once [n, hs], then the private channels [T, n, h - hs]; valid for this p only
            hs = hs_of(cfg)
            self.r = B.to_device(np.concatenate([np.ascontiguousarray(d["R"][0, :, :hs]).ravel(),
                                                 np.ascontiguousarray(d["R"][:, :, hs:]).ravel()]))
        else:
            self.r = B.to_device(d["R"])
        del d
        desc = B.make_desc(cfg)
        self.kc = torch.zeros((cfg.T, cfg.batch, cfg.kv_heads // cfg.T, desc.kv_cap, cfg.head_dim), dtype=torch.bfloat16,
                              device="cuda")
        self.vc = torch.zeros_like(self.kc)
        self.r_out = torch.empty_like(self.r)
        self.ws = torch.empty(B.workspace_bytes(desc), dtype=torch.uint8, device="cuda")

    def step(self, desc):
        self.B.block_fwd(desc, self.weights, None, self.r, self.r_out, None, self.ws, kv_k=self.kc, kv_v=self.vc)


def bench_attention_kinds(args, cfg, base):
    """JSON for the attention sub-block (C4, TFLOP/s) and the decode layer (C5, GB/s and per-token latency)."""
    from paper_2506_19645_amd import binding as B
    T, n, h, hd = cfg.T, cfg.tokens, cfg.h, cfg.hd_r
    if args.config == "C4":
        bwd = not args.fwd_only
        bench = AttnBench(cfg, backward=bwd)
        s = cfg.seq
        fl = {"gemm_nt_qkv": 2.0 * n * h * 3 * h, "flash_attn_fwd": 2.0 * cfg.batch * s * s * h,   # causal half of 4 s^2 h
              "gemm_nt_rowpar": 2.0 * n * h * h}
        by = {"rope": 2.0 * T * n * 2 * hd * 2, "partial_sync_fwd": 3.0 * T * n * hs_of(cfg) * 2,
              "norm_fwd": 2.0 * T * n * h * 2,
              "partial_sync_norm_fwd": (3.0 * T * n * hs_of(cfg) + T * n * (h - hs_of(cfg)) + T * n * h) * 2}
        work = sum(fl.values())
        if bwd:
            # five contractions instead of two in the attention core; the two NN and the two TN launches of a step
            # (o_proj: 2nh^2, qkv: 6nh^2) share a kernel family, so the per-launch figure is their mean
            fl.update({"flash_attn_bwd": 5.0 * cfg.batch * s * s * h, "gemm_nn_dgrad": 4.0 * n * h * h,
                       "gemm_tn_wgrad": 4.0 * n * h * h})
            by.update({"rope_bwd": 2.0 * T * n * 2 * hd * 2, "partial_sync_bwd": 2.0 * T * n * hs_of(cfg) * 2,
                       "norm_bwd_sync": 5.0 * T * n * h * 2,
                       "norm_bwd": 5.0 * T * n * h * 2 - (T * n * hs_of(cfg) * 2 if hs_of(cfg) % 8 == 0 else 0)})
            work += 5.0 * cfg.batch * s * s * h + 16.0 * n * h * h
        unit, peak = "TFLOP/s", MFMA_BF16_PEAK_TFLOPS
        workload = "%s attention sub-block %s: h=%d heads=%d d=%d RoPE causal seq=%d batch=%d T=%d p=%g (hs=%d)" % (
            cfg.name, "fwd+bwd" if bwd else "fwd", h, cfg.n_heads, cfg.head_dim, s, cfg.batch, T, cfg.p, hs_of(cfg))
    elif args.config in ("C6", "C7"):
        bench = PrefillBench(cfg, dedup=args.dedup_shared)
        s, f = cfg.seq, cfg.ffn
        qkv_cols = T * cfg.qkv_r                    # h + 2 * (key/value width); 3h without grouped-query attention
        kvd = cfg.kvd_r
        # the two row-parallel launches of a step (o_proj 2nh^2, down projection 2nhf) share a kernel family
        fl = {"gemm_nt_qkv": 2.0 * n * h * qkv_cols, "flash_attn_fwd": 2.0 * cfg.batch * s * s * h,
              "gemm_nt_rowpar": n * h * h + n * h * f, "gemm_nt_swiglu_fwd": 4.0 * n * h * f}
        # RoPE rewrites q and k in place and the same kernel stores k and v into the caches: read q, k, v; write q, k, K, V
        by = {"rope_kv_append": T * n * (2.0 * hd + 5.0 * kvd) * 2, "partial_sync_fwd": 3.0 * T * n * hs_of(cfg) * 2,
              "norm_fwd": 2.0 * T * n * h * 2,
              # reduce + residual + RMSNorm in one launch (as in the decode layer)
              "partial_sync_norm_fwd": (3.0 * T * n * hs_of(cfg) + T * n * (h - hs_of(cfg)) + T * n * h) * 2}
        work = n * (2.0 * h * qkv_cols + 2.0 * h * h + 6.0 * h * f) + 2.0 * cfg.batch * s * s * h
        unit, peak = "TFLOP/s", MFMA_BF16_PEAK_TFLOPS
        workload = ("%s prefill decoder layer fwd: h=%d ffn=%d heads=%d kv_heads=%d d=%d RoPE causal, %d prompts x %d tokens, "
                    "T=%d p=%g (hs=%d)" % (cfg.name, h, f, cfg.n_heads, cfg.kv_heads, cfg.head_dim, cfg.batch, s, T, cfg.p,
                                           hs_of(cfg)))
    else:
        bench = DecodeBench(cfg)
        fr = cfg.f_r
        kv_bytes = 2.0 * T * cfg.batch * (cfg.n_heads // T) * (cfg.kv_len + 1) * cfg.head_dim * 2
        w_bytes = 2.0 * T * (3 * hd * h + h * hd + 2 * fr * h + h * fr)
        fl = {}
        by = {"decode_attn": kv_bytes, "gemm_nt_qkv": 2.0 * T * 3 * hd * h, "gemm_nt_swiglu_fwd": 2.0 * T * 2 * fr * h,
              "gemm_nt_rowpar": 2.0 * T * (h * hd + h * fr) / 2, "partial_sync_fwd": 3.0 * T * n * hs_of(cfg) * 2,
              "norm_fwd": 2.0 * T * n * h * 2,
              # reduce + residual + RMSNorm in one launch: T partials and T residual slices and the private columns read,
              # R' shared columns and the whole normalised copy written
              "partial_sync_norm_fwd": (3.0 * T * n * hs_of(cfg) + T * n * (h - hs_of(cfg)) + T * n * h) * 2}
        work, unit, peak = kv_bytes + w_bytes, "GB/s", HBM_PEAK_GBS
        workload = "%s decode layer: h=%d ffn=%d heads=%d d=%d batch=%d kv_len=%d T=%d p=%g (hs=%d)" % (
            cfg.name, h, cfg.ffn, cfg.n_heads, cfg.head_dim, cfg.batch, cfg.kv_len, T, cfg.p, hs_of(cfg))
    desc = B.make_desc(cfg, reduce_in_gemm=args.reduce_in_gemm, dedup_shared=args.dedup_shared)
    ms, wall_ms = bench.time_steps(desc, args.steps, args.warmup)
    prof = bench.profile_steps(desc, max(3, min(args.steps, 10)))
    kernels = {}
    for name, v in prof.items():
        e = {"avg_ms": round(v["avg_ms"], 5), "launches_per_step": v["launches_per_step"]}
        if name in fl:
            e["TFLOP/s"] = round(fl[name] / v["avg_ms"] / 1e9, 1)
            e["frac_mfma_peak"] = round(fl[name] / v["avg_ms"] / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)
        if name in by:
            e["GB/s"] = round(by[name] / v["avg_ms"] / 1e6, 1)
            e["frac_hbm_peak"] = round(by[name] / v["avg_ms"] / 1e6 / HBM_PEAK_GBS, 4)
        kernels[name] = e
    dom = max(prof, key=lambda k: prof[k]["avg_ms"] * prof[k]["launches_per_step"])
    if args.config in ("C4", "C6", "C7"):
        value = work / ms / 1e9
        ach = fl.get(dom, 0.0) / prof[dom]["avg_ms"] / 1e9
        roof = {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
                "traffic": pmc_traffic_bytes(args.config, args.p, dom),
                "avg_launch_ms": prof[dom]["avg_ms"], "flops_per_launch": fl.get(dom, 0.0)}
    else:
        value = work / ms / 1e6
        ach = by.get(dom, 0.0) / prof[dom]["avg_ms"] / 1e6
        roof = {"bound": "hbm", "kernel": dom, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
                "traffic": pmc_traffic_bytes(args.config, args.p, dom),
                "avg_launch_ms": prof[dom]["avg_ms"], "bytes_per_launch": by.get(dom, 0.0)}
    out = {"metric": "partial-sync TP block TFLOP/s (% MFMA peak) + sync GB/s (% HBM) vs p, 1 GPU",
           "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": workload + (" [reduce in GEMM]" if args.reduce_in_gemm else "") +
                                  (" [shared channels stored once]" if args.dedup_shared else "") +
                                  (" [HIP graph replay]" if args.graph else ""), "work_per_step": work,
                      "frac_peak": value / peak, "wall_ms_per_step": wall_ms},
           "roofline": roof, "kernels": kernels}
    if args.config in ("C6", "C7"):
        # time to first token of a model made of this layer, and the paper's analytic model (App. C) next to the
        # measured p sweep.  On one GPU the "communication" is the in-HBM reduce over the T emulated ranks, so the
        # compute / communication capacity ratio C of the model is not a property of this machine; the model's linear
        # dependence on (1 - p) is what can be compared, with C fitted from the two end points p = 1 and p = 0.
        layers = 32 if args.config == "C6" else 80
        out["config"]["ttft_ms_%d_layers" % layers] = ms * layers
        sweep = []
        if not args.no_sweep and not args.dedup_shared:
            t = {}
            for p in (1.0, 0.5, 0.25, 0.0):
                c = base.with_(p=p)
                t[p], _ = bench.time_steps(B.make_desc(c, reduce_in_gemm=args.reduce_in_gemm), max(3, args.steps // 2), max(2, args.warmup // 2))
            s0 = (t[1.0] - t[0.0]) / t[1.0]                       # measured speed-up at p = 0 = 1 / (1 + (12h+2s)/(C r))
            c_fit = (12.0 * h + 2.0 * cfg.seq) / (T * (1.0 / s0 - 1.0)) if 0.0 < s0 < 1.0 else None
            for p in (1.0, 0.5, 0.25, 0.0):
                c = base.with_(p=p)
                sweep.append({"p": p, "hs": hs_of(c), "ms_per_layer": round(t[p], 4), "ttft_ms_%d_layers" % layers: round(t[p] * layers, 2),
                              "TFLOP/s": round(work / t[p] / 1e9, 1),
                              "speedup_vs_p1_measured": round((t[1.0] - t[p]) / t[1.0], 5),
                              "speedup_vs_p1_model": round((1.0 - p) * s0, 5),
                              "synced_payload_bytes_per_token_per_layer": 2 * 2 * hs_of(c)})
            out["analytic_model"] = {"form": "(T(1)-T(p))/T(1) = (1-p) / (1 + (12h+2s)/(C r)), G = (24sh^2+4s^2h)/r, P(p) = 2shp",
                                     "r": T, "h": h, "s": cfg.seq, "C_fitted_from_p1_and_p0": c_fit,
                                     "p_star_at_fitted_C": None if c_fit is None else min((12.0 * h + 2.0 * cfg.seq) / (c_fit * T), 1.0)}
        out["p_sweep"] = sweep
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline_other_kinds(args.config if args.config != "C7" else "C6", cfg,
                                                       args.config == "C4" and not args.fwd_only)
    if args.config == "C5":
        out["config"]["latency_us_per_token_step"] = ms * 1e3
        sweep = []
        if not args.no_sweep:
            for p in (1.0, 0.5, 0.25, 0.0):
                c = base.with_(p=p)
                ms_p, _ = bench.time_steps(B.make_desc(c, reduce_in_gemm=args.reduce_in_gemm), args.steps, args.warmup)
                sweep.append({"p": p, "hs": hs_of(c), "ms_per_step": round(ms_p, 5), "GB/s": round(work / ms_p / 1e6, 1),
                              "synced_payload_bytes_per_token_per_reduce": 2 * hs_of(c)})
        out["p_sweep"] = sweep
    return out


def other_configs(args):
    """Condensed records of the other benchmark configurations measured in the same run as the C2 headline: the 7B
    SwiGLU MLP block (C3, forward + backward) and the decode layer (C5) at p = 0.5, and C5's p sweep."""
    import copy
    import gc
    import torch
    from paper_2506_19645_amd import inputs as I
    out = {}
    for name in ("C3", "C5"):
        a = copy.copy(args)
        a.config, a.p, a.no_cpu = name, 0.5, True
        a.no_sweep = name != "C5"
        a.steps, a.warmup = (20, 8) if name == "C3" else (50, 10)
        base = I.CONFIGS[name]
        r = bench_mlp(a, base.with_(p=0.5), base) if name == "C3" else bench_attention_kinds(a, base.with_(p=0.5), base)
        rf = r["roofline"]
        e = {"workload": r["config"]["workload"], "value": round(r["value"], 1), "unit": r["unit"],
             "ms_per_step": round(r["ms_per_step"], 5), "steps": a.steps, "warmup": a.warmup,
             "frac_of_peak": round(r["value"] / (MFMA_BF16_PEAK_TFLOPS if r["unit"] == "TFLOP/s" else HBM_PEAK_GBS), 4),
             "dominant_kernel": {"kernel": rf["kernel"], "bound": rf["bound"], "achieved": round(rf["achieved"], 1),
                                 "unit": rf["unit"], "frac": round(rf["frac"], 4),
                                 "avg_launch_ms": round(rf["avg_launch_ms"], 5), "traffic": rf["traffic"]},
             "kernels": {k: {kk: vv for kk, vv in v.items() if kk in ("avg_ms", "launches_per_step", "frac_mfma_peak", "frac_hbm_peak")}
                         for k, v in r["kernels"].items()}}
        if name == "C5":
            e["latency_us_per_token_step"] = round(r["config"]["latency_us_per_token_step"], 2)
            e["p_sweep"] = r.get("p_sweep")
        out[name] = e
        del r
        gc.collect()
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "C6", "C7"])
    ap.add_argument("--p", type=float, default=0.5)
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--fwd-only", action="store_true", help="C4: time the forward alone")
    ap.add_argument("--reduce-in-gemm", action="store_true",
                    help="single-device serving mode: the sum over ranks of the shared channels is taken inside one "
                         "GEMM (no partial sums in HBM, no reduce pass) instead of the default reduce kernel")
    ap.add_argument("--cpu-sample-tokens", type=int, default=8192)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (known size) so that a rocprofv3 --pmc run can scale "
                         "FETCH_SIZE / WRITE_SIZE against it")
    ap.add_argument("--dedup-shared", action="store_true",
                    help="C6 / C7, implies --reduce-in-gemm: the residual stream stores its shared channels once "
                         "instead of T copies (no p sweep: the layout is tied to p)")
    ap.add_argument("--probe-hbm", action="store_true",
                    help="no workload: time the library's HBM streaming probe (read / copy, access pattern, "
                         "non-temporal hint) on a 2 GiB buffer and print one JSON line")
    ap.add_argument("--no-others", action="store_true",
                    help="default C2 run: leave out the condensed C3 / C5 records (other_configs)")
    ap.add_argument("--graph", action="store_true",
                    help="record one step into a HIP graph and time its replays (launch-bound small configs)")
    args = ap.parse_args()
    MlpBench.use_graph = args.graph
    if args.probe_hbm:
        import torch
        from paper_2506_19645_amd import binding as B
        nbytes = 1 << 31
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        names = ["read_chunk_per_workgroup", "read_chunk_per_workgroup_nontemporal", "read_grid_stride",
                 "copy_chunk_per_workgroup", "copy_chunk_per_workgroup_nontemporal"]
        res = {}
        for mode, name in enumerate(names):
            for _ in range(3):
                B.hbm_probe(src, dst, nbytes, mode)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                B.hbm_probe(src, dst, nbytes, mode)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 10
            moved = nbytes * (2 if mode >= 3 else 1)
            res[name] = {"ms": round(ms, 4), "GB/s": round(moved / ms / 1e6, 1), "frac_hbm_peak": round(moved / ms / 1e6 / HBM_PEAK_GBS, 4)}
        print(json.dumps({"probe": "hbm streaming, 2 GiB buffer, 16-byte accesses", "results": res}))
        return
    if args.dedup_shared:
        if args.config not in ("C6", "C7"):
            ap.error("--dedup-shared is for the prefill layer configs C6 / C7")
        args.reduce_in_gemm = True
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (all T tensor-parallel ranks are emulated on it); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_19645_amd import binding as B
    from paper_2506_19645_amd import inputs as I
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()
    base = I.CONFIGS[args.config]
    cfg = base.with_(p=args.p)
    if args.config in ("C4", "C5", "C6", "C7"):
        print(json.dumps(bench_attention_kinds(args, cfg, base)))
        return
    out = bench_mlp(args, cfg, base)
    if args.config == "C2" and not args.no_others:
        out["other_configs"] = other_configs(args)
    print(json.dumps(out))


def bench_mlp(args, cfg, base):
    """JSON for the MLP block configurations (C1-C3): forward + backward per step, TFLOP/s."""
    import torch
    from paper_2506_19645_amd import binding as B
    from paper_2506_19645_amd import inputs as I
    bench = MlpBench(cfg, seed=0)
    desc = B.make_desc(cfg, reduce_in_gemm=args.reduce_in_gemm, dedup_shared=args.dedup_shared)
    k = 3 if cfg.kind == I.KIND_MLP_SWIGLU else 2
    step_flops = 6.0 * cfg.tokens * cfg.h * cfg.ffn * k

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)          # the calibration kernel: reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst

    ms, wall_ms = bench.time_steps(desc, args.steps, args.warmup)
    value = step_flops / ms / 1e9     # TFLOP/s

    # per-kernel durations, live, HIP events on the launch stream
    prof = bench.profile_steps(desc, max(3, min(args.steps, 10)))
    gemms = {n: v for n, v in prof.items() if n.startswith("gemm")}
    dom = max(gemms, key=lambda n: gemms[n]["avg_ms"] * gemms[n]["launches_per_step"])
    dom_flops = flops_per_launch(dom, cfg)
    achieved = dom_flops / prof[dom]["avg_ms"] / 1e9
    roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                "traffic": pmc_traffic_bytes(args.config, args.p, dom),
                "avg_launch_ms": prof[dom]["avg_ms"], "flops_per_launch": dom_flops}
    if not args.no_sweep:
        roofline["power_check"] = gemm_power_check(torch, B, bench, cfg)
    kernels = {}
    for name, v in prof.items():
        e = {"avg_ms": round(v["avg_ms"], 5), "launches_per_step": v["launches_per_step"]}
        fl, by = flops_per_launch(name, cfg), sync_bytes(name, cfg, hs_of(cfg))
        if fl:
            e["TFLOP/s"] = round(fl / v["avg_ms"] / 1e9, 1)
            e["frac_mfma_peak"] = round(fl / v["avg_ms"] / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)
        if by:
            e["GB/s"] = round(by / v["avg_ms"] / 1e6, 1)
            e["frac_hbm_peak"] = round(by / v["avg_ms"] / 1e6 / HBM_PEAK_GBS, 4)
        kernels[name] = e

    sweep = []
    if not args.no_sweep:
        for p in (1.0, 0.5, 0.25, 0.0):
            c = base.with_(p=p)
            dsc = B.make_desc(c, reduce_in_gemm=args.reduce_in_gemm)
            ms_p, _ = bench.time_steps(dsc, args.steps, args.warmup)   # same warm-up as the headline: the clocks ramp
            # the reduce as a kernel of its own (the in-HBM stand-in for the collective): its time in the step against p
            dsep = B.make_desc(c, reduce_in_gemm=args.reduce_in_gemm, separate_reduce=True)
            ms_sep, _ = bench.time_steps(dsep, max(5, args.steps // 2), max(3, args.warmup // 2))
            pr = bench.profile_steps(dsep, 5)
            sa_ms, sa_gbs = standalone_sync(torch, B, c, hs_of(c))
            sc_ms, sc_gbs = standalone_sync(torch, B, c, hs_of(c), compact=True)
            e = {"p": p, "hs": hs_of(c), "ms_per_step": round(ms_p, 4), "TFLOP/s": round(step_flops / ms_p / 1e9, 1),
                 "ms_per_step_reduce_as_own_kernel": round(ms_sep, 4),
                 "synced_payload_bytes_per_token_per_reduce": 2 * hs_of(c),
                 "in_hbm_sync_bytes_per_token_fwd": 6 * c.T * hs_of(c), "in_hbm_sync_bytes_per_token_bwd": 4 * c.T * hs_of(c),
                 "standalone_sync_ms": round(sa_ms, 5), "standalone_sync_GB/s": round(sa_gbs, 1),
                 "standalone_sync_frac_hbm": round(sa_gbs / HBM_PEAK_GBS, 4),
                 "standalone_sync_compact_ms": round(sc_ms, 5), "standalone_sync_compact_GB/s": round(sc_gbs, 1),
                 "standalone_sync_compact_frac_hbm": round(sc_gbs / HBM_PEAK_GBS, 4)}
            for nm in ("partial_sync_fwd", "partial_sync_bwd"):
                if nm in pr:
                    e[nm + "_ms"] = round(pr[nm]["avg_ms"], 5)
                    e[nm + "_GB/s"] = round(sync_bytes(nm, c, hs_of(c)) / pr[nm]["avg_ms"] / 1e6, 1)
                else:
                    e[nm + "_ms"] = 0.0
            sweep.append(e)

    # time to sync against p: least-squares line through the four sweep points (slope = time per unit of p, i.e. the
    # part that scales with the synced volume; intercept = what a launch costs when nothing is synced)
    sync_fit = None
    if len(sweep) >= 3:
        ps = [e["p"] for e in sweep]
        fit = {}
        for key in ("partial_sync_fwd_ms", "partial_sync_bwd_ms", "standalone_sync_ms", "standalone_sync_compact_ms"):
            ts = [e[key] for e in sweep]
            pm, tm = sum(ps) / len(ps), sum(ts) / len(ts)
            sxx = sum((a - pm) ** 2 for a in ps)
            slope = sum((a - pm) * (b - tm) for a, b in zip(ps, ts)) / sxx
            icpt = tm - slope * pm
            ss_res = sum((b - (icpt + slope * a)) ** 2 for a, b in zip(ps, ts))
            ss_tot = sum((b - tm) ** 2 for b in ts)
            fit[key] = {"slope_ms_per_unit_p": round(slope, 5), "intercept_ms": round(icpt, 5),
                        "r2": round(1.0 - ss_res / ss_tot, 4) if ss_tot > 0 else None}
        sync_fit = fit

    out = {
        "metric": "partial-sync TP block TFLOP/s (% MFMA peak) + sync GB/s (% HBM) vs p, 1 GPU",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "%s MLP block fwd+bwd: h=%d ffn=%d %s %s T=%d p=%g (hs=%d) tokens=%d, seed 0, "
                               "x~N(0,1) w~N(0,0.02^2)" % (cfg.name, cfg.h, cfg.ffn, "SwiGLU" if k == 3 else "GELU",
                                                            "LayerNorm" if cfg.norm == 0 else "RMSNorm", cfg.T, cfg.p,
                                                            hs_of(cfg), cfg.tokens),
                   "flops_per_step": step_flops, "frac_mfma_peak": value / MFMA_BF16_PEAK_TFLOPS,
                   "wall_ms_per_step": wall_ms},
        "roofline": roofline, "kernels": kernels, "p_sweep": sweep, "sync_time_vs_p_fit": sync_fit,
    }
    if not args.no_sweep:
        out["hbm_copy_ceiling"] = copy_ceiling(torch, B)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, bench.host, args.cpu_sample_tokens)
    return out


if __name__ == "__main__":
    main()
