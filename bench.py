#!/usr/bin/env python3
"""Benchmark of the SwiftDiffusion base-model hot path on one MI355X.

One step = one call of the whole spatial-transformer stack (GroupNorm, proj_in, the
LoRA-augmented blocks: self-attention, cross-attention, GEGLU feed-forward, proj_out) on
the classifier-free-guidance pair, at the SDXL 64x64-latent configuration (C = 640,
2 blocks, rank-64 adapters on every attention and feed-forward projection), inputs resident
in HBM.  The JSON line also carries the LoRA patch / unpatch sweep (GB/s), the multi-LoRA
projection batch (TFLOP/s), the roofline of the dominant kernel measured with HIP events,
and the CPU oracle timed on the host cores as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0    # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E
# HBM bytes per lora_patch launch on the 310-matrix sweep, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs of this file, each scaled by the same counter's reading on a pure copy of
# known size (lora_unpatch): see profiles/lora_patch_hbm_traffic.txt
PATCH_TRAFFIC_BYTES = 10.64e9   # FETCH_SIZE + WRITE_SIZE per patch launch, scaled (profiles/lora_patch_hbm_traffic.txt)
# the same two counters for the kernels that can be the stack's dominant one (same file), bytes per launch
STACK_TRAFFIC_BYTES = {"self_attention": 59.8e6, "ff1": 142.9e6}


def stack_flops(cfg) -> float:
    """Algorithmic FLOPs of one stack call: 2 per multiply-add, GEMM and attention work only,
    adapters counted in their unmerged rank-r form."""
    M, C, T, Bn, Tc, Dc, F, r = cfg.M, cfg.C, cfg.T, cfg.Bn, cfg.Tc, cfg.Dc, cfg.F, cfg.r
    Mc = Bn * Tc
    lin = 6 * 2 * M * C * C + 2 * 2 * Mc * Dc * C + 2 * M * C * 2 * F + 2 * M * F * C
    attn = 4 * Bn * T * T * C + 4 * Bn * T * Tc * C
    lora = 0
    if r:
        lora += 6 * 2 * M * r * (C + C)            # q1 k1 v1 o1 q2 o2
        lora += 2 * 2 * Mc * r * (Dc + C)          # k2 v2
        if cfg.lora_ff:
            lora += 2 * M * r * (C + 2 * F) + 2 * M * r * (F + C)
    return float(cfg.depth * (lin + attn + lora) + 2 * 2 * M * C * C)


def self_attention_flops(cfg) -> float:
    return float(4 * cfg.Bn * cfg.T * cfg.T * cfg.C)


def time_events(fn, iters: int):
    """Per-launch durations (ms) with HIP events on the stream the work is launched on
    (torch's current stream, which is the stream the binding passes to the library)."""
    import torch
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(iters)]
    for i in range(iters):
        starts[i].record()
        fn()
        ends[i].record()
    torch.cuda.synchronize()
    return [s.elapsed_time(e) for s, e in zip(starts, ends)]


GROUPS = 5     # timed groups of K steps each; the median group is the figure reported

KERNEL_NAMES = {
    "self_attention": "attention_kernel, latent self-attention",
    "cross_attention": "attention_kernel, cross-attention to the text tokens",
    "qkv": "gemm_kernel, grouped q/k/v^T projections (+ the next cross-attention's text k/v)",
    "attn_out": "gemm_kernel, attention output projection + residual",
    "cross_q": "gemm_kernel, cross-attention query projection",
    "ff1": "gemm_kernel, feed-forward in-projection with GEGLU epilogue",
    "ff2": "gemm_kernel, feed-forward out-projection + residual",
    "proj_io": "gemm_kernel, proj_in / proj_out",
    "layernorm": "layernorm_kernel",
    "groupnorm": "groupnorm_partial_kernel + groupnorm_apply_kernel",
}


class StackLeg:
    """One stack workload resident on the device: inputs, parameters, workspace, output."""

    def __init__(self, B, G, cfg, seed=0):
        import torch
        self.B, self.cfg = B, cfg
        self.p = G.make_stack_inputs(cfg, seed=seed)
        self.sp = B.StackParams(self.p)
        self.x, self.ctx = B.to_bf16(self.p["x"]), B.to_bf16(self.p["ctx"])
        self.y = torch.empty_like(self.x)
        self.ws = torch.empty(B.spatial_transformer_workspace_bytes(cfg.Bn, cfg.T, cfg.C, cfg.Tc, cfg.Dc, self.sp.r_max),
                              dtype=torch.uint8, device="cuda")

    def step(self):
        self.B.spatial_transformer_fwd(self.x, self.ctx, self.sp, self.cfg.heads, out=self.y, ws=self.ws)

    def param_bytes(self):
        """bf16 bytes of every parameter tensor of the stack"""
        n = 0
        stack = [self.p]
        while stack:
            d = stack.pop()
            for k, v in (d.items() if isinstance(d, dict) else enumerate(d)):
                if k in ("x", "ctx", "cfg"):
                    continue
                if isinstance(v, (dict, list)):
                    stack.append(v)
                elif hasattr(v, "size"):
                    n += int(v.size) * 2
        return n


def time_steps(step_fns, K, W, use_graph):
    """GROUPS groups of K steps (the step functions taken in turn), each group bracketed by a
    device synchronisation; returns (median ms per step, every group's ms per step, launch kind).
    With a graph, one replay runs every step function once."""
    import torch
    n = len(step_fns)
    if use_graph:
        for f in step_fns:
            f()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for f in step_fns:
                f()
        reps = max(1, K // n)

        def run_group():
            for _ in range(reps):
                graph.replay()
        steps_per_group = reps * n
    else:
        def run_group():
            for i in range(K):
                step_fns[i % n]()
        steps_per_group = K
    for _ in range(max(1, W // n) if use_graph else W):
        (graph.replay() if use_graph else step_fns[0]())
    torch.cuda.synchronize()
    groups = []
    for _ in range(GROUPS):
        t0 = time.perf_counter()
        run_group()
        torch.cuda.synchronize()
        groups.append((time.perf_counter() - t0) * 1e3 / steps_per_group)
    return float(sorted(groups)[len(groups) // 2]), groups, ("hipgraph" if use_graph else "stream")


def kernel_table(B, leg, K, ms_per_step):
    """Per-launch HIP-event durations of every kernel of the stack inside K eager steps."""
    import numpy as np
    import torch
    cfg = leg.cfg
    d = cfg.depth
    per_step = {"self_attention": d, "cross_attention": d, "qkv": d, "attn_out": 2 * d, "cross_q": d, "ff1": d, "ff2": d,
                "proj_io": 2, "layernorm": 3 * d, "groupnorm": 1}
    M, C, T, Bn, F, r = cfg.M, cfg.C, cfg.T, cfg.Bn, cfg.F, cfg.r
    rl = r if cfg.lora_ff else 0

    # every projection launch holds its down-projection tiles (x A^T), its base GEMM with the
    # K segment extended by r, and nothing else; the q/k/v launch also holds the next
    # cross-attention's text keys / values
    def proj(m, k, n, rr):
        return 2.0 * m * k * n + (2.0 * m * k * rr + 2.0 * m * rr * n if rr else 0.0)
    flop_per_launch = {
        "self_attention": 4.0 * Bn * T * T * C,
        "cross_attention": 4.0 * Bn * T * cfg.Tc * C,
        "qkv": 3 * proj(M, C, C, r) + 2 * proj(Bn * cfg.Tc, cfg.Dc, C, r),
        "attn_out": proj(M, C, C, r),
        "cross_q": proj(M, C, C, r),
        "ff1": proj(M, C, 2 * F, rl),
        "ff2": proj(M, F, C, rl),
        "proj_io": proj(M, C, C, 0),
    }
    # HBM-bound kernels: algorithmic bytes per launch (LayerNorm: fp32 stream in, bf16 out;
    # GroupNorm: bf16 in twice (statistics, apply), bf16 out)
    bytes_per_launch = {"layernorm": 6.0 * M * C, "groupnorm": 6.0 * M * C}
    B.timing_enable(K * max(per_step.values()) + 8)
    for _ in range(K):
        leg.step()
    torch.cuda.synchronize()
    kernels = {}
    for tag, n in per_step.items():
        dd = B.timing_collect(tag)
        ms = float(np.mean(dd))
        e = {"launches": len(dd), "launches_per_step": n, "avg_launch_ms": round(ms, 4), "share_of_step": round(n * ms / ms_per_step, 3)}
        if tag in flop_per_launch:
            e["tflops"] = round(flop_per_launch[tag] / (ms * 1e-3) / 1e12, 1)
            e["frac_of_bf16_peak"] = round(e["tflops"] / PEAK_BF16_TFLOPS, 4)
        else:
            e["gbs"] = round(bytes_per_launch[tag] / (ms * 1e-3) / 1e9, 1)
        kernels[tag] = e
    B.timing_disable()
    tagged = sum(k["share_of_step"] for k in kernels.values())
    return kernels, per_step, round(tagged, 3)


def vendor_gemm_context():
    """torch.matmul (bf16, [M, K] x [N, K]^T) on the shapes of ff1, q/k/v, an N = 640 projection and ff2 at config 2."""
    import numpy as np
    import torch
    res = {"what": "torch.matmul bf16, plain GEMM, 30 launches per graph replay, median of 5 replays", "us": {}, "tflops": {}}
    for name, (M, N, K) in (("ff1_8192x5120x704", (8192, 5120, 704)), ("qkv_8192x1920x704", (8192, 1920, 704)),
                            ("proj_8192x640x704", (8192, 640, 704)), ("ff2_8192x640x2624", (8192, 640, 2624))):
        a = torch.randn(M, K, device="cuda").to(torch.bfloat16)
        b = torch.randn(N, K, device="cuda").to(torch.bfloat16)
        c = torch.empty(M, N, device="cuda", dtype=torch.bfloat16)
        for _ in range(5):
            torch.matmul(a, b.t(), out=c)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            with torch.cuda.graph(g, stream=st):
                for _ in range(30):
                    torch.matmul(a, b.t(), out=c)
        g.replay()
        torch.cuda.synchronize()
        ts = []
        for _ in range(5):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / 30)
        ms = float(np.median(ts))
        res["us"][name] = round(ms * 1e3, 1)
        res["tflops"][name] = round(2.0 * M * N * K / (ms * 1e-3) / 1e12, 1)
        del g, a, b, c
    return res


def stack_leg_report(B, leg, K, W, use_graph):
    cfg = leg.cfg
    ms, groups, launch = time_steps([leg.step], K, W, use_graph)
    flops = stack_flops(cfg)
    tfl = flops / (ms * 1e-3) / 1e12
    kernels, per_step, tagged = kernel_table(B, leg, min(K, 20), ms)
    return {"workload": cfg.name, "ms_per_step": round(ms, 4), "group_ms_per_step": [round(g, 4) for g in groups],
            "gflop_per_step": round(flops / 1e9, 1), "tflops": round(tfl, 2), "frac_of_bf16_peak": round(tfl / PEAK_BF16_TFLOPS, 4),
            "launch": launch, "kernels": kernels, "tagged_share": tagged,
            "untagged_share": round(1.0 - tagged, 3)}, per_step


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-patch", action="store_true")
    ap.add_argument("--no-vendor-context", action="store_true", help="skip the vendor GEMM library timings (context only)")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the legs for the tiny and the 32x32 configuration")
    ap.add_argument("--no-graph", action="store_true", help="launch every step kernel by kernel instead of replaying a HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2407_02031_amd import binding as B
    from workloads import sdxl_inputs as G

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = G.SDXL64
    K, W = args.steps, args.warmup
    use_graph = not args.no_graph

    # ---------------------------------------------------------------- the stack (metric)
    # The library only enqueues kernels on the stream it is given (no allocation, no
    # synchronisation), so one step can be captured once into a HIP graph and replayed: the
    # same launch-overhead removal the paper applies to the base model (Section 4.3).
    leg = StackLeg(B, G, cfg, seed=0)
    p = leg.p
    rep, per_step = stack_leg_report(B, leg, K, W, use_graph)
    ms_per_step, tflops, kernels, flops = rep["ms_per_step"], rep["tflops"], rep["kernels"], stack_flops(cfg)
    dom = max((k for k in kernels if "tflops" in kernels[k]), key=lambda k: kernels[k]["share_of_step"])
    roofline = {"kernel": KERNEL_NAMES[dom], "bound": "mfma", "achieved": kernels[dom]["tflops"], "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(kernels[dom]["tflops"] / PEAK_BF16_TFLOPS, 4),
                "traffic": STACK_TRAFFIC_BYTES.get(dom),
                "avg_launch_ms": kernels[dom]["avg_launch_ms"], "launches_per_step": per_step[dom],
                "share_of_step": kernels[dom]["share_of_step"],
                "measured": "HIP events around every launch of this kernel in %d eager steps" % min(K, 20)}

    out = {
        "metric": "SDXL transformer-block TFLOP/s (% bf16 MFMA peak); LoRA patch GB/s (% HBM)",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.Bn, "tokens": cfg.T, "channels": cfg.C, "heads": cfg.heads,
                   "blocks": cfg.depth, "lora_rank": cfg.r, "text_ctx": [cfg.Tc, cfg.Dc], "gflop_per_step": round(flops / 1e9, 1),
                   "launch": rep["launch"], "timed": "median of %d groups of %d steps" % (GROUPS, K),
                   "cache_resident": True,
                   "cache_note": "weights %.0f MB + workspace %.0f MB < 256 MB last-level cache; see rotated_weights for the leg that is not"
                                 % (leg.param_bytes() / 1e6, leg.ws.numel() / 1e6)},
        "group_ms_per_step": rep["group_ms_per_step"],
        "frac_of_bf16_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline,
        "kernels": kernels,
        "tagged_share": rep["tagged_share"], "untagged_share": rep["untagged_share"],
    }

    # ---------------------- the same step with weights, inputs and workspaces rotated past the cache
    # In a UNet step the next block's weights are not the ones just used.  Three independent
    # sets (parameters drawn with other seeds, own workspace and I/O: 3 x ~190 MB > 256 MB) take
    # turns inside one captured graph, so no set finds its data in the last-level cache.
    legs = [leg] + [StackLeg(B, G, cfg, seed=s) for s in (1, 2)]
    rms, rgroups, _ = time_steps([l.step for l in legs], K, W, use_graph)
    out["rotated_weights"] = {"workload": cfg.name, "sets": len(legs),
                              "footprint_mb": round(sum(l.ws.numel() + 2 * l.x.numel() * 2 + l.param_bytes() for l in legs) / 1e6, 0),
                              "ms_per_step": round(rms, 4), "group_ms_per_step": [round(g, 4) for g in rgroups],
                              "tflops": round(flops / (rms * 1e-3) / 1e12, 2),
                              "frac_of_bf16_peak": round(flops / (rms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                              "vs_cache_resident": round(rms / ms_per_step, 3)}
    del legs

    # one step as a replayable graph for the loops below
    run = leg.step
    if use_graph:
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            leg.step()
        run = graph.replay

    # ------------------------------------------- the other stack configurations (report only)
    other = {}
    if not args.no_other_configs:
        for ocfg, oK in ((G.SDXL32, max(5, K // 5)), (G.TINY, K)):
            oleg = StackLeg(B, G, ocfg, seed=0)
            orep, _ = stack_leg_report(B, oleg, oK, W, use_graph)
            orep["steps_per_group"] = oK
            other[ocfg.name] = (oleg, orep)
            out.setdefault("other_configs", {})[ocfg.name] = orep

    # ------------------------------------------------------------ multi-LoRA projections
    mcfg = G.MULTI_LORA
    mp = G.make_multi_lora_inputs(mcfg, seed=0, n_proj=4)
    mx = B.to_bf16(mp["x"])
    mproj = [(B.to_bf16(pr["W"]), [B.to_bf16(a) for a in pr["A"]], [B.to_bf16(b) for b in pr["B"]], pr["scales"]) for pr in mp["projs"]]
    my = torch.empty((mx.shape[0], mcfg.C), dtype=torch.bfloat16, device="cuda")
    mws = torch.empty(B.lib().sd_multi_lora_linear_workspace_bytes(mx.shape[0], max(mcfg.ranks)), dtype=torch.uint8, device="cuda")

    def mstep():
        for Wd, Ad, Bd, sc in mproj:
            B.multi_lora_linear_fwd(mx, Wd, None, Ad, Bd, sc, mp["seg_offsets"], mp["seg_adapter"], out=my, ws=mws)

    for _ in range(3):
        mstep()
    md = float(np.mean(time_events(mstep, 20)))
    Mm = mx.shape[0]
    mfl = 4 * 2.0 * Mm * mcfg.C * mcfg.C
    for i, a in enumerate(mp["seg_adapter"]):
        rows = int(mp["seg_offsets"][i + 1] - mp["seg_offsets"][i])
        mfl += 4 * 2.0 * rows * mcfg.ranks[a] * (mcfg.C + mcfg.C)
    out["multi_lora"] = {"workload": mcfg.name, "ms": round(md, 4), "tflops": round(mfl / (md * 1e-3) / 1e12, 2),
                         "frac_of_bf16_peak": round(mfl / (md * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}
    del mx, my, mws, mproj

    # --------------------------------------------------------------- patch / unpatch sweep
    if not args.no_patch:
        gen = torch.Generator(device="cuda")
        gen.manual_seed(0)
        mats = []
        elems = 0
        ab = 0
        for count, o, i in G.PATCH_SWEEP:
            for _ in range(count):
                Wt = torch.randn((o, i), device="cuda", generator=gen) * 0.02
                At = torch.randn((G.PATCH_RANK, i), device="cuda", generator=gen) * 0.02
                Bt = torch.randn((o, G.PATCH_RANK), device="cuda", generator=gen) * 0.02
                mats.append((Wt, At, Bt, torch.empty_like(Wt), G.PATCH_ALPHA / G.PATCH_RANK))
                elems += o * i
                ab += G.PATCH_RANK * (o + i)
        plan = B.PatchPlan(mats)
        for _ in range(2):
            B.lora_patch(plan)
            B.lora_unpatch(plan)
        pt, ut = [], []
        for _ in range(10):
            pt += time_events(lambda: B.lora_patch(plan), 1)
            ut += time_events(lambda: B.lora_unpatch(plan), 1)
        pms, ums = float(np.mean(pt)), float(np.mean(ut))
        pbytes = elems * 12.0 + ab * 4.0     # read W, write W', write undo, read A and B once
        ubytes = elems * 8.0                 # read undo, write W
        out["patch"] = {"workload": "patch_sweep_310_matrices_r32_fp32", "elements": elems, "undo": "full fp32 snapshot written in the patch pass",
                        "patch_ms": round(pms, 4), "patch_gbs": round(pbytes / (pms * 1e-3) / 1e9, 1),
                        "patch_frac_of_hbm": round(pbytes / (pms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                        "unpatch_ms": round(ums, 4), "unpatch_gbs": round(ubytes / (ums * 1e-3) / 1e9, 1),
                        "unpatch_frac_of_hbm": round(ubytes / (ums * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                        "roofline": {"kernel": "lora_patch_kernel", "bound": "hbm", "achieved": round(pbytes / (pms * 1e-3) / 1e9, 1),
                                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(pbytes / (pms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                     "algorithmic_bytes": pbytes, "traffic": PATCH_TRAFFIC_BYTES}}
        # bounded asynchronous loading around a denoising loop: 50 stack steps (graph replays, the host
        # waits for each step as a sampler that reads the latent would), the
        # sweep's adapters (131 MB of A and B) arrive from two loader threads into pinned memory
        # while the loop runs unpatched; when the scheduler orders it, the loop copies them to the
        # device and patches all 310 matrices.  eps_patch = loop time with the patch minus without.
        n_loop, k_bound = 50, 30
        hostA = [torch.empty(m[1].shape, dtype=torch.float32).pin_memory() for m in mats]
        hostB = [torch.empty(m[2].shape, dtype=torch.float32).pin_memory() for m in mats]
        srcA = [m[1].cpu() for m in mats]
        srcB = [m[2].cpu() for m in mats]

        def loader(i):                                   # half of the matrices each
            for j in range(i, len(mats), 2):
                hostA[j].copy_(srcA[j])
                hostB[j].copy_(srcB[j])
            return 0

        def loop(with_bal):
            bal = B.Bal(2, loader) if with_bal else None
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            if bal:
                bal.start()
            for stp in range(1, n_loop + 1):
                if bal and bal.before_step(stp, k_bound):
                    for j, m in enumerate(mats):
                        m[1].copy_(hostA[j], non_blocking=True)
                        m[2].copy_(hostB[j], non_blocking=True)
                    B.lora_patch(plan)
                run()
                torch.cuda.synchronize()
            t1 = time.perf_counter()
            st = None
            if bal:
                st = bal.stats()
                if bal.finish():
                    B.lora_unpatch(plan)
                bal.close()
                torch.cuda.synchronize()
            return (t1 - t0) * 1e3, st

        loop(False)
        base_ms = min(loop(False)[0] for _ in range(3))
        bal_runs = [loop(True) for _ in range(3)]
        bal_ms, bal_st = min(bal_runs, key=lambda t: t[0])
        out["bal"] = {"workload": "50 stack steps with a host sync each, 310-matrix rank-32 adapter set (131 MB) loaded by 2 threads, bound k=30",
                      "loop_ms_without_lora": round(base_ms, 3), "loop_ms_with_bal": round(bal_ms, 3),
                      "eps_patch_ms": round(bal_ms - base_ms, 3), "patched_at_step": bal_st["patched_at_step"],
                      "load_ms": round(bal_st["load_s"] * 1e3, 2), "stall_ms": round(bal_st["stall_s"] * 1e3, 3)}
        del hostA, hostB, srcA, srcB

        # two adapters per matrix in one pass, with the bf16 serving copy (the production norm is
        # one or two LoRAs per request): W read once, W', undo and the bf16 copy written once
        multi = []
        for (Wt, At, Bt, Ut, sc) in mats:
            A2 = torch.randn(At.shape, device="cuda", generator=gen) * 0.02
            B2 = torch.randn(Bt.shape, device="cuda", generator=gen) * 0.02
            multi.append((Wt, Ut, torch.empty(Wt.shape, dtype=torch.bfloat16, device="cuda"), [(At, Bt, sc), (A2, B2, sc)]))
        mplan = B.PatchMultiPlan(multi)
        for _ in range(2):
            B.lora_patch_multi(mplan)
            B.lora_unpatch_multi(mplan)
        mt, mu = [], []
        for _ in range(6):
            mt += time_events(lambda: B.lora_patch_multi(mplan), 1)
            mu += time_events(lambda: B.lora_unpatch_multi(mplan), 1)
        mms, mus = float(np.mean(mt)), float(np.mean(mu))
        mbytes = elems * 14.0 + 2 * ab * 4.0
        out["patch_multi"] = {"workload": "patch_sweep_310_matrices_2_adapters_r32_fp32_plus_bf16_serving_copy",
                              "patch_ms": round(mms, 4), "patch_gbs": round(mbytes / (mms * 1e-3) / 1e9, 1),
                              "patch_frac_of_hbm": round(mbytes / (mms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                              "unpatch_ms": round(mus, 4), "unpatch_gbs": round(elems * 10.0 / (mus * 1e-3) / 1e9, 1),
                              "vs_two_single_passes": round(2 * pms / mms, 2)}
        del mats, plan, multi, mplan
        torch.cuda.empty_cache()

    # ------------------------------------------ classifier-free-guidance weighted sum (tiny)
    lat = torch.randn(2, 4 * 128 * 128, device="cuda").to(torch.bfloat16)     # the SDXL latent pair at 1024 x 1024
    lout = torch.empty_like(lat[0])
    B.cfg_combine(lat[0], lat[1], 7.5, out=lout)
    out["cfg_combine"] = {"elements": lat[0].numel(), "us": round(1e3 * float(np.median(time_events(lambda: B.cfg_combine(lat[0], lat[1], 7.5, out=lout), 20))), 2),
                          "note": "launch-bound: 384 KiB of traffic"}

    # ------------------------- ControlNet outputs summed into a skip connection (HBM-bound)
    # the largest SDXL injection point at 1024 x 1024: [2, 320, 128, 128] bf16, three ControlNets
    hsk = torch.randn(2 * 320 * 128 * 128, device="cuda").to(torch.bfloat16)
    rsk = [torch.randn_like(hsk) for _ in range(3)]
    osk = torch.empty_like(hsk)
    B.controlnet_residual_add(hsk, rsk, out=osk)
    rms = float(np.median(time_events(lambda: B.controlnet_residual_add(hsk, rsk, out=osk), 20)))
    rbytes = hsk.numel() * 2.0 * (len(rsk) + 2)
    out["controlnet_residual_add"] = {"workload": "skip_2x320x128x128_bf16_3_controlnets", "us": round(1e3 * rms, 2),
                                      "gbs": round(rbytes / (rms * 1e-3) / 1e9, 1), "frac_of_hbm": round(rbytes / (rms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                      "bytes_per_element": 2 * (len(rsk) + 2)}
    del hsk, rsk, osk

    # ---------------------------------------------------------------- measured ceilings
    # what this device sustains: a register-resident bf16 MFMA loop and a streaming fp32
    # copy, to set beside the vendor peaks the fractions above are quoted against
    cout = torch.empty(1024 * 256, dtype=torch.float32, device="cuda")
    cfl = [0.0]

    def mfma_loop():
        cfl[0] = B.ceiling_mfma_bf16(cout, 1024, 4000)

    mfma_loop()
    cm = float(np.median(time_events(mfma_loop, 5)))
    # vector-ALU issue rates (attention's other bound): one exponential in FMA slots, and whether
    # exponentials and FMAs overlap (mixed / (exp + fma) = 1: one port, no overlap)
    valu_ms, valu_n = [], []
    for mode in range(3):
        cnt = [None]

        def valu_loop(mode=mode, cnt=cnt):
            cnt[0] = B.ceiling_valu(cout, 1024, 4000, mode)

        valu_loop()
        valu_ms.append(float(np.median(time_events(valu_loop, 5))))
        valu_n.append(cnt[0])
    simds = 1024.0
    exp_ns = valu_ms[0] * 1e6 * simds / valu_n[0][0]
    fma_ns = valu_ms[1] * 1e6 * simds / valu_n[1][1]
    # 16 exponentials dealt between the 4 MFMAs of the matrix-core loop's trip, 3 wavefronts per SIMD
    # (attention's residency), against the MFMAs alone and the exponentials alone
    B.ceiling_valu(cout, 768, 4000, 3)
    t_both = float(np.median(time_events(lambda: B.ceiling_valu(cout, 768, 4000, 3), 5)))
    t_mfma = float(np.median(time_events(lambda: B.ceiling_mfma_bf16(cout, 768, 4000), 5)))
    t_exps = float(np.median(time_events(lambda: B.ceiling_valu(cout, 768, 8000, 0), 5)))
    valu = {"v_fma_f32_ns_per_wave_instruction_per_simd": round(fma_ns, 3), "v_exp_f32_ns_per_wave_instruction_per_simd": round(exp_ns, 3),
            "exp_in_fma_slots": round(exp_ns / fma_ns, 2), "mixed_over_sum_of_parts": round(valu_ms[2] / (valu_ms[0] + valu_ms[1]), 3),
            "mfma4_exp16_trip_over_mfma4_trip": round(t_both / t_mfma, 3), "mfma4_exp16_trip_over_sum_of_parts": round(t_both / (t_mfma + t_exps), 3)}
    csrc = torch.randn(1 << 28, device="cuda")           # 1 GiB, well past the last-level cache
    cdst = torch.empty_like(csrc)
    B.ceiling_copy_f32(csrc, cdst)
    cc = float(np.median(time_events(lambda: B.ceiling_copy_f32(csrc, cdst), 5)))
    mfma_ceiling = cfl[0] / (cm * 1e-3) / 1e12
    copy_ceiling = 8.0 * csrc.numel() / (cc * 1e-3) / 1e9
    del csrc, cdst
    # the same copy at the patch sweep's own footprint (3.3 GB each way): the 256 MB last-level
    # cache no longer helps, and this is the rate the patch kernels are up against
    big = 830668800
    csrc = torch.empty(big, device="cuda").normal_()
    cdst = torch.empty_like(csrc)
    B.ceiling_copy_f32(csrc, cdst)
    cb = float(np.median(time_events(lambda: B.ceiling_copy_f32(csrc, cdst), 5)))
    copy_large = 8.0 * big / (cb * 1e-3) / 1e9
    # ... and with two destinations: one read and two writes per element, the patch pass's mix
    cdst2 = torch.empty_like(csrc)
    B.ceiling_copy_1r2w_f32(csrc, cdst, cdst2)
    c2 = float(np.median(time_events(lambda: B.ceiling_copy_1r2w_f32(csrc, cdst, cdst2), 5)))
    copy_1r2w = 12.0 * big / (c2 * 1e-3) / 1e9
    del cdst2
    out["ceilings"] = {"mfma_bf16_tflops": round(mfma_ceiling, 1), "copy_f32_gbs": round(copy_ceiling, 1),
                       "copy_f32_gbs_at_patch_footprint": round(copy_large, 1),
                       "copy_1r2w_f32_gbs_at_patch_footprint": round(copy_1r2w, 1),
                       "valu": valu,
                       "value_frac_of_mfma_ceiling": round(tflops / mfma_ceiling, 4),
                       "dominant_kernel_frac_of_mfma_ceiling": round(kernels[dom]["tflops"] / mfma_ceiling, 4)}
    if "patch" in out:
        out["ceilings"]["patch_frac_of_copy_ceiling"] = round(out["patch"]["patch_gbs"] / copy_ceiling, 4)
        out["ceilings"]["unpatch_frac_of_copy_ceiling"] = round(out["patch"]["unpatch_gbs"] / copy_ceiling, 4)
        out["ceilings"]["patch_frac_of_copy_at_patch_footprint"] = round(out["patch"]["patch_gbs"] / copy_large, 4)
        out["ceilings"]["unpatch_frac_of_copy_at_patch_footprint"] = round(out["patch"]["unpatch_gbs"] / copy_large, 4)
        out["ceilings"]["patch_frac_of_1r2w_copy_at_patch_footprint"] = round(out["patch"]["patch_gbs"] / copy_1r2w, 4)
    del csrc, cdst, cout

    # --------------------------------------------------------------------- CPU baseline
    # The oracle as it stands (numpy in float64, one BLAS matmul per contraction) on the host
    # cores of this machine, on a bounded sample of each workload.  A baseline only.
    if not args.no_cpu_baseline:
        from oracle import sdxl_block_oracle as O
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        kind = "oracle (numpy fp64, BLAS)"

        def timed(fn, budget_s, max_calls):
            calls, c0 = 0, time.perf_counter()
            while calls == 0 or (time.perf_counter() - c0 < budget_s and calls < max_calls):
                fn()
                calls += 1
            return calls, time.perf_counter() - c0

        calls, dt = timed(lambda: O.spatial_transformer(p["x"], p["ctx"], p, cfg.heads), 8.0, 8)
        out["cpu_baseline"] = {"value": round(calls * flops / dt / 1e12, 4), "unit": "TFLOP/s", "cores": threads, "kind": kind,
                               "sample": "%d full stack call(s) of %s, %.1f s" % (calls, cfg.name, dt)}
        more = {}
        for name, (oleg, orep) in other.items():
            ocfg = oleg.cfg
            calls, dt = timed(lambda: O.spatial_transformer(oleg.p["x"], oleg.p["ctx"], oleg.p, ocfg.heads), 3.0, 3 if ocfg is G.TINY else 1)
            more[name] = {"value": round(calls * stack_flops(ocfg) / dt / 1e12, 4), "unit": "TFLOP/s", "cores": threads, "kind": kind,
                          "sample": "%d full stack call(s), %.1f s" % (calls, dt)}
        # one multi-LoRA projection of the batch (of the four the GPU leg runs)
        pr = mp["projs"][0]
        calls, dt = timed(lambda: O.multi_lora_linear(mp["x"], pr["W"], None, pr["A"], pr["B"], pr["scales"], mp["seg_offsets"], mp["seg_adapter"]), 2.0, 3)
        more[mcfg.name] = {"value": round(calls * (mfl / 4) / dt / 1e12, 4), "unit": "TFLOP/s", "cores": threads, "kind": kind,
                           "sample": "%d call(s) of one of the 4 projections (32768 rows), %.1f s" % (calls, dt)}
        # the patch sweep: every tenth matrix of the 310 (31 matrices, all five shapes), patch then unpatch, 3 passes
        sample = [(14, 1280, 1280), (6, 640, 640), (7, 1280, 2048), (2, 10240, 1280), (2, 1280, 5120)]
        pm = G.make_patch_inputs(sample, r=G.PATCH_RANK, alpha=G.PATCH_ALPHA, seed=0)
        pel = sum(d["W"].size for d in pm)
        pab = sum(d["A"].size + d["B"].size for d in pm)

        def patch_pass():
            for d in pm:
                w2, undo = O.lora_patch(d["W"], d["A"], d["B"], d["scale"])
                O.lora_unpatch(w2, undo)
        calls, dt = timed(patch_pass, 6.0, 3)
        more["patch_sweep"] = {"value": round(calls * (pel * 20.0 + pab * 4.0) / dt / 1e9, 2), "unit": "GB/s", "cores": threads, "kind": "oracle (numpy fp32, BLAS)",
                               "sample": "%d pass(es) of patch + unpatch over every tenth matrix (31 matrices, %.0f M elements; 12 + 8 B per element), %.1f s"
                                         % (calls, pel / 1e6, dt)}
        out["cpu_baselines_other_workloads"] = more
    # ------------------------------------------------------------ vendor library, context only
    # What the vendor's GEMM library (through torch.matmul) reaches on this machine on the plain GEMMs
    # underneath the block's largest projections: no LayerNorm, adapter, GEGLU or residual.  Not a
    # target and not part of the product path; it says how far the shapes themselves are from the
    # matrix cores' peak.
    if not args.no_vendor_context:
        try:
            out["vendor_library_context"] = vendor_gemm_context()
        except Exception as e:   # the library is not ours: report, do not fail the benchmark
            out["vendor_library_context"] = {"error": str(e)[:200]}
    out["context"] = "paper reports up to 7.8x latency / 1.6x throughput for SDXL end to end on H800; no kernel-level figure"
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
