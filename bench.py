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
STACK_TRAFFIC_BYTES = {"self_attention": 65.3e6, "ff1": 122.6e6}


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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-patch", action="store_true")
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

    # ---------------------------------------------------------------- the stack (metric)
    p = G.make_stack_inputs(cfg, seed=0)
    sp = B.StackParams(p)
    x, ctx = B.to_bf16(p["x"]), B.to_bf16(p["ctx"])
    y = torch.empty_like(x)
    ws = torch.empty(B.spatial_transformer_workspace_bytes(cfg.Bn, cfg.T, cfg.C, cfg.Tc, cfg.Dc, sp.r_max), dtype=torch.uint8, device="cuda")

    def step():
        B.spatial_transformer_fwd(x, ctx, sp, cfg.heads, out=y, ws=ws)

    # The library only enqueues kernels on the stream it is given (no allocation, no
    # synchronisation), so one step can be captured once into a HIP graph and replayed: the
    # same launch-overhead removal the paper applies to the base model (Section 4.3).
    run = step
    launch = "stream"
    if not args.no_graph:
        step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run = graph.replay
        launch = "hipgraph"
    for _ in range(W):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        run()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    flops = stack_flops(cfg)
    tflops = flops / (ms_per_step * 1e-3) / 1e12

    # ---------------- per-kernel durations inside real steps (HIP events, eager launches)
    # The library records an event pair around each tagged kernel launch on the stream it is
    # given; K more steps of the same workload run eagerly for this (events cannot be read
    # back from a replayed graph).
    per_step = {"self_attention": cfg.depth, "cross_attention": cfg.depth, "qkv": cfg.depth,
                "attn_out": 2 * cfg.depth, "ff1": cfg.depth, "ff2": cfg.depth}
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
        "ff1": proj(M, C, 2 * F, rl),
        "ff2": proj(M, F, C, rl),
    }
    B.timing_enable(K * max(per_step.values()) + 8)
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    kernels = {}
    for tag, n in per_step.items():
        d = B.timing_collect(tag)
        ms = float(np.mean(d))
        kernels[tag] = {"launches": len(d), "avg_launch_ms": round(ms, 4),
                        "tflops": round(flop_per_launch[tag] / (ms * 1e-3) / 1e12, 1),
                        "share_of_step": round(n * ms / ms_per_step, 3)}
    B.timing_disable()
    dom = max(kernels, key=lambda k: kernels[k]["share_of_step"])
    names = {"self_attention": "attention_kernel, latent self-attention (2 x 10 heads x 4096 x 4096 x 64)",
             "ff1": "gemm_kernel, feed-forward in-projection with GEGLU epilogue",
             "ff2": "gemm_kernel, feed-forward out-projection", "qkv": "gemm_kernel, grouped q/k/v^T projections",
             "attn_out": "gemm_kernel, attention output projection", "cross_attention": "attention_kernel, cross-attention"}
    roofline = {"kernel": names[dom], "bound": "mfma", "achieved": kernels[dom]["tflops"], "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(kernels[dom]["tflops"] / PEAK_BF16_TFLOPS, 4),
                "traffic": STACK_TRAFFIC_BYTES.get(dom) if cfg is G.SDXL64 else None,
                "avg_launch_ms": kernels[dom]["avg_launch_ms"], "launches_per_step": per_step[dom],
                "share_of_step": kernels[dom]["share_of_step"],
                "measured": "HIP events around every launch of this kernel in %d eager steps" % K}

    out = {
        "metric": "SDXL transformer-block TFLOP/s (% bf16 MFMA peak); LoRA patch GB/s (% HBM)",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "batch": cfg.Bn, "tokens": cfg.T, "channels": cfg.C, "heads": cfg.heads,
                   "blocks": cfg.depth, "lora_rank": cfg.r, "text_ctx": [cfg.Tc, cfg.Dc], "gflop_per_step": round(flops / 1e9, 1),
                   "launch": launch},
        "frac_of_bf16_peak": round(tflops / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline,
        "kernels": kernels,
    }

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
    if not args.no_cpu_baseline:
        from oracle import sdxl_block_oracle as O
        # whole stack calls of the same workload until about 10 s of CPU work are done (at least one)
        calls, c0 = 0, time.perf_counter()
        while calls == 0 or (time.perf_counter() - c0 < 10.0 and calls < 8):
            O.spatial_transformer(p["x"], p["ctx"], p, cfg.heads)
            calls += 1
        c1 = time.perf_counter()
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        out["cpu_baseline"] = {"value": round(calls * flops / (c1 - c0) / 1e12, 4), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
                               "sample": "%d full stack call(s) of the same workload (fp64 numpy oracle), %.1f s" % (calls, c1 - c0)}
    out["context"] = "paper reports up to 7.8x latency / 1.6x throughput for SDXL end to end on H800; no kernel-level figure"
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
