#!/usr/bin/env python3
"""Benchmark of the GaLore optimizer step on one MI355X.

A "step" is one pass of the whole hot path (project, low-rank Adam, project back + apply; the
subspace refresh falls on step 0 and is timed apart) over every GaLore matrix of a synthetic
LLaMA-7B-shaped stack (32 layers x {4x 4096x4096, 2x 4096x11008, 11008x4096}, bf16 W/G, fp32
M/V, r = 1024), called one layer at a time in backward order, the way a per-layer weight update
during back-propagation calls it; consecutive calls overlap on the library's streams, which
are joined into the caller's stream once per step (galore_join), when the next forward pass
needs the weights.  On the step that carries the refresh a call takes two layers (the refresh is
latency-bound and cheaper per tensor with more tensors per launch).  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch (one LLaMA-7B layer set, r = 1024) from two rocprofv3 --pmc runs (FETCH_SIZE, then
# WRITE_SIZE) of `python3 bench.py --probe-traffic`, each scaled by what the same counter reads for the 1 GiB
# copy at the end of that run (profiles/step_llama7b_hbm_traffic.md has the commands and the table).  Counters
# cannot be read inside a timed run, so the figures are tied to the kernel sources they were measured on:
# `sources` is the digest of the files named in TRAFFIC_SOURCES at that time, and roofline.traffic is reported
# only while the digest still matches (null otherwise: re-run the probe and update both together).
TRAFFIC_SOURCES = ["gemm_mfma_dl.hpp", "gemm_proj_dl.hpp", "proj.hip", "gemm_mfma.hpp", "gemm_dispatch.hpp", "common.hpp", "adam.hip", "adam_entry.hpp"]
MEASURED_TRAFFIC_7B = {
    "sources": "7f1842964fa89488",
    "bytes": {   # read (2 x FETCH_SIZE KiB x 1024) + written (WRITE_SIZE KiB x 1024)
        "project_left": (708.1e6 + 218.9e6) + (16.8e6 + 1.0e6),   # the grouped projection launch of both orientations + the sum of the split tiles' slabs
        "project_left_fused_adam": (1420.5e6 + 636.7e6) + (19.0e6 + 2.6e6),
        "back": 1124.7e6 + 404.8e6,
        "adam": (471.9e6 + 135.3e6) + (393.2e6 + 112.7e6),
    },
}


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    for name in TRAFFIC_SOURCES:
        with open(os.path.join(ROOT, "paper_2403_03507_amd", "csrc", name), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def probe_traffic(layers=3, steps=2, fused_adam=False):
    """Workload of the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs: a few strictly serial steps of the library on
    LLaMA-7B-shaped layer sets with given projectors (no refresh: its thousands of short launches would only slow
    the counter run down), then ONE 1 GiB device-to-device copy whose traffic is known exactly (2^30 bytes read,
    2^30 written) and calibrates the counter."""
    import torch
    from paper_2403_03507_amd import binding as gb
    from paper_2403_03507_amd import workloads as wl
    torch.cuda.set_device(0)
    c = wl.CONFIGS["llama7b"]
    shapes = wl.layer_shapes(c["d"], c["f"])
    r = c["rank"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    W = [(torch.randn(m, n, generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(layers) for (m, n) in shapes]
    G = [(torch.randn(m, n, generator=gen, device="cuda") * 0.01).to(torch.bfloat16) for _ in range(layers) for (m, n) in shapes]
    opt = gb.GaLore(W, r, auto_refresh=False)
    gb.galore_set_concurrency(opt.ctx, 1)
    opt.set_fused_adam(fused_adam)
    for p in opt.proj:  # traffic does not depend on the values: a scaled Gaussian block stands in for a projector
        p.copy_((torch.randn(p.shape, generator=gen, device="cuda") / 64).to(torch.bfloat16))
    n7 = len(shapes)
    for s in range(steps):
        for l in reversed(range(layers)):
            opt.step(W[n7 * l: n7 * (l + 1)], G[n7 * l: n7 * (l + 1)], 1e-3, first=n7 * l)
        torch.cuda.synchronize()
        print("step", s, "done", flush=True)
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()
    print("copy done; kernel sources digest", kernel_sources_digest(), flush=True)


def probe_refresh():
    """Workload of the rocprofv3 --pmc runs that read the traffic of ONE subspace refresh: the seven tensors of a
    LLaMA-7B-shaped layer set (Gaussian bf16 gradients generated on the device; the launch sequence of a refresh does not
    depend on the values, only the number of Jacobi sweeps that still rotate does), r = 1024, four rounds, then the same
    1 GiB calibration copy as probe_traffic."""
    import torch
    from paper_2403_03507_amd import binding as gb
    from paper_2403_03507_amd import workloads as wl
    torch.cuda.set_device(0)
    c = wl.CONFIGS["llama7b"]
    shapes = wl.layer_shapes(c["d"], c["f"])
    gen = torch.Generator(device="cuda")
    gen.manual_seed(6)
    W = [(torch.randn(m, n, generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for (m, n) in shapes]
    G = [(torch.randn(m, n, generator=gen, device="cuda") * 0.01).to(torch.bfloat16) for (m, n) in shapes]
    opt = gb.GaLore(W, c["rank"], auto_refresh=False, refresh_iters=4)
    gb.galore_set_concurrency(opt.ctx, 1)
    opt.refresh(G)
    torch.cuda.synchronize()
    print("refresh done", flush=True)
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()
    print("copy done", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="llama7b")
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers (debug)")
    ap.add_argument("--refresh-iters", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--probe-traffic", action="store_true",
                    help="run only the workload of the rocprofv3 --pmc traffic runs (see probe_traffic) and exit")
    ap.add_argument("--probe-refresh", action="store_true",
                    help="run only one subspace refresh of a 7B layer set plus the calibration copy (see probe_refresh) and exit")
    ap.add_argument("--lanes", type=int, default=3, help="concurrent chains inside one galore_step call (1 = serial)")
    ap.add_argument("--moments", choices=["f32", "q8"], default="f32",
                    help="f32: fp32 moments (the headline configuration); q8: 8-bit block-wise moments (reported under its own metric name)")
    ap.add_argument("--fused-adam", type=int, choices=[0, 1], default=None,
                    help="1: Adam in the epilogue of the projection GEMM (two kernels per step); 0: separate Adam kernel (three).  Same "
                         "bits either way.  Default: whichever is faster in the stack's schedule (measured): 1 for llama7b, llama350m and "
                         "llama130m, 0 for llama1b; the fp32 llama60m stack has no fused epilogue")
    ap.add_argument("--in-flight", type=int, choices=[2, 3], default=None,
                    help="overlapped calls: calls in flight (library streams used) on ordinary steps.  Default: 2 for llama7b (measured "
                         "faster than 3 there: the tail of one call's GEMM hides under the next call's, a third call only adds "
                         "pressure on L2), 3 for the smaller stacks")
    ap.add_argument("--refresh-in-flight", type=int, choices=[2, 3], default=3,
                    help="calls in flight on the steps that carry a subspace refresh (its launches leave most of the chip idle, so three overlap well)")
    ap.add_argument("--layers-per-call", type=int, default=None,
                    help="layers handed to one galore_step call (0 = the whole stack in one call; the library cuts a call "
                         "into launch groups of at most 16 tensors).  Default: 1 for llama7b (the per-layer update the "
                         "headline configuration names), 2 for the smaller stacks, whose launches fill the chip better then")
    ap.add_argument("--refresh-layers-per-call", type=int, default=None,
                    help="layers handed to one call on the steps that carry a subspace refresh (t mod T == 0).  The refresh is a "
                         "long chain of short launches whose cost per tensor falls with the tensors per launch, so a training loop "
                         "can batch two layers on those steps only.  Default: 2 (or --layers-per-call if that is larger)")
    ap.add_argument("--join-every-call", action="store_true",
                    help="join the library streams at the end of every per-layer call (3 chains inside each call) "
                         "instead of overlapping consecutive calls and joining once per step")

    args = ap.parse_args()
    if args.layers_per_call is None:
        args.layers_per_call = 1 if args.config == "llama7b" else 2
    probe_fused = bool(args.fused_adam)  # the counter probes run the separate Adam kernel unless --fused-adam 1 is given
    if args.fused_adam is None:
        args.fused_adam = 1 if args.config in ("llama7b", "llama350m", "llama130m") else 0
    if args.in_flight is None:
        args.in_flight = 2 if args.config == "llama7b" else 3
    if args.refresh_layers_per_call is None:
        args.refresh_layers_per_call = max(args.layers_per_call, 2) if args.layers_per_call > 0 else 0
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (nothing here uses a "
              "second GPU)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2403_03507_amd import binding as gb
    from paper_2403_03507_amd import workloads as wl
    if not os.path.exists(gb.LIB_PATH):
        from paper_2403_03507_amd import build as lib_build
        lib_build.build()
    gb.lib()
    if args.probe_traffic:
        probe_traffic(fused_adam=probe_fused)
        return
    if args.probe_refresh:
        probe_refresh()
        return
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    dev = "cuda"

    cfg = dict(wl.CONFIGS[args.config])
    if args.layers is not None:
        cfg["layers"] = args.layers
    L, d, f, r = cfg["layers"], cfg["d"], cfg["f"], cfg["rank"]
    dtype = cfg["dtype"]
    tdt = wl.TORCH_DTYPE[dtype]
    shapes = wl.layer_shapes(d, f)
    n_per_layer = len(shapes)
    lr = 1e-3

    # ---- synthetic inputs, resident in HBM before anything is timed ------------------------------
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    W = []
    for _ in range(L):
        for (m, n) in shapes:
            W.append((torch.randn(m, n, generator=gen, device=dev, dtype=torch.float32) * 0.02).to(tdt))
    POOL = 4  # gradient layer-sets cycled through, so no step re-reads a cache-warm gradient
    srcs = wl.make_sources(cfg, seed=7, device=dev, layers=1)
    Gpool = [[s.grad(slot) for s in srcs] for slot in range(POOL)]
    del srcs
    torch.cuda.synchronize()

    # one call's workspace per call in flight: overlapped calls then overlap their subspace refreshes as well
    opt = gb.GaLore(W, r, update_gap=cfg["update_gap"], refresh_iters=args.refresh_iters, auto_refresh=True, moments=args.moments,
                    workspace_factor=max(args.in_flight, args.refresh_in_flight) * min(max(args.layers_per_call, args.refresh_layers_per_call, 1), 2))
    gb.galore_set_concurrency(opt.ctx, args.lanes)
    gb.galore_set_fused_adam(opt.ctx, args.fused_adam)
    overlap = args.in_flight if (not args.join_every_call and args.lanes > 1) else 0
    overlap_refresh = args.refresh_in_flight if overlap else 0
    gb.galore_set_call_overlap(opt.ctx, overlap)
    w_descs = [[gb.desc(w) for w in W[n_per_layer * l: n_per_layer * (l + 1)]] for l in range(L)]
    g_descs = [[gb.desc(g) for g in Gpool[s]] for s in range(POOL)]
    LPC = args.layers_per_call if args.layers_per_call > 0 else L
    LPC_REFRESH = args.refresh_layers_per_call if args.refresh_layers_per_call > 0 else L

    def call_arrays(lpc):
        # argument arrays are marshalled once: weights and pooled gradients stay where they are
        cw = {l: gb.tensor_array(x for k in range(l, min(l + lpc, L)) for x in w_descs[k]) for l in range(0, L, lpc)}
        # the layers of one call take consecutive gradient sets of the pool
        cg = [{l: gb.tensor_array(x for k in range(l, min(l + lpc, L)) for x in g_descs[(s + k - l) % POOL])
               for l in range(0, L, lpc)} for s in range(POOL)]
        return cw, cg

    grouping = {LPC: call_arrays(LPC)}
    if LPC_REFRESH not in grouping:
        grouping[LPC_REFRESH] = call_arrays(LPC_REFRESH)

    def one_step(step_index, refresh=False, serial=False):
        lpc = LPC_REFRESH if refresh else LPC
        call_w, call_g = grouping[lpc]
        if refresh and not serial and overlap_refresh != overlap:  # everything is joined between steps
            gb.galore_set_call_overlap(opt.ctx, overlap_refresh)
        for l in reversed(range(0, L, lpc)):  # backward order, one layer (or lpc layers) per call
            gb.galore_step(opt.ctx, call_w[l], call_g[(l // lpc + step_index) % POOL][l], n_per_layer * l, len(call_w[l]), lr)
        gb.galore_join(opt.ctx)  # the next forward pass needs the weights: one join per step
        if refresh and not serial and overlap_refresh != overlap:
            gb.galore_set_call_overlap(opt.ctx, overlap)

    def timed(fn):
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    # step 0: t mod T == 0 for every tensor, so it carries the subspace refresh (in the default schedule
    # the refreshes of consecutive calls overlap like the steps do)
    first_ms = timed(lambda: one_step(0, refresh=True))
    for w in range(1, max(args.warmup, 1)):
        one_step(w)
    K = args.steps
    base = max(args.warmup, 1)
    total_ms = timed(lambda: [one_step(base + i) for i in range(K)])
    ms_per_step = total_ms / K

    # Same K steps again, serial (one chain) and with every kernel group bracketed by HIP events on
    # the library's stream: concurrent chains share the CUs, so per-kernel durations are only
    # meaningful without overlap.
    gb.galore_set_call_overlap(opt.ctx, False)
    gb.galore_set_concurrency(opt.ctx, 1)
    serial_ms = timed(lambda: [one_step(base + K + i) for i in range(K)]) / K
    gb.galore_profile_start(opt.ctx)
    prof_total_ms = timed(lambda: [one_step(base + 2 * K + i) for i in range(K)])
    prof = gb.galore_profile_stop(opt.ctx)
    # one more refresh step, serial and bracketed by events: the refresh of one call on its own
    for i in range(len(W)):
        opt.set_step(i, 0)
    gb.galore_profile_start(opt.ctx)
    one_step(0, refresh=True, serial=True)
    torch.cuda.synchronize()
    refresh_serial_ms = gb.galore_profile_stop(opt.ctx)["refresh"][0]
    gb.galore_set_concurrency(opt.ctx, args.lanes)
    gb.galore_set_call_overlap(opt.ctx, overlap)

    # ---- roofline of the dominant kernel -----------------------------------------------------------
    left = [(m, n) for (m, n) in shapes if m <= n]
    right = [(m, n) for (m, n) in shapes if m > n]
    flops = {"project_left": sum(2.0 * m * n * r for m, n in left), "project_right": sum(2.0 * m * n * r for m, n in right)}
    flops["back"] = flops["project_left"] + flops["project_right"]
    if prof["project_right"][1] == 0:  # both orientations ran in the one grouped projection launch (recorded as project_left)
        flops["project_left"] += flops["project_right"]
    # work of ONE launch: a call's tensors are cut into launch groups of at most 16, so with several layers per call the
    # launches of a step share its work evenly enough for an average (the 7B default, one layer per call, is exact)
    flops = {k: v * L * K / max(prof[k][1], 1) for k, v in flops.items()}
    sN = 2 if dtype == "bf16" else 4
    if args.moments == "q8":  # read R and two code bytes, write two code bytes and N; four scale accesses per 256 elements
        adam_bytes = sum(r * max(m, n) * (4 + 4 + sN + 16.0 / 256) for m, n in shapes)
    else:
        adam_bytes = sum(r * max(m, n) * (4 * 5 + sN) for m, n in shapes)  # read R, M, V; write M, V, N
    stage_ms = {k: v[0] / max(v[1], 1) for k, v in prof.items()}        # average duration of one launch
    stage_ms["adam"] = prof["adam"][0] / max(K * L, 1)                  # Adam: two launches (one per orientation) per layer; 0 when fused
    gemm_stages = ["project_left", "project_right", "back"]
    dominant = max(gemm_stages + ["adam"], key=lambda k: prof[k][0])
    if dominant == "adam":
        achieved = adam_bytes / (stage_ms["adam"] * 1e-3) / 1e9
        roofline = {"kernel": "adam_group_kernel", "bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": achieved / PEAK_HBM_GBS, "traffic": None}
    else:
        peak = PEAK_BF16_TFLOPS if dtype == "bf16" else PEAK_F32_TFLOPS
        achieved = flops[dominant] / (stage_ms[dominant] * 1e-3) / 1e12
        # bf16 tensors of these shapes run on the large-tile kernel, fp32 tensors on the general one
        kname = {"project_left": "proj_dl_kernel/project", "project_right": "gemm_dl_kernel/project_right", "back": "gemm_dl_kernel/back"}
        roofline = {"kernel": kname[dominant] if dtype == "bf16" else "gemm_group_kernel/" + dominant, "bound": "mfma",
                    "achieved": achieved, "peak": peak,
                    "unit": "TFLOP/s", "frac": achieved / peak, "traffic": None}
    roofline["launch_ms"] = stage_ms[dominant]
    if dominant == "project_left" and args.fused_adam and args.moments == "f32" and dtype == "bf16":
        roofline["note"] = ("this launch also runs the Adam update of Algorithm 2 in its epilogue (18 bytes of moments and N per entry of R, "
                            "%.2f GB per launch: %.3f ms at the HBM peak) beside the flops counted here; the other GEMM of the step is "
                            "stages.back" % (sum(r * max(m, n) * (16 + sN) for m, n in shapes) * L * K / max(prof["project_left"][1], 1) / 1e9,
                                             sum(r * max(m, n) * (16 + sN) for m, n in shapes) * L * K / max(prof["project_left"][1], 1) / PEAK_HBM_GBS / 1e6))
    if args.config == "llama7b":
        if MEASURED_TRAFFIC_7B["sources"] == kernel_sources_digest():
            key = "project_left_fused_adam" if (dominant == "project_left" and args.fused_adam) else dominant
            roofline["traffic"] = MEASURED_TRAFFIC_7B["bytes"].get(key) if LPC == 1 else None
            roofline["traffic_unit"] = ("bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE of `bench.py --probe-traffic%s`, scaled by a " % (" --fused-adam 1" if key == "project_left_fused_adam" else "") +
                                        "1 GiB copy; hits in the 256 MB MALL are included; read on these kernel sources, not in this run)")
        else:
            roofline["traffic_unit"] = "null: the kernel sources changed since the counters were last read"
    per_stage = {}
    for k in gemm_stages:
        if prof[k][1]:
            per_stage[k] = {"ms_per_launch": stage_ms[k], "tflops": flops[k] / (stage_ms[k] * 1e-3) / 1e12}
    if prof["adam"][1]:
        per_stage["adam"] = {"ms_per_launch": stage_ms["adam"], "gbs": adam_bytes / (stage_ms["adam"] * 1e-3) / 1e9}

    # ---- CPU baseline: the fp64 oracle on a bounded sample --------------------------------------------
    cpu = None
    if not args.no_cpu_baseline and args.moments == "f32":  # the timed oracle is the fp32-moment step
        from oracle import galore_oracle as orc
        threads = orc.num_threads()

        def oracle_step_seconds(fraction):
            """One oracle step on every tensor of layer 0, one after the other, on the first `fraction` of the
            columns of a LEFT tensor / rows of a RIGHT tensor (the step is separable along the long side: column j
            of W, M, V depends on column j of G only).  Only the step itself is timed."""
            dt = 0.0
            for i, (m, n) in enumerate(shapes):
                left = m <= n
                keep = max(1, int(round(max(m, n) * fraction)))
                cut = (lambda x: x[:, :keep]) if left else (lambda x: x[:keep, :])
                Gs = cut(Gpool[0][i]).to("cpu").to(torch.float64).numpy()
                Ws = cut(W[i]).to("cpu").to(torch.float64).numpy()
                Ps = opt.proj[i].to("cpu").to(torch.float64).numpy()
                rr = orc.round_storage
                t0 = time.time()
                R = orc.project_left(Ps, Gs) if left else orc.project_right(Ps, Gs)
                Mo, Vo = np.zeros_like(R), np.zeros_like(R)
                N = orc.adam(R, Mo, Vo, 0.9, 0.999, 1e-8, 1)
                (orc.apply_left if left else orc.apply_right)(Ws, Ps, N, lr, 0.25, 0.0)
                Ws = rr(Ws, dtype)
                dt += time.time() - t0
            return dt

        import numpy as np
        dt_all = oracle_step_seconds(1.0)
        ONE_CORE_FRACTION = 1.0 / 32
        orc.set_num_threads(1)
        dt_one = oracle_step_seconds(ONE_CORE_FRACTION)
        orc.set_num_threads(threads)
        # the oracle's refresh (one-sided Jacobi SVD) on ONE square tensor of side min(d, 2048) at the stack's
        # rank-to-width ratio: its cost grows with the cube of the side, so the 7B stack's 4096 x 4096 would take
        # about 8 times as long (minutes) and is left out of the default run
        side = min(d, 2048)
        rr_rank = max(1, r * side // d)
        Gr = wl.GradientSource(side, side, 99, cfg["grad"], device="cpu", dtype=dtype, noise=cfg["noise"],
                               **{k: cfg[k] for k in ("signal_rank", "sigma0", "decay") if k in cfg}).grad(0)
        t0 = time.time()
        orc.projector(Gr.to(torch.float64).numpy(), rr_rank)
        dt_refresh = time.time() - t0
        cpu = {"value": dt_all * 1e3, "unit": "ms per layer set", "cores": threads, "kind": "oracle",
               "sample": "one oracle step (project, Adam, apply; projectors given) on each of the %d tensors of one layer "
                         "set of this workload, r=%d: %.1f s in all, no scaling" % (n_per_layer, r, dt_all),
               "one_core": {"value": dt_one / ONE_CORE_FRACTION * 1e3, "unit": "ms per layer set", "cores": 1,
                            "sample": "the same step on the first 1/32 of the columns (rows for the tall matrix) of each tensor, "
                                      "%.1f s on one thread, scaled by 32 (the step is separable along the long side)" % dt_one},
               "refresh": {"value": dt_refresh * 1e3, "unit": "ms per tensor", "cores": threads,
                           "sample": "the oracle's Jacobi SVD of ONE %d x %d gradient of this stack's spectrum, r=%d: %.1f s; "
                                     "cost grows with the cube of the side (a %d x %d tensor: about %.0fx)"
                                     % (side, side, rr_rank, dt_refresh, d, d, (d / side) ** 3)}}

    out = {
        # the benchmark's metric on its headline configuration; other stacks are labelled as what they are
        "metric": ("GaLore step ms per LLaMA-7B layer set @r=1024" if args.config == "llama7b"
                   else "GaLore step ms per %s layer set @r=%d" % (args.config, r)) + (" (8-bit moments)" if args.moments == "q8" else ""),
        "value": ms_per_step / L,
        "unit": "ms per layer set (7 matrices)",
        "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": "%s: %d layers x {4x %dx%d, 2x %dx%d, %dx%d}, %s W/G, %s M/V, r=%d, %s calls in "
                               "backward order, gradient pool of %d layer sets" % (args.config, L, d, d, d, f, f, d, dtype,
                                                                                   "fp32" if args.moments == "f32" else "8-bit", r,
                                                                                   "per-layer" if LPC == 1 else "%d-layer" % LPC, POOL),
                   "tensors": L * n_per_layer, "rank": r, "update_gap": cfg["update_gap"], "refresh_iters": args.refresh_iters,
                   "adam": ("in the projection GEMM's epilogue" if (args.fused_adam and args.moments == "f32" and dtype == "bf16")
                            else "separate kernel"),  # the fused epilogue exists for fp32 moments on the large-tile kernel only
                   "schedule": ("consecutive calls overlap on %d library streams (%d on a step with a refresh), one join per step" % (overlap, overlap_refresh)) if overlap else
                               "%d concurrent chains inside each call, joined every call" % args.lanes},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "stages": per_stage,
        "ms_per_step_serial": serial_ms,
        "ms_per_step_serial_with_events": prof_total_ms / K,
        # step 0 = refresh + step in the timed schedule; the serial figure is the sum of the refresh launches alone
        # amortised: the refresh of the whole stack spread over the T = update_gap steps between two refreshes, in
        # ms per step and as a fraction of the ordinary step next to it
        "refresh": {"step0_ms": first_ms, "ms_per_layer_set": (first_ms - ms_per_step) / L,
                    "ms_per_layer_set_serial": refresh_serial_ms / L,
                    "layers_per_call": min(LPC_REFRESH, L),
                    "amortised_ms_per_step": (first_ms - ms_per_step) / cfg["update_gap"],
                    "amortised_frac_of_step": (first_ms - ms_per_step) / cfg["update_gap"] / ms_per_step},
        "step_flops": 4.0 * sum(m * n for m, n in shapes) * r * L,
        "step_tflops": 4.0 * sum(m * n for m, n in shapes) * r * L / (ms_per_step * 1e-3) / 1e12,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
