#!/usr/bin/env python3
"""Benchmark of the GaLore optimizer step on one MI355X.

A "step" is one pass of the whole hot path (project, low-rank Adam, project back + apply; the
subspace refresh falls on step 0 and is timed apart) over every GaLore matrix of a synthetic
LLaMA-7B-shaped stack (32 layers x {4x 4096x4096, 2x 4096x11008, 11008x4096}, bf16 W/G, fp32
M/V, r = 1024), called one layer at a time in backward order, the way a per-layer weight update
during back-propagation calls it; consecutive calls overlap on the library's streams, which
are joined into the caller's stream once per step (galore_join), when the next forward pass
needs the weights.  Prints ONE JSON line.
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

# HBM bytes per launch (one LLaMA-7B layer set, r = 1024) from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# runs of paper_2403_03507_amd/traffic_probe.py, calibrated with a 1 GiB copy (see
# profiles/step_llama7b_hbm_traffic.md).  Reported as roofline.traffic; null for other shapes.
MEASURED_TRAFFIC_BYTES_7B = {
    "project_left": 590.0e6 + 157.6e6,
    "project_right": 205.7e6 + 45.1e6,
    "back": 1090.4e6 + 404.8e6,
    "adam": (472.0e6 + 135.3e6) + (393.2e6 + 112.7e6),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="llama7b")
    ap.add_argument("--layers", type=int, default=None, help="override the number of layers (debug)")
    ap.add_argument("--refresh-iters", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--lanes", type=int, default=3, help="concurrent chains inside one galore_step call (1 = serial)")
    ap.add_argument("--moments", choices=["f32", "q8"], default="f32",
                    help="f32: fp32 moments (the headline configuration); q8: 8-bit block-wise moments (reported under its own metric name)")
    ap.add_argument("--in-flight", type=int, choices=[2, 3], default=3, help="overlapped calls: calls in flight (library streams used)")
    ap.add_argument("--layers-per-call", type=int, default=1, choices=[1, 2],
                    help="layers handed to one galore_step call (the small stacks fill the chip better with 2)")
    ap.add_argument("--join-every-call", action="store_true",
                    help="join the library streams at the end of every per-layer call (3 chains inside each call) "
                         "instead of overlapping consecutive calls and joining once per step")

    args = ap.parse_args()
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
                    workspace_factor=args.in_flight * args.layers_per_call)
    gb.galore_set_concurrency(opt.ctx, args.lanes)
    overlap = args.in_flight if (not args.join_every_call and args.lanes > 1) else 0
    gb.galore_set_call_overlap(opt.ctx, overlap)
    w_descs = [[gb.desc(w) for w in W[n_per_layer * l: n_per_layer * (l + 1)]] for l in range(L)]
    g_descs = [[gb.desc(g) for g in Gpool[s]] for s in range(POOL)]
    LPC = args.layers_per_call
    # argument arrays are marshalled once: weights and pooled gradients stay where they are
    call_w = {l: gb.tensor_array(x for k in range(l, min(l + LPC, L)) for x in w_descs[k]) for l in range(0, L, LPC)}
    # the layers of one call take consecutive gradient sets of the pool
    call_g = [{l: gb.tensor_array(x for k in range(l, min(l + LPC, L)) for x in g_descs[(s + k - l) % POOL])
               for l in range(0, L, LPC)} for s in range(POOL)]

    def one_step(step_index):
        for l in reversed(range(0, L, LPC)):  # backward order, one layer (or LPC layers) per call
            gb.galore_step(opt.ctx, call_w[l], call_g[(l // LPC + step_index) % POOL][l], n_per_layer * l, len(call_w[l]), lr)
        gb.galore_join(opt.ctx)  # the next forward pass needs the weights: one join per step

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
    first_ms = timed(lambda: one_step(0))
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
    one_step(0)
    torch.cuda.synchronize()
    refresh_serial_ms = gb.galore_profile_stop(opt.ctx)["refresh"][0]
    gb.galore_set_concurrency(opt.ctx, args.lanes)
    gb.galore_set_call_overlap(opt.ctx, overlap)

    # ---- roofline of the dominant kernel -----------------------------------------------------------
    left = [(m, n) for (m, n) in shapes if m <= n]
    right = [(m, n) for (m, n) in shapes if m > n]
    flops = {"project_left": sum(2.0 * m * n * r for m, n in left), "project_right": sum(2.0 * m * n * r for m, n in right)}
    flops["back"] = flops["project_left"] + flops["project_right"]
    if L % LPC == 0:  # a launch covers the tensors of LPC layers
        flops = {k: v * LPC for k, v in flops.items()}
    sN = 2 if dtype == "bf16" else 4
    if args.moments == "q8":  # read R and two code bytes, write two code bytes and N; four scale accesses per 256 elements
        adam_bytes = sum(r * max(m, n) * (4 + 4 + sN + 16.0 / 256) for m, n in shapes)
    else:
        adam_bytes = sum(r * max(m, n) * (4 * 5 + sN) for m, n in shapes)  # read R, M, V; write M, V, N
    stage_ms = {k: v[0] / max(v[1], 1) for k, v in prof.items()}        # average duration of one launch
    stage_ms["adam"] = prof["adam"][0] / max(K * L, 1)                  # Adam: two launches (one per orientation) per layer
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
        roofline = {"kernel": ("gemm_dl_kernel/" if dtype == "bf16" else "gemm_group_kernel/") + dominant, "bound": "mfma",
                    "achieved": achieved, "peak": peak,
                    "unit": "TFLOP/s", "frac": achieved / peak, "traffic": None}
    roofline["launch_ms"] = stage_ms[dominant]
    if args.config == "llama7b":
        roofline["traffic"] = MEASURED_TRAFFIC_BYTES_7B[dominant] * (LPC if L % LPC == 0 else 1)
        roofline["traffic_unit"] = "bytes per launch (L2 fetch + write-back counters; cache hits in the 256 MB MALL are included)"
    per_stage = {}
    for k in gemm_stages:
        if prof[k][1]:
            per_stage[k] = {"ms_per_launch": stage_ms[k], "tflops": flops[k] / (stage_ms[k] * 1e-3) / 1e12}
    per_stage["adam"] = {"ms_per_launch": stage_ms["adam"], "gbs": adam_bytes / (stage_ms["adam"] * 1e-3) / 1e9}

    # ---- CPU baseline: the fp64 oracle on a bounded sample --------------------------------------------
    cpu = None
    if not args.no_cpu_baseline and args.moments == "f32":  # the timed oracle is the fp32-moment step
        from oracle import galore_oracle as orc
        dt = 0.0
        for i in range(n_per_layer):  # layer 0, one tensor after the other; only the step itself is timed
            Gs = Gpool[0][i].to("cpu").to(torch.float64).numpy()
            Ps = opt.proj[i].to("cpu").to(torch.float64).numpy()
            o = orc.GaLoreTensor(W[i].to("cpu").to(torch.float64).numpy(), r, dtype=dtype, auto_refresh=False)
            o.set_projector(Ps)
            t0 = time.time()
            o.step(Gs, lr)
            dt += time.time() - t0
            del o, Gs, Ps
        cpu = {"value": dt * 1e3, "unit": "ms per layer set", "cores": orc.num_threads(), "kind": "oracle",
               "sample": "one oracle step (project, Adam, apply; projectors given) on each of the %d tensors of one layer "
                         "set of this workload, r=%d: %.1f s in all, no scaling" % (n_per_layer, r, dt)}

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
                   "schedule": "consecutive calls overlap on %d library streams, one join per step" % overlap if overlap else
                               "%d concurrent chains inside each call, joined every call" % args.lanes},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "stages": per_stage,
        "ms_per_step_serial": serial_ms,
        "ms_per_step_serial_with_events": prof_total_ms / K,
        # step 0 = refresh + step in the timed schedule; the serial figure is the sum of the refresh launches alone
        "refresh": {"step0_ms": first_ms, "ms_per_layer_set": (first_ms - ms_per_step) / L,
                    "ms_per_layer_set_serial": refresh_serial_ms / L},
        "step_flops": 4.0 * sum(m * n for m, n in shapes) * r * L,
        "step_tflops": 4.0 * sum(m * n for m, n in shapes) * r * L / (ms_per_step * 1e-3) / 1e12,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
