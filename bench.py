"""Benchmark of the learned-optimizer step on one MI355X.

One "step" = one lopt_step() over the whole synthetic parameter set (all passes of the hot path),
with parameters, gradients and optimizer state already resident in HBM. Prints ONE JSON line: the headline
workload (default: configuration 2, small_fc_lopt on ViT-B/16 shapes) and, with the default workload, an `also`
list with VeLO on the same shapes (configuration 3) and VeLO on the Llama-1.3B-shaped set with 2000 tiny tensors
(configuration 5), each timed the same way.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2|3|4|5] [--optimizer small_fc_lopt|velo]
                  [--no-cpu-baseline] [--no-also] [--micro NAME] [--graph]
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

import numpy as np

HBM_PEAK_GBS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3      # fp32 matrix (= packed fp32 vector) peak
MFMA_F16_PEAK_TFLOPS = 2500.0     # dense fp16/bf16 matrix peak

# Algorithmic work per element of the streaming passes:
#   apply pass, small_fc_lopt hidden 32: MLP contraction 28*32 + 32*32 + 32*2 MACs = 3968 FLOP
#   rowcol_sums: read g = 4 B. The pass that writes the new M1..3, V reads g, p, M1..3, V (24 B) and writes 16 B more:
#     state written by accum_stats (LOPT_STATE_PASS=stats, or an apply kernel other than the two default ones):
#       accum_stats 24 + 16 = 40 B, apply 24 + 4 (write p) = 28 B
#     state written by the apply pass (k_apply_f16s and k_apply_velo4, the default): accum_stats 24 B, apply 24 + 20 = 44 B
#   whole step: 44 B compulsory (24 read + 20 written), 72 B when the three dependent sweeps all go to HBM
APPLY_FLOP_SMALL_FC = 2 * (28 * 32 + 32 * 32 + 32 * 2)


def state_in_apply(apply_kernel):
    return apply_kernel in ("k_apply_f16s", "k_apply_velo4") and os.environ.get("LOPT_STATE_PASS", "auto") != "stats"


def pass_bytes(apply_kernel):
    in_apply = state_in_apply(apply_kernel)
    return {"rowcol_sums": 4, "accum_stats": 24 if in_apply else 40, "apply": 44 if in_apply else 28}


# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by what the same counters read
# for a plain 256 MiB copy: 2.0 and 1.0), keyed by (element count of the list, kernel, pass that writes the
# accumulators). A kernel or list that was not profiled reports null. Source: profiles/hbm_traffic_vit_b16.md.
MEASURED_TRAFFIC_BYTES = {
    (86_567_656, "k_apply_f16s", "apply"): (1_048_339 * 2.0 + 1_691_076) * 1024,
    (86_567_656, "k_apply_velo4", "apply"): (1_024_092 * 2.0 + 1_690_784) * 1024,
    (86_567_656, "k_accum_stats", "apply"): (1_019_353 * 2.0 + 540) * 1024,
    (86_567_656, "k_rowcol_sums", "apply"): (169_592 * 2.0 + 7_108) * 1024,
    (86_567_656, "k_apply_f16s", "stats"): (1_044_874 * 2.0 + 338_455) * 1024,
    (86_567_656, "k_apply_velo4", "stats"): (1_024_085 * 2.0 + 338_155) * 1024,
    (86_567_656, "k_accum_stats", "stats"): (1_020_449 * 2.0 + 1_353_160) * 1024,
    (86_567_656, "k_rowcol_sums", "stats"): (169_589 * 2.0 + 7_108) * 1024,
}

APPLY_KERNEL = {"auto": "k_apply_f16s", "mfma_f16s": "k_apply_f16s", "mfma_f32": "k_apply_mfma", "valu": "k_apply"}
APPLY_ARITH = {"k_apply_f16s": "fp16 hi+lo operands, 3 MFMA terms per product, fp32 accumulate (column strips, software-pipelined)",
               "k_apply_mfma": "fp32 MFMA", "k_apply": "fp32 vector ALU",
               "k_apply_velo4": "fp32 4x4x1 MFMA, per-tensor weights"}


def cpu_baseline(config_id: int, optimizer: str):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    import workloads as W
    from oracle import lopt_oracle as O
    wl = W.get_workload(config_id, optimizer)
    kind = O.KIND_SMALL_FC if optimizer == "small_fc_lopt" else O.KIND_VELO
    cfg = O.OracleConfig(kind=kind, hidden=32 if kind == O.KIND_SMALL_FC else 4)
    weights = W.small_fc_weights(0, 32) if kind == O.KIND_SMALL_FC else W.velo_weights(0)
    # sample: the tensors of the first four transformer blocks (every shape class of the repeated part;
    # sized for roughly 10-30 s of oracle time on the GPU machine's host cores)
    prefixes = tuple(f"{p}{i}." for p in ("blocks.", "h.", "layers.") for i in range(4))
    idx = [i for i, t in enumerate(wl.tensors) if t.name.startswith(prefixes)]
    ps = [W.init_param(config_id, i, wl.tensors[i]) for i in idx]
    gs = [W.grad(config_id, i, 0, wl.tensors[i], wl.grad_kind) for i in idx]
    sts = [O.init_state(*p.shape, cfg) for p in ps]
    n_el = sum(p.size for p in ps)
    t0 = time.perf_counter()
    O.list_step(ps, gs, sts, weights, cfg, 0, 1.0, 0.0, [wl.tensors[i].as_2d()[0] for i in idx], loss=W.loss_at(config_id, 0))
    dt = time.perf_counter() - t0
    try:
        import threadpoolctl
        cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": n_el / dt / 1e9, "unit": "Gparams/s", "cores": int(cores), "kind": "oracle",
            "sample": f"one oracle step over the {len(idx)} tensors of the first four blocks "
                      f"({n_el} elements) of {wl.name}, {dt:.1f} s"}


def measure(wl, config_id, steps, warmup, device_draws=False, graph=False):
    """Time `steps` steps of workload `wl` (after `warmup` untimed ones) and, in a second run of the same number of
    steps, every pass with HIP events recorded by lopt_step on the stream it launches on. Returns the measurement and
    the roofline view of the pass with the longest launches."""
    import torch
    import workloads as W
    import paper_2506_10315_amd as P

    optimizer = wl.optimizer
    dev = "cuda:0"
    kind = P.LOPT_SMALL_FC if optimizer == "small_fc_lopt" else P.LOPT_VELO
    cfg = P.default_config(kind)
    weights = W.small_fc_weights(0, 32) if kind == P.LOPT_SMALL_FC else W.velo_weights(0)
    shapes = [t.shape for t in wl.tensors]
    n = len(shapes)
    n_el = wl.numel
    n_sets = 2 if n_el < 500_000_000 else 1
    if device_draws:
        # the 1.3 G-element set: seeded draws of the same families made on the device (host draws take minutes)
        gen = torch.Generator(device=dev)
        gen.manual_seed(W.BASE_SEED + config_id)
        params, grads = [], [[] for _ in range(n_sets)]
        for i, t in enumerate(wl.tensors):
            _, rows, cols = t.as_2d()
            params.append(torch.randn(rows, cols, generator=gen, device=dev) * 0.02)
            sc = W.grad_scale(config_id, i, wl.grad_kind)
            for s in range(n_sets):
                grads[s].append(torch.randn(rows, cols, generator=gen, device=dev) * sc)
    else:
        params = [torch.from_numpy(W.init_param(config_id, i, t)).to(dev) for i, t in enumerate(wl.tensors)]
        grads = [[torch.from_numpy(W.grad(config_id, i, s, t, wl.grad_kind)).to(dev) for i, t in enumerate(wl.tensors)]
                 for s in range(n_sets)]
    opt = P.LearnedOptimizer(cfg, weights, shapes, device=dev)
    step = 0

    def run(k):
        nonlocal step
        for _ in range(k):
            opt.step(params, grads[step % n_sets], lr=W.lr_at(wl, step % wl.steps), weight_decay=wl.weight_decay,
                     step=step, loss=W.loss_at(config_id, step))
            step += 1

    # clocks settle after some tens of milliseconds of load: on the small sets, untimed extra steps make up for a
    # short --warmup (none with the defaults); the timed region is exactly `steps` steps either way
    settle = max(0, 20 - warmup) if n_el < 200_000_000 else 0
    run(settle)
    run(warmup)
    graph_info = None
    if graph:
        # one step captured into a HIP graph (static-scratch entry point: nothing allocates), replayed `steps` times
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            opt.step(params, grads[0], lr=W.lr_at(wl, 0), weight_decay=wl.weight_decay, step=step, static=True)
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                opt.step(params, grads[0], lr=W.lr_at(wl, 0), weight_decay=wl.weight_decay, step=step, static=True)
        torch.cuda.synchronize()
        for _ in range(5):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        graph_info = {"ms_per_replay": (time.perf_counter() - t0) / steps * 1e3,
                      "note": "one lopt_step_static captured in a HIP graph, same step replayed"}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # second pass of the same K steps with HIP events around every launch (on the same stream)
    opt.profile_enable(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    dt_prof = time.perf_counter() - t1
    pass_ms, k = opt.profile_read()
    opt.profile_enable(False)
    pass_ms = {name: v / max(k, 1) for name, v in pass_ms.items()}
    finite = all(bool(torch.isfinite(p).all()) for p in params)
    opt.close()
    del params, grads, opt
    torch.cuda.empty_cache()

    dominant = max(pass_ms, key=pass_ms.get)
    dur_s = pass_ms[dominant] * 1e-3
    variant = os.environ.get("LOPT_APPLY", "auto")
    apply_kernel = APPLY_KERNEL[variant] if optimizer == "small_fc_lopt" else ("k_apply_velo4" if variant != "valu" else "k_apply")
    kernel = apply_kernel if dominant == "apply" else "k_" + dominant
    PASS_BYTES = pass_bytes(apply_kernel)
    # the two roofs of that kernel: HBM at its algorithmic bytes, and (for the MLP contraction on the matrix cores) the
    # dense peak of the operand type the contraction runs in; the one that allows less is the bound
    hbm_gbs = PASS_BYTES.get(dominant, 0) * n_el / dur_s / 1e9
    roofline = {"kernel": kernel, "avg_launch_ms": pass_ms[dominant]}
    if dominant == "apply" and optimizer == "small_fc_lopt" and kernel != "k_apply":
        peak_tf = MFMA_F16_PEAK_TFLOPS if kernel == "k_apply_f16s" else MFMA_F32_PEAK_TFLOPS
        tflops = APPLY_FLOP_SMALL_FC * n_el / dur_s / 1e12
        t_hbm = PASS_BYTES["apply"] * n_el / (HBM_PEAK_GBS * 1e9)
        t_mfma = APPLY_FLOP_SMALL_FC * n_el / (peak_tf * 1e12)
        if t_hbm >= t_mfma:
            roofline.update(bound="hbm", achieved=hbm_gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=hbm_gbs / HBM_PEAK_GBS)
        else:
            roofline.update(bound="mfma", achieved=tflops, peak=peak_tf, unit="TFLOP/s", frac=tflops / peak_tf)
        roofline["roofs"] = {
            "hbm": {"algorithmic_bytes_per_element": PASS_BYTES["apply"], "achieved_GBs": hbm_gbs, "frac": hbm_gbs / HBM_PEAK_GBS},
            "mfma": {"algorithmic_flop_per_element": APPLY_FLOP_SMALL_FC, "operand_dtype_peak_TFLOPs": peak_tf,
                     "achieved_TFLOPs": tflops, "frac": tflops / peak_tf},
            "note": f"arithmetic intensity 3968 FLOP / {PASS_BYTES['apply']} B = {APPLY_FLOP_SMALL_FC / PASS_BYTES['apply']:.0f} FLOP/B; the ridge of the fp16 matrix roof is 312 FLOP/B, "
                    "so with the contraction on the fp16 matrix cores the HBM roof is the lower one; what occupies the "
                    "kernel in fact is vector-instruction issue (operand splits, ReLU, layer 3): profiles/sq_counters_vit_b16.md"}
        roofline["contraction"] = APPLY_ARITH[kernel]
    else:
        roofline.update(bound="hbm", achieved=hbm_gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=hbm_gbs / HBM_PEAK_GBS)
    roofline["traffic"] = MEASURED_TRAFFIC_BYTES.get((n_el, kernel, "apply" if state_in_apply(apply_kernel) else "stats"))
    roofline["state_written_by"] = "apply pass" if state_in_apply(apply_kernel) else "statistics pass"
    roofline["traffic_unit"] = "HBM bytes per launch of this kernel on this list (rocprofv3 FETCH_SIZE x2 + WRITE_SIZE, profiles/); null = not profiled"
    roofline["pass_ms"] = pass_ms
    roofline["ms_per_step_with_events"] = dt_prof / steps * 1e3
    roofline["hbm_frac_by_pass"] = {name: (b * n_el / (pass_ms[name] * 1e-3) / 1e9) / HBM_PEAK_GBS
                                    for name, b in PASS_BYTES.items() if pass_ms[name] > 0}
    # the whole step against the HBM roof: 44 B per element compulsory, 72 B when all three dependent sweeps go to HBM
    per_step_s = dt / steps
    roofline["step_hbm_frac_44B"] = (44.0 * n_el / per_step_s / 1e9) / HBM_PEAK_GBS
    roofline["step_hbm_frac_72B"] = (72.0 * n_el / per_step_s / 1e9) / HBM_PEAK_GBS
    roofline["timing_note"] = ("pass_ms / avg_launch_ms: second run of the same K steps with per-pass HIP events recorded by "
                               "lopt_step on its stream, every pass over the whole list (the tensor-group pipeline is off "
                               "while events are on)")
    res = {"optimizer": optimizer, "n_tensors": n, "n_elements": n_el, "ms_per_step": per_step_s * 1e3,
           "value": n_el / per_step_s / 1e9, "settle_steps": settle, "finite": finite, "roofline": roofline,
           "hidden": int(cfg.hidden), "dtype": dtype_of(optimizer, apply_kernel)}
    if graph_info:
        res["graph"] = graph_info
    return res


def dtype_of(optimizer, apply_kernel):
    if optimizer == "small_fc_lopt" and apply_kernel == "k_apply_f16s":
        return "f32 storage and arithmetic; MLP contraction as 3 fp16 MFMA terms on hi+lo operand pairs, fp32 accumulate"
    return "f32"


def workload_name(wl, config_id, micro):
    return (f"{'micro' if micro else 'config ' + str(config_id)}: {wl.optimizer} on {wl.name} shapes "
            f"({len(wl.tensors)} tensors, {wl.numel} fp32 elements), all tensors in one lopt_step")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: the chip needs some tens of milliseconds of load before its clocks settle (with 3 warm-up steps the
    # first timed steps of the ViT-B/16 set run about 15 % slow and a 20-step average comes out 5 % high)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=None)
    ap.add_argument("--optimizer", default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="default workload only: skip the `also` list")
    ap.add_argument("--micro", default=None,
                    help="time a micro-workload instead of a numbered config: layer1000, layer8192 or mlp_w<W>_d<D>")
    ap.add_argument("--graph", action="store_true",
                    help="also time one step captured in a HIP graph (lopt_step_static) and replayed")
    ap.add_argument("--n-tiny", type=int, default=None,
                    help="config 5 only: number of extra tiny 1-D tensors (default 2000)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device-to-device copy kernel (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; --gpus must be 1 (no collectives, no sharding here)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as W

    default_workload = args.config is None and args.micro is None and args.optimizer is None
    config_id = 2 if args.config is None else args.config
    wl = W.get_workload(config_id, args.optimizer)
    if args.micro:
        wl = W.micro_workload(args.micro, args.optimizer or "small_fc_lopt")
        config_id = wl.config_id
    if config_id == 5 and args.n_tiny is not None:
        wl.tensors = W.llama_1p3b_shapes(args.n_tiny)
    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")   # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    m = measure(wl, config_id, args.steps, args.warmup, device_draws=wl.numel > 500_000_000, graph=args.graph)
    out = {
        "metric": "optimizer-step throughput", "value": m["value"], "unit": "Gparams/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_steps": m["settle_steps"],
        "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": m["dtype"], "data": "synthetic",
        "config": {"workload": workload_name(wl, config_id, args.micro), "optimizer": wl.optimizer, "hidden": m["hidden"],
                   "launch": "lopt_step defaults (tensor-group pipeline on two streams for large small_fc_lopt lists)"
                             if not os.environ.get("LOPT_GROUPS") else "LOPT_GROUPS=" + os.environ["LOPT_GROUPS"]},
        "finite": m["finite"],
        "roofline": m["roofline"],
    }
    if "graph" in m:
        out["graph"] = m["graph"]
    if default_workload and not args.no_also:
        # the rest of the metric: VeLO on the same shapes, and VeLO on the 1.3B-shaped set (fewer steps: 20 ms each)
        also = []
        for cid, steps, warmup in ((3, args.steps, args.warmup), (5, max(3, args.steps // 4), max(2, args.warmup // 4))):
            w2 = W.get_workload(cid)
            r = measure(w2, cid, steps, warmup, device_draws=w2.numel > 500_000_000)
            rf = r["roofline"]
            also.append({"workload": workload_name(w2, cid, None), "optimizer": r["optimizer"], "steps": steps, "warmup": warmup,
                         "ms_per_step": r["ms_per_step"], "value": r["value"], "unit": "Gparams/s", "dtype": r["dtype"],
                         "data": "synthetic" + (" (seeded on-device draws)" if w2.numel > 500_000_000 else ""),
                         "finite": r["finite"],
                         "roofline": {k: rf[k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic",
                                                         "avg_launch_ms", "pass_ms", "hbm_frac_by_pass",
                                                         "step_hbm_frac_44B", "step_hbm_frac_72B")}})
        out["also"] = also
    if not args.no_cpu_baseline and not args.micro:
        out["cpu_baseline"] = cpu_baseline(config_id, wl.optimizer)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
