"""Benchmark of the learned-optimizer step on one MI355X.

One "step" = one lopt_step() over the whole synthetic parameter set (all passes of the hot path),
with parameters, gradients and optimizer state already resident in HBM. Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2|3|4|5] [--optimizer small_fc_lopt|velo]
                  [--no-cpu-baseline]
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

# Vector-ALU instruction issue: 256 CUs x 4 SIMDs, one wave64 instruction per 4 cycles and SIMD, 2.4 GHz
VALU_ISSUE_PEAK_GINST = 256 * 4 * 2.4 / 4          # 614.4 G wave-instructions/s
# k_apply_f16s executes 320 vector instructions (20 of them MFMAs) per round of 64 elements, per-tile set-up and
# pipeline fill included (profiles/sq_counters_vit_b16.md)
APPLY_F16S_INST_PER_ROUND = 320

# Algorithmic work per element of the dominant pass:
#   apply pass, small_fc_lopt hidden 32: MLP contraction 28*32 + 32*32 + 32*2 MACs = 3968 FLOP
#   apply pass bytes: read g, p, M1..3, V (24 B) + write p (4 B) = 28 B
#   accum_stats pass bytes: read g, p, M1..3, V (24 B) + write M1..3, V (16 B) = 40 B
APPLY_FLOP_SMALL_FC = 2 * (28 * 32 + 32 * 32 + 32 * 2)
APPLY_BYTES = 28
ACCUM_BYTES = 40

# HBM bytes per launch of the dominant kernel, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and
# scaled by the factors a plain 256 MiB copy gives (2.0 / 1.0): see profiles/hbm_traffic_vit_b16.md.
# Keyed by (config, pass); other configurations report null.
MEASURED_TRAFFIC_BYTES = {
    (2, "apply"): (1_044_777 * 2.0 + 338_455) * 1024,
    (2, "accum_stats"): (1_020_355 * 2.0 + 1_353_160) * 1024,
    (3, "apply"): (1_024_089 * 2.0 + 338_155) * 1024,
    (3, "accum_stats"): (1_020_277 * 2.0 + 1_353_160) * 1024,
}


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
    inputs = []
    for i in idx:
        s = wl.tensors[i]
        inputs.append((W.init_param(config_id, i, s), W.grad(config_id, i, 0, s, wl.grad_kind), s.as_2d()[0]))
    n_el = sum(p.size for p, _, _ in inputs)
    t0 = time.perf_counter()
    for p, g, nd in inputs:
        st = O.init_state(*p.shape, cfg)
        O.tensor_step(p, g, st, weights, cfg, 0, 1.0, 0.0, ndim=nd)
    dt = time.perf_counter() - t0
    try:
        import threadpoolctl
        cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": n_el / dt / 1e9, "unit": "Gparams/s", "cores": int(cores), "kind": "oracle",
            "sample": f"one oracle step over the {len(idx)} tensors of the first four blocks "
                      f"({n_el} elements) of {wl.name}, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: the chip needs some tens of milliseconds of load before its clocks settle (with 3 warm-up steps the
    # first timed steps of the ViT-B/16 set run about 15 % slow and a 20-step average comes out 5 % high)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--optimizer", default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--micro", default=None,
                    help="time a micro-workload instead of a numbered config: layer1000 or mlp_w<W>_d<D>")
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
    import paper_2506_10315_amd as P

    wl = W.get_workload(args.config, args.optimizer)
    if args.micro:
        wl = W.micro_workload(args.micro, args.optimizer or "small_fc_lopt")
        args.config = wl.config_id
    if args.config == 5 and args.n_tiny is not None:
        wl.tensors = W.llama_1p3b_shapes(args.n_tiny)
    optimizer = wl.optimizer
    dev = "cuda:0"
    kind = P.LOPT_SMALL_FC if optimizer == "small_fc_lopt" else P.LOPT_VELO
    cfg = P.default_config(kind)
    weights = W.small_fc_weights(0, 32) if kind == P.LOPT_SMALL_FC else W.velo_weights(0)
    shapes = [t.shape for t in wl.tensors]
    n = len(shapes)
    n_el = wl.numel
    # inputs: seeded host draws, uploaded once; two gradient sets alternate between steps
    params = [torch.from_numpy(W.init_param(args.config, i, t)).to(dev) for i, t in enumerate(wl.tensors)]
    n_sets = 2 if n_el < 500_000_000 else 1
    grads = [[torch.from_numpy(W.grad(args.config, i, s, t, wl.grad_kind)).to(dev) for i, t in enumerate(wl.tensors)]
             for s in range(n_sets)]
    opt = P.LearnedOptimizer(cfg, weights, shapes, device=dev)
    step = 0

    def run(k):
        nonlocal step
        for _ in range(k):
            opt.step(params, grads[step % n_sets], lr=W.lr_at(wl, step % wl.steps), weight_decay=wl.weight_decay,
                     step=step)
            step += 1

    if args.calibrate_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)   # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # clocks settle after some tens of milliseconds of load: on the small sets, untimed extra steps make up for a
    # short --warmup (none with the defaults); the timed region is exactly --steps steps either way
    settle = max(0, 20 - args.warmup) if n_el < 200_000_000 else 0
    run(settle)
    run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # second pass of the same K steps with HIP events around every launch (on the same stream)
    opt.profile_enable(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    dt_prof = time.perf_counter() - t1
    pass_ms, k = opt.profile_read()
    opt.profile_enable(False)
    pass_ms = {name: v / max(k, 1) for name, v in pass_ms.items()}
    finite = all(bool(torch.isfinite(p).all()) for p in params[:8])

    dominant = max(pass_ms, key=pass_ms.get)
    dur_s = pass_ms[dominant] * 1e-3
    variant = os.environ.get("LOPT_APPLY", "auto")
    if dominant == "apply" and optimizer == "small_fc_lopt" and variant != "valu":
        # the MLP contraction runs on the matrix cores: fp32 MFMA (variant mfma_f32) or three fp16 MFMA terms
        # per product (default); either way the algorithmic work is the fp32 contraction of the paper's MLP
        f16 = variant in ("auto", "mfma_f16x3", "mfma_f16s")
        bound, unit = "mfma", "TFLOP/s"
        peak = MFMA_F16_PEAK_TFLOPS if f16 else MFMA_F32_PEAK_TFLOPS
        achieved = APPLY_FLOP_SMALL_FC * n_el / dur_s / 1e12
        kernel = ("apply (k_apply_f16x3: fp16 hi+lo operands, 3 MFMA terms, fp32 accumulate, row form)"
                  if variant == "mfma_f16x3" else
                  "apply (k_apply_f16s: fp16 hi+lo operands, 3 MFMA terms, fp32 accumulate, column strips, "
                  "software-pipelined)" if f16 else "apply (k_apply_mfma: fp32 MFMA)")
    else:
        bound, unit, peak = "hbm", "GB/s", HBM_PEAK_GBS
        per = APPLY_BYTES if dominant == "apply" else ACCUM_BYTES if dominant == "accum_stats" else 4
        achieved = per * n_el / dur_s / 1e9
        kernel = dominant
    roofline = {"bound": bound, "kernel": kernel, "achieved": achieved, "peak": peak, "unit": unit,
                "frac": achieved / peak, "traffic": MEASURED_TRAFFIC_BYTES.get((args.config, dominant)),
                "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE x2 + WRITE_SIZE, see profiles/)",
                "avg_launch_ms": pass_ms[dominant], "pass_ms": pass_ms,
                "ms_per_step_with_events": dt_prof / args.steps * 1e3}
    if dominant == "apply" and optimizer == "small_fc_lopt" and variant in ("auto", "mfma_f16s"):
        # what actually binds this kernel: vector-instruction issue (executed instructions, not algorithmic work)
        ginst = APPLY_F16S_INST_PER_ROUND * (n_el / 64) / dur_s / 1e9
        roofline["valu_issue"] = {"achieved": ginst, "peak": VALU_ISSUE_PEAK_GINST, "unit": "G wave-instructions/s",
                                  "frac": ginst / VALU_ISSUE_PEAK_GINST,
                                  "note": "executed vector instructions per 64 elements x rounds / launch time"}
        roofline["binding_resource"] = ("vector-instruction issue (valu_issue.frac): the matrix unit is busy about 43 % of the "
                                        "launch, HBM about 29 %; `frac` prices the algorithmic MLP FLOPs against the fp16 "
                                        "matrix peak because that is the unit the contraction runs on")
    if bound == "mfma":
        # the same algorithmic FLOP rate against the fp32 vector-ALU peak (what a kernel without matrix cores could reach)
        roofline["frac_of_fp32_vector_peak"] = achieved / MFMA_F32_PEAK_TFLOPS
    # whole step against the HBM roof at 72 algorithmic bytes per element (three sweeps: 4 + 40 + 28)
    roofline["step_hbm_frac"] = (72.0 * n_el / (dt / args.steps) / 1e9) / HBM_PEAK_GBS
    roofline["timing_note"] = ("pass_ms / avg_launch_ms: second run of the same K steps with per-pass HIP events, every pass "
                               "over the whole list on one stream (the tensor-group pipeline is off while events are on)")
    # every HBM-bound pass against the 8 TB/s roof (algorithmic bytes per element: 4 / 40 / 28)
    roofline["hbm_frac_by_pass"] = {
        name: (b * n_el / (pass_ms[name] * 1e-3) / 1e9) / HBM_PEAK_GBS
        for name, b in (("rowcol_sums", 4), ("accum_stats", ACCUM_BYTES), ("apply", APPLY_BYTES)) if pass_ms[name] > 0}
    out = {
        "metric": "optimizer-step throughput", "value": n_el / (dt / args.steps) / 1e9, "unit": "Gparams/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_steps": settle, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{'micro' if args.micro else 'config ' + str(args.config)}: {optimizer} on {wl.name} shapes "
                               f"({n} tensors, {n_el} fp32 elements), all tensors in one lopt_step",
                   "optimizer": optimizer, "hidden": int(cfg.hidden),
                   "launch": "lopt_step defaults (tensor-group pipeline on two streams for large small_fc_lopt lists)"
                             if not os.environ.get("LOPT_GROUPS") else "LOPT_GROUPS=" + os.environ["LOPT_GROUPS"]},
        "finite": finite,
        "roofline": roofline,
    }
    if not args.no_cpu_baseline and not args.micro:
        out["cpu_baseline"] = cpu_baseline(args.config, optimizer)
    opt.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
