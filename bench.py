#!/usr/bin/env python3
"""Benchmark of the sparse Winograd forward pass on one MI355X.

A "step" is one pass of the whole hot path (input transform, per-position sparse product,
output transform) over one batch of seeded synthetic input that is already resident in HBM.
Metric: effective TFLOP/s = FLOPs a dense direct convolution would execute / time (the paper's
Fig. 2 definition).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--density D] [--rotate R] [--backward]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
FP32_VECTOR_TFLOPS = 157.3  # MI355X fp32 vector, published (256 CU x 128 FMA lanes x 2 x 2.4 GHz)
STAGES = ("input_transform_kernel", "spmm_kernel", "output_transform_kernel")
# HBM-side bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a plain
# copy of known size (profiles/pmc_traffic_alexnet_conv3_n32_f4.md); known for the default workload only.
MEASURED_TRAFFIC = {
    ("alexnet_conv3_n32_f4", 0.10): {"input_transform_kernel": 24.51e6, "spmm_kernel": 51.77e6,
                                     "output_transform_kernel": 37.72e6},
}


def stage_models(cfg, nnz):
    """Algorithmic bytes and flops of each of the three kernels for one launch."""
    N, C, H, W, K = cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"]
    P, T, Ho, Wo = cfg["P"], cfg["T"], cfg["Ho"], cfg["Wo"]
    return [
        dict(bytes=4 * (N * C * H * W + P * C * T), flops=0),
        dict(bytes=4 * (P * C * T + P * K * T) + 8 * nnz, flops=2 * nnz * T),
        dict(bytes=4 * (P * K * T + N * K * Ho * Wo), flops=0),
    ]


def backward_stage_models(cfg, nnz, padded_entries):
    """Algorithmic bytes and flops of the seven backward kernels for one launch (launch order)."""
    N, C, H, W, K = cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"]
    P, T, Ho, Wo = cfg["P"], cfg["T"], cfg["Ho"], cfg["Wo"]
    ntb = (T + 63) // 64
    return [
        dict(bytes=4 * (N * K * Ho * Wo + P * K * T), flops=0),                      # dZ = A dO A^T
        dict(bytes=4 * (N * C * H * W + P * C * T), flops=0),                        # I_F again
        dict(bytes=4 * (P * C * T + P * K * T) + 8 * nnz + 4 * ntb * nnz, flops=2 * nnz * T),  # sampled products
        dict(bytes=4 * ntb * nnz + 8 * nnz, flops=0),                                # reduction to CSR order
        dict(bytes=4 * (P * K * T + P * C * T) + 8 * nnz, flops=2 * nnz * T),        # dI_F = W_F^T dZ
        dict(bytes=8 * P * C * T, flops=0),                                          # patches = B dI_F B^T
        dict(bytes=4 * (P * C * T + N * C * H * W), flops=0),                        # gather
    ]


def run_backward(args, sw, synth, torch, np, plan, cfg, name, x, xd, rp, ci, va, nnz, flops_direct, sp):
    """The backward pass (Section 3, Eq. 5 and Eq. 6): dL/dI and dL/dW_F (stored entries) from dL/dO."""
    dev = xd.device
    sw.swconv_set_weights(plan, rp, ci, va)
    G = np.random.default_rng(cfg["seed"] + 5).standard_normal((cfg["N"], cfg["K"], cfg["Ho"], cfg["Wo"])).astype(
        np.float32)
    gd = torch.from_numpy(G).to(dev)
    din = torch.empty_like(xd)
    dvals = torch.empty((max(1, nnz),), dtype=torch.float32, device=dev)
    a = (plan, sp, xd.data_ptr(), gd.data_ptr(), din.data_ptr(), dvals.data_ptr())
    for _ in range(args.warmup):
        sw.swconv_backward(*a)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sw.swconv_backward(*a)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    # the two gradients each cost what the forward pass costs as a direct convolution
    flops = 2 * flops_direct
    result = {
        "metric": "effective TFLOP/s of the backward pass (2 x direct-conv FLOPs / time), 1 MI355X",
        "value": round(flops / (elapsed / args.steps) / 1e12, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": name, "N": cfg["N"], "C": cfg["C"], "H": cfg["H"], "W": cfg["W"], "K": cfg["K"],
                   "winograd": "F(%dx%d,%dx%d)" % (cfg["m"], cfg["m"], cfg["r"], cfg["r"]), "pad": cfg["pad"],
                   "density": (nnz / float(cfg["P"] * cfg["K"] * cfg["C"])), "nnz": nnz,
                   "path": "backward (dL/dI and dL/dW_F)"},
    }
    stage_ms = sw.swconv_profile_backward(*a, args.steps)
    st = sw.swconv_plan_weight_stats(plan)
    models = backward_stage_models(cfg, nnz, st["padded_nnz"])
    names = list(sw.BACKWARD_STAGES)
    if stage_ms[6] == 0 and stage_ms[5] > 0:
        # Eq. 6's last two lines ran as one kernel (image planes in LDS, no patch buffer)
        names[5] = "input_grad_kernel"
        models[5] = dict(bytes=4 * (cfg["P"] * cfg["C"] * cfg["T"] + cfg["N"] * cfg["C"] * cfg["H"] * cfg["W"]), flops=0)
    stages = []
    ran = [i for i in range(len(names)) if stage_ms[i] > 0]     # kernels of the pass that were launched
    names, models, stage_ms = [names[i] for i in ran], [models[i] for i in ran], stage_ms[ran]
    for nm, ms, mdl in zip(names, stage_ms.tolist(), models):
        gbs = mdl["bytes"] / (ms * 1e-3) / 1e9 if ms > 0 else 0.0
        tfl = mdl["flops"] / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
        stages.append({"kernel": nm, "ms": round(ms, 6), "alg_bytes": mdl["bytes"], "alg_flops": mdl["flops"],
                       "GBps": round(gbs, 1), "hbm_frac": round(gbs / HBM_PEAK_GBS, 4), "TFLOPs": round(tfl, 3),
                       "fp32_frac": round(tfl / FP32_VECTOR_TFLOPS, 4)})
    dom = max(range(len(stages)), key=lambda i: stage_ms[i])
    d, mdl = stages[dom], models[dom]
    if mdl["bytes"] / (HBM_PEAK_GBS * 1e9) >= mdl["flops"] / (FP32_VECTOR_TFLOPS * 1e12):
        roof = {"bound": "hbm", "achieved": d["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": d["hbm_frac"]}
    else:
        roof = {"bound": "alu", "achieved": d["TFLOPs"], "peak": FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                "frac": d["fp32_frac"]}
    roof.update({"kernel": d["kernel"], "avg_ms": d["ms"], "traffic": None})
    result["roofline"] = roof
    result["stages"] = stages
    if not args.no_cpu_baseline:
        import oracle

        times = []
        t_start = time.perf_counter()
        while True:
            t0 = time.perf_counter()
            oracle.backward_f32(x, rp, ci, va, G, cfg["K"], cfg["m"], cfg["r"], cfg["pad"])
            times.append(time.perf_counter() - t0)
            if len(times) >= 5 or time.perf_counter() - t_start > 20.0:
                break
        t_med = sorted(times)[len(times) // 2]
        result["cpu_baseline"] = {"value": round(flops / t_med / 1e12, 5), "unit": "TFLOP/s",
                                  "cores": oracle.num_threads(), "kind": "oracle",
                                  "sample": "full workload (%d images), median of %d runs, fp32 instantiation"
                                            % (cfg["N"], len(times)),
                                  "seconds": round(t_med, 4)}
    sw.swconv_plan_destroy(plan)
    print(json.dumps(result))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default=None)
    ap.add_argument("--density", type=float, default=None)
    ap.add_argument("--dense", action="store_true", help="time the 0%%-sparsity MFMA comparison path instead")
    ap.add_argument("--backward", action="store_true",
                    help="time the backward pass of the layer (dL/dI and dL/dW_F from dL/dO) instead of the forward pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rotate", type=int, default=1, metavar="R",
                    help="cold-cache regime: step i runs on the i %% R-th of R independent sets of plan, workspaces, "
                         "input and output (choose R so that the sets exceed the 256 MB Infinity Cache)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="instead of the benchmark, run 20 plain device copies of this many MiB (a kernel of known "
                         "HBM traffic, used to scale the FETCH_SIZE / WRITE_SIZE counters of rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the forward path has no multi-GPU part); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1702_08597_amd import binding as sw
    from paper_1702_08597_amd import synth

    if args.copy_calibration > 0:
        n = args.copy_calibration * (1 << 20) // 4
        a = torch.ones(n, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        for _ in range(20):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_MiB": args.copy_calibration, "copies": 20,
                          "bytes_read_per_copy": n * 4, "bytes_written_per_copy": n * 4}))
        return

    name = args.workload or synth.BENCH_CONFIG
    cfg, x, rp, ci, va = synth.make_layer(name, density=args.density)
    nnz = int(rp[-1])
    flops_direct = synth.direct_conv_flops(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"], cfg["r"],
                                           cfg["pad"])

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    plan = sw.swconv_plan_create(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"], cfg["r"], cfg["pad"])
    xd = torch.from_numpy(x).to(dev)
    out = torch.empty((cfg["N"], cfg["K"], cfg["Ho"], cfg["Wo"]), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    sp, xp, op = stream.cuda_stream, xd.data_ptr(), out.data_ptr()
    if args.backward:
        run_backward(args, sw, synth, torch, np, plan, cfg, name, x, xd, rp, ci, va, nnz, flops_direct, sp)
        return
    if args.dense:
        wf = synth.dense_weights(cfg["P"], cfg["K"], cfg["C"], cfg["seed"] + 2000)
        sw.swconv_set_weights_dense(plan, wf)
        step = lambda i: sw.swconv_forward_dense(plan, sp, xp, op)
    else:
        t0 = time.perf_counter()
        sw.swconv_set_weights(plan, rp, ci, va)
        set_weights_ms = (time.perf_counter() - t0) * 1e3      # first call: allocates the workspaces too
        t0 = time.perf_counter()
        sw.swconv_set_weights(plan, rp, ci, va)
        update_weights_ms = (time.perf_counter() - t0) * 1e3   # a weight update: validate, re-pack, schedule, copy
        vd = torch.from_numpy(va).to(dev)
        sw.swconv_update_values(plan, sp, vd.data_ptr())
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(100):
            sw.swconv_update_values(plan, sp, vd.data_ptr())
        torch.cuda.synchronize()
        update_values_us = (time.perf_counter() - t0) / 100 * 1e6   # same pattern, new values, in place on the device
        sets = [(plan, xp, op)]
        keep = []
        for _ in range(1, max(1, args.rotate)):
            p2 = sw.swconv_plan_create(cfg["N"], cfg["C"], cfg["H"], cfg["W"], cfg["K"], cfg["m"], cfg["r"], cfg["pad"])
            sw.swconv_set_weights(p2, rp, ci, va)
            x2, o2 = xd.clone(), torch.empty_like(out)
            keep.append((x2, o2))
            sets.append((p2, x2.data_ptr(), o2.data_ptr()))
        step = lambda i: sw.swconv_forward(sets[i % len(sets)][0], sp, sets[i % len(sets)][1], sets[i % len(sets)][2])

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    value = flops_direct / (elapsed / args.steps) / 1e12

    result = {
        "metric": "effective TFLOP/s (direct-conv FLOPs / time), 1 MI355X",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": name, "N": cfg["N"], "C": cfg["C"], "H": cfg["H"], "W": cfg["W"], "K": cfg["K"],
                   "winograd": "F(%dx%d,%dx%d)" % (cfg["m"], cfg["m"], cfg["r"], cfg["r"]), "pad": cfg["pad"],
                   "density": (nnz / float(cfg["P"] * cfg["K"] * cfg["C"])), "nnz": nnz,
                   "path": "dense-mfma-comparison" if args.dense else "sparse",
                   "cache_regime": "warm (one buffer set)" if args.rotate <= 1 or args.dense
                                   else "cold (%d buffer sets in rotation)" % args.rotate},
        "paper_context": {"value": 31.7, "unit": "effective TFLOP/s fp32", "hardware": "2x Xeon Platinum 8180 (56 cores)",
                          "note": "paper's peak on pruned AlexNet 3x3 layers, batch 56; another machine and model"},
    }

    if not args.dense:
        # per-kernel durations: a pair of HIP events attached to every kernel launch on the launch
        # stream (the kernel's own start and end time stamps), over as many steps as the timed region
        stage_ms = sw.swconv_profile_forward(plan, sp, xp, op, args.steps)
        models = stage_models(cfg, nnz)
        names = list(STAGES)
        if stage_ms[2] == 0:
            # steps 2 and 3 ran as one kernel (m = 2, few input channels): the products stay on chip,
            # its algorithmic traffic is the transformed input, the weights and the output
            N, K, T = cfg["N"], cfg["K"], cfg["T"]
            names = [STAGES[0], "product_output_kernel"]
            models = [models[0], dict(bytes=4 * (cfg["P"] * cfg["C"] * T + N * K * cfg["Ho"] * cfg["Wo"]) + 8 * nnz,
                                      flops=2 * nnz * T)]
            stage_ms = stage_ms[:2]
        stages = []
        for nm, ms, mdl in zip(names, stage_ms.tolist(), models):
            gbs = mdl["bytes"] / (ms * 1e-3) / 1e9
            tfl = mdl["flops"] / (ms * 1e-3) / 1e12
            stages.append({"kernel": nm, "ms": round(ms, 6), "alg_bytes": mdl["bytes"], "alg_flops": mdl["flops"],
                           "GBps": round(gbs, 1), "hbm_frac": round(gbs / HBM_PEAK_GBS, 4),
                           "TFLOPs": round(tfl, 3), "fp32_frac": round(tfl / FP32_VECTOR_TFLOPS, 4)})
        dom = max(range(len(stages)), key=lambda i: stage_ms[i])
        d, mdl = stages[dom], models[dom]
        t_hbm = mdl["bytes"] / (HBM_PEAK_GBS * 1e9)
        t_alu = mdl["flops"] / (FP32_VECTOR_TFLOPS * 1e12)
        if t_hbm >= t_alu:
            roof = {"bound": "hbm", "achieved": d["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(d["GBps"] / HBM_PEAK_GBS, 4)}
        else:
            roof = {"bound": "alu", "achieved": d["TFLOPs"], "peak": FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(d["TFLOPs"] / FP32_VECTOR_TFLOPS, 4)}
        traffic = MEASURED_TRAFFIC.get((name, 0.10 if args.density is None else args.density), {}).get(d["kernel"])
        roof.update({"kernel": d["kernel"], "avg_ms": d["ms"], "traffic": traffic})
        result["roofline"] = roof
        result["stages"] = stages
        st = sw.swconv_plan_weight_stats(plan)
        result["weights"] = {"set_weights_ms": round(set_weights_ms, 3),
                             "update_weights_ms": round(update_weights_ms, 3),
                             "update_values_us": round(update_values_us, 2), "padded_nnz": st["padded_nnz"],
                             "work_items": st["work_items"]}

    if not args.no_cpu_baseline:
        import oracle

        # the oracle's float instantiation, as it stands, on the host cores of this machine
        n_img = cfg["N"]
        xs = x
        t_one = None
        times = []
        budget = 20.0
        t_start = time.perf_counter()
        while True:
            t0 = time.perf_counter()
            oracle.forward_f32(xs, rp, ci, va, cfg["K"], cfg["m"], cfg["r"], cfg["pad"])
            times.append(time.perf_counter() - t0)
            if len(times) >= 5 or time.perf_counter() - t_start > budget:
                break
        t_med = sorted(times)[len(times) // 2]
        result["cpu_baseline"] = {"value": round(flops_direct / t_med / 1e12, 5), "unit": "TFLOP/s",
                                  "cores": oracle.num_threads(), "kind": "oracle",
                                  "sample": "full workload (%d images), median of %d runs, fp32 instantiation"
                                            % (n_img, len(times)),
                                  "seconds": round(t_med, 4)}

    if not args.dense:
        for p2, _, _ in sets[1:]:
            sw.swconv_plan_destroy(p2)
    sw.swconv_plan_destroy(plan)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
