#!/usr/bin/env python3
"""Benchmark of the sparse Winograd forward pass on one MI355X.

A "step" is one pass of the whole hot path (input transform, per-position sparse product,
output transform) over one batch of seeded synthetic input that is already resident in HBM.
Metric: effective TFLOP/s = FLOPs a dense direct convolution would execute / time (the paper's
Fig. 2 definition).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--batches B] [--workload NAME] [--density D] [--rotate R]
                  [--no-cold] [--backward] [--dense]
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


def timed_batches(torch, step, stream, steps, batches, first=0):
    """`batches` runs of `steps` back-to-back launches, each between two HIP events recorded on the launch
    stream; returns the list of milliseconds per batch."""
    out = []
    i = first
    for _ in range(batches):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            step(i)
            i += 1
        e1.record(stream)
        e1.synchronize()
        out.append(e0.elapsed_time(e1))
    return out


def median(v):
    v = sorted(v)
    return v[len(v) // 2] if len(v) % 2 else 0.5 * (v[len(v) // 2 - 1] + v[len(v) // 2])


def oracle_baseline(oracle, cfg, x, rp, ci, va, flops_direct, budget_s=12.0):
    """The oracle's fp32 instantiation as it stands, on all host cores and on one, each on a bounded sample of
    the workload's images (the layer treats images independently; the rate is scaled by the image share)."""
    N = cfg["N"]

    def run(n_img, threads):
        oracle.set_num_threads(threads)
        t0 = time.perf_counter()
        oracle.forward_f32(x[:n_img], rp, ci, va, cfg["K"], cfg["m"], cfg["r"], cfg["pad"])
        return time.perf_counter() - t0

    all_threads = oracle.num_threads()
    res = {}
    for label, threads in (("all", all_threads), ("one", 1)):
        t_probe = run(1, threads)                       # one image: sizes the sample
        n_img = int(max(1, min(N, budget_s / 3.0 / max(t_probe, 1e-6))))
        times = []
        t_start = time.perf_counter()
        while len(times) < 3 and (not times or time.perf_counter() - t_start < budget_s):
            times.append(run(n_img, threads))
        t_med = median(times)
        res[label] = dict(value=round(flops_direct * (n_img / N) / t_med / 1e12, 5), cores=threads, images=n_img,
                          runs=len(times), seconds=round(t_med, 4))
    oracle.set_num_threads(all_threads)
    a, o = res["all"], res["one"]
    return {"value": a["value"], "unit": "TFLOP/s", "cores": a["cores"], "kind": "oracle",
            "sample": "%d of %d images, median of %d runs, fp32 instantiation (%.3f s per run)"
                      % (a["images"], N, a["runs"], a["seconds"]),
            "single_thread": {"value": o["value"], "cores": 1,
                              "sample": "%d of %d images, median of %d runs (%.3f s per run)"
                                        % (o["images"], N, o["runs"], o["seconds"])}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100, help="launches per timed batch")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batches", type=int, default=5,
                    help="timed batches of --steps launches, each between two HIP events; the median is reported")
    ap.add_argument("--workload", default=None)
    ap.add_argument("--density", type=float, default=None)
    ap.add_argument("--dense", action="store_true", help="time the 0%%-sparsity MFMA comparison path instead")
    ap.add_argument("--backward", action="store_true",
                    help="time the backward pass of the layer (dL/dI and dL/dW_F from dL/dO) instead of the forward pass")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold-cache measurement")
    ap.add_argument("--rotate", type=int, default=0, metavar="R",
                    help="cold-cache regime: step i runs on the i %% R-th of R independent sets of plan, workspaces, "
                         "input and output; 0 = as many as put three times the 256 MB Infinity Cache between two "
                         "uses of a buffer (at least 2)")
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
    N, C, K, P, T = cfg["N"], cfg["C"], cfg["K"], cfg["P"], cfg["T"]
    in_bytes, out_bytes = 4 * N * C * cfg["H"] * cfg["W"], 4 * N * K * cfg["Ho"] * cfg["Wo"]
    v_bytes, m_bytes, w_bytes = 4 * P * C * T, 4 * P * K * T, 8 * nnz
    set_bytes = in_bytes + out_bytes + v_bytes + m_bytes + w_bytes
    sets = [(plan, xp, op)]
    if args.dense:
        wf = synth.dense_weights(P, K, C, cfg["seed"] + 2000)
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
        step = lambda i: sw.swconv_forward(plan, sp, xp, op)

    # warm regime (one buffer set): W untimed steps, then `batches` x K steps, each batch between two HIP
    # events on the launch stream; the whole timed region also sits between two host clock readings with
    # the device synchronised on both sides
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    batch_ms = timed_batches(torch, step, stream, args.steps, args.batches)
    torch.cuda.synchronize()
    wall_ms_per_step = (time.perf_counter() - t0) / (args.steps * args.batches) * 1e3
    ms_per_step = median(batch_ms) / args.steps
    value = flops_direct / (ms_per_step * 1e-3) / 1e12

    result = {
        "metric": "effective TFLOP/s (direct-conv FLOPs / time), 1 MI355X",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": name, "N": N, "C": C, "H": cfg["H"], "W": cfg["W"], "K": K,
                   "winograd": "F(%dx%d,%dx%d)" % (cfg["m"], cfg["m"], cfg["r"], cfg["r"]), "pad": cfg["pad"],
                   "density": (nnz / float(P * K * C)), "nnz": nnz,
                   "path": "dense-mfma-comparison" if args.dense else "sparse",
                   "cache_regime": "warm (one buffer set of %.0f MB; the Infinity Cache holds 256 MB)" % (set_bytes / 1e6)},
        "timing": {"method": "median of %d batches of %d launches, each batch between two HIP events on the launch stream"
                             % (args.batches, args.steps),
                   "batch_ms_per_step": [round(b / args.steps, 6) for b in batch_ms],
                   "host_clock_ms_per_step": round(wall_ms_per_step, 6)},
        "paper_context": {"value": 31.7, "unit": "effective TFLOP/s fp32", "hardware": "2x Xeon Platinum 8180 (56 cores)",
                          "note": "paper's peak on pruned AlexNet 3x3 layers, batch 56; another machine and model"},
    }

    if not args.dense:
        # per-kernel durations: a pair of HIP events attached to every kernel launch on the launch
        # stream (the kernel's own start and end time stamps), over as many steps as one timed batch
        stage_ms = sw.swconv_profile_forward(plan, sp, xp, op, args.steps)
        models = stage_models(cfg, nnz)
        names = list(STAGES)
        if stage_ms[2] == 0:
            # steps 2 and 3 ran as one kernel: the products stay on chip, its algorithmic traffic is
            # the transformed input, the weights and the output
            names = [STAGES[0], "product_output_kernel"]
            models = [models[0], dict(bytes=v_bytes + out_bytes + w_bytes, flops=2 * nnz * T)]
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
        # HBM-side traffic is not measured inside this run (it needs rocprofv3 --pmc); the counter
        # summaries of the same command are under profiles/
        roof.update({"kernel": d["kernel"], "avg_ms": d["ms"], "traffic": None})
        result["roofline"] = roof
        result["stages"] = stages
        # the whole layer against its roofs: t_roof = max(bytes / HBM peak, non-zero FLOPs / fp32 peak), with
        # the bytes of the pass as built (every intermediate stored once and read once, minus what the fused
        # kernel keeps on chip), of three separate kernels, and of a fully fused pass (input, output, weights)
        built_bytes = sum(mm["bytes"] for mm in models)
        unfused_bytes = in_bytes + 2 * v_bytes + 2 * m_bytes + out_bytes + w_bytes
        fused_min_bytes = in_bytes + out_bytes + w_bytes
        t_meas = ms_per_step * 1e-3
        t_fma = 2 * nnz * T / (FP32_VECTOR_TFLOPS * 1e12)

        def layer_frac(b):
            return round(max(b / (HBM_PEAK_GBS * 1e9), t_fma) / t_meas, 4)

        result["whole_layer"] = {
            "as_built": {"bytes": built_bytes, "frac": layer_frac(built_bytes)},
            "unfused": {"bytes": unfused_bytes, "frac": layer_frac(unfused_bytes)},
            "fused_minimum": {"bytes": fused_min_bytes, "frac": layer_frac(fused_min_bytes)},
            "nonzero_flops": 2 * nnz * T, "nonzero_TFLOPs": round(2 * nnz * T / t_meas / 1e12, 3)}
        st = sw.swconv_plan_weight_stats(plan)
        result["weights"] = {"set_weights_ms": round(set_weights_ms, 3),
                             "update_weights_ms": round(update_weights_ms, 3),
                             "update_values_us": round(update_values_us, 2), "padded_nnz": st["padded_nnz"],
                             "work_items": st["work_items"]}

        if not args.no_cold:
            # cold regime: R independent sets of plan, workspaces, input and output in rotation, so that
            # every buffer has left the caches before it is used again
            R = args.rotate if args.rotate > 0 else max(2, -(-3 * 256 * (1 << 20) // set_bytes))
            keep = []
            for _ in range(1, R):
                p2 = sw.swconv_plan_create(N, C, cfg["H"], cfg["W"], K, cfg["m"], cfg["r"], cfg["pad"])
                sw.swconv_set_weights(p2, rp, ci, va)
                x2, o2 = xd.clone(), torch.empty_like(out)
                keep.append((x2, o2))
                sets.append((p2, x2.data_ptr(), o2.data_ptr()))
            cold_step = lambda i: sw.swconv_forward(sets[i % R][0], sp, sets[i % R][1], sets[i % R][2])
            for i in range(max(R, args.warmup)):
                cold_step(i)
            torch.cuda.synchronize()
            cold_ms = median(timed_batches(torch, cold_step, stream, args.steps, args.batches)) / args.steps
            result["cold"] = {"value": round(flops_direct / (cold_ms * 1e-3) / 1e12, 3), "ms_per_step": round(cold_ms, 6),
                              "buffer_sets": R, "bytes_in_rotation": R * set_bytes}
            for p2, _, _ in sets[1:]:
                sw.swconv_plan_destroy(p2)
            del keep

    if not args.dense:
        # What this machine's memory system gives a plain device-to-device copy of 1 GiB (read + written bytes per
        # second): the practical ceiling next to the published 8 TB/s that the fractions above are taken against.
        n = (1 << 30) // 4
        src = torch.ones(n, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(2):
            dst.copy_(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(10):
            dst.copy_(src)
        e1.record(stream)
        e1.synchronize()
        copy_gbs = 2 * n * 4 * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        result["device_copy"] = {"GBps": round(copy_gbs, 1), "frac_of_peak": round(copy_gbs / HBM_PEAK_GBS, 4),
                                 "what": "torch copy_ of 1 GiB, bytes read + written"}
        del src, dst

    if not args.no_cpu_baseline:
        import oracle

        result["cpu_baseline"] = oracle_baseline(oracle, cfg, x, rp, ci, va, flops_direct)

    sw.swconv_plan_destroy(plan)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
