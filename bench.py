#!/usr/bin/env python3
"""Stage-training throughput on one MI355X: forward + loss + backward + SGD update of one
pipeline stage on seeded synthetic data, through the C-ABI library.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config {1,2,5,6}] [--also 2 1] [--graph]

Prints ONE JSON line: samples/s of the whole step (inputs resident in HBM; K steps between two
device synchronisations, plus the median of the K per-step times from HIP events on the stream),
the roofline of the kernel family that takes the most time (HIP events around every launch in a
second pass, less the measured cost of the event pair) and the CPU oracle timed on this host as
a baseline.  The headline workload is the largest single-GPU configuration, config 5 (MobileNetV2
w1.4 at 224x224, batch 128, bf16); config 2 (32x32, batch 32, fp32, launch-latency bound) and
config 1 (the 1-D CNN) are measured in the same run and reported under "also".
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}

WORKLOADS = {
    1: dict(name="config1: 1D-CNN 9x128 -> 32/64/64 -> 6 classes, batch 8, fp32, whole model",
            net="cnn1d", batch=8, in_shape=(1, 128, 9), classes=6, dtype="f32", lr=0.01, mu=0.9, wd=0.0),
    2: dict(name="config2: MobileNetV2 w1.0, 32x32x3, 10 classes, batch 32, fp32, whole model as one stage",
            net="mbv2", width=1.0, stem_stride=1, batch=32, in_shape=(32, 32, 3), classes=10, dtype="f32",
            lr=0.01, mu=0.9, wd=4e-5),
    6: dict(name="1D-CNN 9x128 -> 32/64/64 -> 6 classes at batch 256 (sensor-window workload at a realistic batch), fp32, whole model",
            net="cnn1d", batch=256, in_shape=(1, 128, 9), classes=6, dtype="f32", lr=0.01, mu=0.9, wd=0.0),
    5: dict(name="config5: MobileNetV2 w1.4, 224x224x3, 1000 classes, batch 128, bf16 (fp32 masters), whole model",
            net="mbv2", width=1.4, stem_stride=2, batch=128, in_shape=(224, 224, 3), classes=1000, dtype="bf16",
            lr=0.01, mu=0.9, wd=4e-5),
}


def build_units(P, w):
    if w["net"] == "cnn1d":
        return P.models.cnn1d_units()
    return P.models.mobilenet_v2_units(w["width"], w["classes"], w["stem_stride"])


def oracle_baseline(w, seed, budget_s=10.0, one_thread=False):
    """Training steps of the CPU oracle (float64, as it stands) on a bounded sample of the
    same workload: the batch is cut so that a step takes seconds, and whole steps are repeated
    for about budget_s.  one_thread: with the numerical library held to one thread."""
    import synth
    from oracle import models as OM
    from oracle.stage import Stage
    from threadpoolctl import threadpool_info, threadpool_limits
    if one_thread:
        with threadpool_limits(limits=1):
            return oracle_baseline(w, seed, budget_s)
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    units = OM.cnn1d() if w["net"] == "cnn1d" else OM.mobilenet_v2(w["width"], w["classes"], w["stem_stride"])
    # rough cost model: config-2 batch 32 takes a few seconds; 224x224 images cost 49x more per sample
    per_sample = (w["in_shape"][0] * w["in_shape"][1]) / 1024.0 * (w.get("width", 1.0) ** 2)
    batch = int(max(2, min(w["batch"], 48.0 / max(per_sample, 1e-3))))
    st = Stage(units, w["in_shape"], 0, len(units))
    P = OM.init_params(units, seed)
    for i in range(len(units)):
        st.set_params(i, P[i])
    x = synth.normal(seed, "x", (batch,) + tuple(w["in_shape"]))
    labels = synth.labels(seed, "labels", batch, w["classes"])
    # repeat whole steps until about 10 s of CPU work have been timed
    t0 = time.perf_counter()
    nsteps = 0
    while True:
        st.forward(0, x)
        st.loss(0, labels)
        st.backward(0)
        st.update(w["lr"], w["mu"], w["wd"])
        nsteps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or nsteps >= 200:
            break
    return dict(value=batch * nsteps / dt, unit="samples/s", cores=int(threads), kind="oracle",
                sample=f"{nsteps} full training steps (fwd+loss+bwd+update) of the same network at batch {batch} "
                       f"of {w['batch']}, float64 numpy, {dt:.2f} s")


def load_traffic(config):
    """HBM bytes per launch per kernel family from the committed rocprofv3 --pmc summary
    (profiles/config<N>_pmc_traffic.txt: family fetch_bytes write_bytes, already scaled by the copy yardstick)."""
    path = os.path.join(ROOT, "profiles", f"config{config}_pmc_traffic.txt")
    out = {}
    if os.path.exists(path):
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and not line.startswith("#"):
                try:
                    out[f[0]] = float(f[1]) + float(f[2])
                except ValueError:
                    pass
    return out


def fused_rule_step_bytes(units, in_shape, batch, es):
    """Bytes a training step must move under the best legal fusion (the accounting the roofline of the WHOLE step
    uses): per convolution + BatchNorm (+ activation) with input `i` and output `z`, forward i + z, backward
    2 i + 3 z; a residual block 2 |out| more each way; global average pool its input each way; FC its operands;
    the update 20 bytes per parameter (+ 2 for the bfloat16 copy)."""
    import paper_2110_02781_amd.binding as B
    H, W, C = in_shape
    fwd = bwd = 0.0
    n_param = 0
    for u in units:
        k = u["kind"]
        if k == B.UNIT_CONV:
            Ho = (H + 2 * u.get("pad_h", 0) - u["kh"]) // u["stride"] + 1
            Wo = (W + 2 * u.get("pad_w", 0) - u["kw"]) // u["stride"] + 1
            i, z = batch * H * W * C * es, batch * Ho * Wo * u["cout"] * es
            fwd += i + z; bwd += 2 * i + 3 * z
            n_param += u["cout"] * u["kh"] * u["kw"] * C + 2 * u["cout"]
            H, W, C = Ho, Wo, u["cout"]
        elif k == B.UNIT_INVRES:
            ce, s_ = C * u["expand"], u["stride"]
            Ho, Wo = (H + 2 - 3) // s_ + 1, (W + 2 - 3) // s_ + 1
            xin = batch * H * W * C * es
            if u["expand"] != 1:
                z = batch * H * W * ce * es
                fwd += xin + z; bwd += 2 * xin + 3 * z
                n_param += ce * C + 2 * ce
            i, z = batch * H * W * ce * es, batch * Ho * Wo * ce * es
            fwd += i + z; bwd += 2 * i + 3 * z
            n_param += 9 * ce + 2 * ce
            i, z = z, batch * Ho * Wo * u["cout"] * es
            fwd += i + z; bwd += 2 * i + 3 * z
            n_param += u["cout"] * ce + 2 * u["cout"]
            if s_ == 1 and C == u["cout"]:
                fwd += 2 * z; bwd += 2 * z
            H, W, C = Ho, Wo, u["cout"]
        elif k == B.UNIT_GAP:
            fwd += batch * H * W * C * es; bwd += batch * H * W * C * es
            H = W = 1
        elif k == B.UNIT_FC:
            fwd += (batch * C + batch * u["cout"] + C * u["cout"]) * es
            bwd += 2 * (batch * C + batch * u["cout"] + C * u["cout"]) * es
            n_param += u["cout"] * C + u["cout"]
            C = u["cout"]
    upd = n_param * (20.0 + (2.0 if es == 2 else 0.0))
    return dict(forward=fwd, backward=bwd, update=upd, total=fwd + bwd + upd)


SPINUP_S = 1.0


def run_workload(config, steps, warmup, use_graph, ktrace, calibrate, seed):
    import torch
    import synth
    import paper_2110_02781_amd as P

    w = WORKLOADS[config]
    dev = torch.device("cuda:0")
    tdt = torch.float32 if w["dtype"] == "f32" else torch.bfloat16
    units = build_units(P, w)
    H, W_, C = w["in_shape"]
    model = P.model_create(units, H, W_, C, P.F32 if w["dtype"] == "f32" else P.BF16)
    L = P.model_num_units(model)
    stage = P.stage_create(model, 0, L, w["batch"], 1)
    params = P.models.init_unit_params(units, seed)
    for i in range(L):
        P.stage_import_weights(stage, i, params[i])
    x = torch.from_numpy(synth.normal(seed, "x", (w["batch"], H, W_, C)).astype(np.float32)).to(dev).to(tdt)
    labels = torch.from_numpy(synth.labels(seed, "labels", w["batch"], w["classes"])).to(dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    stream = torch.cuda.Stream()
    sp = stream.cuda_stream

    def step():
        P.stage_forward(stage, 0, x, None, sp)
        P.stage_loss(stage, 0, labels, loss, sp)
        P.stage_backward(stage, 0, None, None, sp)
        P.stage_update(stage, w["lr"], w["mu"], w["wd"], sp)

    run = step
    if use_graph:
        # the library only enqueues kernels and device-to-device copies, so a step can be captured
        step()
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step()
        run = graph.replay

    if calibrate:
        ca = torch.ones(1 << 26, dtype=torch.float32, device=dev)       # 256 MiB
        cb = torch.empty_like(ca)
        P.calibration_copy(cb, ca, ca.numel() * 4, sp)
        stream.synchronize()
        del ca, cb
    # untimed spin-up so that the clocks have ramped before the W warm-up steps (short kernels, cold box)
    t_spin = time.perf_counter()
    while time.perf_counter() - t_spin < SPINUP_S:
        for _ in range(10):
            run()
        torch.cuda.synchronize()
    for _ in range(warmup):
        run()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        for k in range(steps):
            marks[k].record(stream)          # on the stream the kernels are launched on
            run()
        marks[steps].record(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(steps))
    median_ms = per_step[len(per_step) // 2] if steps % 2 else 0.5 * (per_step[steps // 2 - 1] + per_step[steps // 2])
    final_loss = float(loss.item())
    es = 4 if w["dtype"] == "f32" else 2
    rule = fused_rule_step_bytes(units, w["in_shape"], w["batch"], es)
    res = dict(workload=w["name"], batch=w["batch"], units=L, dtype=w["dtype"], hip_graph=bool(use_graph),
               value=round(w["batch"] * steps / dt, 2), ms_per_step=round(dt / steps * 1e3, 4),
               median_ms_per_step=round(median_ms, 4), min_ms_per_step=round(per_step[0], 4),
               final_loss=round(final_loss, 4), roofline=None, kernels=[],
               whole_step=dict(alg_bytes=round(rule["total"]), alg_bytes_forward=round(rule["forward"]),
                               alg_bytes_backward=round(rule["backward"]), alg_bytes_update=round(rule["update"]),
                               achieved_GBps=round(rule["total"] / (median_ms * 1e-3) / 1e9, 1),
                               frac_of_hbm_peak=round(rule["total"] / (median_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                               note="bytes under the best legal fusion (conv+BN: forward in+z, backward 2in+3z; residual 2 out each "
                                    "way; update 20-22 B/param) / median step time / 8 TB/s"))

    # second pass: HIP events around every launch -> the dominant kernel family and its roofline
    if ktrace:
        traffic = load_traffic(config)
        P.ktrace_begin(1 << 16)
        nsteps = max(1, min(steps, 20))
        for _ in range(nsteps):
            step()
        rows = P.ktrace_end()
        pair_ms = sum(r["total_ms"] for r in rows if r["name"] == "__event_pair_overhead")
        rows = [r for r in rows if r["name"] != "__event_pair_overhead"]
        for r in rows:                       # take the cost of the event pair off every launch
            r["raw_total_ms"] = r["total_ms"]
            r["total_ms"] = max(r["total_ms"] - pair_ms * r["launches"], 0.05 * r["total_ms"])
        rows.sort(key=lambda r: -r["total_ms"])
        tot = sum(r["total_ms"] for r in rows) or 1.0
        for r in rows:
            avg_us = r["total_ms"] / r["launches"] * 1e3
            gbs = r["alg_bytes"] / (r["total_ms"] * 1e-3) / 1e9 if r["total_ms"] > 0 else 0.0
            tfs = r["flops"] / (r["total_ms"] * 1e-3) / 1e12 if r["total_ms"] > 0 else 0.0
            res["kernels"].append(dict(name=r["name"], launches_per_step=r["launches"] / nsteps, avg_us=round(avg_us, 2),
                                       share=round(r["total_ms"] / tot, 4), alg_GBps=round(gbs, 1), TFLOPs=round(tfs, 2)))
        d = rows[0]
        ai = d["flops"] / max(d["alg_bytes"], 1.0)
        balance = PEAK_TFLOPS[w["dtype"]] * 1e12 / (PEAK_HBM_GBS * 1e9)
        tr = traffic.get(d["name"])
        if d["name"].startswith("pw_") and ai >= balance:
            ach = d["flops"] / (d["total_ms"] * 1e-3) / 1e12
            roof = dict(bound="mfma", achieved=round(ach, 3), peak=PEAK_TFLOPS[w["dtype"]], unit="TFLOP/s",
                        frac=round(ach / PEAK_TFLOPS[w["dtype"]], 4), traffic=tr)
        else:
            ach = d["alg_bytes"] / (d["total_ms"] * 1e-3) / 1e9
            roof = dict(bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(ach / PEAK_HBM_GBS, 4), traffic=tr)
        roof.update(kernel=d["name"], avg_launch_us=round(d["total_ms"] / d["launches"] * 1e3, 2),
                    launches_per_step=d["launches"] / nsteps,
                    alg_bytes_per_launch=round(d["alg_bytes"] / d["launches"]),
                    event_pair_overhead_us=round(pair_ms * 1e3, 2),
                    avg_launch_us_with_event_pair=round(d["raw_total_ms"] / d["launches"] * 1e3, 2),
                    note="algorithmic bytes = every operand of a launch once; durations from HIP events around each "
                         "launch on its stream, in a separate traced pass, less the cost of the event pair itself "
                         "(measured on empty kernels when the trace starts); traffic = HBM bytes per launch from "
                         f"profiles/config{config}_pmc_traffic.txt (rocprofv3 FETCH_SIZE + WRITE_SIZE scaled by a plain "
                         "copy; a committed measurement, not taken in this run) or null")
        res["roofline"] = roof
    P.stage_destroy(stage)
    P.model_destroy(model)
    del x
    torch.cuda.empty_cache()
    return res


def bench_aggregate(config, versions=3, reps=50, seed=2110):
    """Weight aggregation (mean of `versions` stashed weight versions into the live weights) timed on its own:
    an HBM-bound pass over (versions + 1) fp32 copies of the parameters (+ the bfloat16 copy)."""
    import torch
    import synth
    import paper_2110_02781_amd as P

    w = WORKLOADS[config]
    dev = torch.device("cuda:0")
    tdt = torch.float32 if w["dtype"] == "f32" else torch.bfloat16
    units = build_units(P, w)
    H, W_, C = w["in_shape"]
    batch = min(w["batch"], 8)                      # the pass does not depend on the batch
    model = P.model_create(units, H, W_, C, P.F32 if w["dtype"] == "f32" else P.BF16)
    L = P.model_num_units(model)
    stage = P.stage_create(model, 0, L, batch, versions)
    params = P.models.init_unit_params(units, seed)
    n_param = 0
    for i in range(L):
        P.stage_import_weights(stage, i, params[i])
        n_param += len(params[i])
    x = torch.from_numpy(synth.normal(seed, "x", (batch, H, W_, C)).astype(np.float32)).to(dev).to(tdt)
    stream = torch.cuda.Stream()
    sp = stream.cuda_stream
    for sl in range(versions):
        P.stage_forward(stage, sl, x, None, sp)
        P.stage_snapshot_weights(stage, sl, sp)
    slots = list(range(versions))
    for _ in range(5):
        P.stage_aggregate_weights(stage, slots, sp)
    stream.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        e0.record(stream)
        for _ in range(reps):
            P.stage_aggregate_weights(stage, slots, sp)
        e1.record(stream)
    stream.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / reps
    nbytes = n_param * (4.0 * (versions + 1) + (2.0 if w["dtype"] == "bf16" else 0.0))
    P.stage_destroy(stage)
    P.model_destroy(model)
    return dict(workload=w["name"], params=n_param, versions=versions, us_per_call=round(us, 2),
                alg_GBps=round(nbytes / (us * 1e-6) / 1e9, 1), frac_of_hbm_peak=round(nbytes / (us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4))


def bench_recompute(config, micro=4, reps=3, seed=2110):
    """Recomputation as a memory / time trade: `micro` micro-batches forwarded, then backwarded, then one update
    (the synchronous pipeline order), once with stages that keep every intermediate per micro-batch and once with
    slots that keep only their input and run the forward again in the backward."""
    import torch
    import synth
    import paper_2110_02781_amd as P

    w = WORKLOADS[config]
    dev = torch.device("cuda:0")
    tdt = torch.float32 if w["dtype"] == "f32" else torch.bfloat16
    units = build_units(P, w)
    H, W_, C = w["in_shape"]
    batch = w["batch"]
    model = P.model_create(units, H, W_, C, P.F32 if w["dtype"] == "f32" else P.BF16)
    L = P.model_num_units(model)
    params = P.models.init_unit_params(units, seed)
    x = torch.from_numpy(synth.normal(seed, "x", (batch, H, W_, C)).astype(np.float32)).to(dev).to(tdt)
    labels = torch.from_numpy(synth.labels(seed, "labels", batch, w["classes"]).astype(np.int32)).to(dev)
    loss = torch.zeros(1, dtype=torch.float32, device=dev)
    stream = torch.cuda.Stream()
    sp = stream.cuda_stream
    res = {}
    for name, flags in (("keep", 0), ("recompute", P.STAGE_RECOMPUTE)):
        stage = P.stage_create(model, 0, L, batch, micro, flags)
        for i in range(L):
            P.stage_import_weights(stage, i, params[i])

        def mini_batch():
            for sl in range(micro):
                P.stage_forward(stage, sl, x, None, sp)
                P.stage_loss(stage, sl, labels, loss, sp)
            for sl in range(micro):
                P.stage_backward(stage, sl, None, None, sp)
            P.stage_update(stage, 0.01 / micro, 0.9, 4e-5, sp)
        mini_batch()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(stream):
            e0.record(stream)
            for _ in range(reps):
                mini_batch()
            e1.record(stream)
        stream.synchronize()
        res[name] = dict(ms_per_mini_batch=round(e0.elapsed_time(e1) / reps, 3), device_GiB=round(P.stage_device_bytes(stage) / 2**30, 2))
        P.stage_destroy(stage)
        torch.cuda.synchronize()
    P.model_destroy(model)
    return dict(workload=w["name"], micro_batches=micro, **res,
                time_ratio=round(res["recompute"]["ms_per_mini_batch"] / res["keep"]["ms_per_mini_batch"], 3),
                memory_ratio=round(res["recompute"]["device_GiB"] / res["keep"]["device_GiB"], 3))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=5, choices=sorted(WORKLOADS))
    ap.add_argument("--also", type=int, nargs="*", default=None,
                    help="further configs reported under 'also' (default: 2 and 1 when --config is 5)")
    ap.add_argument("--graph", action="store_true", help="replay the step from a captured HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ktrace", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch one plain 256 MiB copy (a dispatch of known traffic for counter scaling)")
    ap.add_argument("--seed", type=int, default=2110)
    ap.add_argument("--spinup", type=float, default=1.0, help="seconds of untimed steps before the warm-up (0 for profiler runs)")
    args = ap.parse_args()
    global SPINUP_S
    SPINUP_S = args.spinup
    if args.gpus != 1:
        print("bench.py: this build runs one pipeline stage on ONE GPU; --gpus must be 1 "
              "(no multi-GPU path exists: a pipeline would put one stage on each GPU and exchange only the boundary tensors)", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    main_res = run_workload(args.config, args.steps, args.warmup, args.graph, not args.no_ktrace, args.calibrate, args.seed)
    also_cfgs = args.also if args.also is not None else ([2, 1] if args.config == 5 else [])
    also = []
    for c in also_cfgs:
        if c == args.config or c not in WORKLOADS:
            continue
        small = WORKLOADS[c]["batch"] * WORKLOADS[c]["in_shape"][0] * WORKLOADS[c]["in_shape"][1] <= (1 << 16)
        r = run_workload(c, 200 if small else 20, 20 if small else 5, False, not args.no_ktrace, False, args.seed)
        r["kernels"] = r["kernels"][:12]
        if not args.no_cpu_baseline and small:
            r["cpu_baseline"] = oracle_baseline(WORKLOADS[c], args.seed, 3.0)
            r["cpu_baseline_one_thread"] = oracle_baseline(WORKLOADS[c], args.seed, 3.0, one_thread=True)
        also.append(r)

    # the widened rows: weight aggregation over three stashed versions and recomputation, on the headline workload
    agg = rec = None
    if args.config == 5 and not args.no_ktrace:
        agg = bench_aggregate(args.config, 3, 50, args.seed)
        rec = bench_recompute(args.config, 4, 3, args.seed)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = oracle_baseline(WORKLOADS[args.config], args.seed)

    out = {
        "metric": "stage train samples/sec (fwd+bwd+update) at 1 MI355X; % HBM/MFMA roofline",
        "value": main_res["value"], "unit": "samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "median_ms_per_step": main_res["median_ms_per_step"],
        "min_ms_per_step": main_res["min_ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": main_res["dtype"], "data": "synthetic (seeded N(0,1) inputs, uniform labels, He-normal weights)",
        "config": {"workload": main_res["workload"], "batch": main_res["batch"], "units": main_res["units"],
                   "hip_graph": main_res["hip_graph"], "final_loss": main_res["final_loss"]},
        "roofline": main_res["roofline"], "whole_step": main_res["whole_step"], "cpu_baseline": cpu,
        "kernels": main_res["kernels"], "also": also,
        "aggregate": agg, "recompute": rec,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
