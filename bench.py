#!/usr/bin/env python3
"""Benchmark of the stacked-LSTM forward pass on one MI355X.

A "step" is one lstm_forward (input projection of every layer + the whole recurrence) over one seeded synthetic
batch that is already resident in device memory.  Default workload: the 2-layer 1500-wide language-model-shaped
stack with 90 % masked weights at batch 1, T = 35 (the configuration the latency metric is quoted on).

Prints ONE JSON line.  `value` = microseconds per sequence (lower is better).
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

HBM_PEAK_GBS = 8000.0


def counter_traffic_bytes(workload_name):
    """HBM bytes per launch of the dominant kernel from the committed profiler counters, or None when the kernel
    sources have changed since they were taken (or none were taken for this workload)."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "traffic_counters.txt")
    try:
        kv = dict(line.strip().split("=", 1) for line in open(path) if "=" in line and not line.startswith("#"))
        h = hashlib.sha256()
        for f in ("persist_b1.hip", "exchange.h", "device_math.h"):
            h.update(open(os.path.join(ROOT, "paper_1901_10997_amd", "csrc", f), "rb").read())
        if kv.get("workload") != workload_name or kv.get("source_sha256") != h.hexdigest():
            return None
        return (float(kv["fetch_kib"]) * float(kv["fetch_scale"]) + float(kv["write_kib"]) * float(kv["write_scale"])) * 1024.0
    except (OSError, KeyError, ValueError):
        return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2_b1", choices=["c1", "c2_b1", "c2_b20", "c4", "c4_dense", "c5", "h1", "h2"],
                    help="c4_dense: the c4 stack with its weights held dense (the unpruned model; --format dense implied)")
    ap.add_argument("--format", default="auto", choices=["auto", "dense", "csr"])
    ap.add_argument("--plan", default="auto", choices=["auto", "stepwise", "persistent"])
    ap.add_argument("--waves", type=int, default=0)
    ap.add_argument("--launch", default="ordinary", choices=["ordinary", "cooperative"],
                    help="launch mode of the persistent kernels (ordinary, the library's default: residency by grid <= "
                         "compute units; cooperative: guaranteed by the runtime, slower dispatch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep-fine", action="store_true",
                    help="fine-grained batch-1 latency profile around the register-tier boundaries (writes "
                         "latency_sweep_fine.json into --out) and the growth targets of a few pruned dimensions")
    ap.add_argument("--sweep-matmul", action="store_true",
                    help="stand-alone product latency against the dimension for dense and row-compressed weights at "
                         "batch 16 (writes matmul_sweep.json into --out)")
    ap.add_argument("--sweep-speech", action="store_true",
                    help="model-level latency profile of the bidirectional speech stack at batch 16 over the hidden "
                         "width (writes latency_sweep_speech.json into --out)")
    ap.add_argument("--sweep-exchange", action="store_true",
                    help="the exchange inside groups of workgroups with no arithmetic: groups dealt over all XCDs, groups "
                         "placed on one XCD each, and those with workgroup-scope stores (writes exchange_groups.json "
                         "into --out)")
    ap.add_argument("--no-compare-launch-modes", action="store_true", help="do not time the loop in the other launch mode")
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip the 63-point hidden-size latency sweep (on by default for the default workload)")
    ap.add_argument("--sweep", action="store_true", help="run the hidden-size latency sweep for a non-default workload too")
    ap.add_argument("--no-yardsticks", action="store_true", help="skip the achievable-peak yardsticks and the cold-weights figure")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run the 1 GiB device copy kernel (known traffic, for scaling profiler byte counters)")
    ap.add_argument("--out", default=os.path.join(ROOT, "bench_out"))
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_1901_10997_amd import binding as B
    from paper_1901_10997_amd import inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.load(build_if_missing=True)
    dev = torch.device("cuda:0")
    if args.calibrate_copy:
        n = 1 << 30
        src = torch.zeros(n, dtype=torch.uint8, device=dev)
        dst = torch.empty(n, dtype=torch.uint8, device=dev)
        us = B.lstm_bench_copy(dst.data_ptr(), src.data_ptr(), n, 10)
        print(json.dumps({"metric": "device_copy_bandwidth", "value": 2 * n / us / 1e3, "unit": "GB/s",
                          "bytes_read": n, "bytes_written": n, "avg_us": us}))
        return
    if args.workload == "c4_dense":
        args.format = "dense"
    wl = {"c1": inputs.c1(), "c2_b1": inputs.c2(1), "c2_b20": inputs.c2(20), "c4": inputs.c4(), "c4_dense": inputs.c4(),
          "c5": inputs.c5(), "h1": inputs.h1(), "h2": inputs.h2()}[args.workload]
    hl = wl.gate_hidden > 0     # H-LSTM cell: one hidden layer of that width inside each gate
    case = inputs.make_case(wl, 0)
    dtype = B.LSTM_BF16 if wl.dtype == "bf16" else B.LSTM_F32
    fmt = {"auto": B.LSTM_FMT_AUTO, "dense": B.LSTM_FMT_DENSE_MASKED, "csr": B.LSTM_FMT_ROW_COMPRESSED}[args.format]
    plan = {"auto": B.LSTM_PLAN_AUTO, "stepwise": B.LSTM_PLAN_STEPWISE, "persistent": B.LSTM_PLAN_PERSISTENT}[args.plan]
    m = B.Lstm(wl.layers, wl.input_dim, wl.hidden, wl.bidirectional, dtype, gate_hidden=wl.gate_hidden)
    m.set_weights_from(case.weights, fmt)
    B.lstm_set_plan(m.handle, plan, args.waves)
    B.lstm_set_launch_mode(m.handle, args.launch == "cooperative")
    x = torch.from_numpy(case.x).to(dev)
    if dtype == B.LSTM_BF16:
        x = x.to(torch.bfloat16)
    x = x.contiguous()
    T, Bn, H = wl.T, wl.B, wl.hidden
    n = wl.layers * wl.ndir
    y = torch.empty((T, Bn, wl.ndir * H), dtype=torch.float32, device=dev)
    hT = torch.empty((n, Bn, H), dtype=torch.float32, device=dev)
    cT = torch.empty((n, Bn, H), dtype=torch.float32, device=dev)
    ws_bytes = B.lstm_workspace_bytes(m.handle, T, Bn)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream

    def step():
        B.lstm_forward(m.handle, T, Bn, x.data_ptr(), None, None, y.data_ptr(), hT.data_ptr(), cT.data_ptr(),
                       ws.data_ptr(), ws_bytes, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize(dev)
    B.lstm_check(m.handle)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize(dev)
    wall = time.perf_counter() - t0
    B.lstm_check(m.handle)
    ms_per_step = wall * 1e3 / args.steps
    us_per_seq = ms_per_step * 1e3 / Bn
    plan_desc = B.lstm_describe_plan(m.handle)

    # distribution over single forwards: each bracketed by its own event pair on the stream the library launches on
    # (torch's current stream), and, separately, host wall-clock of forward + synchronise (what a caller waits for)
    def percentiles(v):
        v = sorted(v)
        pick = lambda q: v[min(len(v) - 1, int(q * len(v)))]
        return {"median": pick(0.5), "p10": pick(0.1), "p90": pick(0.9), "n": len(v)}

    n_dist = max(20, min(200, args.steps))
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_dist)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize(dev)
    B.lstm_check(m.handle)
    dist_events = percentiles([e0.elapsed_time(e1) * 1e3 / Bn for e0, e1 in evs])
    walls = []
    for _ in range(n_dist):
        t1 = time.perf_counter()
        step()
        torch.cuda.synchronize(dev)
        walls.append((time.perf_counter() - t1) * 1e6 / Bn)
    dist_wall = percentiles(walls)

    other_mode = None
    if not args.no_compare_launch_modes and "persist" in plan_desc:
        other = "cooperative" if args.launch == "ordinary" else "ordinary"
        B.lstm_set_launch_mode(m.handle, other == "cooperative")
        for _ in range(min(args.warmup, 5)):
            step()
        torch.cuda.synchronize(dev)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize(dev)
        other_mode = {other: (time.perf_counter() - t0) * 1e6 / args.steps / Bn}
        B.lstm_check(m.handle)
        B.lstm_set_launch_mode(m.handle, args.launch == "cooperative")

    # per-kernel durations from events the library records on the same stream (separate pass: the event
    # pairs perturb the stream, so they stay out of the latency figure above)
    B.lstm_set_profiling(m.handle, True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize(dev)
    prof = B.lstm_get_profile(m.handle)
    B.lstm_set_profiling(m.handle, False)
    rec_us = prof["rec_us"] / max(prof["rec_launches"], 1)      # average per recurrence launch (one layer-direction)
    proj_us = prof["proj_us"] / max(prof["proj_launches"], 1)

    # Algorithmic bytes of one recurrence launch, for the plan that ran:
    #  * on-chip-resident plans (persistent kernels) read each kept weight once per launch:
    #    row-compressed: nnz * (4 B value + 2 B column); dense: 4H*K * sizeof(w);
    #    plus, per timestep, the input row (fused input side) or the projected row P[t], and the h_t written;
    #  * stepwise plans read W_h once per timestep.
    persistent = "persist" in plan_desc
    wavefront = "wavefront" in plan_desc
    wsize = 2 if dtype == B.LSTM_BF16 else 4

    def mat_bytes(p, wn, mn, compressed):
        Wm = p[wn]
        if compressed:
            nnz = int(p[mn].sum()) if p[mn] is not None else Wm.size
            return nnz * (4 + 2) + (Wm.shape[0] + 1) * 4
        return Wm.size * wsize

    layers_per_launch = 2 if wavefront else 1
    rec_launches_per_fwd = max(prof["rec_launches"] // max(args.steps, 1), 1)
    alg_bytes = 0.0
    keys = sorted(case.weights.keys())
    G = wl.gate_hidden
    for (l, d) in keys if hl else []:
        # H-LSTM: hidden layers (W1x fused at batch 1, W1h) and gate outputs (W2); stepwise also moves the
        # projected rows P1[t] and the hidden activations u_t (written by stage 1, read by stage 2)
        p = case.weights[(l, d)]
        comp = B.lstm_is_compressed(m.handle, l, d, 1)
        w1h, w2 = mat_bytes(p, "W1h", "M1h", comp), mat_bytes(p, "W2", "M2", comp)
        if persistent:
            alg_bytes += mat_bytes(p, "W1x", "M1x", comp) + w1h + w2 + T * Bn * (p["W1x"].shape[1] * 4 + H * 4)
        else:
            alg_bytes += T * (w1h + w2 + Bn * (4 * G * 4 * 3 + H * 4 * 3))
    for (l, d) in [] if hl else keys:
        p = case.weights[(l, d)]
        rec_compressed = B.lstm_is_compressed(m.handle, l, d, 1)
        wh = mat_bytes(p, "Wh", "Mh", rec_compressed)
        fused = "fused" in plan_desc
        wx = mat_bytes(p, "Wx", "Mx", rec_compressed) if fused else 0
        D_l = p["Wx"].shape[1]
        per_step_in = D_l * 4 if (fused and (l == 0 or not wavefront)) else (0 if fused else 4 * H * 4)
        per_step_out = H * 4 if not (wavefront and l == 0) else 0
        if persistent:
            alg_bytes += wh + wx + T * Bn * (per_step_in + per_step_out)
        else:
            alg_bytes += T * (wh + Bn * (4 * H * 4 + H * 4 + H * 4))
    alg_bytes /= rec_launches_per_fwd
    achieved = alg_bytes / (rec_us * 1e-6) / 1e9 if rec_us > 0 else 0.0
    roofline = {"bound": "hbm",
                "kernel": "recurrence (" + ("persistent, weights resident on chip" + (", 2-layer wavefront" if wavefront else "")
                                            if persistent else "one launch per step") + ")",
                "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                "traffic": counter_traffic_bytes(wl.name) if (args.format == "auto" and args.plan == "auto") else None,
                "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_us": rec_us,
                "launches_per_forward": rec_launches_per_fwd, "proj_avg_launch_us": proj_us}
    coop = args.launch == "cooperative"
    if persistent and Bn == 1:
        # latency criterion of the on-chip-resident plan: time per sequential step against (a) a device-wide barrier
        # of the same grid that carries no data (one tagged slot per workgroup) and (b) the bare exchange of the same
        # number of hidden values between the same number of workgroups
        try:
            slots = H * layers_per_launch
            waves = 12 if wavefront else 0
            ex_us = B.lstm_bench_exchange(slots, waves, 200, 5, stream, coop)
            if hl:   # a step of the H-LSTM kernel has two exchanges (h: H values; hidden activations: 4G values);
                ex_us *= 2.0   # the yardstick counts both at the size of the smaller one, i.e. it is a lower bound
            ncu = torch.cuda.get_device_properties(dev).multi_processor_count
            wpg = waves if waves else 16
            groups = min(ncu, 256, (slots + wpg - 1) // wpg)
            bar_us = B.lstm_bench_barrier(groups, wpg, 200, 5, coop, stream) * (2.0 if hl else 1.0)
            steps_seq = T + layers_per_launch - 1
            roofline["sequential_steps_per_launch"] = steps_seq
            roofline["step_us"] = rec_us / steps_seq
            roofline["barrier_only_step_us"] = bar_us
            roofline["barrier_workgroups"] = groups
            roofline["step_over_barrier"] = (rec_us / steps_seq) / bar_us if bar_us > 0 else None
            roofline["exchange_only_step_us"] = ex_us
            roofline["step_over_exchange"] = (rec_us / steps_seq) / ex_us if ex_us > 0 else None
        except B.LstmError as e:
            roofline["exchange_only_step_us"] = None
            roofline["exchange_error"] = str(e)
    # input projection on the matrix cores (the contraction of the large-batch workloads): flops of all projection
    # launches of a forward over their summed duration, against the spec-sheet peak of the operand type
    proj = None
    if prof["proj_launches"] > 0 and T * Bn >= 256:
        flops = sum(2.0 * T * Bn * wl.layer_input_dim(l) * (4 * (G if hl else H)) for (l, d) in keys)
        per_fwd_us = prof["proj_us"] / max(args.steps, 1)
        if "proj=q16" in plan_desc:
            # projection over the kept entries only: vector multiply-adds, two flops per kept weight and input row;
            # peak = the fp32 vector rate of the spec sheet (256 compute units x 4 SIMDs x 32 multiply-adds per clock at
            # 2.4 GHz with packed instructions; this library is compiled without them, which halves what it can reach)
            kept = sum(float(case.weights[k]["Mx"].sum()) if case.weights[k].get("Mx") is not None
                       else float(case.weights[k]["Wx"].size) for k in keys)
            sflops = 2.0 * T * Bn * kept
            tf = sflops / (per_fwd_us * 1e-6) / 1e12
            proj = {"bound": "alu", "achieved": tf, "peak": 157.3, "unit": "TFLOP/s", "frac": tf / 157.3,
                    "peak_without_packed_fp32": 78.6, "frac_without_packed_fp32": tf / 78.6,
                    "flops_per_forward": sflops, "dense_flops_per_forward": flops,
                    "dense_equivalent_TFLOPs": flops / (per_fwd_us * 1e-6) / 1e12,
                    "us_per_forward": per_fwd_us, "launches_per_forward": prof["proj_launches"] // max(args.steps, 1)}
        else:
            tf = flops / (per_fwd_us * 1e-6) / 1e12
            peak = 2500.0 if dtype == B.LSTM_BF16 else 157.3
            proj = {"bound": "mfma", "achieved": tf, "peak": peak, "unit": "TFLOP/s", "frac": tf / peak,
                    "flops_per_forward": flops, "us_per_forward": per_fwd_us, "launches_per_forward": prof["proj_launches"] // max(args.steps, 1)}
    measured = None
    cold = None
    if not args.no_yardsticks:
        # achievable peaks measured in this run, next to the spec-sheet ones
        nbytes = 1 << 29
        src = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        copy_us = B.lstm_bench_copy(dst.data_ptr(), src.data_ptr(), nbytes, 5, stream)
        bf_c, bf_c_ghz = B.lstm_bench_mfma(B.LSTM_BF16, 20000, 3, stream, False, True)
        bf_r, bf_r_ghz = B.lstm_bench_mfma(B.LSTM_BF16, 20000, 3, stream, True, True)
        f_c, f_c_ghz = B.lstm_bench_mfma(B.LSTM_F32, 5000, 3, stream, False, True)
        f_r, f_r_ghz = B.lstm_bench_mfma(B.LSTM_F32, 5000, 3, stream, True, True)
        measured = {"copy_GBps": 2 * nbytes / copy_us / 1e3, "copy_bytes_each_way": nbytes,
                    "mfma_bf16_TFLOPs": bf_c, "mfma_bf16_clock_GHz": bf_c_ghz,
                    "mfma_bf16_random_operands_TFLOPs": bf_r, "mfma_bf16_random_operands_clock_GHz": bf_r_ghz,
                    "mfma_f32_TFLOPs": f_c, "mfma_f32_clock_GHz": f_c_ghz,
                    "mfma_f32_random_operands_TFLOPs": f_r, "mfma_f32_random_operands_clock_GHz": f_r_ghz}
        roofline["frac_of_measured_copy"] = achieved / measured["copy_GBps"]
        if proj and proj["bound"] == "mfma":
            key = "mfma_bf16" if dtype == B.LSTM_BF16 else "mfma_f32"
            proj["measured_peak"] = measured[key + "_TFLOPs"]
            proj["frac_of_measured"] = proj["achieved"] / proj["measured_peak"]
            proj["measured_peak_random_operands"] = measured[key + "_random_operands_TFLOPs"]
            proj["frac_of_measured_random_operands"] = proj["achieved"] / proj["measured_peak_random_operands"]
            # the vendor library's product of the first layer's projection shape, same operand and output types (fp32
            # out), as a yardstick of what this shape reaches on this device; it is not part of the path
            try:
                Mr, Kr, Nr = T * Bn, wl.layer_input_dim(0), 4 * (G if hl else H)
                tdt = torch.bfloat16 if dtype == B.LSTM_BF16 else torch.float32
                ga = torch.randn(Mr, Kr, device=dev).to(tdt)
                gb = ((torch.rand(Nr, Kr, device=dev) * 2 - 1) * wl.a).to(tdt).t()
                mm = (lambda: torch.mm(ga, gb, out_dtype=torch.float32)) if tdt == torch.bfloat16 else (lambda: torch.mm(ga, gb))
                for _ in range(3):
                    mm()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(10):
                    mm()
                e1.record()
                torch.cuda.synchronize(dev)
                lib_us = e0.elapsed_time(e1) * 1e3 / 10
                proj["library_gemm"] = {"shape_MKN": [Mr, Kr, Nr], "us": lib_us, "TFLOPs": 2.0 * Mr * Kr * Nr / lib_us / 1e6,
                                        "kind": "torch.mm (hipBLASLt), fp32 output"}
                del ga, gb
            except Exception as e:   # older torch without out_dtype, or no library kernel for the shape
                proj["library_gemm"] = {"error": str(e)[:200]}
        # cold weights: one forward right after a 2 x 512 MiB device copy has swept the caches
        colds = []
        for _ in range(5):
            B.lstm_bench_copy(dst.data_ptr(), src.data_ptr(), nbytes, 1, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            step()
            e1.record()
            torch.cuda.synchronize(dev)
            colds.append(e0.elapsed_time(e1) * 1e3 / Bn)
        cold = {"median_us_per_seq": sorted(colds)[len(colds) // 2], "min": min(colds), "max": max(colds), "n": len(colds),
                "swept_bytes": 2 * nbytes}
        del src, dst

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import hlstm_oracle, lstm_oracle
        import dataclasses
        # bounded sample of the same workload: a few sequences (batch columns are independent), all T steps
        # except for the 1500-step bidirectional stack, which is cut to T'=30 and scaled (cost is linear in T)
        nseq = {1: 64, 2: 8, 4: 2, 5: 8, 6: 32, 7: 2}.get(wl.cid, 4)
        big = inputs.make_case(dataclasses.replace(wl, B=max(nseq, 1)), 0) if Bn < nseq else case
        sub = inputs.select_batch(big, list(range(nseq)))
        Tc = T
        if wl.cid in (4, 7):
            Tc = 30
            sub = dataclasses.replace(sub, x=sub.x[:Tc].copy())
        oracle_forward = (hlstm_oracle if hl else lstm_oracle).forward_case
        nthreads = lstm_oracle.max_threads()
        t1 = time.perf_counter()
        oracle_forward(sub, nthreads)
        cpu_s = time.perf_counter() - t1
        cpu_us_per_seq = cpu_s * 1e6 / nseq * (T / Tc)
        # one thread: fewer sequences and, for the long workloads, fewer steps (cost is linear in both)
        n1 = max(1, nseq // 8)
        sub1 = inputs.select_batch(sub, list(range(n1)))
        T1 = min(Tc, 8) if wl.cid in (4, 5, 7) else Tc
        sub1 = dataclasses.replace(sub1, x=sub1.x[:T1].copy())
        t1 = time.perf_counter()
        oracle_forward(sub1, 1)
        cpu1_s = time.perf_counter() - t1
        cpu = {"value": cpu_us_per_seq, "unit": "us/seq", "cores": nthreads, "kind": "oracle",
               "sample": f"{nseq} sequence(s) of the same workload, T={Tc} of {T}" + (" (scaled linearly in T)" if Tc != T else ""),
               "wall_s": cpu_s, "nproc": os.cpu_count(),
               "one_thread": {"value": cpu1_s * 1e6 / n1 * (T / T1), "unit": "us/seq", "cores": 1,
                              "sample": f"{n1} sequence(s), T={T1} of {T}" + (" (scaled linearly in T)" if T1 != T else ""),
                              "wall_s": cpu1_s}}

    out = {
        "metric": "lstm_fwd_latency_us_per_seq", "value": us_per_seq, "unit": "us/seq", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if dtype == B.LSTM_BF16 else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.layers, "bidirectional": wl.bidirectional, "input_dim": wl.input_dim,
                   "hidden": H, "gate_hidden": wl.gate_hidden, "T": T, "batch": Bn, "mask_keep": wl.keep, "format": args.format, "plan": plan_desc, "launch": args.launch},
        "us_per_seq_other_launch_mode": other_mode,
        "us_per_seq_single_forward_events": dist_events, "us_per_seq_single_forward_host_wall": dist_wall,
        "us_per_seq_cold_weights": cold,
        "timestep_batch_per_s": T * Bn / (ms_per_step * 1e-3),
        "roofline": roofline, "projection": proj, "measured_peaks": measured, "cpu_baseline": cpu,
    }
    if (args.workload == "c2_b1" and not args.no_sweep) or args.sweep:
        os.makedirs(args.out, exist_ok=True)
        Hs = inputs.c3_hidden_sizes()
        B.lstm_set_default_launch_mode(args.launch == "cooperative")
        med, p10, p90, flags = B.lstm_latency_sweep(Hs, 35, 1, B.LSTM_F32, 1, 10, 100, stream)
        f2, red2 = B.lstm_find_lhp(Hs, med, 0.02)
        f0, red0 = B.lstm_find_lhp(Hs, med, 0.0)
        with open(os.path.join(args.out, "latency_sweep.json"), "w") as fh:
            json.dump({"launch": args.launch, "T": 35, "batch": 1, "H": Hs, "median_us": list(med), "p10_us": list(p10), "p90_us": list(p90),
                       "is_lhp_eps0": [int(v) for v in f0], "is_lhp_eps2pct": [int(v) for v in f2],
                       "redundancy_pct_eps0": red0, "redundancy_pct_eps2pct": red2}, fh)
        out["sweep"] = {"workload": "c3: 1 layer, input_dim = H, T=35, batch 1, fp32, dense", "launch": args.launch,
                        "points": len(Hs), "H": Hs, "median_us": [round(float(v), 2) for v in med],
                        "p10_us": [round(float(v), 2) for v in p10], "p90_us": [round(float(v), 2) for v in p90],
                        "lhp_eps0": [h for h, f in zip(Hs, f0) if f], "lhp_eps2pct": [h for h, f in zip(Hs, f2) if f],
                        "redundancy_pct_eps0": red0, "redundancy_pct_eps2pct": red2,
                        "min_us": float(min(med)), "max_us": float(max(med))}
    if args.sweep_fine:
        # batch 1, dense, step 4 around the tier boundaries of the fused persistent kernel, plus the language-model
        # pair (hidden, input) = (H, H * 4 / 15) of the paper's pruned gates (1197 / 317 -> 1200 / 320)
        os.makedirs(args.out, exist_ok=True)
        B.lstm_set_default_launch_mode(args.launch == "cooperative")
        res = {"launch": args.launch, "T": 35, "batch": 1, "curves": {}}
        for name, Hs in (("dense_1x_H", list(range(960, 1089, 4)) + list(range(1216, 1377, 4))),
                         ("dense_1x_H_in_4H15", list(range(1100, 1301, 4)) + [1197])):
            Hs = sorted(set(Hs))
            Ds = None if name == "dense_1x_H" else [max(1, round(h * 4 / 15)) for h in Hs]
            med, p10, p90, _ = B.lstm_latency_sweep_model(Hs, Ds, T=35, B=1, warmup=10, iters=100, stream=stream)
            f2, red2 = B.lstm_find_lhp(Hs, med, 0.02)
            res["curves"][name] = {"H": Hs, "D": Ds, "median_us": list(med), "p10_us": list(p10), "p90_us": list(p90),
                                   "is_lhp_eps2pct": [int(v) for v in f2], "redundancy_pct_eps2pct": red2}
            if name == "dense_1x_H_in_4H15":
                res["growth_targets_eps2pct"] = {str(d): B.lstm_grow_to_lhp(Hs, med, d, 0.02) for d in (1197, 1150, 1262)}
        with open(os.path.join(args.out, "latency_sweep_fine.json"), "w") as fh:
            json.dump(res, fh)
        out["sweep_fine"] = {k: {"points": len(v["H"]), "redundancy_pct_eps2pct": v["redundancy_pct_eps2pct"]}
                             for k, v in res["curves"].items()}
        out["sweep_fine"]["growth_targets_eps2pct"] = res["growth_targets_eps2pct"]
    if args.sweep_matmul:
        os.makedirs(args.out, exist_ok=True)
        ns = list(range(256, 4097, 128))
        keeps = [0.5, 0.3, 0.1, 0.05]
        res = {"batch": 16, "n": ns, "dense_us": [B.lstm_bench_matmul(n, 16, 1.0, B.LSTM_FMT_DENSE_MASKED, iters=50, stream=stream) for n in ns],
               "compressed_us": {str(k): [B.lstm_bench_matmul(n, 16, k, B.LSTM_FMT_ROW_COMPRESSED, iters=50, stream=stream) for n in ns]
                                 for k in keeps}}
        f2, red2 = B.lstm_find_lhp(ns, res["dense_us"], 0.02)
        res["dense_is_lhp_eps2pct"] = [int(v) for v in f2]
        res["dense_redundancy_pct_eps2pct"] = red2
        with open(os.path.join(args.out, "matmul_sweep.json"), "w") as fh:
            json.dump(res, fh)
        out["sweep_matmul"] = {"points": len(ns), "dense_redundancy_pct_eps2pct": red2}
    if args.sweep_exchange:
        os.makedirs(args.out, exist_ok=True)
        coop = args.launch == "cooperative"
        # (slots, members, groups): the shapes of the kernels that exchange inside groups
        shapes = [(200, 13, 1), (1024, 32, 8), (1600, 16, 16), (3200, 25, 8), (6000, 30, 8), (800, 8, 8), (3000, 24, 10)]
        rows = []
        for slots, members, groups in shapes:
            row = {"slots": slots, "members": members, "groups": groups}
            row["spread_us"], _ = B.lstm_bench_group_exchange(slots, members, groups, False, False, cooperative=coop, stream=stream)
            if ((groups + 7) // 8) * members <= 32:
                row["placed_us"], row["verified"] = B.lstm_bench_group_exchange(slots, members, groups, True, False,
                                                                                cooperative=coop, stream=stream)
                row["placed_l2_us"], _ = B.lstm_bench_group_exchange(slots, members, groups, True, True, cooperative=coop,
                                                                     stream=stream)
            rows.append(row)
        with open(os.path.join(args.out, "exchange_groups.json"), "w") as fh:
            json.dump({"launch": args.launch, "rows": rows}, fh)
        out["sweep_exchange"] = rows
    if args.sweep_speech:
        # the paper's model-level figure: latency of the bidirectional speech stack at batch 16 against the hidden
        # width (here: 5 layers, 15 % kept weights as in workload c4, T = 100)
        os.makedirs(args.out, exist_ok=True)
        B.lstm_set_default_launch_mode(args.launch == "cooperative")
        Hs = list(range(512, 1025, 32))
        Ds = [640] * len(Hs)
        med, p10, p90, _ = B.lstm_latency_sweep_model(Hs, Ds, layers=5, bidirectional=True, keep=0.15, T=100, B=16,
                                                      warmup=2, iters=10, stream=stream)
        f2, red2 = B.lstm_find_lhp(Hs, med, 0.02)
        # the same stack with dense weights (keep = 0 means no masks): the unpruned model, and what a row/column-pruned
        # model is once it has been compacted to its smaller dimensions
        dmed, dp10, dp90, _ = B.lstm_latency_sweep_model(Hs, Ds, layers=5, bidirectional=True, keep=0.0, T=100, B=16,
                                                         warmup=2, iters=10, stream=stream)
        df2, dred2 = B.lstm_find_lhp(Hs, dmed, 0.02)
        with open(os.path.join(args.out, "latency_sweep_speech.json"), "w") as fh:
            json.dump({"launch": args.launch, "layers": 5, "bidirectional": True, "keep": 0.15, "T": 100, "batch": 16,
                       "H": Hs, "median_us": list(med), "p10_us": list(p10), "p90_us": list(p90),
                       "is_lhp_eps2pct": [int(v) for v in f2], "redundancy_pct_eps2pct": red2,
                       "dense": {"median_us": list(dmed), "p10_us": list(dp10), "p90_us": list(dp90),
                                 "is_lhp_eps2pct": [int(v) for v in df2], "redundancy_pct_eps2pct": dred2}}, fh)
        out["sweep_speech"] = {"points": len(Hs), "redundancy_pct_eps2pct": red2, "min_us": float(min(med)), "max_us": float(max(med)),
                               "dense_redundancy_pct_eps2pct": dred2, "dense_min_us": float(min(dmed)), "dense_max_us": float(max(dmed))}
    m.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
