#!/usr/bin/env python3
"""Benchmark of the per-layer DP weight-gradient path (Algorithm 1 of FlashDP) on one MI355X.

A step is one pass of the whole path - per-sample contraction, norm reduction, clip factors, clipped
batch sum, Philox noise, store - over every linear layer of the workload (default: the seven linears of
a Llama-13B decoder block, B = 8, T = 2048, bf16), inputs resident in HBM.  Prints one JSON line:
throughput in algorithmic TFLOP/s (2*B*T*d_in*d_out per layer, one contraction per layer whatever the
schedule does), its fraction of the dense bf16 MFMA peak, the ratio against the plain non-DP dY^T X
weight-gradient GEMM timed in the same run (the fastest of the vendor BLAS through torch.matmul, this library's
own contraction with norm/clip/noise switched off, and the same with its work balanced over the chip), a roofline object for the dominant kernel
(timed alone, live, with events on the launch stream) and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X dense MFMA peaks by input type (TFLOP/s); bf16 and fp16 share one figure
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "fp32": 157.3}
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of the dominant kernel are not measurable from inside this script: they come from two
# rocprofv3 --pmc runs of it (FETCH_SIZE, WRITE_SIZE), scaled by what the same counters read for a copy of known
# size, and are kept with their command, date and source commit in profiles/traffic.json.  A workload / schedule /
# kernel without an entry there reports traffic = null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def measured_traffic(workload, schedule, kernel):
    try:
        with open(TRAFFIC_FILE) as f:
            table = json.load(f)
    except (OSError, ValueError):
        return None
    for e in table.get("entries", []):
        if e.get("workload") == workload and e.get("schedule") == schedule and e.get("kernel") == kernel:
            return e
    return None


def write_traffic(fetch_dir, write_dir, workload, schedule, kernel):
    """Reads the p_counter_collection.csv of two rocprofv3 --pmc runs of this script (FETCH_SIZE in one, WRITE_SIZE in
    the other, both with --copy-probe) and records, in profiles/traffic.json, the average HBM-side bytes per launch of
    `kernel` (a substring of the profiler's kernel name), scaled by what the same counter read for the 1 GiB copy of
    --copy-probe.  No GPU needed."""
    import csv
    import datetime
    import subprocess

    def read(d, counter):
        rows = [r for r in csv.DictReader(open(os.path.join(d, "p_counter_collection.csv"))) if r["Counter_Name"] == counter]
        copies = [float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"]]
        mine = [float(r["Counter_Value"]) for r in rows if kernel in r["Kernel_Name"]]
        if not copies or not mine:
            raise SystemExit(f"{d}: no {counter} rows for the copy probe or for a kernel named like {kernel!r}")
        scale = float(1 << 20) / max(copies)          # KiB the 1 GiB copy moved each way / KiB the counter read
        return sum(mine) / len(mine) * 1024.0 * scale, scale, len(mine)

    rd, rscale, n_r = read(fetch_dir, "FETCH_SIZE")
    wr, wscale, n_w = read(write_dir, "WRITE_SIZE")
    try:
        commit = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short", "HEAD"], capture_output=True, text=True).stdout.strip()
    except OSError:
        commit = ""
    try:
        with open(TRAFFIC_FILE) as f:
            table = json.load(f)
    except (OSError, ValueError):
        table = {"entries": []}
    name = kernel.split("<")[0]
    entry = {"workload": workload, "schedule": schedule, "kernel": name, "profiler_kernel_match": kernel,
             "read_bytes": round(rd), "write_bytes": round(wr), "fetch_size_scale": round(rscale, 4), "write_size_scale": round(wscale, 4),
             "dispatches_averaged": [n_r, n_w], "commit": commit, "date": datetime.date.today().isoformat(),
             "command": "rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE -d <dir> -o p --output-format csv -- python3 bench.py --steps 3 --warmup 1 "
                        f"--no-cpu-baseline --no-comparators --no-schedule-comparison --copy-probe --workload {workload} --schedule {schedule}"}
    table["entries"] = [e for e in table.get("entries", []) if not (e.get("workload") == workload and e.get("schedule") == schedule and e.get("kernel") == name)]
    table["entries"].append(entry)
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(table, f, indent=1)
        f.write("\n")
    print(json.dumps(entry))


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama13b_block")
    ap.add_argument("--schedule", default="auto", choices=["auto", "twopass", "scratch", "explicit", "overlap", "ghost", "fused"])
    ap.add_argument("--no-schedule-comparison", action="store_true",
                    help="skip timing the other schedules (two-pass recompute, explicit four-stage) beside the default")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--share-x", action="store_true",
                    help="secondary variant: q/k/v (and gate/up) read the same X tensor, as in a real decoder block; "
                         "the default gives every layer its own tensors, as the workload states")
    ap.add_argument("--no-comparators", action="store_true")
    ap.add_argument("--timeline", action="store_true",
                    help="also run the traced instantiation of the contraction kernel on the workload's largest layer (its data, "
                         "then all-zero operands) and report where a workgroup's time goes and the clock it ran at")
    ap.add_argument("--traffic-from", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no benchmark: read two rocprofv3 --pmc output folders (FETCH_SIZE, WRITE_SIZE runs of this script with "
                         "--copy-probe) and record the dominant kernel's measured bytes per launch in profiles/traffic.json")
    ap.add_argument("--traffic-kernel", default="gemm_mfma_dma16_kernel<flashdp::DmaCfg<4>, 1,",
                    help="substring of the profiler's kernel name to average over (default: the contraction kernel in its parking mode)")
    ap.add_argument("--vendor-envelope", action="store_true",
                    help="also time the vendor GEMM (torch.matmul) on 8192^3 bf16 in its best layout (reduction index contiguous for both "
                         "operands) and in this path's layout (reduction index slowest for both), on N(0,1) data and on zeros")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device-to-device copy: a kernel of known traffic to scale profiler byte counters by")
    return ap.parse_args()


def time_steps(fn, steps, warmup):
    """Wall-clock over exactly `steps` calls, bracketed by device synchronisation; ms per step."""
    import torch
    # untimed: bring the clocks up first (a sub-millisecond step would otherwise be timed on a GPU that is
    # still ramping), then the W warm-up steps proper
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < 0.05:
        fn()
        torch.cuda.synchronize()
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def time_events(fn, steps, warmup):
    """Device time per call from events recorded on the current stream (the stream the library launches on)."""
    import torch
    for _ in range(warmup):
        fn()
    s = torch.cuda.Event(enable_timing=True)
    e = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    s.record()
    for _ in range(steps):
        fn()
    e.record()
    torch.cuda.synchronize()
    return s.elapsed_time(e) / steps


def time_each(fn, steps, warmup):
    """Device time of every single call (events on the current stream between calls): (median, min) in ms."""
    import torch
    for _ in range(warmup):
        fn()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for k in range(steps):
        fn()
        ev[k + 1].record()
    torch.cuda.synchronize()
    ts = sorted(ev[k].elapsed_time(ev[k + 1]) for k in range(steps))
    return ts[len(ts) // 2], ts[0]


def mfma_only(F, torch, dev):
    """The matrix cores alone (register-resident operands, the contraction kernel's instruction mix, no memory),
    and with the operand fragments re-read from LDS as the kernel does (lds_*): what this part sustains on all-zero
    and on random operands, in TFLOP/s.  ~0.1 s of GPU time each."""
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    wgs, iters = 1024, 20000
    flop = wgs * 8 * iters * 16 * 32768.0
    out = {}
    for name, pattern in (("zeros", 0), ("random", 1), ("lds_zeros", 2), ("lds_random", 3), ("random_shared_operand_order", 4),
                          ("random_one_operand_pair", 5), ("random_wide_exponents", 6), ("random_16x16x32", 7), ("lds_random_16x16x32", 8), ("zeros_16x16x32", 9), ("random_16x16x32_acc_regs", 10), ("random_16x16x32_in_place", 11), ("lds_random_16x16x32_fewer_reads", 12)):
        ms = time_events(lambda: F.flashdp_mfma_probe(pattern, iters, wgs, sink), 3, 2)
        out[name + "_tflops"] = round(flop / ms / 1e9, 1)
    return out


def contraction_timeline(F, torch, X, dY, B, T, P, D, park, reps=8):
    """Per-workgroup timeline of the contraction kernel (flashdp_contraction_timeline), summarised: mean microseconds per
    phase, main-loop shader cycles per k-tile (1024 = matrix cores never idle), the clock the main loop ran at, the gap
    between two workgroups on a CU, and the share of a CU's time that is not main loop."""
    import numpy as np
    L = [dict(X=X, dY=dY, d_in=P, d_out=D, C=1.0, sigma=0.0, seed=0, layer=0, out_grad=None)]
    ws = torch.empty(F.flashdp_workspace_bytes(L, B, T, F.BF16, "scratch"), dtype=torch.uint8, device=X.device)
    tiles = ((D + 255) // 256) * ((P + 255) // 256)
    n = 8 * ((B * ((tiles + 31) // 32) + 7) // 8) * 32
    trace = torch.zeros(8 * n, dtype=torch.int64, device=X.device)
    for _ in range(reps):      # the last repetition is the one read: clocks have settled by then
        trace.zero_()
        F.flashdp_contraction_timeline(X, dY, B, T, P, D, park, ws, trace)
    torch.cuda.synchronize()
    t = trace.cpu().numpy().reshape(-1, 8)
    t = t[t[:, 7] == 1]
    us = 0.01
    st, first, loop, issued, end = [t[:, k].astype(np.float64) * us for k in range(5)]
    cyc = t[:, 6].astype(np.float64)
    nk = (T + 31) // 32
    key = ((t[:, 5] >> 32) << 8) | ((t[:, 5] & 0xFFFFFFFF) >> 8 & 0xFF)
    gaps = []
    for k in np.unique(key):
        m = key == k
        o = np.argsort(st[m])
        s_, e_ = st[m][o], end[m][o]
        gaps.extend(s_[1:] - e_[:-1])
    span = end.max() - st.min()
    gap = float(np.mean(gaps)) if gaps else 0.0
    whole = float((end - st).mean()) + gap
    return {
        "workgroups": int(len(t)), "span_us": round(float(span), 1),
        "tflops": round(2.0 * B * T * P * D / span / 1e6, 1),
        "fill_us": round(float((first - st).mean()), 2), "main_loop_us": round(float((loop - first).mean()), 2),
        "epilogue_until_stores_issued_us": round(float((issued - loop).mean()), 2),
        "store_drain_us": round(float((end - issued).mean()), 2), "gap_to_next_workgroup_us": round(gap, 2),
        "not_main_loop_share": round(1.0 - float((loop - first).mean()) / whole, 4),
        "main_loop_cycles_per_k_tile": round(float(cyc.mean()) / nk, 1),
        "main_loop_matrix_core_busy": round(1024.0 * nk / float(cyc.mean()), 4),
        "main_loop_clock_ghz": round(float(cyc.mean()) / float((loop - first).mean()) / 1e3, 3),
        "last_round_idle_share": round(1.0 - float(np.mean([end[key == k].max() for k in np.unique(key)]) - st.min()) / float(span), 4),
    }


def cpu_baseline(w, target_flop=6e12):
    """The oracle as it stands on the host cores, on a bounded sample of the same workload: whole layers
    (all samples, full T), largest first, until about target_flop of work (10-30 s) has been timed."""
    import numpy as np
    import workloads as W
    from oracle import flashdp_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    order = sorted(range(len(w.layers)), key=lambda k: -w.layers[k].d_in * w.layers[k].d_out)
    done_flop, dt, names = 0.0, 0.0, []
    for l in order:
        spec = w.layers[l]
        X, dY = W.make_layer(w, l)
        if X.dtype == np.float16:     # the oracle takes stored values widened exactly
            X, dY = X.astype(np.float32), dY.astype(np.float32)
        t0 = time.perf_counter()
        O.linear_dp_grad(X, dY, w.C, w.sigma, w.layer_seed(l), l)
        dt += time.perf_counter() - t0
        done_flop += 2.0 * w.B * w.T * spec.d_in * spec.d_out
        names.append(spec.name)
        if done_flop >= target_flop:
            break
    return {"value": round(done_flop / dt / 1e12, 5), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": f"layers {'+'.join(names)} of {w.name} (all {w.B} samples, T={w.T}), fp64 numpy oracle incl. noise field"}


def main():
    args = parse()
    if args.traffic_from:
        write_traffic(args.traffic_from[0], args.traffic_from[1], args.workload, "scratch" if args.schedule in ("auto", "overlap") else args.schedule,
                      args.traffic_kernel)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import workloads as W
    import paper_2507_01154_amd as F

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    F.lib()   # fail loudly if the HIP library is missing
    w = W.WORKLOADS[args.workload]
    dev = "cuda:0"
    dtype_code = {"bf16": F.BF16, "f16": F.F16, "fp32": F.F32}[w.dtype]
    peak = PEAK_MFMA_TFLOPS[w.dtype]
    layers, keep = [], []
    shared = {}
    for l, spec in enumerate(w.layers):
        X, dY = W.make_layer_device(w, l, dev)
        if args.share_x:
            group = {"q_proj": "attn", "k_proj": "attn", "v_proj": "attn", "gate_proj": "mlp", "up_proj": "mlp"}.get(spec.name)
            if group is not None:
                X = shared.setdefault(group, X)
        out = torch.empty((spec.d_out, spec.d_in), dtype=torch.float32, device=dev)
        norms = torch.empty((w.B,), dtype=torch.float32, device=dev)
        layers.append(dict(X=X, dY=dY, d_in=spec.d_in, d_out=spec.d_out, C=w.C, sigma=w.sigma,
                           seed=w.layer_seed(l), layer=l, out_grad=out, out_norms=norms))
        keep.append((X, dY, out, norms))
    arr = F.make_layers(layers)
    sched = args.schedule
    ws = None
    if sched != "twopass":
        ws_kind = {"explicit": "explicit", "scratch": "scratch", "ghost": "ghost", "fused": "fused"}.get(sched, "overlap")
        ws = torch.empty(F.flashdp_workspace_bytes(arr, w.B, w.T, dtype_code, ws_kind), dtype=torch.uint8, device=dev)

    def step():
        F.flashdp_block_dp_grad(arr, w.B, w.T, dtype_code, sched, ws)

    ms = time_steps(step, args.steps, args.warmup)
    used = F.flashdp_last_schedule()
    kernel = F.flashdp_last_kernel()
    flops = float(w.flops())
    tflops = flops / ms / 1e9
    ms_median, ms_min = time_each(step, args.steps, 2)   # spread of single steps, outside the timed region above

    # dominant kernel alone (the per-sample contraction + intra-block norm), same launches, same stream
    if used == "fused":      # one kernel does everything: there are no stages to time apart
        ms_contract, ms_aggregate = time_events(step, args.steps, 2), 0.0
    else:
        F.flashdp_set_stages(F.STAGE_CONTRACT)
        ms_contract = time_events(step, args.steps, 2)
        F.flashdp_set_stages(F.STAGE_AGGREGATE)
        ms_aggregate = time_events(step, args.steps, 2)
        F.flashdp_set_stages(F.STAGE_ALL)
        step()
        torch.cuda.synchronize()
    hw_flops = flops * (2.0 if used == "twopass" else 1.0)
    if used == "ghost":   # upper-triangular blocks of both T x T Gram matrices, then the gradient itself
        hw_flops = flops + sum(float(w.B) * w.T * (w.T + 128) * (s.d_in + s.d_out) for s in w.layers)
    traffic_key = "scratch" if used == "overlap" else used
    n_launch = len(w.layers)
    what = {"scratch": "per-sample contraction + norm + spill", "twopass": "per-sample contraction + norm (first of two passes)",
            "explicit": "per-sample contraction, fp32 gradients materialised", "ghost": "Gram-matrix norms",
            "fused": "the whole of Algorithm 1 in one launch"}[traffic_key]
    roofline = {
        "bound": "mfma", "kernel": f"{'gram_norm_mfma_kernel' if used == 'ghost' else kernel} ({what})",
        "achieved": round(flops / ms_contract / 1e9, 2), "peak": peak, "unit": "TFLOP/s",
        "frac": round(flops / ms_contract / 1e9 / peak, 4),
        "launches_per_step": n_launch, "avg_launch_ms": round(ms_contract / n_launch, 4),
        "flops_per_launch": flops / n_launch, "traffic": None,
    }
    if w.dtype == "bf16":
        probe = mfma_only(F, torch, dev)
        roofline["mfma_only"] = probe
        # against what the matrix cores alone sustain on random operands through the instruction this kernel uses
        key = "random_16x16x32_tflops" if "dma16" in kernel else "random_tflops"
        roofline["frac_of_mfma_only_random"] = round(flops / ms_contract / 1e9 / probe[key], 4)
        roofline["mfma_only_reference"] = key
    mt = measured_traffic(w.name, traffic_key, kernel)
    if mt:
        roofline["traffic"] = mt["read_bytes"] + mt["write_bytes"]
        esz = 4.0 if w.dtype == "fp32" else 2.0
        roofline["traffic_detail"] = {
            "read_bytes": mt["read_bytes"], "write_bytes": mt["write_bytes"], "source": "profiles/traffic.json",
            "measured_at_commit": mt.get("commit"), "measured_on": mt.get("date"),
            "algorithmic_read_bytes": sum(esz * w.B * w.T * (s.d_in + s.d_out) for s in w.layers) / n_launch,
            "algorithmic_write_bytes": sum(esz * w.B * s.d_in * s.d_out for s in w.layers) / n_launch}

    result = {
        "metric": "dp_weight_grad_tflops", "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "T": w.T,
                   "layers": [f"{s.name}:{s.d_in}->{s.d_out}" for s in w.layers],
                   "C": w.C, "sigma": w.sigma, "schedule": used, "shared_x": bool(args.share_x)},
        "ms_per_step_median": round(ms_median, 4), "ms_per_step_min": round(ms_min, 4),
        "frac_of_mfma_peak": round(tflops / peak, 4),
        "hardware_flops_per_step": hw_flops,
        "stage_ms": {"contract": round(ms_contract, 4), "aggregate_and_noise": round(ms_aggregate, 4),
                     "exposed_beyond_contract": round(ms - ms_contract, 4)},
        "roofline": roofline,
    }

    if not args.no_comparators:
        # non-DP comparators: dY^T X over K = B*T (Eq. batched-grad), same inputs
        def blas():
            for (X, dY, out, _) in keep:
                torch.matmul(dY.view(-1, dY.shape[-1]).t(), X.view(-1, X.shape[-1]))

        def own():
            for (X, dY, out, _), spec in zip(keep, w.layers):
                F.flashdp_plain_grad(X, dY, w.B, w.T, spec.d_in, spec.d_out, dtype_code, out)

        ws_bal = torch.empty(F.flashdp_plain_grad_balanced_workspace_bytes(), dtype=torch.uint8, device=dev)

        def own_balanced():
            for (X, dY, out, _), spec in zip(keep, w.layers):
                F.flashdp_plain_grad_balanced(X, dY, w.B, w.T, spec.d_in, spec.d_out, dtype_code, out, ws_bal)

        ms_blas = time_steps(blas, args.steps, 3)
        ms_own = time_steps(own, args.steps, 3)
        ms_bal = time_steps(own_balanced, args.steps, 3)
        del ws_bal
        best = min(ms_blas, ms_own, ms_bal)
        result["nondp"] = {"torch_matmul_ms": round(ms_blas, 4), "torch_matmul_tflops": round(flops / ms_blas / 1e9, 2),
                           "own_plain_ms": round(ms_own, 4), "own_plain_tflops": round(flops / ms_own / 1e9, 2),
                           "own_balanced_ms": round(ms_bal, 4), "own_balanced_tflops": round(flops / ms_bal / 1e9, 2),
                           "fastest": min((ms_blas, "torch_matmul"), (ms_own, "own_plain"), (ms_bal, "own_balanced"))[1]}
        result["ratio_vs_nondp"] = round(best / ms, 4)
        # restore the outputs of a full DP step
        step()
        torch.cuda.synchronize()

    if not args.no_schedule_comparison:
        # the same step under the other schedules: two-pass recompute (the paper's "implicit" class) and the
        # explicit four-stage flow with materialised fp32 per-sample gradients (its "explicit" class), and the
        # ghost-norm route (norms from T x T Gram matrices, then one clipped accumulation)
        cmp = {used: round(ms, 4)}
        for other in ("overlap", "scratch", "twopass", "explicit", "ghost", "fused"):
            if other in cmp:
                continue
            ws_o = torch.empty(F.flashdp_workspace_bytes(arr, w.B, w.T, dtype_code, other), dtype=torch.uint8, device=dev)
            cmp[other] = round(time_steps(lambda: F.flashdp_block_dp_grad(arr, w.B, w.T, dtype_code, other, ws_o),
                                          max(3, args.steps // 4), 2), 4)
            del ws_o
        result["schedule_ms"] = cmp
        step()
        torch.cuda.synchronize()

    if args.timeline and w.dtype == "bf16":
        big = max(range(len(w.layers)), key=lambda k: w.layers[k].d_in * w.layers[k].d_out)
        X, dY, _, _ = keep[big]
        spec = w.layers[big]
        tl = {"layer": spec.name, "B": w.B, "T": w.T, "d_in": spec.d_in, "d_out": spec.d_out}
        tl["workload_data_park"] = contraction_timeline(F, torch, X, dY, w.B, w.T, spec.d_in, spec.d_out, True)
        tl["workload_data_norm_only"] = contraction_timeline(F, torch, X, dY, w.B, w.T, spec.d_in, spec.d_out, False)
        Xz, dYz = torch.zeros_like(X), torch.zeros_like(dY)
        tl["zero_operands_park"] = contraction_timeline(F, torch, Xz, dYz, w.B, w.T, spec.d_in, spec.d_out, True)
        tl["zero_operands_norm_only"] = contraction_timeline(F, torch, Xz, dYz, w.B, w.T, spec.d_in, spec.d_out, False)
        del Xz, dYz
        result["timeline"] = tl
        step()
        torch.cuda.synchronize()

    if args.vendor_envelope:
        env = {}
        n = 8192
        for kind in ("randn", "zeros"):
            mk = (lambda *sh: torch.randn(*sh, device=dev).bfloat16()) if kind == "randn" else (lambda *sh: torch.zeros(*sh, device=dev, dtype=torch.bfloat16))
            a_mk, b_nk, a_km, b_kn = mk(n, n), mk(n, n), mk(n, n), mk(n, n)
            t_best = time_events(lambda: torch.matmul(a_mk, b_nk.t()), 10, 3)
            t_ours = time_events(lambda: torch.matmul(a_km.t(), b_kn), 10, 3)
            env[kind] = {"k_contiguous_tflops": round(2.0 * n ** 3 / t_best / 1e9, 1), "k_slowest_tflops": round(2.0 * n ** 3 / t_ours / 1e9, 1)}
            del a_mk, b_nk, a_km, b_kn
        result["vendor_gemm_8192_cubed"] = env

    if args.copy_probe:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        result["copy_probe_bytes_each_way"] = 1 << 30

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
