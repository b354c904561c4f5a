#!/usr/bin/env python3
"""Benchmark of the stochastic pulsed update on one MI355X.

A step = one aht_pulsed_update call (line scaling + pulse trains + cell update) on the
headline workload: 4096x4096 LinearStep tile, update management, B = 256 update vectors,
BL = 63, fresh seeded synthetic x ~ N(0,1), d ~ N(0,0.01) already resident in HBM.
Prints ONE JSON line: Gcell-pulse-updates/s (cells * B * BL per call / time), the roofline
of the dominant kernel (the cell update, bound by plain vector-ALU issue) and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# ---- roofline model of the cell-update kernel ------------------------------------------------
# The kernel is bound by plain vector-ALU issue.  Peak = one lane-op per lane and clock:
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz (the rate of v_fma_f32, i.e. half the 157.3 TFLOP/s
# packed-fp32 figure).  Algorithmic work = the minimal ISA instruction stream of the method,
# one lane-op per instruction and lane:
#   per (cell, sample), 64-bit words: 2 AND + 2 BCNT + 1 XOR (direction) + 1 to record  = 6
#   per (cell, sample), 32-bit words: 1 AND + 1 BCNT + 1 XOR + 1                       = 4
#   per applied pulse with pulse-to-pulse noise:
#       1/4 Philox4x32-10 block  (20 v_mad_u64_u32 + 20 three-input XOR) / 4           = 10
#       1/2 Box-Muller pair      (2 shift, add, 2 cvt, 5 mul, log, sqrt, sin, cos) / 2 = 7
#       device step: ConstantStep 4 (select, noise fma, w fma, clamp); LinearStep/SoftBounds 8
#       (two selects, slope fma, max, mul, noise fma, w fma, clamp)
PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
C_CS = {8: 6.0, 4: 4.0}
C_PULSE_NOISE = 10.0 + 7.0
C_STEP = {0: 4.0, 1: 8.0, 2: 8.0}
# HBM-side bytes of one headline call of the cell-update kernel, from rocprofv3 --pmc
# FETCH_SIZE and WRITE_SIZE (profiles/cell_update_cfg5_counters.md; FETCH_SIZE scaled by the
# factor a plain copy of known size gives).  None for other workloads.
MEASURED_TRAFFIC_BYTES = {"cfg5_4096x4096_linearstep": 717.0e6}


def algorithmic_lane_ops(w, pulses_per_call):
    word_bytes = 4 if w.bl <= 31 else 8
    c_p = C_STEP[w.device["kind"]] + (C_PULSE_NOISE if w.device["dw_min_std"] > 0 else 0.0)
    if not w.device["dw_min_std"] > 0:
        c_p -= 1.0                                   # no noise fma
    return C_CS[word_bytes] * w.rows * w.cols * w.batch + c_p * pulses_per_call


def host_cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def oracle_call(w, rows, threads):
    """One oracle call on the first `rows` rows of workload `w`; returns (work, pulses, seconds)."""
    import numpy as np

    import oracle
    from paper_2104_02184_amd import workloads as wl

    s = wl.scaled(w, rows=rows, steps=1, name=w.name + "_cpu_sample")
    p = oracle.DeviceParams(**s.device)
    planes = oracle.device_planes(p, s.seed, s.rows, s.cols)
    W = np.clip(wl.initial_weights(s), planes["b_min"], planes["b_max"]).astype(np.float32)
    _, x, d = next(iter(wl.input_stream(s)))
    oracle.set_num_threads(threads)
    t0 = time.perf_counter()
    pulses = oracle.pulsed_update(W, planes, p, s.bl, s.update_management, x, d, s.lr, s.seed, 0)
    dt = time.perf_counter() - t0
    return s, pulses, dt


def cpu_baseline(w, target_rows):
    """The oracle, as it stands, on a row slice of the same workload (same device law, same
    input law, same B and BL): all host threads on `target_rows` rows, then one thread on an
    quarter of them (the pulse words of all 4096 columns are part of both samples)."""
    import oracle

    all_threads = oracle.num_threads()
    s, pulses, dt = oracle_call(w, target_rows, all_threads)
    s1, pulses1, dt1 = oracle_call(w, max(1, target_rows // 4), 1)
    oracle.set_num_threads(all_threads)
    return {
        "value": s.cell_pulse_updates_per_call / dt / 1e9,
        "unit": "Gcell-pulse-updates/s",
        "cores": all_threads,
        "kind": "oracle",
        "sample": f"{s.rows}x{s.cols} row slice of the headline tile, B={s.batch}, BL={s.bl}, 1 call "
                  f"({pulses} pulses, {dt:.2f} s wall)",
        "single_thread_value": s1.cell_pulse_updates_per_call / dt1 / 1e9,
        "single_thread_sample": f"{s1.rows}x{s1.cols} row slice, 1 call ({pulses1} pulses, {dt1:.2f} s wall)",
        "host": f"{host_cpu_model()}, {os.cpu_count()} logical CPUs",
    }


def bench_decay_diffuse(args):
    """Side benchmark: the once-per-mini-batch decay + diffusion pass on the headline tile
    (HBM bound: 20 bytes read and 4 written per cell)."""
    import torch

    import paper_2104_02184_amd as aht
    from paper_2104_02184_amd import workloads as wl

    w = wl.WORKLOADS[args.workload or wl.HEADLINE]
    tile = aht.Tile(w.rows, w.cols, aht.DeviceParams(**w.device), w.bl, w.update_management, w.seed)
    tile.set_temporal(decay_rate=0.001, decay_rate_dtod=0.1, diffusion=0.0005, diffusion_dtod=0.3)
    tile.set_weights(torch.from_numpy(wl.initial_weights(w)).cuda())
    for _ in range(args.warmup):
        tile.decay_diffuse()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        tile.decay_diffuse()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    tile.close()
    cells = w.rows * w.cols
    bytes_alg = cells * 24.0
    print(json.dumps({
        "metric": "Gcell/s of decay_diffuse", "value": cells / (ms * 1e-3) / 1e9, "unit": "Gcell/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "dtype": "f32",
        "data": "synthetic", "config": {"workload": w.name + " decay_diffuse"},
        "roofline": {"bound": "hbm", "achieved": bytes_alg / (ms * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                     "frac": bytes_alg / (ms * 1e-3) / 8e12, "traffic": None},
    }), flush=True)


def bench_mvm(args, transposed):
    """Side benchmark: the analog matrix-vector product of a batch (Eq. (1)) on the headline tile
    (2*B*R*C flops per call; the roofline counts the flops the chosen path executes on the matrix cores)."""
    import torch

    import paper_2104_02184_amd as aht
    from paper_2104_02184_amd import workloads as wl

    w = wl.WORKLOADS[args.workload or wl.HEADLINE]
    tile = aht.Tile(w.rows, w.cols, aht.DeviceParams(**w.device), w.bl, w.update_management, w.seed)
    tile.set_weights(torch.from_numpy(wl.initial_weights(w)).cuda())
    g = wl.rng_for(w, 3)
    n_in = w.rows if transposed else w.cols
    x = torch.from_numpy(g.standard_normal((w.batch, n_in), dtype="float32")).cuda()
    io = aht.IOParams(inp_noise=args.inp_noise, w_noise=0.02)
    fn = tile.backward if transposed else tile.forward
    for _ in range(args.warmup):
        fn(x, io)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        fn(x, io)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    tile.close()
    flops = 2.0 * w.batch * w.rows * w.cols
    # quantised inputs without input noise: the product runs as three passes of the bf16 matrix
    # cores (integer DAC codes, fp32 weights cut into three bf16 terms, fp32 sums); other inputs as
    # three bf16 terms too, six passes; where the shape rules both out, one pass of the fp32 cores
    n_out = w.cols if transposed else w.rows
    codes = args.inp_noise == 0.0 and os.environ.get("AHT_MVM_CODES", "1") != "0" and n_in % 32 == 0 and n_out % 16 == 0
    planes = (not codes and os.environ.get("AHT_MVM_PLANES", "1") != "0" and n_in % 32 == 0 and n_out % 64 == 0)
    executed = 3.0 * flops if codes else 6.0 * flops if planes else flops
    peak = 2500.0 if (codes or planes) else 157.3
    dtype = "bf16 x 3 terms, f32 sums" if codes else "bf16 x 3 x 3 terms (6 products), f32 sums" if planes else "f32"
    print(json.dumps({
        "metric": "TFLOP/s of analog " + ("backward" if transposed else "forward"), "value": flops / (ms * 1e-3) / 1e12,
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{w.name} analog MVM, B={w.batch}, inp_noise={args.inp_noise}"},
        "roofline": {"bound": "mfma", "achieved": executed / (ms * 1e-3) / 1e12, "peak": peak, "unit": "TFLOP/s",
                     "frac": executed / (ms * 1e-3) / (peak * 1e12), "traffic": None},
    }), flush=True)


def bench_transfer(args):
    """Side benchmark: one transfer event between two coupled tiles of the headline shape (analog read
    of one column of the fast tile, pulsed write onto the slow tile)."""
    import torch

    import paper_2104_02184_amd as aht
    from paper_2104_02184_amd import workloads as wl

    w = wl.WORKLOADS[args.workload or wl.HEADLINE]
    fast = aht.Tile(w.rows, w.cols, aht.DeviceParams(**w.device), w.bl, w.update_management, w.seed)
    slow = aht.Tile(w.rows, w.cols, aht.DeviceParams(**w.device), w.bl, w.update_management, w.seed + 1)
    fast.set_weights(torch.from_numpy(wl.initial_weights(w)).cuda())
    io = aht.IOParams(inp_noise=0.0, w_noise=0.0, out_noise=0.02)
    cols = [(7919 * k) % w.cols for k in range(args.warmup + args.steps)]
    for k in range(args.warmup):
        fast.transfer_column_to(slow, cols[k], 0.1, io)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for k in range(args.steps):
        fast.transfer_column_to(slow, cols[args.warmup + k], 0.1, io)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    pulses = slow.pulse_count()
    fast.close()
    slow.close()
    print(json.dumps({
        "metric": "transfer events/s", "value": 1e3 / ms, "unit": "events/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name} transfer of one column", "pulses_total": pulses},
    }), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=None, help="workload name (default: the headline one)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--cpu-rows", type=int, default=512)
    ap.add_argument("--inp-noise", type=float, default=0.01,
                    help="input noise of the forward/backward side benchmarks (0: quantised inputs only)")
    ap.add_argument("--op", default="pulsed_update", choices=["pulsed_update", "decay_diffuse", "forward", "backward", "transfer"],
                    help="side benchmarks of other operations; the default is the headline metric")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the pulsed update of one tile runs on a single MI355X "
              "(it would shard by blocks of rows of the tile, not by batch); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2104_02184_amd as aht
    from paper_2104_02184_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    aht.load_library()
    if args.op == "decay_diffuse":
        bench_decay_diffuse(args)
        return
    if args.op == "transfer":
        bench_transfer(args)
        return
    if args.op in ("forward", "backward"):
        bench_mvm(args, args.op == "backward")
        return
    w = wl.WORKLOADS[args.workload or wl.HEADLINE]
    K, Wm = args.steps, args.warmup

    tile = aht.Tile(w.rows, w.cols, aht.DeviceParams(**w.device), w.bl, w.update_management, w.seed)
    bmax, bmin = tile.get_plane("b_max"), tile.get_plane("b_min")
    W0 = torch.from_numpy(wl.initial_weights(w)).cuda()
    tile.set_weights(torch.minimum(torch.maximum(W0, bmin), bmax))
    del bmax, bmin, W0

    # fresh inputs for every step, uploaded before the timed region
    g = wl.rng_for(w, 2)
    pool = min(K + Wm, 24 if w.batch <= 1024 else 4)
    xs = [torch.from_numpy(wl.draw_x(w, g)).cuda() for _ in range(pool)]
    ds = [torch.from_numpy(wl.draw_d(w, g)).cuda() for _ in range(pool)]

    for i in range(Wm):
        tile.pulsed_update(xs[i % pool], ds[i % pool], w.lr)
    torch.cuda.synchronize()
    p0 = tile.pulse_count()
    tile.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        tile.pulsed_update(xs[(Wm + i) % pool], ds[(Wm + i) % pool], w.lr)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_words, ms_cells, calls = tile.profile_read()
    tile.profile_enable(False)
    pulses = (tile.pulse_count() - p0) / max(K, 1)
    # The same K calls once more without the three event records per call that the kernel times above
    # come from: on small tiles those records cost more than the gaps between the kernels.
    torch.cuda.synchronize()
    u0 = time.perf_counter()
    for i in range(K):
        tile.pulsed_update(xs[(Wm + i) % pool], ds[(Wm + i) % pool], w.lr)
    torch.cuda.synchronize()
    ms_per_step_plain = (time.perf_counter() - u0) / K * 1e3
    tile.close()

    sec = t1 - t0
    ms_per_step = sec / K * 1e3
    value = w.cell_pulse_updates_per_call * K / sec / 1e9
    cell_ms = ms_cells / max(calls, 1)
    ops = algorithmic_lane_ops(w, pulses)
    achieved = ops / (cell_ms * 1e-3)
    out = {
        "metric": "Gcell-pulse-updates/s of pulsed_update",
        "value": value,
        "unit": "Gcell-pulse-updates/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": ms_per_step,
        "ms_per_step_without_event_records": ms_per_step_plain,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "rows": w.rows, "cols": w.cols, "batch": w.batch, "bl": w.bl,
                   "update_management": w.update_management, "lr": w.lr,
                   "pulses_per_call": pulses, "applied_pulses_per_s": pulses / (sec / K)},
        "roofline": {
            "bound": "alu",
            "kernel": "k_cell_update",
            "achieved": achieved / 1e12,
            "peak": PEAK_LANE_OPS / 1e12,
            "unit": "Tlane-op/s",
            "frac": achieved / PEAK_LANE_OPS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
            "kernel_ms": cell_ms,
            "words_ms": ms_words / max(calls, 1),
            "algorithmic_lane_ops_per_launch": ops,
        },
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_rows)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
