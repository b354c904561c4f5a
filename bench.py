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
# Measured issue rate of every instruction of that minimal stream, as a multiple of the nominal one
# lane-op per lane and clock (profiles/valu_issue_rates_gfx950.md).  The plain count above treats them
# all as 1.0; weighting the same stream by these gives the time the vector ALU needs at least for it
# (`rate_weighted_bound_ms`): simple two-operand operations issue faster than nominal, the 64-bit
# multiply-add and the population count a little slower, transcendentals at half rate.
RATE = {"and": 1.58, "xor": 1.69, "bcnt": 0.895, "alignbit": 0.95, "mad_u64_u32": 0.823, "bitop3": 1.027,
        "shift": 1.73, "add": 1.54, "cvt": 0.949, "mul": 1.58, "trans": 0.49, "bfi": 0.91, "fma": 0.99,
        "max": 0.97, "med3": 0.93}
# minimal stream: (instruction, how many) per unit
STREAM_CELL_SAMPLE = {8: [("and", 2), ("bcnt", 2), ("xor", 1), ("alignbit", 1)],
                      4: [("and", 1), ("bcnt", 1), ("xor", 1), ("alignbit", 1)]}
STREAM_PHILOX_QUARTER = [("mad_u64_u32", 5), ("bitop3", 5)]                       # 20 + 20 per block of four
STREAM_BOX_MULLER_HALF = [("shift", 1), ("add", 0.5), ("cvt", 1), ("mul", 2.5), ("trans", 2)]
STREAM_STEP = {0: [("bfi", 1), ("fma", 2), ("med3", 1)],                          # ConstantStep: select, noise, w, clamp
               1: [("bfi", 2), ("fma", 3), ("max", 1), ("mul", 1), ("med3", 1)],  # LinearStep / SoftBounds: + slope select,
               2: [("bfi", 2), ("fma", 3), ("max", 1), ("mul", 1), ("med3", 1)]}  #   slope fma, max, mul
COUNTERS_JSON = os.path.join(ROOT, "profiles", "cell_update_counters.json")


def _count(stream):
    return sum(n for _, n in stream)


def _weighted(stream):
    return sum(n / RATE[i] for i, n in stream)


def lane_ops_model(w, pulses_per_call, cell_samples=None):
    """(plain count, rate-weighted count) of the minimal instruction stream of one call; `cell_samples`
    overrides the number of (cell, sample) pairs counted (row lists visit only part of them)."""
    word_bytes = 4 if w.bl <= 31 else 8
    noise = w.device["dw_min_std"] > 0
    per_pulse = list(STREAM_STEP[w.device["kind"]])
    if noise:
        per_pulse += STREAM_PHILOX_QUARTER + STREAM_BOX_MULLER_HALF
    else:
        per_pulse = [(i, n - 1 if i == "fma" else n) for i, n in per_pulse]      # no noise fma
    cs = w.rows * w.cols * w.batch if cell_samples is None else cell_samples
    a = STREAM_CELL_SAMPLE[word_bytes]
    return (_count(a) * cs + _count(per_pulse) * pulses_per_call,
            _weighted(a) * cs + _weighted(per_pulse) * pulses_per_call)


def algorithmic_lane_ops(w, pulses_per_call):
    return lane_ops_model(w, pulses_per_call)[0]


def stored_counters(name):
    """hardware counters of the cell-update kernel on workload `name`, per dispatch, from the last
    rocprofv3 --pmc runs that `bench.py --pmc-summary` turned into profiles/cell_update_counters.json"""
    try:
        with open(COUNTERS_JSON) as f:
            return json.load(f).get(name)
    except (OSError, ValueError):
        return None


def pmc_summary(root_dir):
    """Turns rocprofv3 counter runs of this program into profiles/cell_update_counters.json (+ .md).

    Expected layout, one run per counter group and workload (rocprofv3 does not split counters over passes):
        <root_dir>/<workload>/fetch/*_counter_collection.csv   rocprofv3 --pmc FETCH_SIZE  -- python3 bench.py --workload <workload> --steps 3 --warmup 2 --no-cpu
        <root_dir>/<workload>/write/*_counter_collection.csv   rocprofv3 --pmc WRITE_SIZE  -- (same program)
        <root_dir>/<workload>/valu/*_counter_collection.csv    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_VALU_TRANS_F32 SQ_INSTS_SALU SQ_WAVES SQ_BUSY_CYCLES -- (same program)
    Per workload: the mean per dispatch of the cell-update kernel of the timed calls (the most frequent
    instantiation), and the byte counters' scale factors from the plain device-to-device copies of the
    weight matrix that the same run makes (rows x cols x 4 bytes read and written each)."""
    import csv
    import datetime
    import glob
    from collections import Counter, defaultdict

    from paper_2104_02184_amd import workloads as wl

    def rows_of(d):
        files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
        out = []
        for f in files:
            with open(f, newline="") as fh:
                out += list(csv.DictReader(fh))
        return out

    def per_kernel(rows, want):
        """kernel name -> counter -> list of per-dispatch values, for kernels whose name contains `want`"""
        acc = defaultdict(lambda: defaultdict(list))
        for r in rows:
            if want in r["Kernel_Name"]:
                acc[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
        return acc

    result, lines = {}, []
    for name, w in wl.WORKLOADS.items():
        base = os.path.join(root_dir, name)
        if not os.path.isdir(base):
            continue
        entry = {"date": datetime.date.today().isoformat(),
                 "command": f"rocprofv3 --pmc <counters> -- python3 bench.py --workload {name} --steps 3 --warmup 2 --no-cpu"}
        copy_bytes = w.rows * w.cols * 4.0
        for leg, counter, factor_key, kib_key in (("fetch", "FETCH_SIZE", "fetch_factor", "fetch_kib"),
                                                  ("write", "WRITE_SIZE", "write_factor", "write_kib")):
            rows = rows_of(os.path.join(base, leg))
            cells = per_kernel(rows, "k_cell_update")
            if not cells:
                continue
            kname = Counter({k: len(v[counter]) for k, v in cells.items()}).most_common(1)[0][0]
            vals = cells[kname][counter]
            entry[kib_key] = sum(vals) / len(vals)
            entry["kernel"] = kname.split("(")[0]
            entry["dispatches"] = len(vals)
            copies = [v for k, c in per_kernel(rows, "copyBuffer").items() for v in c[counter]]
            entry[factor_key] = (copy_bytes / 1024.0) / max(copies) if copies and max(copies) > 0 else None
        rows = rows_of(os.path.join(base, "valu"))
        cells = per_kernel(rows, "k_cell_update")
        if cells:
            kname = Counter({k: len(v["SQ_INSTS_VALU"]) for k, v in cells.items()}).most_common(1)[0][0]
            for counter, key in (("SQ_INSTS_VALU", "insts_valu"), ("SQ_INSTS_VALU_TRANS_F32", "insts_trans"),
                                 ("SQ_INSTS_SALU", "insts_salu"), ("SQ_WAVES", "waves"), ("SQ_BUSY_CYCLES", "busy_cycles")):
                v = cells[kname].get(counter)
                if v:
                    entry[key] = sum(v) / len(v)
        if "fetch_kib" in entry and "write_kib" in entry:
            result[name] = entry
    # scale factors of the byte counters: small tiles' copies are too short to calibrate on; they take the
    # factors of the largest tile measured (the counters' units do not depend on the kernel)
    ref = max(result, key=lambda n: wl.WORKLOADS[n].rows * wl.WORKLOADS[n].cols, default=None)
    for name, e in result.items():
        for k in ("fetch_factor", "write_factor"):
            small = wl.WORKLOADS[name].rows * wl.WORKLOADS[name].cols < (1 << 20)
            if e.get(k) is None or small:
                e[k] = result[ref][k]
            e[k] = round(e[k], 3)
    with open(COUNTERS_JSON, "w") as f:
        json.dump(result, f, indent=1, sort_keys=True)
        f.write("\n")
    lines.append("# Cell-update kernel: HBM-side bytes and executed vector instructions per dispatch, all workloads\n")
    lines.append("Written by `python bench.py --pmc-summary <dir>` from these runs (on the MI355X box, from /tmp with TMPDIR=/tmp,")
    lines.append("one counter group per run; W = a workload name, P = `python3 bench.py --workload W --steps 3 --warmup 2 --no-cpu`):\n")
    lines.append("    rocprofv3 --pmc FETCH_SIZE -d <dir>/W/fetch -o fetch --output-format csv -- P")
    lines.append("    rocprofv3 --pmc WRITE_SIZE -d <dir>/W/write -o write --output-format csv -- P")
    lines.append("    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_VALU_TRANS_F32 SQ_INSTS_SALU SQ_WAVES SQ_BUSY_CYCLES -d <dir>/W/valu -o valu --output-format csv -- P\n")
    lines.append("The byte counters are scaled by what the same counters read for the run's plain copies of the weight matrix")
    lines.append("(rows x cols x 4 bytes read and written).  `bench.py` reads the JSON beside this file for `roofline.traffic` and")
    lines.append("`roofline.executed_over_minimal`; algorithmic bytes = cells x (8 + 4 planes) + one read of the pulse words.\n")
    lines.append("| workload | kernel | FETCH_SIZE KiB x factor | WRITE_SIZE KiB x factor | HBM bytes | algorithmic bytes | vector instructions | x64 / minimal stream |")
    lines.append("|---|---|---|---|---|---|---|---|")
    for name, e in result.items():
        w = wl.WORKLOADS[name]
        traffic = e["fetch_kib"] * 1024 * e["fetch_factor"] + e["write_kib"] * 1024 * e["write_factor"]
        planes = 6 if w.device["kind"] == 1 else 4
        wb = 4 if w.bl <= 31 else 8
        alg = w.rows * w.cols * (8 + 4 * planes) + wb * w.batch * (w.rows + w.cols)
        lines.append(f"| {name} | `{e['kernel'].replace('aht::', '')}` | {e['fetch_kib']:.0f} x {e['fetch_factor']} | "
                     f"{e['write_kib']:.0f} x {e['write_factor']} | {traffic / 1e6:.1f} MB | {alg / 1e6:.1f} MB | "
                     f"{e.get('insts_valu', float('nan')):.4g} | see the bench line (needs the pulses of the timed calls) |")
    with open(os.path.join(ROOT, "profiles", "cell_update_counters.md"), "w") as f:
        f.write("\n".join(lines) + "\n")
    print(json.dumps(result, indent=1, sort_keys=True))


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
    info = tile.launch_info()
    tile.close()
    flops = 2.0 * w.batch * w.rows * w.cols             # the method's work: one multiply-add per weight and vector
    # Which path the library took is asked of the library.  Quantised inputs without input noise: three
    # passes of the bf16 matrix cores (integer DAC codes, fp32 weights cut into three bf16 terms, fp32
    # sums); other inputs as three bf16 terms too, six passes; where the shape rules both out, one pass of
    # the fp32 cores.  `frac` prices the method's flops against the peak of the cores used; the passes the
    # path executes for them are reported beside it, not in it.
    path, passes = info["mvm_path"], {1: 1, 2: 3, 3: 6}[info["mvm_path"]]
    peak = 157.3 if path == 1 else 2500.0
    dtype = {1: "f32", 2: "bf16 x 3 terms, f32 sums", 3: "bf16 x 3 x 3 terms (6 products), f32 sums"}[path]
    hbm_bytes = 4.0 * (w.rows * w.cols + w.batch * (w.rows + w.cols))
    print(json.dumps({
        "metric": "TFLOP/s of analog " + ("backward" if transposed else "forward"), "value": flops / (ms * 1e-3) / 1e12,
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": True, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{w.name} analog MVM, B={w.batch}, inp_noise={args.inp_noise}",
                   "path": {1: "fp32 matrix cores", 2: "bf16 matrix cores, DAC codes", 3: "bf16 matrix cores, input planes"}[path],
                   "slices": info["mvm_splits"]},
        "roofline": {"bound": "mfma", "achieved": flops / (ms * 1e-3) / 1e12, "peak": peak, "unit": "TFLOP/s",
                     "frac": flops / (ms * 1e-3) / (peak * 1e12), "traffic": None,
                     "matrix_passes_executed": passes,
                     "executed_matrix_flops_frac": passes * flops / (ms * 1e-3) / (peak * 1e12),
                     "bound_ms": {"matrix_cores_at_executed_passes": passes * flops / (peak * 1e12) * 1e3,
                                  "hbm_weights_and_vectors_once": hbm_bytes / 8e12 * 1e3}},
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


def bench_many(args):
    """N tiles of one workload per step (the layers of a network), updated through aht_pulsed_update_many and,
    for comparison, one after the other.  Kernels of different tiles overlap, so there is no per-kernel time:
    the roofline of this line prices the whole round (pulse-train kernels and gaps included) against the ALU."""
    import torch

    import paper_2104_02184_amd as aht
    from paper_2104_02184_amd import workloads as wl

    w = wl.WORKLOADS[args.workload or wl.HEADLINE]
    N, K, Wm = args.tiles, args.steps, args.warmup
    tiles, xs, ds = [], [], []
    g = wl.rng_for(w, 2)
    for i in range(N):
        t = aht.Tile(w.rows, w.cols, aht.DeviceParams(**w.device), w.bl, w.update_management, w.seed + i)
        bmax, bmin = t.get_plane("b_max"), t.get_plane("b_min")
        t.set_weights(torch.minimum(torch.maximum(torch.from_numpy(wl.initial_weights(w)).cuda(), bmin), bmax))
        tiles.append(t)
        xs.append([torch.from_numpy(wl.draw_x(w, g)).cuda() for _ in range(4)])
        ds.append([torch.from_numpy(wl.draw_d(w, g)).cuda() for _ in range(4)])
    lrs = [w.lr] * N

    def together(k):
        aht.pulsed_update_many(tiles, [x[k % 4] for x in xs], [d[k % 4] for d in ds], lrs)

    def in_turn(k):
        for t, x, d in zip(tiles, xs, ds):
            t.pulsed_update(x[k % 4], d[k % 4], w.lr)

    times = {}
    for name, fn in (("in_turn", in_turn), ("together", together)):
        for k in range(max(Wm, 20)):                     # (the launch shapes settle on the tiles' own pulse rates)
            fn(k)
        torch.cuda.synchronize()
        p0 = sum(t.pulse_count() for t in tiles)
        t0 = time.perf_counter()
        for k in range(K):
            fn(k)
        torch.cuda.synchronize()
        times[name] = (time.perf_counter() - t0) / K
        pulses = (sum(t.pulse_count() for t in tiles) - p0) / K / N
    info = tiles[0].launch_info()
    ms_graph = None
    if args.graph:
        # the same K rounds recorded once into a HIP graph and replayed: what a round costs without the host
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            for k in range(K):
                together(k)
        graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - g0) / K * 1e3
        for t in tiles:
            t.sync_step()
    for t in tiles:
        t.close()
    sec = times["together"]
    sparse = bool(info["row_lists"]) and info["row_fill"] >= 0
    ops, ops_weighted = lane_ops_model(w, pulses, w.rows * w.cols * w.batch * info["row_fill"] if sparse else None)
    print(json.dumps({
        "metric": "Gcell-pulse-updates/s of pulsed_update", "value": N * w.cell_pulse_updates_per_call / sec / 1e9,
        "unit": "Gcell-pulse-updates/s", "n_gpus": 1, "steps": K, "warmup": max(Wm, 20), "ms_per_step": sec * 1e3,
        "ms_per_tile": sec * 1e3 / N, "ms_per_tile_one_after_the_other": times["in_turn"] * 1e3 / N,
        "ms_per_tile_graph_replay": ms_graph / N if ms_graph is not None else None,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{N} tiles of {w.name} per step (aht_pulsed_update_many)", "tiles": N, "rows": w.rows,
                   "cols": w.cols, "batch": w.batch, "bl": w.bl, "pulses_per_tile_and_call": pulses},
        "roofline": {"bound": "alu", "kernel": "whole round: pulse-train and cell kernels of all tiles, overlapping",
                     "achieved": N * ops / sec / 1e12, "peak": PEAK_LANE_OPS / 1e12, "unit": "Tlane-op/s",
                     "frac": N * ops / sec / PEAK_LANE_OPS,
                     "frac_one_after_the_other": N * ops / times["in_turn"] / PEAK_LANE_OPS,
                     "algorithmic_lane_ops_per_tile": ops, "traffic": None, "launch": info},
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
    ap.add_argument("--tiles", type=int, default=1,
                    help="pulsed_update only: that many tiles of the workload per step, through aht_pulsed_update_many")
    ap.add_argument("--graph", action="store_true",
                    help="also record the timed calls into a HIP graph and time a replay (ms_per_step_graph_replay)")
    ap.add_argument("--pmc-summary", default=None, metavar="DIR",
                    help="no benchmark: turn rocprofv3 --pmc runs of this program under DIR into profiles/cell_update_counters.json")
    args = ap.parse_args()
    if args.pmc_summary:
        pmc_summary(args.pmc_summary)
        return
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
    if args.tiles > 1:
        bench_many(args)
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
    info = tile.launch_info()
    ms_per_step_graph = None
    if args.graph:
        # the same K calls recorded once into a HIP graph (through the entry point that allocates nothing: the
        # step counter is read and advanced on the device) and replayed: what a call costs without the host
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            for i in range(K):
                tile.pulsed_update_noalloc(xs[(Wm + i) % pool], ds[(Wm + i) % pool], w.lr)
        graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        graph.replay()
        torch.cuda.synchronize()
        ms_per_step_graph = (time.perf_counter() - g0) / K * 1e3
        tile.sync_step()
    tile.close()

    sec = t1 - t0
    ms_per_step = sec / K * 1e3
    value = w.cell_pulse_updates_per_call * K / sec / 1e9
    cell_ms = ms_cells / max(calls, 1)
    # Walking row lists, the kernel never looks at the (cell, sample) pairs whose row train is empty: the dense
    # count is then no lower bound of its work (the kernel can, and on workload 4 does, finish sooner than the
    # ALU could run the dense stream).  The roofline of such a launch counts the visited pairs only; the dense
    # count's figure stays beside it under a name of its own.
    ops_dense = lane_ops_model(w, pulses)[0]
    sparse = bool(info["row_lists"]) and info["row_fill"] >= 0
    visited = w.rows * w.cols * w.batch * info["row_fill"] if sparse else None
    ops, ops_weighted = lane_ops_model(w, pulses, visited)
    achieved = ops / (cell_ms * 1e-3)
    kernel = ("k_cell_update_rowlists" if info["row_lists"] else
              "k_cell_update_pair" if info["side_rows_per_lane"] else "k_cell_update")
    # Counters of the same kernel on the same workload from the last profiler runs (bench.py cannot read them
    # while it times): HBM-side bytes, and the vector instructions executed, which say how much of what the
    # kernel issues is the minimal stream.  null where no such run is on file.
    pmc = stored_counters(w.name)
    traffic = executed_over_minimal = None
    if pmc:
        traffic = pmc["fetch_kib"] * 1024.0 * pmc["fetch_factor"] + pmc["write_kib"] * 1024.0 * pmc["write_factor"]
        if pmc.get("insts_valu"):
            executed_over_minimal = pmc["insts_valu"] * 64.0 / ops
    out = {
        "metric": "Gcell-pulse-updates/s of pulsed_update",
        "value": value,
        "unit": "Gcell-pulse-updates/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": Wm,
        "ms_per_step": ms_per_step,
        "ms_per_step_without_event_records": ms_per_step_plain,
        "ms_per_step_graph_replay": ms_per_step_graph,
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
            "kernel": kernel,
            "achieved": achieved / 1e12,
            "peak": PEAK_LANE_OPS / 1e12,
            "unit": "Tlane-op/s",
            "frac": achieved / PEAK_LANE_OPS,
            "traffic": traffic,
            "traffic_source": (f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of {pmc['date']}, kernel {pmc['kernel']}"
                               if pmc else None),
            "kernel_ms": cell_ms,
            "words_ms": ms_words / max(calls, 1),
            "algorithmic_lane_ops_per_launch": ops,
            # the same minimal stream with every instruction at its measured issue rate: the least time the
            # vector ALU needs for it, and the kernel's time against that
            "rate_weighted_bound_ms": ops_weighted / PEAK_LANE_OPS * 1e3,
            "frac_rate_weighted": ops_weighted / PEAK_LANE_OPS * 1e3 / cell_ms,
            "executed_over_minimal": executed_over_minimal,
            "launch": info,
        },
    }
    if sparse:
        out["roofline"]["row_trains_with_a_pulse"] = info["row_fill"]
        out["roofline"]["frac_on_dense_count"] = ops_dense / (cell_ms * 1e-3) / PEAK_LANE_OPS
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_rows)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
