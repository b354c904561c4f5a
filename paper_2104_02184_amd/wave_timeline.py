"""Where the waves of the cell kernel spend their time (a profiling aid, not part of the update path).

    python -m paper_2104_02184_amd.wave_timeline --build            # no GPU needed: libaht_stamps.so beside libaht.so
    python -m paper_2104_02184_amd.wave_timeline WORKLOAD [...]     # on the GPU

The library is built once more with -DAHT_WAVE_STAMPS: lane 0 of every wave of the cell kernel then
writes the 100 MHz wall clock at seven points (start, weights loaded, phase A over, device parameters
loaded, cells dealt, pulses applied, weights stored) and the hardware's id of the SIMD it ran on.  After
some warm-up calls (the launch shape settles on the tile's own pulse rate) one call is stamped, and the
report gives, per workload: how the waves were spread over compute units and SIMDs, when the k-th wave
to finish on a SIMD passed each point (mean over the SIMDs), and the duration of each part.
The stamps wait for the wave's outstanding memory operations, so the stamped call is a little slower
than a plain one.
"""
from __future__ import annotations

import ctypes
import os
import sys
from collections import Counter

HERE = os.path.dirname(os.path.abspath(__file__))
STAMPS_LIB = os.path.join(HERE, "libaht_stamps.so")
POINTS = ["start", "weights loaded", "phase A over", "parameters loaded", "cells dealt", "pulses applied",
          "weights stored"]
PARTS = [(0, 1, "load weights"), (1, 2, "phase A (and earlier drains)"), (2, 3, "parameters, close streams"),
         (3, 4, "deal cells"), (4, 5, "apply pulses"), (5, 6, "cells home, store"), (0, 6, "whole wave")]


def timeline(name: str) -> None:
    import numpy as np
    import torch

    import paper_2104_02184_amd as aht
    from paper_2104_02184_amd import workloads as wl

    lib = aht.load_library()
    lib.aht_debug_set_wave_stamps.argtypes = [ctypes.c_void_p]
    w = wl.WORKLOADS[name]
    tile = aht.Tile(w.rows, w.cols, aht.DeviceParams(**w.device), w.bl, w.update_management, w.seed)
    bmax, bmin = tile.get_plane("b_max"), tile.get_plane("b_min")
    tile.set_weights(torch.minimum(torch.maximum(torch.from_numpy(wl.initial_weights(w)).cuda(), bmin), bmax))
    g = wl.rng_for(w, 2)
    xs = [torch.from_numpy(wl.draw_x(w, g)).cuda() for _ in range(4)]
    ds = [torch.from_numpy(wl.draw_d(w, g)).cuda() for _ in range(4)]
    max_waves = 1 << 19
    buf = torch.zeros(max_waves * 8, dtype=torch.int64, device="cuda")
    for i in range(24):
        tile.pulsed_update(xs[i % 4], ds[i % 4], w.lr)
        torch.cuda.synchronize()
    if lib.aht_debug_set_wave_stamps(ctypes.c_void_p(buf.data_ptr())) != 0:
        raise RuntimeError("aht_debug_set_wave_stamps failed")
    tile.pulsed_update(xs[0], ds[0], w.lr)
    torch.cuda.synchronize()
    lib.aht_debug_set_wave_stamps(None)
    info = tile.launch_info()
    raw = buf.cpu().numpy().reshape(max_waves, 8)
    raw = raw[(raw[:, 6] > 0) & (raw[:, 1] > 0)]
    t = (raw[:, :7] - raw[:, 0].min()).astype(np.float64) / 100.0          # microseconds since the first start
    hw, xcc = raw[:, 7] & 0xFFFFFFFF, (raw[:, 7] >> 32) & 0xF
    simd, cu, sh, se = (hw >> 4) & 3, (hw >> 8) & 15, (hw >> 12) & 1, (hw >> 13) & 7
    cu_key = ((xcc * 8 + se) * 2 + sh) * 16 + cu
    simd_key = cu_key * 4 + simd
    per_cu, per_simd = Counter(cu_key.tolist()), Counter(simd_key.tolist())
    print(f"== {name}: {info['rows_per_lane']} rows per lane, row lists {info['row_lists']}, {len(raw)} waves")
    print(f"  compute units used {len(per_cu)}, waves per compute unit {sorted(Counter(per_cu.values()).items())}; "
          f"SIMDs used {len(per_simd)}, waves per SIMD {sorted(Counter(per_simd.values()).items())}")
    print("  point, microseconds after the first wave's start:     min     p10     p50     p90     max")
    for k, label in enumerate(POINTS):
        v = t[:, k]
        print(f"    {label:44s} {v.min():7.1f} {np.percentile(v, 10):7.1f} {np.percentile(v, 50):7.1f} "
              f"{np.percentile(v, 90):7.1f} {v.max():7.1f}")
    print("  part, microseconds:                                  mean     p10     p50     p90     max")
    for a, b, label in PARTS:
        v = t[:, b] - t[:, a]
        print(f"    {label:44s} {v.mean():7.2f} {np.percentile(v, 10):7.2f} {np.percentile(v, 50):7.2f} "
              f"{np.percentile(v, 90):7.2f} {v.max():7.2f}")
    counts = set(per_simd.values())
    if len(counts) == 1 and len(raw) <= 16 * len(per_simd):                # one round: every wave resident from the start
        k = counts.pop()
        order = np.lexsort((t[:, 6], simd_key))
        by_rank = t[order].reshape(-1, k, 7).mean(axis=0)
        print("  k-th wave to finish on its SIMD, mean over the SIMDs, microseconds at each point:")
        for r in range(k):
            print(f"    {r + 1}. " + " ".join(f"{v:7.1f}" for v in by_rank[r]))
    tile.close()


def main(argv) -> int:
    if argv and argv[0] == "--build":
        from paper_2104_02184_amd import build as hip_build
        print(hip_build.build(force=True, extra=["-DAHT_WAVE_STAMPS"], out=STAMPS_LIB))
        return 0
    if not argv:
        print(__doc__)
        return 2
    if not os.path.exists(STAMPS_LIB):
        print("build the profiling library first: python -m paper_2104_02184_amd.wave_timeline --build", file=sys.stderr)
        return 2
    from paper_2104_02184_amd import binding
    binding._LIB_PATH = STAMPS_LIB            # (before the first load_library() of this process)
    for name in argv:
        timeline(name)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
