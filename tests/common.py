"""Helpers shared by the GPU parity tests: build the HIP tile and the oracle's
description from one workload, and run both sides on the same seeded inputs."""
import numpy as np

import oracle
import paper_2104_02184_amd as aht
from paper_2104_02184_amd import workloads as wl


def oracle_params(dev: dict) -> oracle.DeviceParams:
    return oracle.DeviceParams(**dev)


def gpu_params(dev: dict) -> aht.DeviceParams:
    return aht.DeviceParams(**dev)


def make_tile(w: wl.Workload, seed=None) -> aht.Tile:
    return aht.Tile(w.rows, w.cols, gpu_params(w.device), w.bl, w.update_management,
                    seed=w.seed if seed is None else seed)


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def words_to_np(t):
    """int64 device tensor holding uint64 bit patterns -> numpy uint64"""
    return t.cpu().numpy().view(np.uint64)


def run_gpu(w: wl.Workload, W0, steps=None, tile=None, collect_words_step=None):
    """Run `steps` update calls of workload w on the GPU; returns final weights (numpy)."""
    import torch
    own = tile is None
    tile = tile or make_tile(w)
    tile.set_weights(to_dev(W0))
    n = 0
    for t, x, d in wl.input_stream(w):
        if steps is not None and t >= steps:
            break
        tile.pulsed_update(to_dev(x), to_dev(d), w.lr)
        n += 1
    out = tile.get_weights().cpu().numpy()
    torch.cuda.synchronize()
    pulses = tile.pulse_count()
    if own:
        tile.close()
    return out, pulses


def run_oracle(w: wl.Workload, W0, planes, steps=None, cells=None):
    p = oracle_params(w.device)
    W = W0.copy()
    pulses = 0
    for t, x, d in wl.input_stream(w):
        if steps is not None and t >= steps:
            break
        pulses += oracle.pulsed_update(W, planes, p, w.bl, w.update_management, x, d, w.lr, w.seed, t,
                                       cells=cells)
    return W, pulses


def gpu_planes(tile) -> dict:
    return {n: tile.get_plane(n).cpu().numpy() for n in aht.PLANE_NAMES}
