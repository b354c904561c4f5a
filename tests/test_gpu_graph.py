"""A sequence of update calls recorded once into a HIP graph and replayed.

The step counter lives in device memory and every full update advances it itself, so each replay
continues the random streams where the last one stopped; the recorded entry point is the one that
allocates nothing.  The graph is replayed several times with eager work and synchronisations in
between, and every replay is checked against a tile that makes the same calls eagerly (bit for bit)
and, at the end, against the oracle."""
import numpy as np
import pytest

import oracle
import paper_2104_02184_amd as aht
from paper_2104_02184_amd import workloads as wl

from common import gpu_params, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("R,C,B,bl,um,kind", [
    (64, 64, 1, 31, False, aht.CONSTANT_STEP),          # the whole call in one launch
    (200, 333, 48, 63, True, aht.LINEAR_STEP),          # line scaling + pulse trains + cell update
    (96, 640, 300, 31, False, aht.SOFT_BOUNDS),         # a long batch of 32-bit words
])
def test_recorded_sequence_of_updates_replays_like_eager_calls(R, C, B, bl, um, kind):
    import torch
    dev = dict(kind=kind, dw_min=0.003, dw_min_dtod=0.3, dw_min_std=0.3, w_max=0.6, w_max_dtod=0.2, w_min=-0.6,
               w_min_dtod=0.2, gamma_up=0.4, gamma_down=0.6, gamma_dtod=0.1)
    g = np.random.default_rng(R + B)
    W0 = g.uniform(-0.3, 0.3, size=(R, C)).astype(np.float32)
    per_graph, replays = 3, 3
    xs = [g.normal(size=(B, C)).astype(np.float32) for _ in range(per_graph * replays)]
    ds = [(g.normal(size=(B, R)) * 0.2).astype(np.float32) for _ in range(per_graph * replays)]
    eager = aht.Tile(R, C, gpu_params(dev), bl, um, 3)
    graphed = aht.Tile(R, C, gpu_params(dev), bl, um, 3)
    eager.set_weights(to_dev(W0))
    graphed.set_weights(to_dev(W0))
    # static input buffers of the recorded calls, refilled before every replay
    xbuf = [torch.zeros((B, C), dtype=torch.float32, device="cuda") for _ in range(per_graph)]
    dbuf = [torch.zeros((B, R), dtype=torch.float32, device="cuda") for _ in range(per_graph)]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for k in range(per_graph):
            graphed.pulsed_update_noalloc(xbuf[k], dbuf[k], 0.1)
    torch.cuda.synchronize()
    # recording launched nothing: weights and the device's counter are untouched; the host's copy has counted
    # the recorded calls and is put right by reading the device's counter back
    assert (graphed.get_weights().cpu().numpy() == W0).all()
    assert graphed.sync_step() == 0
    for r in range(replays):
        for k in range(per_graph):
            n = r * per_graph + k
            xbuf[k].copy_(to_dev(xs[n]))
            dbuf[k].copy_(to_dev(ds[n]))
            eager.pulsed_update(to_dev(xs[n]), to_dev(ds[n]), 0.1)             # eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        We, Wg = eager.get_weights().cpu().numpy(), graphed.get_weights().cpu().numpy()
        assert (We.view(np.uint32) == Wg.view(np.uint32)).all(), f"replay {r}"
        assert eager.pulse_count() == graphed.pulse_count()
        assert graphed.sync_step() == eager.step == (r + 1) * per_graph
    # an eager call after the replays continues the same sequence
    x, d = g.normal(size=(B, C)).astype(np.float32), (g.normal(size=(B, R)) * 0.2).astype(np.float32)
    eager.pulsed_update(to_dev(x), to_dev(d), 0.1)
    graphed.pulsed_update(to_dev(x), to_dev(d), 0.1)
    We, Wg = eager.get_weights().cpu().numpy(), graphed.get_weights().cpu().numpy()
    assert (We.view(np.uint32) == Wg.view(np.uint32)).all()
    assert graphed.step == eager.step == replays * per_graph + 1
    pg = graphed.pulse_count()
    eager.close()
    graphed.close()
    # the oracle on the same sequence
    planes = oracle.device_planes(oracle.DeviceParams(**dev), 3, R, C)
    Wo, po = W0.copy(), 0
    for t, (xx, dd) in enumerate(zip(xs + [x], ds + [d])):
        po += oracle.pulsed_update(Wo, planes, oracle.DeviceParams(**dev), bl, um, xx, dd, 0.1, 3, t)
    assert po == pg
    assert np.abs(Wg.astype(np.float64) - Wo).max() / 0.6 <= 1e-5
