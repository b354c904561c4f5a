"""GPU parity of one transfer event between two coupled tiles (Tiki-Taka): analog read of a
column of the fast tile, pulsed write onto the slow tile; the oracle composes its own analog
product and pulsed update."""
import numpy as np
import pytest

import oracle
import paper_2104_02184_amd as aht

from common import gpu_params, oracle_params, to_dev

pytestmark = pytest.mark.gpu


# without input noise the library reads the column directly, with it through the full analog product
@pytest.mark.parametrize("inp_noise,w_noise", [(0.0, 0.0), (0.0, 0.03), (0.01, 0.03)])
@pytest.mark.parametrize("R,C", [(64, 64), (70, 131), (300, 70)])
def test_transfer_events_match_the_oracle_composition(R, C, inp_noise, w_noise):
    dev = dict(kind=aht.SOFT_BOUNDS, dw_min=0.002, dw_min_dtod=0.3, dw_min_std=0.3, w_max=0.6, w_max_dtod=0.2,
               w_min=-0.6, w_min_dtod=0.2)
    io_kw = dict(inp_res=1.0 / 126.0, inp_bound=1.0, inp_noise=inp_noise, w_noise=w_noise, out_noise=0.02,
                 out_res=2.0 / 254.0, out_bound=2.0, noise_management=True)
    g = np.random.default_rng(R)
    A0 = g.uniform(-0.3, 0.3, size=(R, C)).astype(np.float32)
    seed_a, seed_c, bl, lr = 5, 6, 31, 0.05
    planes_c = oracle.device_planes(oracle_params(dev), seed_c, R, C)
    Co = np.zeros((R, C), dtype=np.float32)
    fast = aht.Tile(R, C, gpu_params(dev), bl, False, seed_a)
    slow = aht.Tile(R, C, gpu_params(dev), bl, True, seed_c)
    fast.set_weights(to_dev(A0))
    cols = [0, 3, C - 1, 3]
    pulses = 0
    for k, col in enumerate(cols):
        fast.transfer_column_to(slow, col, lr, aht.IOParams(**io_kw))
        e = np.zeros((1, C), dtype=np.float32)
        e[0, col] = 1.0
        read = oracle.analog_mvm(A0, e, oracle.IOParams(**io_kw), seed_a, k)
        pulses += oracle.pulsed_update(Co, planes_c, oracle_params(dev), bl, True, e, -read, lr, seed_c, k)
    Cg = slow.get_weights().cpu().numpy()
    assert slow.pulse_count() == pulses and pulses > 0
    assert fast.mvm_steps[0] == len(cols) and slow.step == len(cols)
    assert np.abs(Cg.astype(np.float64) - Co).max() / 0.6 <= 1e-5
    untouched = np.setdiff1d(np.arange(C), cols)
    assert (Cg[:, untouched] == 0).all()
    # the written column follows the read column's sign
    assert np.sign(Cg[:, 0]).astype(int).tolist().count(0) < R
    with pytest.raises(aht.AhtError):
        fast.transfer_column_to(slow, C, lr, aht.IOParams(**io_kw))
    with pytest.raises(aht.AhtError):
        fast.transfer_column_to(fast, 0, lr, aht.IOParams(**io_kw))
    fast.close()
    slow.close()
