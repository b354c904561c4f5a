"""Seeded synthetic workloads: tile shapes, device descriptions and the
``x`` / ``d`` / initial-weight generators.

This module holds NO arithmetic of the update method (no pulse probabilities,
no device steps, no random streams of the method itself); it only draws
inputs with numpy's seeded generator.  It is the one module that both the
HIP path's callers and the CPU oracle's callers use, so that they see the
same inputs.

The five workloads are layer-shaped tiles of the kind the paper trains
(arXiv 2104.02184, Sec. 3: fully connected and convolution layers mapped on
tiles; mini-batches and convolutions give many update vectors per step).
They stand in for the paper's VGG-8/CIFAR-10 run, whose data is not used.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

CONSTANT_STEP, LINEAR_STEP, SOFT_BOUNDS = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    rows: int                 # R = length of d (outputs)
    cols: int                 # C = length of x (inputs)
    batch: int                # update vectors per call
    bl: int                   # pulse-train length
    steps: int                # update calls
    lr: float
    update_management: bool
    device: dict = field(default_factory=dict)   # scalar device description
    x_dist: str = "normal"    # normal | uniform | relu_normal
    d_std: float = 1.0
    w_init: float = 0.3       # W0 ~ U(-w_init, w_init) * w_max ; 0 -> zeros
    seed: int = 0

    @property
    def cell_pulse_updates_per_call(self) -> int:
        return self.rows * self.cols * self.batch * self.bl


def _dev(kind, **kw):
    base = dict(kind=kind, dw_min=0.001, dw_min_dtod=0.0, dw_min_std=0.0, up_down=0.0,
                up_down_dtod=0.0, w_max=1.0, w_max_dtod=0.0, w_min=-1.0, w_min_dtod=0.0,
                gamma_up=0.0, gamma_down=0.0, gamma_dtod=0.0)
    base.update(kw)
    return base


_D2D_CONSTANT = _dev(CONSTANT_STEP, dw_min=0.001, dw_min_dtod=0.3, dw_min_std=0.3,
                     up_down_dtod=0.01, w_max=0.6, w_max_dtod=0.3, w_min=-0.6, w_min_dtod=0.3)

WORKLOADS = {
    # 1: small noiseless constant-step tile
    "cfg1_64x64_constant": Workload(
        "cfg1_64x64_constant", 64, 64, 1, 31, 10, 0.1, False,
        _dev(CONSTANT_STEP, dw_min=0.01, w_max=1.0, w_min=-1.0),
        x_dist="normal", d_std=1.0, w_init=0.0),
    # 2: constant step with device-to-device and pulse-to-pulse variation
    "cfg2_512x512_constant_d2d": Workload(
        "cfg2_512x512_constant_d2d", 512, 512, 64, 31, 100, 0.1, False, _D2D_CONSTANT,
        x_dist="uniform", d_std=0.1),
    # 3: soft bounds, ReLU-sparse inputs
    "cfg3_1024x1024_softbounds": Workload(
        "cfg3_1024x1024_softbounds", 1024, 1024, 128, 31, 100, 0.1, False,
        _dev(SOFT_BOUNDS, dw_min=0.001, dw_min_std=0.3, w_max=0.6, w_min=-0.6),
        x_dist="relu_normal", d_std=0.05),
    # 4: convolution-shaped tile: 256 output channels x (3*3*256) inputs,
    #    64 images x 14x14 positions = 12544 update vectors per step
    "cfg4_conv_256x2304": Workload(
        "cfg4_conv_256x2304", 256, 2304, 12544, 31, 10, 0.1, False, _D2D_CONSTANT,
        x_dist="relu_normal", d_std=0.01),
    # 5: headline: large linear-step tile with update management, BL = 63
    "cfg5_4096x4096_linearstep": Workload(
        "cfg5_4096x4096_linearstep", 4096, 4096, 256, 63, 20, 0.1, True,
        _dev(LINEAR_STEP, dw_min=0.001, dw_min_dtod=0.3, dw_min_std=0.3, up_down_dtod=0.01,
             w_max=0.6, w_max_dtod=0.3, w_min=-0.6, w_min_dtod=0.3, gamma_up=0.1,
             gamma_down=0.1, gamma_dtod=0.3),
        x_dist="normal", d_std=0.01),
}

HEADLINE = "cfg5_4096x4096_linearstep"
SMALL = "cfg1_64x64_constant"


def scaled(w: Workload, rows=None, cols=None, batch=None, steps=None, name=None) -> Workload:
    """Same device and input law on another shape (parity cases, CPU timing samples)."""
    from dataclasses import replace
    return replace(w, rows=rows or w.rows, cols=cols or w.cols, batch=batch or w.batch,
                   steps=steps or w.steps, name=name or (w.name + "_scaled"))


def rng_for(w: Workload, stream: int = 0) -> np.random.Generator:
    return np.random.default_rng([w.seed, stream])


def initial_weights(w: Workload) -> np.ndarray:
    """float32 [R][C]; uniform in +-w_init*w_max (zeros when w_init == 0)."""
    if w.w_init == 0.0:
        return np.zeros((w.rows, w.cols), dtype=np.float32)
    g = rng_for(w, 1)
    wm = w.device["w_max"]
    return (g.uniform(-w.w_init, w.w_init, size=(w.rows, w.cols)) * wm).astype(np.float32)


def draw_x(w: Workload, g: np.random.Generator) -> np.ndarray:
    shape = (w.batch, w.cols)
    if w.x_dist == "normal":
        x = g.standard_normal(shape, dtype=np.float32)
    elif w.x_dist == "uniform":
        x = g.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    elif w.x_dist == "relu_normal":
        x = np.maximum(g.standard_normal(shape, dtype=np.float32), np.float32(0))
    else:
        raise ValueError(w.x_dist)
    return np.ascontiguousarray(x, dtype=np.float32)


def draw_d(w: Workload, g: np.random.Generator) -> np.ndarray:
    d = g.standard_normal((w.batch, w.rows), dtype=np.float32) * np.float32(w.d_std)
    return np.ascontiguousarray(d, dtype=np.float32)


def input_stream(w: Workload):
    """Yields (step, x[B][C], d[B][R]) with fresh inputs every step."""
    g = rng_for(w, 2)
    for t in range(w.steps):
        yield t, draw_x(w, g), draw_d(w, g)
