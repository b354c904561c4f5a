"""ctypes front-end of the CPU oracle (``pulsed_update_oracle.c``).

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product package never does.
Nothing here touches the HIP library.

Every function marshals numpy arrays into the C oracle and returns numpy
arrays; the arithmetic lives in the C file, which cites the passages of
arXiv 2104.02184 (Sec. 3, Eq. (2)) it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pulsed_update_oracle.c")
# AHT_ORACLE_LIB names an already built oracle library to load instead (the sanitizer and
# mutation checks of the test-suite build their own copies elsewhere and point here).
_LIB = os.environ.get("AHT_ORACLE_LIB") or os.path.join(_HERE, "liboracle.so")

CONSTANT_STEP, LINEAR_STEP, SOFT_BOUNDS = 0, 1, 2
TAG_X, TAG_D, TAG_C2C, TAG_D2D = 1, 2, 3, 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no FMA contraction, no fast-math)."""
    if os.environ.get("AHT_ORACLE_LIB"):
        return _LIB                    # a library built by the caller: never overwritten
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = ctypes.CDLL(_LIB)
        _declare(_lib)
    return _lib


_u32p = ctypes.POINTER(ctypes.c_uint32)
_u64p = ctypes.POINTER(ctypes.c_uint64)
_i64p = ctypes.POINTER(ctypes.c_int64)
_i8p = ctypes.POINTER(ctypes.c_int8)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_f, _i, _u32, _u64 = ctypes.c_float, ctypes.c_int, ctypes.c_uint32, ctypes.c_uint64


def _declare(L):
    L.orc_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
    L.orc_philox4x32_10.restype = None
    L.orc_gauss_block_f64.argtypes = [_u64, _u32, _u32, _u32, _u32, _f64p]
    L.orc_gauss_block_f64.restype = None
    L.orc_gauss.argtypes = [_u64, _u32, _u32, _u32, _u32]
    L.orc_gauss.restype = _f
    L.orc_device_planes.argtypes = [_i] + [_f] * 11 + [_u64, _i, _i] + [_f32p] * 6
    L.orc_device_planes.restype = None
    L.orc_line_scale.argtypes = [_f32p, _f32p, _i, _i, _i, _f, _f, _i, _i, _f64p, _f64p]
    L.orc_line_scale.restype = None
    L.orc_threshold.argtypes = [ctypes.c_double, _f]
    L.orc_threshold.restype = _u64
    L.orc_pulse_word.argtypes = [_u64, _u32, _u32, _u32, _u32, ctypes.c_double, _f, _i]
    L.orc_pulse_word.restype = _u64
    L.orc_pulse_words.argtypes = [_f32p, _f32p, _i, _i, _i, _f, _f, _i, _i, _u64, _u32, _u64p, _u64p]
    L.orc_pulse_words.restype = None
    L.orc_counts.argtypes = [_u64p, _u64p, _i, _i, _i, _i, _i8p]
    L.orc_counts.restype = None
    L.orc_device_step.argtypes = [_i, _f, _i, _f, _f, _f, _f, _f, _f, _f, _f]
    L.orc_device_step.restype = _f
    L.orc_apply_words.argtypes = ([_f32p] * 7 + [_i, _f, _u64p, _u64p, _i, _i, _i, _i, _u64, _u32,
                                                 _i64p, ctypes.c_int64])
    L.orc_apply_words.restype = ctypes.c_int64
    L.orc_pulsed_update.argtypes = ([_f32p] * 7 + [_i, _f, _f, _i, _i, _f32p, _f32p, _i, _i, _i, _f,
                                                   _u64, _u32, _i64p, ctypes.c_int64])
    L.orc_pulsed_update.restype = ctypes.c_int64
    L.orc_line_scale_ex.argtypes = [_f32p, _f32p, _i, _i, _i, _f, _f, _i, _i, _i, _f64p, _f64p,
                                    ctypes.POINTER(ctypes.c_int32)]
    L.orc_line_scale_ex.restype = None
    L.orc_pulse_word_deterministic.argtypes = [_u32, ctypes.c_double, _f, _i]
    L.orc_pulse_word_deterministic.restype = _u64
    L.orc_pulse_words_ex.argtypes = [_f32p, _f32p, _i, _i, _i, _f, _f, _i, _i, _i, _i, _u64, _u32, _u64p, _u64p]
    L.orc_pulse_words_ex.restype = None
    L.orc_pulsed_update_ex.argtypes = ([_f32p] * 7 + [_i, _f, _f, _i, _i, _i, _i, _f32p, _f32p, _i, _i, _i, _f,
                                                      _u64, _u32, _i64p, ctypes.c_int64])
    L.orc_pulsed_update_ex.restype = ctypes.c_int64
    L.orc_analog_mvm.argtypes = [_f32p, _i, _i, _i, _f32p, _i] + [_f] * 7 + [_i, _u64, _u32, _f32p, _f32p]
    L.orc_analog_mvm.restype = None
    L.orc_analog_mvm_cellwise.argtypes = L.orc_analog_mvm.argtypes
    L.orc_analog_mvm_cellwise.restype = None
    L.orc_conv_patches.argtypes = [_f32p] + [_i] * 8 + [_f32p]
    L.orc_conv_patches.restype = None
    L.orc_conv_rows.argtypes = [_f32p, _i, _i, _i, _i, _f32p]
    L.orc_conv_rows.restype = None
    L.orc_temporal_planes.argtypes = [_f] * 6 + [_u64, _i, _i] + [_f32p] * 3
    L.orc_temporal_planes.restype = None
    L.orc_decay_diffuse.argtypes = [_f32p] * 5 + [_u64, _u32, _i, _i]
    L.orc_decay_diffuse.restype = None
    L.orc_reset_columns.argtypes = [_f32p, _f32p, _f, _f32p, _f32p, _u64, _u32, _i, _i, _i, _i]
    L.orc_reset_columns.restype = None
    L.orc_num_threads.argtypes = []
    L.orc_num_threads.restype = _i
    L.orc_set_num_threads.argtypes = [_i]
    L.orc_set_num_threads.restype = None


def _p(a, typ):
    return a.ctypes.data_as(typ)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


@dataclass
class DeviceParams:
    """Scalar device description in normalised units (names after the paper's
    ``dw_min``, ``dw_min_dtod``, ``dw_min_std`` of its Tiki-Taka listing)."""
    kind: int = CONSTANT_STEP
    dw_min: float = 0.001
    dw_min_dtod: float = 0.0
    dw_min_std: float = 0.0      # pulse-to-pulse (cycle-to-cycle) relative std
    up_down: float = 0.0
    up_down_dtod: float = 0.0
    w_max: float = 1.0
    w_max_dtod: float = 0.0
    w_min: float = -1.0
    w_min_dtod: float = 0.0
    gamma_up: float = 0.0
    gamma_down: float = 0.0
    gamma_dtod: float = 0.0


PLANE_NAMES = ("dw_up", "dw_down", "b_max", "b_min", "slope_up", "slope_down")


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c, _u32p), _p(k, _u32p), _p(out, _u32p))
    return out


def gauss_block_f64(seed, index, t, blk, tag):
    z = np.zeros(4, dtype=np.float64)
    lib().orc_gauss_block_f64(seed, index, t, blk, tag, _p(z, _f64p))
    return z


def gauss(seed, index, t, q, tag):
    return float(lib().orc_gauss(seed, index, t, q, tag))


def device_planes(p: DeviceParams, seed: int, R: int, C: int):
    """dict name -> float32 [R][C] plane."""
    planes = {n: np.zeros((R, C), dtype=np.float32) for n in PLANE_NAMES}
    lib().orc_device_planes(p.kind, p.dw_min, p.dw_min_dtod, p.up_down, p.up_down_dtod, p.w_max,
                            p.w_max_dtod, p.w_min, p.w_min_dtod, p.gamma_up, p.gamma_down,
                            p.gamma_dtod, seed, R, C, *[_p(planes[n], _f32p) for n in PLANE_NAMES])
    return planes


def line_scale(x, d, lr, dw_min, BL, update_management):
    x, d = _f32(x), _f32(d)
    B, C = x.shape
    R = d.shape[1]
    a_x = np.zeros(B, dtype=np.float64)
    a_d = np.zeros(B, dtype=np.float64)
    lib().orc_line_scale(_p(x, _f32p), _p(d, _f32p), B, R, C, lr, dw_min, BL,
                         int(update_management), _p(a_x, _f64p), _p(a_d, _f64p))
    return a_x, a_d


STOCHASTIC, DETERMINISTIC = 0, 1


def line_scale_ex(x, d, lr, dw_min, BL, update_management, dynamic_bl):
    """(a_x, a_d, bl_b): per-sample probability factors and train lengths."""
    x, d = _f32(x), _f32(d)
    B, C = x.shape
    R = d.shape[1]
    a_x = np.zeros(B, dtype=np.float64)
    a_d = np.zeros(B, dtype=np.float64)
    bl = np.zeros(B, dtype=np.int32)
    lib().orc_line_scale_ex(_p(x, _f32p), _p(d, _f32p), B, R, C, lr, dw_min, BL, int(update_management),
                            int(dynamic_bl), _p(a_x, _f64p), _p(a_d, _f64p),
                            bl.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    return a_x, a_d, bl


def pulse_word_deterministic(tag, a, v, BL):
    return int(lib().orc_pulse_word_deterministic(tag, float(a), float(np.float32(v)), BL))


def threshold(a, v):
    return int(lib().orc_threshold(float(a), float(np.float32(v))))


def pulse_word(seed, t, tag, index, b, a, v, BL):
    return int(lib().orc_pulse_word(seed, t, tag, index, b, float(a), float(np.float32(v)), BL))


def pulse_words(x, d, lr, dw_min, BL, update_management, seed, t, train_kind=STOCHASTIC, dynamic_bl=False):
    """(xw[B][C], dw[B][R]) uint64 pulse words of the call at step t."""
    x, d = _f32(x), _f32(d)
    B, C = x.shape
    R = d.shape[1]
    assert d.shape[0] == B
    xw = np.zeros((B, C), dtype=np.uint64)
    dw = np.zeros((B, R), dtype=np.uint64)
    if train_kind == STOCHASTIC and not dynamic_bl:
        lib().orc_pulse_words(_p(x, _f32p), _p(d, _f32p), B, R, C, lr, dw_min, BL,
                              int(update_management), seed, t, _p(xw, _u64p), _p(dw, _u64p))
    else:
        lib().orc_pulse_words_ex(_p(x, _f32p), _p(d, _f32p), B, R, C, lr, dw_min, BL, int(update_management),
                                 int(train_kind), int(dynamic_bl), seed, t, _p(xw, _u64p), _p(dw, _u64p))
    return xw, dw


def counts(xw, dw, b, BL):
    """int8 [R][C]: +n (UP) / -n (DOWN) coincidences of sample b."""
    xw = np.ascontiguousarray(xw, dtype=np.uint64)
    dw = np.ascontiguousarray(dw, dtype=np.uint64)
    C, R = xw.shape[1], dw.shape[1]
    out = np.zeros((R, C), dtype=np.int8)
    lib().orc_counts(_p(xw, _u64p), _p(dw, _u64p), b, R, C, BL, _p(out, _i8p))
    return out


def device_step(kind, w, up, xi, c2c, s_up, s_dn, bmax, bmin, slope_up=0.0, slope_dn=0.0):
    return float(lib().orc_device_step(kind, w, int(up), xi, c2c, s_up, s_dn, bmax, bmin,
                                       slope_up, slope_dn))


def _plane_ptrs(planes):
    arrs = [_f32(planes[n]) for n in PLANE_NAMES]
    return arrs, [_p(a, _f32p) for a in arrs]


def _cells_arg(cells):
    if cells is None:
        return None, None, 0
    c = np.ascontiguousarray(cells, dtype=np.int64)
    return c, _p(c, _i64p), c.size


def apply_words(W, planes, kind, c2c, xw, dw, BL, seed, t, cells=None):
    """Apply given pulse words in place to W (float32 [R][C]); returns pulses applied."""
    assert W.dtype == np.float32 and W.flags.c_contiguous
    R, C = W.shape
    xw = np.ascontiguousarray(xw, dtype=np.uint64)
    dw = np.ascontiguousarray(dw, dtype=np.uint64)
    B = xw.shape[0]
    assert xw.shape == (B, C) and dw.shape == (B, R)
    keep, ptrs = _plane_ptrs(planes)
    ckeep, cptr, nc = _cells_arg(cells)
    return int(lib().orc_apply_words(_p(W, _f32p), *ptrs, kind, c2c, _p(xw, _u64p), _p(dw, _u64p),
                                     B, R, C, BL, seed, t, cptr, nc))


def pulsed_update(W, planes, p: DeviceParams, BL, update_management, x, d, lr, seed, t,
                  cells=None, train_kind=STOCHASTIC, dynamic_bl=False):
    """One whole update call at step t, in place on W; returns pulses applied.
    With ``cells`` (flat indices) only those cells are updated."""
    assert W.dtype == np.float32 and W.flags.c_contiguous
    R, C = W.shape
    x, d = _f32(x), _f32(d)
    B = x.shape[0]
    assert x.shape == (B, C) and d.shape == (B, R)
    keep, ptrs = _plane_ptrs(planes)
    ckeep, cptr, nc = _cells_arg(cells)
    if train_kind == STOCHASTIC and not dynamic_bl:
        return int(lib().orc_pulsed_update(_p(W, _f32p), *ptrs, p.kind, p.dw_min_std, p.dw_min, BL,
                                           int(update_management), _p(x, _f32p), _p(d, _f32p), B, R, C,
                                           lr, seed, t, cptr, nc))
    return int(lib().orc_pulsed_update_ex(_p(W, _f32p), *ptrs, p.kind, p.dw_min_std, p.dw_min, BL,
                                          int(update_management), int(train_kind), int(dynamic_bl),
                                          _p(x, _f32p), _p(d, _f32p), B, R, C, lr, seed, t, cptr, nc))


@dataclass
class IOParams:
    """Non-idealities of the analog matrix-vector product (Eq. (1) of the paper)."""
    inp_res: float = 1.0 / 126.0      # DAC step of the scaled input (0: no quantisation)
    inp_bound: float = 1.0
    inp_noise: float = 0.0
    w_noise: float = 0.0
    out_noise: float = 0.06
    out_res: float = 12.0 / 254.0     # ADC step (0: no quantisation)
    out_bound: float = 12.0
    noise_management: bool = True


def analog_mvm(W, x, io: IOParams, seed, t, transposed=False, return_pre=False, cellwise_weight_noise=False):
    """y[B][R] = analog product of x[B][C] with W[R][C] (transposed: x[B][R] -> y[B][C]).
    ``cellwise_weight_noise``: a fresh Gaussian for every cell and vector, Eq. (1) as printed,
    instead of the output-referred draw (same law)."""
    W = _f32(W)
    x = _f32(x)
    R, C = W.shape
    B = x.shape[0]
    N = C if transposed else R
    assert x.shape[1] == (R if transposed else C)
    y = np.zeros((B, N), dtype=np.float32)
    pre = np.zeros((B, N), dtype=np.float32)
    fn = lib().orc_analog_mvm_cellwise if cellwise_weight_noise else lib().orc_analog_mvm
    fn(_p(W, _f32p), R, C, int(transposed), _p(x, _f32p), B, io.inp_res, io.inp_bound,
                         io.inp_noise, io.w_noise, io.out_noise, io.out_res, io.out_bound,
                         int(io.noise_management), seed, t, _p(y, _f32p), _p(pre, _f32p))
    return (y, pre) if return_pre else y


def conv_update_vectors(img, dgrad, kh, kw, stride=1, pad=0):
    """(x[B][Cin*kh*kw], d[B][Cout]) of a convolution layer's update: one update vector per image
    and output position.  img [N][Cin][H][W], dgrad [N][Cout][OH][OW]."""
    img, dgrad = _f32(img), _f32(dgrad)
    N, Cin, H, Wd = img.shape
    OH, OW = (H + 2 * pad - kh) // stride + 1, (Wd + 2 * pad - kw) // stride + 1
    assert dgrad.shape[0] == N and dgrad.shape[2:] == (OH, OW)
    Cout = dgrad.shape[1]
    x = np.zeros((N * OH * OW, Cin * kh * kw), dtype=np.float32)
    d = np.zeros((N * OH * OW, Cout), dtype=np.float32)
    lib().orc_conv_patches(_p(img, _f32p), N, Cin, H, Wd, kh, kw, stride, pad, _p(x, _f32p))
    lib().orc_conv_rows(_p(dgrad, _f32p), N, Cout, OH, OW, _p(d, _f32p))
    return x, d


@dataclass
class TemporalParams:
    """Once-per-mini-batch processes: decay toward 0, diffusion, reset (normalised units)."""
    decay_rate: float = 0.0
    decay_rate_dtod: float = 0.0
    diffusion: float = 0.0
    diffusion_dtod: float = 0.0
    reset: float = 0.0
    reset_dtod: float = 0.0
    reset_std: float = 0.0


TEMPORAL_PLANE_NAMES = ("decay", "diffusion", "reset")


def temporal_planes(tp: TemporalParams, seed: int, R: int, C: int):
    planes = {n: np.zeros((R, C), dtype=np.float32) for n in TEMPORAL_PLANE_NAMES}
    lib().orc_temporal_planes(tp.decay_rate, tp.decay_rate_dtod, tp.diffusion, tp.diffusion_dtod, tp.reset,
                              tp.reset_dtod, seed, R, C, *[_p(planes[n], _f32p) for n in TEMPORAL_PLANE_NAMES])
    return planes


def decay_diffuse(W, tplanes, planes, seed, tau):
    """One application (temporal step tau) in place on W."""
    assert W.dtype == np.float32 and W.flags.c_contiguous
    R, C = W.shape
    arrs = [_f32(tplanes["decay"]), _f32(tplanes["diffusion"]), _f32(planes["b_max"]), _f32(planes["b_min"])]
    lib().orc_decay_diffuse(_p(W, _f32p), *[_p(a, _f32p) for a in arrs], seed, tau, R, C)


def reset_columns(W, tplanes, reset_std, planes, seed, tau, c0, ncols):
    assert W.dtype == np.float32 and W.flags.c_contiguous
    R, C = W.shape
    arrs = [_f32(tplanes["reset"]), _f32(planes["b_max"]), _f32(planes["b_min"])]
    lib().orc_reset_columns(_p(W, _f32p), _p(arrs[0], _f32p), reset_std, _p(arrs[1], _f32p), _p(arrs[2], _f32p),
                            seed, tau, R, C, c0, ncols)


def num_threads():
    return int(lib().orc_num_threads())


def set_num_threads(n):
    lib().orc_set_num_threads(int(n))


# ---------------------------------------------------------------------------------------------
# Unit cells of several devices (Sec. 4 of the paper: a cross-point may hold several conductive
# elements with their own material properties, updated one by one or all together).  Reading:
# the devices of a cell share the row and column lines, so one set of pulse trains (drawn with
# device 0's seed at the cell's step) reaches every updated device, which steps through its own
# response model and pulse-to-pulse noise stream; the cell's weight is sum_k gamma_k w^(k).
# ---------------------------------------------------------------------------------------------
def unit_cell_update(Ws, planes, params, seeds, BL, update_management, x, d, lr, t, which=-1):
    """In place on the list of device weights ``Ws``; returns the pulses applied per device."""
    xw, dw = pulse_words(x, d, lr, params[0].dw_min, BL, update_management, seeds[0], t)
    counts = []
    for k, W in enumerate(Ws):
        if which >= 0 and k != which:
            counts.append(0)
            continue
        counts.append(apply_words(W, planes[k], params[k].kind, params[k].dw_min_std, xw, dw, BL, seeds[k], t))
    return counts


def unit_cell_weights(Ws, gamma):
    """float32 [R][C]: sum_k gamma_k W_k, added in device order, every operation rounded to fp32."""
    acc = np.zeros_like(Ws[0], dtype=np.float32)
    for g, W in zip(gamma, Ws):
        acc = (acc + np.float32(g) * W.astype(np.float32)).astype(np.float32)
    return acc
