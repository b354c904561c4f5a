"""ctypes binding of the C ABI declared in ``include/aht.h``.

Argument marshalling only: every function here forwards device pointers of
torch tensors and the current HIP stream to the library.  Function and
structure names follow the header.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, fields

HERE = os.path.dirname(os.path.abspath(__file__))
# AHT_LIB names a library built elsewhere to load instead (the host-sanitizer check of the test-suite)
_LIB_PATH = os.environ.get("AHT_LIB") or os.path.join(HERE, "libaht.so")

CONSTANT_STEP, LINEAR_STEP, SOFT_BOUNDS = 0, 1, 2
PLANE_NAMES = ("dw_up", "dw_down", "b_max", "b_min", "slope_up", "slope_down")
TEMPORAL_PLANE_NAMES = ("decay", "diffusion", "reset")

# every symbol include/aht.h declares
EXPORTS = (
    "aht_tile_create", "aht_tile_destroy", "aht_set_weights", "aht_get_weights", "aht_pulsed_update",
    "aht_pulsed_update_noalloc", "aht_get_launch_info", "aht_sync_step", "aht_pulsed_update_many",
    "aht_get_step", "aht_set_step", "aht_get_pulse_count", "aht_get_device_planes",
    "aht_set_device_planes", "aht_debug_pulse_words", "aht_debug_counts", "aht_debug_apply_words",
    "aht_debug_philox", "aht_debug_gauss", "aht_profile_enable", "aht_profile_read",
    "aht_pulsed_update_conv2d", "aht_debug_pulse_words_conv2d", "aht_forward", "aht_backward",
    "aht_transfer_column", "aht_get_mvm_steps", "aht_set_mvm_steps",
    "aht_unit_cell_update", "aht_unit_cell_weights", "aht_unit_cell_forward", "aht_unit_cell_backward",
    "aht_set_pulse_mode", "aht_set_temporal", "aht_decay_diffuse", "aht_reset_columns", "aht_get_temporal_plane",
    "aht_get_temporal_step", "aht_set_temporal_step",
    "aht_status_string", "aht_last_error", "aht_version",
)


class AhtError(RuntimeError):
    def __init__(self, status, name, message):
        super().__init__(f"{name} ({status}): {message}")
        self.status = status
        self.status_name = name


class aht_device_params(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("dw_min", ctypes.c_float), ("dw_min_dtod", ctypes.c_float),
                ("dw_min_std", ctypes.c_float), ("up_down", ctypes.c_float), ("up_down_dtod", ctypes.c_float),
                ("w_max", ctypes.c_float), ("w_max_dtod", ctypes.c_float), ("w_min", ctypes.c_float),
                ("w_min_dtod", ctypes.c_float), ("gamma_up", ctypes.c_float), ("gamma_down", ctypes.c_float),
                ("gamma_dtod", ctypes.c_float)]


class aht_io_params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_float) for n in ("inp_res", "inp_bound", "inp_noise", "w_noise", "out_noise",
                                               "out_res", "out_bound")] + [("noise_management", ctypes.c_int32)]


@dataclass
class IOParams:
    inp_res: float = 1.0 / 126.0
    inp_bound: float = 1.0
    inp_noise: float = 0.0
    w_noise: float = 0.0
    out_noise: float = 0.06
    out_res: float = 12.0 / 254.0
    out_bound: float = 12.0
    noise_management: bool = True

    def to_c(self) -> "aht_io_params":
        return aht_io_params(self.inp_res, self.inp_bound, self.inp_noise, self.w_noise, self.out_noise,
                             self.out_res, self.out_bound, int(bool(self.noise_management)))


class aht_temporal_params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_float) for n in ("decay_rate", "decay_rate_dtod", "diffusion", "diffusion_dtod",
                                               "reset", "reset_dtod", "reset_std")]


class aht_launch_info(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("rows_per_lane", "side_rows_per_lane", "row_lists", "stream_words",
                                               "mvm_path", "mvm_splits")] + [("pulse_rate", ctypes.c_double),
                                                                             ("row_fill", ctypes.c_double)]


class aht_update_params(ctypes.Structure):
    _fields_ = [("bl", ctypes.c_int32), ("update_management", ctypes.c_int32)]


@dataclass
class DeviceParams:
    kind: int = CONSTANT_STEP
    dw_min: float = 0.001
    dw_min_dtod: float = 0.0
    dw_min_std: float = 0.0
    up_down: float = 0.0
    up_down_dtod: float = 0.0
    w_max: float = 1.0
    w_max_dtod: float = 0.0
    w_min: float = -1.0
    w_min_dtod: float = 0.0
    gamma_up: float = 0.0
    gamma_down: float = 0.0
    gamma_dtod: float = 0.0

    def to_c(self) -> aht_device_params:
        return aht_device_params(**{f.name: getattr(self, f.name) for f in fields(self)})


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libaht.so; raises if it is missing (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime under the same SONAME; load it first so that the tensors
    # torch allocates and the kernels this library launches share one runtime.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2104_02184_amd.build` "
                          "(hipcc, gfx950); there is no CPU fallback")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, u32, u64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float
    L.aht_tile_create.argtypes = [ctypes.POINTER(vp), i32, i32, ctypes.POINTER(aht_device_params),
                                  ctypes.POINTER(aht_update_params), u64]
    L.aht_tile_destroy.argtypes = [vp]
    L.aht_set_weights.argtypes = [vp, vp, vp]
    L.aht_get_weights.argtypes = [vp, vp, vp]
    L.aht_pulsed_update.argtypes = [vp, vp, vp, i32, f32, vp]
    L.aht_pulsed_update_noalloc.argtypes = [vp, vp, vp, i32, f32, vp]
    L.aht_pulsed_update_many.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp),
                                         ctypes.POINTER(i32), ctypes.POINTER(f32), i32, vp]
    L.aht_get_launch_info.argtypes = [vp, ctypes.POINTER(aht_launch_info)]
    L.aht_get_step.argtypes = [vp, ctypes.POINTER(u32)]
    L.aht_set_step.argtypes = [vp, u32]
    L.aht_sync_step.argtypes = [vp, ctypes.POINTER(u32), vp]
    L.aht_get_pulse_count.argtypes = [vp, ctypes.POINTER(u64), vp]
    L.aht_get_device_planes.argtypes = [vp, i32, vp, vp]
    L.aht_set_device_planes.argtypes = [vp, i32, vp, vp]
    L.aht_debug_pulse_words.argtypes = [vp, vp, vp, i32, f32, vp, vp, vp]
    L.aht_debug_counts.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    L.aht_debug_apply_words.argtypes = [vp, vp, vp, i32, u32, vp]
    L.aht_debug_philox.argtypes = [vp, vp, i32, vp, vp]
    L.aht_debug_gauss.argtypes = [u64, u32, u32, u32, u32, i32, i32, vp, vp]
    L.aht_pulsed_update_conv2d.argtypes = [vp, vp, vp] + [i32] * 8 + [f32, vp]
    L.aht_debug_pulse_words_conv2d.argtypes = [vp, vp, vp] + [i32] * 8 + [f32, vp, vp, vp]
    L.aht_forward.argtypes = [vp, ctypes.POINTER(aht_io_params), vp, vp, vp, i32, vp]
    L.aht_backward.argtypes = [vp, ctypes.POINTER(aht_io_params), vp, vp, vp, i32, vp]
    L.aht_transfer_column.argtypes = [vp, vp, i32, f32, ctypes.POINTER(aht_io_params), vp]
    L.aht_unit_cell_update.argtypes = [ctypes.POINTER(vp), i32, i32, vp, vp, i32, f32, vp]
    L.aht_unit_cell_weights.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(f32), i32, vp, vp]
    L.aht_unit_cell_forward.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(f32), i32, ctypes.POINTER(aht_io_params),
                                        vp, vp, vp, i32, vp]
    L.aht_unit_cell_backward.argtypes = L.aht_unit_cell_forward.argtypes
    L.aht_get_mvm_steps.argtypes = [vp, ctypes.POINTER(u32), ctypes.POINTER(u32)]
    L.aht_set_mvm_steps.argtypes = [vp, u32, u32]
    L.aht_set_pulse_mode.argtypes = [vp, i32, i32]
    L.aht_set_temporal.argtypes = [vp, ctypes.POINTER(aht_temporal_params)]
    L.aht_decay_diffuse.argtypes = [vp, vp]
    L.aht_reset_columns.argtypes = [vp, i32, i32, vp]
    L.aht_get_temporal_plane.argtypes = [vp, i32, vp, vp]
    L.aht_get_temporal_step.argtypes = [vp, ctypes.POINTER(u32)]
    L.aht_set_temporal_step.argtypes = [vp, u32]
    L.aht_profile_enable.argtypes = [vp, i32]
    L.aht_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                   ctypes.POINTER(i32)]
    for name in EXPORTS:
        getattr(L, name).restype = ctypes.c_int
    L.aht_status_string.argtypes = [ctypes.c_int]
    L.aht_status_string.restype = ctypes.c_char_p
    L.aht_last_error.argtypes = []
    L.aht_last_error.restype = ctypes.c_char_p
    L.aht_version.argtypes = []
    L.aht_version.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(status: int):
    if status != 0:
        L = load_library()
        raise AhtError(status, L.aht_status_string(status).decode(), L.aht_last_error().decode())


def _stream():
    import torch
    # (the raw handle of the current stream without building a Stream object: this runs once per call)
    return ctypes.c_void_p(torch._C._cuda_getCurrentRawStream(torch.cuda.current_device()))


def _ptr(t, dtype, shape=None):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("expected a CUDA/HIP tensor")
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"expected a contiguous {dtype} tensor, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


class Tile:
    """One analog tile on the current HIP device (wraps ``aht_tile``)."""

    def __init__(self, rows: int, cols: int, device: DeviceParams, bl: int, update_management: bool = False,
                 seed: int = 0):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        self.rows, self.cols, self.bl = int(rows), int(cols), int(bl)
        self.device_params = device
        dp = device.to_c()
        up = aht_update_params(int(bl), int(bool(update_management)))
        _check(self._lib.aht_tile_create(ctypes.byref(self._h), rows, cols, ctypes.byref(dp), ctypes.byref(up),
                                         ctypes.c_uint64(seed & (2**64 - 1))))

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            _check(self._lib.aht_tile_destroy(self._h))
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # -- weights ---------------------------------------------------------------------------
    def set_weights(self, w):
        import torch
        _check(self._lib.aht_set_weights(self._h, _ptr(w, torch.float32, (self.rows, self.cols)), _stream()))

    def get_weights(self, out=None):
        import torch
        if out is None:
            out = torch.empty((self.rows, self.cols), dtype=torch.float32, device="cuda")
        _check(self._lib.aht_get_weights(self._h, _ptr(out, torch.float32, (self.rows, self.cols)), _stream()))
        return out

    # -- the update ------------------------------------------------------------------------
    def pulsed_update(self, x, d, lr: float):
        import torch
        B = int(x.shape[0]) if x.dim() == 2 else -1
        if B > 0:
            xp, dp = _ptr(x, torch.float32, (B, self.cols)), _ptr(d, torch.float32, (B, self.rows))
        else:
            xp = dp = ctypes.c_void_p()
        _check(self._lib.aht_pulsed_update(self._h, xp, dp, B, ctypes.c_float(lr), _stream()))

    def pulsed_update_noalloc(self, x, d, lr: float):
        """aht_pulsed_update_noalloc: the same update out of the library's static device scratch."""
        import torch
        B = int(x.shape[0]) if x.dim() == 2 else -1
        if B > 0:
            xp, dp = _ptr(x, torch.float32, (B, self.cols)), _ptr(d, torch.float32, (B, self.rows))
        else:
            xp = dp = ctypes.c_void_p()
        _check(self._lib.aht_pulsed_update_noalloc(self._h, xp, dp, B, ctypes.c_float(lr), _stream()))

    def launch_info(self) -> dict:
        """what the library chose for the most recent full update and analog product"""
        info = aht_launch_info()
        _check(self._lib.aht_get_launch_info(self._h, ctypes.byref(info)))
        return {n: getattr(info, n) for n, _ in aht_launch_info._fields_}

    # -- analog matrix-vector product ------------------------------------------------------
    def _mvm(self, fn, io, x, n_in, n_out, with_pre):
        import torch
        B = int(x.shape[0])
        y = torch.empty((B, n_out), dtype=torch.float32, device="cuda")
        pre = torch.empty((B, n_out), dtype=torch.float32, device="cuda") if with_pre else None
        c = io.to_c()
        _check(fn(self._h, ctypes.byref(c), _ptr(x, torch.float32, (B, n_in)), _ptr(y, torch.float32),
                  _ptr(pre, torch.float32) if with_pre else ctypes.c_void_p(), B, _stream()))
        return (y, pre) if with_pre else y

    def forward(self, x, io: "IOParams", with_pre: bool = False):
        return self._mvm(self._lib.aht_forward, io, x, self.cols, self.rows, with_pre)

    def backward(self, d, io: "IOParams", with_pre: bool = False):
        return self._mvm(self._lib.aht_backward, io, d, self.rows, self.cols, with_pre)

    def transfer_column_to(self, dst: "Tile", col: int, lr: float, io: "IOParams"):
        """One Tiki-Taka transfer event: read column `col` of this tile, pulse it onto `dst`."""
        c = io.to_c()
        _check(self._lib.aht_transfer_column(self._h, dst._h, col, ctypes.c_float(lr), ctypes.byref(c), _stream()))

    @property
    def mvm_steps(self):
        f, b = ctypes.c_uint32(), ctypes.c_uint32()
        _check(self._lib.aht_get_mvm_steps(self._h, ctypes.byref(f), ctypes.byref(b)))
        return f.value, b.value

    @mvm_steps.setter
    def mvm_steps(self, fb):
        _check(self._lib.aht_set_mvm_steps(self._h, ctypes.c_uint32(fb[0]), ctypes.c_uint32(fb[1])))

    def set_pulse_mode(self, deterministic: bool = False, dynamic_bl: bool = False):
        _check(self._lib.aht_set_pulse_mode(self._h, int(bool(deterministic)), int(bool(dynamic_bl))))

    def _conv_geometry(self, img, grad, kh, kw, stride, pad):
        import torch
        N, Cin, H, W = (int(v) for v in img.shape)
        OH, OW = (H + 2 * pad - kh) // stride + 1, (W + 2 * pad - kw) // stride + 1
        ip = _ptr(img, torch.float32, (N, Cin, H, W))
        gp = _ptr(grad, torch.float32, (N, self.rows, OH, OW))
        return ip, gp, N, Cin, H, W, OH, OW

    def pulsed_update_conv2d(self, img, grad, kh: int, kw: int, stride: int, pad: int, lr: float):
        """img [N][Cin][H][W], grad [N][rows][OH][OW]; one update vector per output position."""
        ip, gp, N, Cin, H, W, _, _ = self._conv_geometry(img, grad, kh, kw, stride, pad)
        _check(self._lib.aht_pulsed_update_conv2d(self._h, ip, gp, N, Cin, H, W, kh, kw, stride, pad,
                                                  ctypes.c_float(lr), _stream()))

    def debug_pulse_words_conv2d(self, img, grad, kh: int, kw: int, stride: int, pad: int, lr: float):
        import torch
        ip, gp, N, Cin, H, W, OH, OW = self._conv_geometry(img, grad, kh, kw, stride, pad)
        B = N * OH * OW
        xw = torch.empty((B, self.cols), dtype=torch.int64, device="cuda")
        dw = torch.empty((B, self.rows), dtype=torch.int64, device="cuda")
        _check(self._lib.aht_debug_pulse_words_conv2d(self._h, ip, gp, N, Cin, H, W, kh, kw, stride, pad,
                                                      ctypes.c_float(lr), _ptr(xw, torch.int64), _ptr(dw, torch.int64),
                                                      _stream()))
        return xw, dw

    # -- state -----------------------------------------------------------------------------
    @property
    def step(self) -> int:
        v = ctypes.c_uint32()
        _check(self._lib.aht_get_step(self._h, ctypes.byref(v)))
        return v.value

    @step.setter
    def step(self, value: int):
        _check(self._lib.aht_set_step(self._h, ctypes.c_uint32(value)))

    def sync_step(self) -> int:
        """reads the device's step counter back into the host's copy (after replaying a recorded graph)"""
        v = ctypes.c_uint32()
        _check(self._lib.aht_sync_step(self._h, ctypes.byref(v), _stream()))
        return v.value

    def pulse_count(self) -> int:
        v = ctypes.c_uint64()
        _check(self._lib.aht_get_pulse_count(self._h, ctypes.byref(v), _stream()))
        return v.value

    def get_plane(self, name):
        import torch
        idx = PLANE_NAMES.index(name) if isinstance(name, str) else int(name)
        out = torch.empty((self.rows, self.cols), dtype=torch.float32, device="cuda")
        _check(self._lib.aht_get_device_planes(self._h, idx, _ptr(out, torch.float32), _stream()))
        return out

    def set_plane(self, name, values):
        import torch
        idx = PLANE_NAMES.index(name) if isinstance(name, str) else int(name)
        _check(self._lib.aht_set_device_planes(self._h, idx, _ptr(values, torch.float32, (self.rows, self.cols)),
                                               _stream()))

    # -- temporal processes ----------------------------------------------------------------
    def set_temporal(self, decay_rate=0.0, decay_rate_dtod=0.0, diffusion=0.0, diffusion_dtod=0.0, reset=0.0,
                     reset_dtod=0.0, reset_std=0.0):
        p = aht_temporal_params(decay_rate, decay_rate_dtod, diffusion, diffusion_dtod, reset, reset_dtod, reset_std)
        _check(self._lib.aht_set_temporal(self._h, ctypes.byref(p)))

    def decay_diffuse(self):
        _check(self._lib.aht_decay_diffuse(self._h, _stream()))

    def reset_columns(self, c0: int, ncols: int):
        _check(self._lib.aht_reset_columns(self._h, c0, ncols, _stream()))

    def get_temporal_plane(self, name):
        import torch
        idx = TEMPORAL_PLANE_NAMES.index(name) if isinstance(name, str) else int(name)
        out = torch.empty((self.rows, self.cols), dtype=torch.float32, device="cuda")
        _check(self._lib.aht_get_temporal_plane(self._h, idx, _ptr(out, torch.float32), _stream()))
        return out

    @property
    def temporal_step(self) -> int:
        v = ctypes.c_uint32()
        _check(self._lib.aht_get_temporal_step(self._h, ctypes.byref(v)))
        return v.value

    @temporal_step.setter
    def temporal_step(self, value: int):
        _check(self._lib.aht_set_temporal_step(self._h, ctypes.c_uint32(value)))

    # -- measurement hook ------------------------------------------------------------------
    def profile_enable(self, enable: bool = True):
        _check(self._lib.aht_profile_enable(self._h, int(bool(enable))))

    def profile_read(self):
        """(ms in line scaling + pulse words, ms in the cell update, calls covered)"""
        a, b, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_int32()
        _check(self._lib.aht_profile_read(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(n)))
        return a.value, b.value, n.value

    # -- test hooks ------------------------------------------------------------------------
    def debug_pulse_words(self, x, d, lr: float):
        """(xw[B][cols], dw[B][rows]) as int64 tensors holding the uint64 bit patterns."""
        import torch
        B = int(x.shape[0])
        xw = torch.empty((B, self.cols), dtype=torch.int64, device="cuda")
        dw = torch.empty((B, self.rows), dtype=torch.int64, device="cuda")
        _check(self._lib.aht_debug_pulse_words(self._h, _ptr(x, torch.float32, (B, self.cols)),
                                               _ptr(d, torch.float32, (B, self.rows)), B, ctypes.c_float(lr),
                                               _ptr(xw, torch.int64), _ptr(dw, torch.int64), _stream()))
        return xw, dw

    def debug_counts(self, xw, dw, b: int):
        import torch
        B = int(xw.shape[0])
        out = torch.empty((self.rows, self.cols), dtype=torch.int8, device="cuda")
        _check(self._lib.aht_debug_counts(self._h, _ptr(xw, torch.int64, (B, self.cols)),
                                          _ptr(dw, torch.int64, (B, self.rows)), B, b, _ptr(out, torch.int8),
                                          _stream()))
        return out

    def debug_apply_words(self, xw, dw, step: int):
        import torch
        B = int(xw.shape[0])
        _check(self._lib.aht_debug_apply_words(self._h, _ptr(xw, torch.int64, (B, self.cols)),
                                               _ptr(dw, torch.int64, (B, self.rows)), B, ctypes.c_uint32(step),
                                               _stream()))


def pulsed_update_many(tiles, xs, ds, lrs) -> None:
    """aht_pulsed_update_many: tile i gets pulsed_update(xs[i], ds[i], lrs[i]); small tiles run side by side."""
    import torch
    n = len(tiles)
    if not (len(xs) == len(ds) == len(lrs) == n):
        raise ValueError("tiles, xs, ds and lrs must have the same length")
    if n == 0:
        return
    vp = ctypes.c_void_p
    h, xp, dp = (vp * n)(), (vp * n)(), (vp * n)()
    Bs, lr = (ctypes.c_int32 * n)(), (ctypes.c_float * n)()
    for i, (t, x, d) in enumerate(zip(tiles, xs, ds)):
        B = int(x.shape[0]) if x.dim() == 2 else -1
        h[i] = t._h
        if B > 0:
            xp[i], dp[i] = _ptr(x, torch.float32, (B, t.cols)), _ptr(d, torch.float32, (B, t.rows))
        Bs[i], lr[i] = B, float(lrs[i])
    _check(tiles[0]._lib.aht_pulsed_update_many(h, xp, dp, Bs, lr, n, _stream()))


class UnitCell:
    """Several tiles used as the devices of one unit cell (wraps the ``aht_unit_cell_*`` calls);
    ``gamma[k]`` weighs device k in the cell's effective weight."""

    def __init__(self, devices, gamma=None):
        self.devices = list(devices)
        self.gamma = [1.0] * len(self.devices) if gamma is None else [float(g) for g in gamma]
        assert len(self.gamma) == len(self.devices)
        self._lib = load_library()

    def _handles(self):
        return (ctypes.c_void_p * len(self.devices))(*[t._h for t in self.devices])

    def _gamma(self):
        return (ctypes.c_float * len(self.gamma))(*self.gamma)

    def pulsed_update(self, x, d, lr: float, which: int = -1):
        """One set of pulse trains for the cell; applied to all devices (which = -1) or to one."""
        import torch
        lead = self.devices[0]
        B = int(x.shape[0])
        _check(self._lib.aht_unit_cell_update(self._handles(), len(self.devices), which,
                                              _ptr(x, torch.float32, (B, lead.cols)),
                                              _ptr(d, torch.float32, (B, lead.rows)), B, ctypes.c_float(lr), _stream()))

    def weights(self):
        import torch
        lead = self.devices[0]
        out = torch.empty((lead.rows, lead.cols), dtype=torch.float32, device="cuda")
        _check(self._lib.aht_unit_cell_weights(self._handles(), self._gamma(), len(self.devices),
                                               _ptr(out, torch.float32), _stream()))
        return out

    def _mvm(self, fn, io, x, n_in, n_out):
        import torch
        B = int(x.shape[0])
        y = torch.empty((B, n_out), dtype=torch.float32, device="cuda")
        c = io.to_c()
        _check(fn(self._handles(), self._gamma(), len(self.devices), ctypes.byref(c), _ptr(x, torch.float32, (B, n_in)),
                  _ptr(y, torch.float32), ctypes.c_void_p(), B, _stream()))
        return y

    def forward(self, x, io: "IOParams"):
        lead = self.devices[0]
        return self._mvm(self._lib.aht_unit_cell_forward, io, x, lead.cols, lead.rows)

    def backward(self, d, io: "IOParams"):
        lead = self.devices[0]
        return self._mvm(self._lib.aht_unit_cell_backward, io, d, lead.rows, lead.cols)


def debug_philox(ctr, key):
    """ctr int32[n][4], key int32[n][2] device tensors (bit patterns) -> int32[n][4]."""
    import torch
    n = int(ctr.shape[0])
    out = torch.empty((n, 4), dtype=torch.int32, device="cuda")
    _check(load_library().aht_debug_philox(_ptr(ctr, torch.int32, (n, 4)), _ptr(key, torch.int32, (n, 2)), n,
                                           _ptr(out, torch.int32), _stream()))
    return out


def debug_gauss(seed: int, index: int, t: int, tag: int, q0: int, n: int, fast: bool):
    import torch
    out = torch.empty((n,), dtype=torch.float32, device="cuda")
    _check(load_library().aht_debug_gauss(ctypes.c_uint64(seed), index, t, tag, q0, n, int(fast),
                                          _ptr(out, torch.float32), _stream()))
    return out
