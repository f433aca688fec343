"""ctypes binding of libabs.so: same names as the C entry points, marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
# PyTorch supplies device memory and streams.  It must be imported before libabs.so is
# loaded: it brings its own copy of the HIP runtime (libamdhip64.so.7), and a process can
# hold only one; loading torch first makes libabs resolve its HIP calls against that copy.
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libabs.so")

ABS_TRACE_HEADER = 12
ABS_MAX_WORKERS = 128


class AbsError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libabs error {code}: {text}")
        self.code = code


class AbsConfig(C.Structure):
    """Mirror of `abs_config` in include/abs.h."""
    _fields_ = [
        ("model", C.c_int32), ("n_layers", C.c_int32), ("dims", C.c_int32 * 8),
        ("x_dtype", C.c_int32), ("N", C.c_int32), ("M", C.c_int64), ("B", C.c_int32),
        ("K0", C.c_int32), ("k_mode", C.c_int32), ("tau_mode", C.c_int32),
        ("tau_cap", C.c_int32), ("a", C.c_int32), ("lr", C.c_float), ("sa_penalty", C.c_int32),
        ("time_dist", C.c_int32), ("n_slow", C.c_int32), ("time_param", C.c_double),
        ("slow_factor", C.c_double), ("seed", C.c_uint64),
        ("k_replay", C.POINTER(C.c_int32)), ("k_replay_len", C.c_int64),
        ("device_mode", C.c_int32), ("profile", C.c_int32), ("U", C.c_int32), ("reserved", C.c_int32),
    ]


class AbsKernelStat(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int64), ("total_ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double), ("timed_launches", C.c_int64),
                ("timed_flops", C.c_double), ("timed_bytes", C.c_double)]


def library_path() -> str:
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'); "
            "there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    cfgp = C.POINTER(AbsConfig)
    lib.abs_config_bytes.restype = i32
    lib.abs_config_bytes.argtypes = []
    lib.abs_workspace_size.restype = sz
    lib.abs_workspace_size.argtypes = [cfgp]
    lib.abs_create.restype = C.c_int
    lib.abs_create.argtypes = [cfgp, vp, vp, vp, vp, sz, vp, C.POINTER(vp)]
    lib.abs_round.restype = C.c_int
    lib.abs_round.argtypes = [vp, i32]
    lib.abs_evaluate.restype = C.c_int
    lib.abs_evaluate.argtypes = [vp, i64, vp, vp, i64, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.abs_evaluate_static.restype = C.c_int
    lib.abs_evaluate_static.argtypes = [vp, i64, vp, vp, i64, vp]
    lib.abs_batch_workspace_size.restype = sz
    lib.abs_batch_workspace_size.argtypes = [C.POINTER(vp), i32]
    lib.abs_batch_create.restype = C.c_int
    lib.abs_batch_create.argtypes = [C.POINTER(vp), i32, vp, sz, C.POINTER(vp)]
    lib.abs_batch_round.restype = C.c_int
    lib.abs_batch_round.argtypes = [vp, i32]
    lib.abs_batch_last_error.restype = C.c_char_p
    lib.abs_batch_last_error.argtypes = [vp]
    lib.abs_batch_destroy.restype = None
    lib.abs_batch_destroy.argtypes = [vp]
    lib.abs_get_model.restype = C.c_int
    lib.abs_get_model.argtypes = [vp, i64, C.POINTER(C.c_float), sz]
    lib.abs_trace.restype = C.c_int
    lib.abs_trace.argtypes = [vp, i64, i64, C.POINTER(i32), sz, C.POINTER(sz)]
    lib.abs_calibrate_mfma.restype = C.c_int
    lib.abs_calibrate_mfma.argtypes = [i32, i32, i32, vp, vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.abs_mlp_round_plan.restype = C.c_int
    lib.abs_mlp_round_plan.argtypes = [cfgp, i32, C.c_char_p, sz]
    lib.abs_rounds_done.restype = i64
    lib.abs_rounds_done.argtypes = [vp]
    lib.abs_kernel_stats.restype = C.c_int
    lib.abs_kernel_stats.argtypes = [vp, C.POINTER(AbsKernelStat), i32, C.POINTER(i32)]
    lib.abs_last_error.restype = C.c_char_p
    lib.abs_last_error.argtypes = [vp]
    lib.abs_destroy.restype = None
    lib.abs_destroy.argtypes = [vp]
    lib.abs_draw_time_ticks.restype = C.c_uint64
    lib.abs_draw_time_ticks.argtypes = [cfgp, i32, i64]
    lib.abs_draw_batch_rows.restype = C.c_int
    lib.abs_draw_batch_rows.argtypes = [cfgp, i32, i64, C.POINTER(i64)]
    if lib.abs_config_bytes() != C.sizeof(AbsConfig):
        raise ImportError("abs_config layout mismatch between binding and library")
    return lib


_lib = _load()


def _check(rc: int, handle=None):
    if rc != 0:
        raise AbsError(rc, _lib.abs_last_error(handle).decode())


def make_config(p: dict, device_mode: int = 1, profile: int = 0, k_replay=None) -> AbsConfig:
    """AbsConfig from a workload record (keys as in workloads.presets).  The replay
    array, if any, is kept alive on the returned object."""
    c = AbsConfig()
    c.model = p["model"]
    # the convolutional model's dims carry its geometry (8 entries); it has five layers
    c.n_layers = 5 if p["model"] == 3 else len(p["dims"]) - 1
    for i, d in enumerate(p["dims"]):
        c.dims[i] = d
    c.x_dtype = p["x_dtype"]
    c.N, c.M, c.B, c.K0 = p["N"], p["M"], p["B"], p["K0"]
    c.k_mode, c.tau_mode, c.tau_cap, c.a = p["k_mode"], p["tau_mode"], p["tau_cap"], p["a"]
    c.lr, c.sa_penalty = p["lr"], p["sa_penalty"]
    c.time_dist, c.time_param = p["time_dist"], p["time_param"]
    c.n_slow, c.slow_factor = p["n_slow"], p["slow_factor"]
    c.seed = p["seed_sim"]
    if k_replay is None and p.get("k_replay") is not None:
        k_replay = p["k_replay"]
    if k_replay is not None:
        arr = np.ascontiguousarray(k_replay, dtype=np.int32)
        c._keep = arr
        c.k_replay = arr.ctypes.data_as(C.POINTER(C.c_int32))
        c.k_replay_len = arr.size
    c.device_mode, c.profile = device_mode, profile
    c.U = int(p.get("U", 1))
    return c


def trace_stride(N: int) -> int:
    return ABS_TRACE_HEADER + 3 * N


def abs_config_bytes() -> int:
    return _lib.abs_config_bytes()


def abs_workspace_size(cfg: AbsConfig) -> int:
    n = _lib.abs_workspace_size(C.byref(cfg))
    if n == 0:
        raise AbsError(-1, _lib.abs_last_error(None).decode())
    return n


def abs_create(cfg: AbsConfig, d_X: int, d_y: int, d_w0: int, d_workspace: int,
               workspace_bytes: int, hip_stream: int) -> int:
    """Device pointers and the stream are plain integers (e.g. tensor.data_ptr())."""
    out = C.c_void_p()
    rc = _lib.abs_create(C.byref(cfg), d_X, d_y, d_w0, d_workspace, workspace_bytes, hip_stream,
                         C.byref(out))
    _check(rc, None)
    return out.value


def abs_round(handle: int, n_rounds: int) -> None:
    _check(_lib.abs_round(handle, n_rounds), handle)


def abs_get_model(handle: int, version: int, n_floats: int) -> np.ndarray:
    out = np.empty(n_floats, dtype=np.float32)
    _check(_lib.abs_get_model(handle, version, out.ctypes.data_as(C.POINTER(C.c_float)), n_floats), handle)
    return out


def abs_batch_workspace_size(handles) -> int:
    """Bytes of device memory a batch of these handles needs; 0 for MLP handles, and 0 as well when
    the handles cannot form a batch (abs_batch_create then says why)."""
    arr = (C.c_void_p * len(handles))(*handles)
    return _lib.abs_batch_workspace_size(arr, len(handles))


def abs_batch_create(handles, d_workspace: int = 0, workspace_bytes: int = 0) -> int:
    arr = (C.c_void_p * len(handles))(*handles)
    out = C.c_void_p()
    rc = _lib.abs_batch_create(arr, len(handles), d_workspace or None, workspace_bytes, C.byref(out))
    if rc != 0:
        raise AbsError(rc, _lib.abs_batch_last_error(None).decode())
    return out.value


def abs_batch_round(batch: int, n_rounds: int) -> None:
    rc = _lib.abs_batch_round(batch, n_rounds)
    if rc != 0:
        raise AbsError(rc, _lib.abs_batch_last_error(batch).decode())


def abs_batch_destroy(batch: int) -> None:
    _lib.abs_batch_destroy(batch)


def abs_evaluate(handle: int, version: int, d_X: int, d_y: int, n_rows: int):
    """(mean loss, accuracy) of model `version` on an evaluation set given by device pointers."""
    loss, acc = C.c_double(), C.c_double()
    _check(_lib.abs_evaluate(handle, version, d_X, d_y, n_rows, C.byref(loss), C.byref(acc)), handle)
    return loss.value, acc.value


def abs_evaluate_static(handle: int, version: int, d_X: int, d_y: int, n_rows: int, d_out: int) -> None:
    """Enqueue the evaluation; (mean loss, accuracy) land in the two doubles at device address d_out."""
    _check(_lib.abs_evaluate_static(handle, version, d_X, d_y, n_rows, d_out), handle)


def abs_trace(handle: int, round_lo: int, round_hi: int, N: int) -> np.ndarray:
    stride = trace_stride(N)
    out = np.empty((max(0, round_hi - round_lo), stride), dtype=np.int32)
    written = C.c_size_t()
    _check(_lib.abs_trace(handle, round_lo, round_hi, out.ctypes.data_as(C.POINTER(C.c_int32)),
                          out.size, C.byref(written)), handle)
    assert written.value == out.size
    return out


def abs_calibrate_mfma(data_mode: int, iters: int, workgroups: int, d_scratch: int, hip_stream: int):
    """(milliseconds, TFLOP/s) of one launch of the MFMA-only loop."""
    ms, tf = C.c_double(), C.c_double()
    rc = _lib.abs_calibrate_mfma(data_mode, iters, workgroups, d_scratch, hip_stream, C.byref(ms), C.byref(tf))
    if rc != 0:
        raise AbsError(rc, "abs_calibrate_mfma failed")
    return ms.value, tf.value


def abs_mlp_round_plan(cfg: AbsConfig, K: int) -> str:
    buf = C.create_string_buffer(4096)
    rc = _lib.abs_mlp_round_plan(C.byref(cfg), K, buf, len(buf))
    if rc != 0:
        raise AbsError(rc, "abs_mlp_round_plan: not an MLP configuration the library supports, or K outside [1, N]")
    return buf.value.decode()


def abs_rounds_done(handle: int) -> int:
    return _lib.abs_rounds_done(handle)


def abs_kernel_stats(handle: int):
    buf = (AbsKernelStat * 32)()
    n = C.c_int32()
    _check(_lib.abs_kernel_stats(handle, buf, 32, C.byref(n)), handle)
    return [dict(name=buf[i].name.decode(), launches=buf[i].launches, total_ms=buf[i].total_ms,
                 flops=buf[i].flops, bytes=buf[i].bytes, timed_launches=buf[i].timed_launches,
                 timed_flops=buf[i].timed_flops, timed_bytes=buf[i].timed_bytes) for i in range(n.value)]


def abs_last_error(handle=None) -> str:
    return _lib.abs_last_error(handle).decode()


def abs_destroy(handle: int) -> None:
    _lib.abs_destroy(handle)


def abs_draw_time_ticks(cfg: AbsConfig, n: int, j: int) -> int:
    return _lib.abs_draw_time_ticks(C.byref(cfg), n, j)


def abs_draw_batch_rows(cfg: AbsConfig, n: int, j: int) -> np.ndarray:
    out = np.empty(cfg.B, dtype=np.int64)
    rc = _lib.abs_draw_batch_rows(C.byref(cfg), n, j, out.ctypes.data_as(C.POINTER(C.c_int64)))
    if rc != 0:
        raise AbsError(rc, "abs_draw_batch_rows: bad argument")
    return out


class Simulation:
    """Harness convenience: owns the device buffers (PyTorch is used for nothing but
    device memory and the stream) and a libabs handle."""

    def __init__(self, p: dict, inputs: dict | None, device_mode: int = 1, profile: int = 0,
                 k_replay=None, device: str = "cuda:0"):
        self.p = p
        self.N = p["N"]
        self.cfg = make_config(p, device_mode, profile, k_replay)
        self.handle = None
        if not device_mode:
            self.handle = abs_create(self.cfg, None, None, None, None, 0, None)
            self.P = None
            return
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: libabs has no CPU path (use device_mode=0 for schedule-only runs)")
        self.torch = torch
        dev = torch.device(device)
        # simulations created from the same `inputs` dict share one device copy of the dataset
        # (a sweep over seeds or settings reads one dataset); the library only reads these buffers
        shared = inputs.setdefault("_device_copies", {})
        X, y, w0 = inputs["X"], inputs["y"], inputs["w0"]
        hit = shared.get(device)
        if hit is None or hit[0] is not X or hit[1] is not y or hit[2] is not w0:
            xt = torch.from_numpy(X.view(np.int16) if X.dtype == np.uint16 else X)
            hit = (X, y, w0, xt.to(dev), torch.from_numpy(y).to(dev), torch.from_numpy(w0).to(dev))
            shared[device] = hit
        self.d_X, self.d_y, self.d_w0 = hit[3:]
        self.P = int(inputs["w0"].size)
        self.ws_bytes = abs_workspace_size(self.cfg)
        self.d_ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=dev)
        base = self.d_ws.data_ptr()
        self.ws_ptr = (base + 255) // 256 * 256
        self.stream = torch.cuda.current_stream(dev)
        torch.cuda.synchronize(dev)
        self.handle = abs_create(self.cfg, self.d_X.data_ptr(), self.d_y.data_ptr(), self.d_w0.data_ptr(),
                                 self.ws_ptr, self.ws_bytes, self.stream.cuda_stream)

    def round(self, n: int = 1):
        abs_round(self.handle, n)
        return self

    def model(self, version: int = -1) -> np.ndarray:
        return abs_get_model(self.handle, version, self.P)

    def evaluate(self, X: np.ndarray, y: np.ndarray, version: int = -1):
        """Held-out loss and accuracy of a model version; X, y are host arrays in the payload's dtypes."""
        dev = self.d_X.device
        xt = self.torch.from_numpy(X.view(np.int16) if X.dtype == np.uint16 else X).to(dev)
        yt = self.torch.from_numpy(y).to(dev)
        return abs_evaluate(self.handle, version, xt.data_ptr(), yt.data_ptr(), int(X.shape[0]))

    def trace(self, lo: int = 0, hi: int | None = None) -> np.ndarray:
        hi = abs_rounds_done(self.handle) if hi is None else hi
        return abs_trace(self.handle, lo, hi, self.N)

    def kernel_stats(self):
        return abs_kernel_stats(self.handle)

    def close(self):
        if self.handle is not None:
            abs_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Batch:
    """S simulations of one shape advanced together (abs_batch_*); sims: Simulation objects."""

    def __init__(self, sims):
        self.sims = list(sims)
        handles = [s.handle for s in self.sims]
        self.handle = None
        self.ws_bytes = abs_batch_workspace_size(handles)
        self.d_ws, ptr = None, 0
        if self.ws_bytes:
            self.d_ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=self.sims[0].d_X.device)
            ptr = (self.d_ws.data_ptr() + 255) // 256 * 256
        self.handle = abs_batch_create(handles, ptr, self.ws_bytes)

    def round(self, n: int = 1):
        abs_batch_round(self.handle, n)
        return self

    def close(self):
        if self.handle is not None:
            abs_batch_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
