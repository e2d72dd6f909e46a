"""ctypes front end of libmultilora.so: the same entry points as ``include/multi_lora.h``.

Argument marshalling only -- every step of the layer runs in the HIP kernels.  Tensors are
passed as anything with ``data_ptr()`` (torch tensors) or as raw integer addresses; torch is
used by callers for device memory and streams, never for compute.  Loading fails loudly if
the shared library has not been built (``python -m paper_2604_05426_amd.build``).
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

F32, BF16 = 0, 1
FLAG_BASE_ONLY, FLAG_LORA_ONLY, FLAG_ACCUM_GRADS, FLAG_GROUP_BANDS = 1, 2, 4, 8
TABLE_ROW_BLOCKS, TABLE_GEMM_ROW_TILES, TABLE_WGRAD_CHUNKS, TABLE_CLASS_BLOCKS, TABLE_GEMM_BAND_ORDER = 0, 1, 2, 3, 4
GEO_BLOCK_ROWS, GEO_GEMM_TILE_ROWS, GEO_GEMM_TILE_COLS, GEO_WGRAD_CHUNK_ROWS = 0, 1, 2, 3
GEO_R1_LO, GEO_R1_HI, GEO_USES_MFMA, GEO_WGRAD_CHUNK_ROWS_WIDE = 4, 5, 6, 7
GEO_BLOCK_ROWS_WIDE, GEO_GEMM_BAND_TILES, GEO_NUM_CUS, GEO_WGRAD_PANEL_COLS, GEO_WGRAD_MIN_CHUNK_ROWS, GEO_COUNT = 8, 9, 10, 11, 12, 13
MAX_RANK, MAX_ADAPTERS = 128, 4096

STATUS_NAMES = {0: "MLORA_OK", -1: "MLORA_ERR_NULL", -2: "MLORA_ERR_SHAPE", -3: "MLORA_ERR_SEGMENTS",
                -4: "MLORA_ERR_RANK", -5: "MLORA_ERR_DTYPE", -6: "MLORA_ERR_ALIGN",
                -7: "MLORA_ERR_WORKSPACE", -8: "MLORA_ERR_HIP", -9: "MLORA_ERR_FLAGS",
                -10: "MLORA_ERR_SCALE"}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmultilora.so")

# every symbol include/multi_lora.h declares
EXPORTS = ["multi_lora_plan_create", "multi_lora_plan_create_like", "multi_lora_plan_destroy", "multi_lora_validate",
           "multi_lora_workspace_bytes", "multi_lora_plan_geometry", "multi_lora_plan_dump",
           "multi_lora_fwd", "multi_lora_bwd", "multi_lora_bwd_static", "multi_lora_last_error", "multi_lora_version",
           "multi_lora_profile_begin", "multi_lora_profile_end",
           "multi_lora_adamw_init", "multi_lora_adamw_step",
           "multi_lora_calib_mfma", "multi_lora_calib_read",
           "multi_lora_monitor_create", "multi_lora_monitor_destroy", "multi_lora_monitor_train_loss",
           "multi_lora_monitor_val_loss", "multi_lora_monitor_warmup_select", "multi_lora_monitor_state",
           "multi_lora_memory_model_fit", "multi_lora_admission_create", "multi_lora_admission_destroy",
           "multi_lora_admission_submit", "multi_lora_admission_fill", "multi_lora_admission_exit",
           "multi_lora_admission_running",
           "multi_lora_schedule_tasks", "multi_lora_cluster_create", "multi_lora_cluster_destroy",
           "multi_lora_cluster_submit", "multi_lora_cluster_complete", "multi_lora_cluster_poll",
           "multi_lora_cluster_plan"]

EXIT_CONTINUE, EXIT_DIVERGING, EXIT_OVERFITTING, EXIT_UNDERPERFORMING = 0, 1, 2, 3

KERNEL_NAMES = {0: "shrink", 1: "gemm_fwd", 2: "dshrink", 3: "gemm_bwd", 4: "wgrad", 5: "wgrad_reduce", 6: "other",
                7: "adamw"}


class MonitorParams(ctypes.Structure):
    """mlora_monitor_params"""
    _fields_ = [("ema_alpha", ctypes.c_double), ("window", ctypes.c_int32), ("patience_div", ctypes.c_int32),
                ("patience_ovf", ctypes.c_int32), ("tau_slope", ctypes.c_double), ("tau_gap", ctypes.c_double)]


class MonitorState(ctypes.Structure):
    """mlora_monitor_state"""
    _fields_ = [("ema_train_loss", ctypes.c_double), ("best_val_loss", ctypes.c_double), ("best_eval_step", ctypes.c_int32),
                ("evaluations", ctypes.c_int32), ("count_diverging", ctypes.c_int32), ("count_overfitting", ctypes.c_int32),
                ("status", ctypes.c_int32)]


class AdmissionParams(ctypes.Structure):
    """mlora_admission_params"""
    _fields_ = [("k0", ctypes.c_double), ("k1", ctypes.c_double), ("capacity_bytes", ctypes.c_double),
                ("safety_margin", ctypes.c_double), ("seq_len", ctypes.c_int64)]


class AdamwHparams(ctypes.Structure):
    """mlora_adamw_hparams: one entry per adapter; `step` is that adapter's 1-based step count."""
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float), ("step", ctypes.c_int32)]


class MultiLoraError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_05426_amd.build`; "
                              "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        i32, i64, vp, u32 = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_uint32
        L.multi_lora_plan_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, i64, i64, i32, vp, vp, vp, vp]
        L.multi_lora_plan_create.restype = ctypes.c_int
        L.multi_lora_plan_create_like.argtypes = [ctypes.POINTER(vp), vp, i64, i64, vp]
        L.multi_lora_plan_create_like.restype = ctypes.c_int
        L.multi_lora_plan_destroy.argtypes = [vp]
        L.multi_lora_plan_destroy.restype = ctypes.c_int
        L.multi_lora_validate.argtypes = [ctypes.c_int, i64, i64, i64, i32, vp, vp, vp]
        L.multi_lora_validate.restype = ctypes.c_int
        L.multi_lora_workspace_bytes.argtypes = [vp]
        L.multi_lora_workspace_bytes.restype = ctypes.c_size_t
        L.multi_lora_plan_geometry.argtypes = [vp, vp]
        L.multi_lora_plan_geometry.restype = ctypes.c_int
        L.multi_lora_plan_dump.argtypes = [vp, ctypes.c_int, vp, i64, ctypes.POINTER(i64)]
        L.multi_lora_plan_dump.restype = ctypes.c_int
        L.multi_lora_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, u32, vp]
        L.multi_lora_fwd.restype = ctypes.c_int
        L.multi_lora_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, u32, vp]
        L.multi_lora_bwd.restype = ctypes.c_int
        L.multi_lora_bwd_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, u32, vp]
        L.multi_lora_bwd_static.restype = ctypes.c_int
        L.multi_lora_profile_begin.argtypes = [vp, i32]
        L.multi_lora_profile_begin.restype = ctypes.c_int
        L.multi_lora_profile_end.argtypes = [vp, vp, vp, i32, ctypes.POINTER(i32)]
        L.multi_lora_profile_end.restype = ctypes.c_int
        L.multi_lora_adamw_init.argtypes = [vp, vp, vp, vp, vp, vp]
        L.multi_lora_adamw_init.restype = ctypes.c_int
        L.multi_lora_adamw_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.multi_lora_adamw_step.restype = ctypes.c_int
        L.multi_lora_calib_mfma.argtypes = [i32, vp, ctypes.POINTER(ctypes.c_float), vp]
        L.multi_lora_calib_mfma.restype = ctypes.c_int
        L.multi_lora_calib_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_float), vp]
        L.multi_lora_calib_read.restype = ctypes.c_int
        L.multi_lora_monitor_create.argtypes = [ctypes.POINTER(vp), i32, ctypes.POINTER(MonitorParams)]
        L.multi_lora_monitor_create.restype = ctypes.c_int
        L.multi_lora_monitor_destroy.argtypes = [vp]
        L.multi_lora_monitor_destroy.restype = ctypes.c_int
        L.multi_lora_monitor_train_loss.argtypes = [vp, i32, ctypes.c_double]
        L.multi_lora_monitor_train_loss.restype = ctypes.c_int
        L.multi_lora_monitor_val_loss.argtypes = [vp, i32, ctypes.c_double, ctypes.POINTER(i32)]
        L.multi_lora_monitor_val_loss.restype = ctypes.c_int
        L.multi_lora_monitor_warmup_select.argtypes = [vp, ctypes.c_double, vp]
        L.multi_lora_monitor_warmup_select.restype = ctypes.c_int
        L.multi_lora_monitor_state.argtypes = [vp, i32, ctypes.POINTER(MonitorState)]
        L.multi_lora_monitor_state.restype = ctypes.c_int
        dp = ctypes.POINTER(ctypes.c_double)
        L.multi_lora_memory_model_fit.argtypes = [i32, dp, dp, dp, dp]
        L.multi_lora_memory_model_fit.restype = ctypes.c_int
        L.multi_lora_admission_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(AdmissionParams)]
        L.multi_lora_admission_create.restype = ctypes.c_int
        L.multi_lora_admission_destroy.argtypes = [vp]
        L.multi_lora_admission_destroy.restype = ctypes.c_int
        L.multi_lora_admission_submit.argtypes = [vp, i32, i32]
        L.multi_lora_admission_submit.restype = ctypes.c_int
        L.multi_lora_admission_fill.argtypes = [vp, vp, i32, ctypes.POINTER(i32)]
        L.multi_lora_admission_fill.restype = ctypes.c_int
        L.multi_lora_admission_exit.argtypes = [vp, i32, vp, i32, ctypes.POINTER(i32)]
        L.multi_lora_admission_exit.restype = ctypes.c_int
        L.multi_lora_admission_running.argtypes = [vp, vp, vp, i32, ctypes.POINTER(i32)]
        L.multi_lora_admission_running.restype = ctypes.c_int
        dbl = ctypes.c_double
        L.multi_lora_schedule_tasks.argtypes = [i32, vp, vp, i32, vp, dbl, vp, vp, dp, ctypes.POINTER(i32)]
        L.multi_lora_schedule_tasks.restype = ctypes.c_int
        L.multi_lora_cluster_create.argtypes = [ctypes.POINTER(vp), i32]
        L.multi_lora_cluster_create.restype = ctypes.c_int
        L.multi_lora_cluster_destroy.argtypes = [vp]
        L.multi_lora_cluster_destroy.restype = ctypes.c_int
        L.multi_lora_cluster_submit.argtypes = [vp, dbl, dbl, i32, ctypes.POINTER(i32)]
        L.multi_lora_cluster_submit.restype = ctypes.c_int
        L.multi_lora_cluster_complete.argtypes = [vp, dbl, i32]
        L.multi_lora_cluster_complete.restype = ctypes.c_int
        L.multi_lora_cluster_poll.argtypes = [vp, dbl, vp, vp, i32, ctypes.POINTER(i32)]
        L.multi_lora_cluster_poll.restype = ctypes.c_int
        L.multi_lora_cluster_plan.argtypes = [vp, vp, vp, i32, ctypes.POINTER(i32), dp]
        L.multi_lora_cluster_plan.restype = ctypes.c_int
        L.multi_lora_last_error.restype = ctypes.c_char_p
        L.multi_lora_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def last_error() -> str:
    return lib().multi_lora_last_error().decode()


def version() -> str:
    return lib().multi_lora_version().decode()


def _check(status: int) -> None:
    if status != 0:
        raise MultiLoraError(status, last_error())


def _addr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _ptr_array(items: Optional[Sequence], n: int):
    if items is None:
        return None
    arr = (ctypes.c_void_p * max(n, 1))()
    for i in range(n):
        arr[i] = _addr(items[i])
    return arr


def _meta(N, ranks, scales, offsets):
    r = (ctypes.c_int32 * max(N, 1))(*[int(x) for x in ranks]) if ranks is not None else None
    s = (ctypes.c_float * max(N, 1))(*[float(x) for x in scales]) if scales is not None else None
    o = (ctypes.c_int64 * (len(offsets)))(*[int(x) for x in offsets]) if offsets is not None else None
    return r, s, o


def multi_lora_validate(dtype: int, T: int, k: int, n: int, N: int, ranks, scales, offsets) -> int:
    """Status code of the argument check alone (touches no GPU)."""
    r, s, o = _meta(N, ranks, scales, offsets)
    return int(lib().multi_lora_validate(dtype, T, k, n, N, r, s, o))


class Plan:
    """Owns one mlora_plan (multi_lora_plan_create / multi_lora_plan_destroy)."""

    def __init__(self, dtype: int, T: int, k: int, n: int, ranks, scales, offsets, stream: int = 0):
        self.dtype, self.T, self.k, self.n = dtype, T, k, n
        self.N = len(ranks)
        self.ranks, self.scales, self.offsets = list(ranks), list(scales or []), list(offsets or [0])
        self._h = ctypes.c_void_p()
        r, s, o = _meta(self.N, ranks, scales, offsets)
        _check(lib().multi_lora_plan_create(ctypes.byref(self._h), dtype, T, k, n, self.N, r, s, o,
                                            ctypes.c_void_p(stream)))

    @classmethod
    def like(cls, base: "Plan", k: int, n: int, stream: int = 0) -> "Plan":
        """multi_lora_plan_create_like: another layer shape over the segmentation tables of `base`."""
        self = cls.__new__(cls)
        self.dtype, self.T, self.k, self.n, self.N = base.dtype, base.T, k, n, base.N
        self.ranks, self.scales, self.offsets = list(base.ranks), list(base.scales), list(base.offsets)
        self._h = ctypes.c_void_p()
        _check(lib().multi_lora_plan_create_like(ctypes.byref(self._h), base.handle, k, n, ctypes.c_void_p(stream)))
        return self

    @property
    def handle(self):
        return self._h

    def workspace_bytes(self) -> int:
        return int(lib().multi_lora_workspace_bytes(self._h))

    def geometry(self) -> List[int]:
        out = (ctypes.c_int32 * GEO_COUNT)()
        _check(lib().multi_lora_plan_geometry(self._h, out))
        return list(out)

    @property
    def R1(self) -> int:
        g = self.geometry()
        return g[GEO_R1_LO] + (g[GEO_R1_HI] << 31)

    def dump(self, table: int) -> List[tuple]:
        cnt = ctypes.c_int64(0)
        _check(lib().multi_lora_plan_dump(self._h, table, None, 0, ctypes.byref(cnt)))
        n = cnt.value
        buf = (ctypes.c_int32 * (4 * max(n, 1)))()
        _check(lib().multi_lora_plan_dump(self._h, table, buf, n, ctypes.byref(cnt)))
        return [tuple(buf[4 * i: 4 * i + 4]) for i in range(n)]

    def profile_begin(self, max_records: int) -> None:
        _check(lib().multi_lora_profile_begin(self._h, max_records))

    def profile_end(self, cap: int) -> List[tuple]:
        """[(kernel id, milliseconds), ...] for every launch recorded since profile_begin."""
        ids = (ctypes.c_int32 * max(cap, 1))()
        ms = (ctypes.c_float * max(cap, 1))()
        cnt = ctypes.c_int32(0)
        _check(lib().multi_lora_profile_end(self._h, ids, ms, cap, ctypes.byref(cnt)))
        return [(int(ids[i]), float(ms[i])) for i in range(min(cnt.value, cap))]

    def destroy(self) -> None:
        if self._h:
            _check(lib().multi_lora_plan_destroy(self._h))
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def multi_lora_fwd(plan: Plan, X, W, A: Optional[Sequence], B: Optional[Sequence], Y, S, workspace,
                   flags: int = 0, stream: int = 0) -> None:
    _check(lib().multi_lora_fwd(plan.handle, _addr(X), _addr(W), _ptr_array(A, plan.N), _ptr_array(B, plan.N),
                                _addr(Y), _addr(S), _addr(workspace), flags, ctypes.c_void_p(stream)))


def multi_lora_bwd(plan: Plan, dY, X, W, A, B, S, dX, dA, dB, workspace, flags: int = 0, stream: int = 0) -> None:
    _check(lib().multi_lora_bwd(plan.handle, _addr(dY), _addr(X), _addr(W), _ptr_array(A, plan.N),
                                _ptr_array(B, plan.N), _addr(S), _addr(dX), _ptr_array(dA, plan.N),
                                _ptr_array(dB, plan.N), _addr(workspace), flags, ctypes.c_void_p(stream)))


STATIC_WORKSPACE_BYTES = 64 << 20


def multi_lora_bwd_static(plan: Plan, dY, X, W, A, B, S, dX, dA, dB, flags: int = 0, stream: int = 0) -> None:
    """multi_lora_bwd with the workspace in the library's static device array (allocates nothing)."""
    _check(lib().multi_lora_bwd_static(plan.handle, _addr(dY), _addr(X), _addr(W), _ptr_array(A, plan.N),
                                       _ptr_array(B, plan.N), _addr(S), _addr(dX), _ptr_array(dA, plan.N),
                                       _ptr_array(dB, plan.N), flags, ctypes.c_void_p(stream)))


def multi_lora_adamw_init(plan: Plan, A, B, stateA, stateB, stream: int = 0) -> None:
    n = plan.N
    _check(lib().multi_lora_adamw_init(plan.handle, _ptr_array(A, n), _ptr_array(B, n), _ptr_array(stateA, n),
                                       _ptr_array(stateB, n), ctypes.c_void_p(stream)))


def multi_lora_adamw_step(plan: Plan, A, B, dA, dB, stateA, stateB, hparams: Sequence, stream: int = 0) -> None:
    """`hparams`: one (lr, beta1, beta2, eps, weight_decay, step) tuple per adapter."""
    n = plan.N
    hp = (AdamwHparams * max(n, 1))()
    for i in range(n):
        lr, b1, b2, eps, wd, step = hparams[i]
        hp[i] = AdamwHparams(lr, b1, b2, eps, wd, int(step))
    _check(lib().multi_lora_adamw_step(plan.handle, _ptr_array(A, n), _ptr_array(B, n), _ptr_array(dA, n),
                                       _ptr_array(dB, n), _ptr_array(stateA, n), _ptr_array(stateB, n), hp,
                                       ctypes.c_void_p(stream)))


def multi_lora_calib_mfma(random_data: bool, scratch, stream: int = 0) -> float:
    """TFLOP/s of the register-only MFMA loop (see include/multi_lora.h)."""
    out = ctypes.c_float(0.0)
    _check(lib().multi_lora_calib_mfma(1 if random_data else 0, _addr(scratch), ctypes.byref(out), ctypes.c_void_p(stream)))
    return float(out.value)


def multi_lora_calib_read(buffer, nbytes: int, scratch, stream: int = 0) -> float:
    """GB/s of a coalesced streaming read of `buffer`."""
    out = ctypes.c_float(0.0)
    _check(lib().multi_lora_calib_read(_addr(buffer), nbytes, _addr(scratch), ctypes.byref(out), ctypes.c_void_p(stream)))
    return float(out.value)


class Monitor:
    """Owns one mlora_monitor (loss-aware early exit; host only)."""

    def __init__(self, n: int, ema_alpha: float, window: int, tau_slope: float, tau_gap: float, patience_div: int,
                 patience_ovf: int):
        self.n = n
        self._h = ctypes.c_void_p()
        p = MonitorParams(ema_alpha, window, patience_div, patience_ovf, tau_slope, tau_gap)
        _check(lib().multi_lora_monitor_create(ctypes.byref(self._h), n, ctypes.byref(p)))

    def train_loss(self, adapter: int, loss: float) -> None:
        _check(lib().multi_lora_monitor_train_loss(self._h, adapter, float(loss)))

    def val_loss(self, adapter: int, val: float) -> int:
        d = ctypes.c_int32(-1)
        _check(lib().multi_lora_monitor_val_loss(self._h, adapter, float(val), ctypes.byref(d)))
        return d.value

    def warmup_select(self, ratio: float) -> List[int]:
        out = (ctypes.c_int32 * max(self.n, 1))()
        _check(lib().multi_lora_monitor_warmup_select(self._h, float(ratio), out))
        return list(out)[: self.n]

    def state(self, adapter: int) -> MonitorState:
        st = MonitorState()
        _check(lib().multi_lora_monitor_state(self._h, adapter, ctypes.byref(st)))
        return st

    def destroy(self) -> None:
        if self._h:
            lib().multi_lora_monitor_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def memory_model_fit(batch_times_seq: Sequence[float], peak_bytes: Sequence[float]):
    """multi_lora_memory_model_fit -> (k0, k1)"""
    n = len(batch_times_seq)
    x = (ctypes.c_double * max(n, 1))(*[float(v) for v in batch_times_seq])
    y = (ctypes.c_double * max(n, 1))(*[float(v) for v in peak_bytes])
    k0, k1 = ctypes.c_double(), ctypes.c_double()
    _check(lib().multi_lora_memory_model_fit(n, x, y, ctypes.byref(k0), ctypes.byref(k1)))
    return k0.value, k1.value


class Admission:
    """Owns one mlora_admission (online greedy intra-task scheduler; host only)."""
    CAP = 4096

    def __init__(self, k0: float, k1: float, capacity_bytes: float, safety_margin: float, seq_len: int):
        self._h = ctypes.c_void_p()
        p = AdmissionParams(k0, k1, capacity_bytes, safety_margin, seq_len)
        _check(lib().multi_lora_admission_create(ctypes.byref(self._h), ctypes.byref(p)))

    def submit(self, job: int, batch: int) -> None:
        _check(lib().multi_lora_admission_submit(self._h, job, batch))

    def fill(self) -> List[int]:
        out, cnt = (ctypes.c_int32 * self.CAP)(), ctypes.c_int32(0)
        _check(lib().multi_lora_admission_fill(self._h, out, self.CAP, ctypes.byref(cnt)))
        return list(out[: cnt.value])

    def exit(self, job: int) -> List[int]:
        out, cnt = (ctypes.c_int32 * self.CAP)(), ctypes.c_int32(0)
        _check(lib().multi_lora_admission_exit(self._h, job, out, self.CAP, ctypes.byref(cnt)))
        return list(out[: cnt.value])

    def running(self) -> List[tuple]:
        ids, bs, cnt = (ctypes.c_int32 * self.CAP)(), (ctypes.c_int32 * self.CAP)(), ctypes.c_int32(0)
        _check(lib().multi_lora_admission_running(self._h, ids, bs, self.CAP, ctypes.byref(cnt)))
        return [(ids[i], bs[i]) for i in range(cnt.value)]

    def destroy(self) -> None:
        if self._h:
            lib().multi_lora_admission_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


MAX_TASKS, MAX_CLUSTER_GPUS = 24, 64


def _mask_to_gpus(mask: int) -> List[int]:
    return [q for q in range(MAX_CLUSTER_GPUS) if mask >> q & 1]


def schedule_tasks(durations: Sequence[float], gpus_needed: Sequence[int], G: int,
                   release: Optional[Sequence[float]] = None, now: float = 0.0, with_proof: bool = False):
    """multi_lora_schedule_tasks: (starts, gpus per task, makespan) of the minimum-makespan schedule; with_proof adds
    whether the search ran to its end (it gives up after about a second and then returns the best schedule found)."""
    n = len(durations)
    d = (ctypes.c_double * max(n, 1))(*[float(x) for x in durations])
    g = (ctypes.c_int32 * max(n, 1))(*[int(x) for x in gpus_needed])
    rel = (ctypes.c_double * G)(*[float(x) for x in release]) if release is not None else None
    starts, masks, mk = (ctypes.c_double * max(n, 1))(), (ctypes.c_uint64 * max(n, 1))(), ctypes.c_double()
    proved = ctypes.c_int32(0)
    _check(lib().multi_lora_schedule_tasks(n, d, g, G, rel, float(now), starts, masks, ctypes.byref(mk), ctypes.byref(proved)))
    out = ([starts[i] for i in range(n)], [_mask_to_gpus(masks[i]) for i in range(n)], mk.value)
    return out + (bool(proved.value),) if with_proof else out


class Cluster:
    """Owns one mlora_cluster (event-driven inter-task scheduler; host only)."""

    def __init__(self, G: int):
        self._h = ctypes.c_void_p()
        _check(lib().multi_lora_cluster_create(ctypes.byref(self._h), G))

    def submit(self, now: float, duration: float, gpus: int) -> int:
        tid = ctypes.c_int32(-1)
        _check(lib().multi_lora_cluster_submit(self._h, float(now), float(duration), int(gpus), ctypes.byref(tid)))
        return tid.value

    def complete(self, now: float, task: int) -> None:
        _check(lib().multi_lora_cluster_complete(self._h, float(now), int(task)))

    def poll(self, now: float) -> List[tuple]:
        ids, masks, cnt = (ctypes.c_int32 * MAX_TASKS)(), (ctypes.c_uint64 * MAX_TASKS)(), ctypes.c_int32(0)
        _check(lib().multi_lora_cluster_poll(self._h, float(now), ids, masks, MAX_TASKS, ctypes.byref(cnt)))
        return [(ids[i], _mask_to_gpus(masks[i])) for i in range(cnt.value)]

    def plan(self):
        ids, st, cnt, mk = (ctypes.c_int32 * MAX_TASKS)(), (ctypes.c_double * MAX_TASKS)(), ctypes.c_int32(0), ctypes.c_double()
        _check(lib().multi_lora_cluster_plan(self._h, ids, st, MAX_TASKS, ctypes.byref(cnt), ctypes.byref(mk)))
        return {ids[i]: st[i] for i in range(cnt.value)}, mk.value

    def destroy(self) -> None:
        if self._h:
            lib().multi_lora_cluster_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
