"""ctypes binding of libinfaas_sel.so.  Same call names as include/infaas_sel.h.

Argument marshalling only.  Device arrays are passed as raw pointers (``tensor.data_ptr()``)
and the HIP stream as ``torch.cuda.current_stream().cuda_stream``.  There is no CPU
fallback: if the library has not been built the import of it fails with an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libinfaas_sel.so")

ENGINE_AUTO = 0
ENGINE_SCAN = 1
ENGINE_INDEX = 2

KERNEL_NAMES = ("update_load", "histogram", "plan", "scatter", "scan_lds", "scan_wide",
                "finish_wide", "index_build", "index_select", "update_state", "worker_report",
                "worker_tables", "step_workers", "scale", "group_bin", "group_lookup",
                "group_finish", "instance_states", "closest_scan", "scale_down")
_K_COUNT = len(KERNEL_NAMES)

_I32P = ctypes.POINTER(ctypes.c_int32)


class InfaasSelError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"infaas_sel status {status}: {text}")
        self.status = status


class _Config(ctypes.Structure):
    _fields_ = [("num_tasks", ctypes.c_int32), ("num_batch_sizes", ctypes.c_int32),
                ("batch_sizes", _I32P), ("device", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("lds_segment_limit", ctypes.c_int32)]


class _Timings(ctypes.Structure):
    _fields_ = [("launches", ctypes.c_int64 * _K_COUNT), ("total_ms", ctypes.c_double * _K_COUNT)]


class _Info(ctypes.Structure):
    _fields_ = [("num_variants", ctypes.c_int32), ("num_slices", ctypes.c_int32),
                ("max_segment", ctypes.c_int32), ("lds_segment_limit", ctypes.c_int32),
                ("wide_segments", ctypes.c_int32), ("index_in_lds", ctypes.c_int32),
                ("index_truncated", ctypes.c_int32), ("index_max_steps", ctypes.c_int32),
                ("index_hot_rows", ctypes.c_int32),
                ("index_bytes", ctypes.c_int64), ("index_steps", ctypes.c_int64),
                ("table_bytes", ctypes.c_int64),
                ("scratch_bytes", ctypes.c_int64),
                ("lookup_parked", ctypes.c_int64), ("lookup_second_body", ctypes.c_int64),
                ("lookup_global_body", ctypes.c_int64), ("lookup_scanned", ctypes.c_int64),
                ("lookup_unanswered", ctypes.c_int64), ("index_groups", ctypes.c_int32), ("reserved0", ctypes.c_int32)]


_lib: Optional[ctypes.CDLL] = None

# every symbol include/infaas_sel.h declares
EXPORTED = ("infaas_sel_create", "infaas_sel_load_variants", "infaas_sel_update_load",
            "infaas_sel_select", "infaas_sel_select_noalloc", "infaas_sel_select_closest", "infaas_sel_load_states",
            "infaas_sel_update_state", "infaas_sel_select_tiered", "infaas_sel_select_tiered_closest",
            "infaas_sel_load_workers",
            "infaas_sel_update_workers", "infaas_sel_load_instance_states", "infaas_sel_update_instance_states",
            "infaas_sel_select_workers", "infaas_sel_select_workers_closest", "infaas_sel_load_scaling",
            "infaas_sel_scale", "infaas_sel_scale_down", "infaas_sel_destroy", "infaas_sel_reserve",
            "infaas_sel_read_load", "infaas_sel_set_timing", "infaas_sel_get_timings",
            "infaas_sel_get_info", "infaas_sel_strerror", "infaas_sel_last_error")


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load the built library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with "
                          "`python -m paper_1905_13348_amd.build` (needs hipcc)")
    # The process must hold ONE HIP runtime.  PyTorch ships its own copy (same soname as the
    # system one); importing torch first makes the loader resolve this library's dependency to
    # the copy torch already mapped, instead of mapping a second runtime beside it.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    vp = ctypes.c_void_p
    lib.infaas_sel_create.argtypes = [ctypes.POINTER(_Config), ctypes.POINTER(vp)]
    lib.infaas_sel_load_variants.argtypes = [vp, ctypes.c_int32, _I32P, _I32P, _I32P, _I32P, _I32P]
    lib.infaas_sel_update_load.argtypes = [vp, ctypes.c_int32, vp, vp, vp]
    lib.infaas_sel_select.argtypes = [vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp]
    lib.infaas_sel_select_noalloc.argtypes = [vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp]
    lib.infaas_sel_select_closest.argtypes = [vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp]
    lib.infaas_sel_load_states.argtypes = [vp, _I32P, _I32P]
    lib.infaas_sel_update_state.argtypes = [vp, ctypes.c_int32, vp, vp, vp]
    lib.infaas_sel_select_tiered.argtypes = [vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp]
    lib.infaas_sel_select_tiered_closest.argtypes = [vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.infaas_sel_load_workers.argtypes = [vp, ctypes.c_int32, _I32P, _I32P, _I32P, ctypes.c_int32, _I32P, _I32P, _I32P]
    lib.infaas_sel_update_workers.argtypes = [vp, ctypes.c_int32, vp, vp, ctypes.c_int32, vp, vp, vp]
    lib.infaas_sel_load_instance_states.argtypes = [vp, _I32P]
    lib.infaas_sel_update_instance_states.argtypes = [vp, ctypes.c_int32, vp, vp, vp]
    lib.infaas_sel_select_workers.argtypes = [vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.infaas_sel_select_workers_closest.argtypes = [vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.infaas_sel_load_scaling.argtypes = [vp, _I32P, _I32P, _I32P, _I32P, ctypes.c_int32, ctypes.c_int32]
    lib.infaas_sel_scale.argtypes = [vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.infaas_sel_scale_down.argtypes = lib.infaas_sel_scale.argtypes
    lib.infaas_sel_destroy.argtypes = [vp]
    lib.infaas_sel_destroy.restype = None
    lib.infaas_sel_reserve.argtypes = [vp, ctypes.c_int64]
    lib.infaas_sel_read_load.argtypes = [vp, _I32P, vp]
    lib.infaas_sel_set_timing.argtypes = [vp, ctypes.c_int32]
    lib.infaas_sel_get_timings.argtypes = [vp, ctypes.POINTER(_Timings)]
    lib.infaas_sel_get_info.argtypes = [vp, ctypes.POINTER(_Info)]
    lib.infaas_sel_strerror.argtypes = [ctypes.c_int]
    lib.infaas_sel_strerror.restype = ctypes.c_char_p
    lib.infaas_sel_last_error.argtypes = []
    lib.infaas_sel_last_error.restype = ctypes.c_char_p
    for name in EXPORTED:
        if name not in ("infaas_sel_destroy", "infaas_sel_strerror", "infaas_sel_last_error"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        lib = load_library()
        text = lib.infaas_sel_strerror(status).decode()
        if status == -4:
            text += " [" + lib.infaas_sel_last_error().decode() + "]"
        raise InfaasSelError(status, text)


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _dev_ptr(t, n: int, name: str) -> int:
    """Raw device pointer of an int32 CUDA/HIP tensor with at least n elements."""
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.int32 \
            or not t.is_contiguous() or t.numel() < n:
        raise TypeError(f"{name}: contiguous int32 device tensor with >= {n} elements expected")
    return t.data_ptr()


def _stream_ptr(stream) -> int:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


class Selector:
    """One handle of the library (infaas_sel_create ... infaas_sel_destroy)."""

    def __init__(self, num_tasks: int, batch_sizes: Sequence[int], device: int = 0,
                 engine: int = ENGINE_AUTO, lds_segment_limit: int = 0):
        lib = load_library()
        bs = _host_i32(batch_sizes)
        cfg = _Config(num_tasks=num_tasks, num_batch_sizes=bs.shape[0],
                      batch_sizes=bs.ctypes.data_as(_I32P), device=device, flags=engine,
                      lds_segment_limit=lds_segment_limit)
        h = ctypes.c_void_p()
        _check(lib.infaas_sel_create(ctypes.byref(cfg), ctypes.byref(h)))
        self._h = h
        self._lib = lib
        self.num_tasks = num_tasks
        self.num_batch_sizes = int(bs.shape[0])
        self.device = device

    # -- the five calls ------------------------------------------------------------
    def load_variants(self, task_id, acc_bp, lat_us, cost, queue_us) -> None:
        task_id, acc_bp, queue_us = _host_i32(task_id), _host_i32(acc_bp), _host_i32(queue_us)
        lat_us, cost = _host_i32(lat_us), _host_i32(cost)
        V = task_id.shape[0]
        if lat_us.shape != (V, self.num_batch_sizes) or cost.shape != lat_us.shape \
                or acc_bp.shape != (V,) or queue_us.shape != (V,):
            raise ValueError("table arrays have inconsistent shapes")
        p = lambda a: a.ctypes.data_as(_I32P)
        _check(self._lib.infaas_sel_load_variants(self._h, V, p(task_id), p(acc_bp), p(lat_us),
                                                  p(cost), p(queue_us)))

    def update_load(self, d_variant_idx, d_queue_us, stream=None) -> None:
        n = int(d_variant_idx.numel())
        _check(self._lib.infaas_sel_update_load(
            self._h, n, _dev_ptr(d_variant_idx, n, "d_variant_idx"),
            _dev_ptr(d_queue_us, n, "d_queue_us"), _stream_ptr(stream)))

    def select(self, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, stream=None,
               n: Optional[int] = None) -> None:
        n = int(d_task.numel()) if n is None else int(n)
        _check(self._lib.infaas_sel_select(
            self._h, n, _dev_ptr(d_task, n, "d_task"), _dev_ptr(d_slo_us, n, "d_slo_us"),
            _dev_ptr(d_min_acc_bp, n, "d_min_acc_bp"), _dev_ptr(d_batch_idx, n, "d_batch_idx"),
            _dev_ptr(d_out_variant, n, "d_out_variant"), _stream_ptr(stream)))

    def select_noalloc(self, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, stream=None,
                       n: Optional[int] = None) -> None:
        """infaas_sel_select through the entry point that allocates nothing (static scratch array)."""
        n = int(d_task.numel()) if n is None else int(n)
        _check(self._lib.infaas_sel_select_noalloc(
            self._h, n, _dev_ptr(d_task, n, "d_task"), _dev_ptr(d_slo_us, n, "d_slo_us"),
            _dev_ptr(d_min_acc_bp, n, "d_min_acc_bp"), _dev_ptr(d_batch_idx, n, "d_batch_idx"),
            _dev_ptr(d_out_variant, n, "d_out_variant"), _stream_ptr(stream)))

    def select_closest(self, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, d_out_closest,
                       stream=None, n: Optional[int] = None) -> None:
        n = int(d_task.numel()) if n is None else int(n)
        _check(self._lib.infaas_sel_select_closest(
            self._h, n, _dev_ptr(d_task, n, "d_task"), _dev_ptr(d_slo_us, n, "d_slo_us"),
            _dev_ptr(d_min_acc_bp, n, "d_min_acc_bp"), _dev_ptr(d_batch_idx, n, "d_batch_idx"),
            _dev_ptr(d_out_variant, n, "d_out_variant"), _dev_ptr(d_out_closest, n, "d_out_closest"),
            _stream_ptr(stream)))

    def load_states(self, state, load_us) -> None:
        """Host arrays [V]: state codes 0..3 (Inactive, Active, Overloaded, Interfered), loading latency."""
        state, load_us = _host_i32(state), _host_i32(load_us)
        assert state.shape == load_us.shape and state.ndim == 1
        _check(self._lib.infaas_sel_load_states(self._h, state.ctypes.data_as(_I32P),
                                                load_us.ctypes.data_as(_I32P)))

    def update_state(self, d_variant_idx, d_state, stream=None, n: Optional[int] = None) -> None:
        n = int(d_variant_idx.numel()) if n is None else int(n)
        _check(self._lib.infaas_sel_update_state(
            self._h, n, _dev_ptr(d_variant_idx, n, "d_variant_idx"), _dev_ptr(d_state, n, "d_state"),
            _stream_ptr(stream)))

    def select_tiered(self, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, d_out_tier,
                      stream=None, n: Optional[int] = None) -> None:
        n = int(d_task.numel()) if n is None else int(n)
        _check(self._lib.infaas_sel_select_tiered(
            self._h, n, _dev_ptr(d_task, n, "d_task"), _dev_ptr(d_slo_us, n, "d_slo_us"),
            _dev_ptr(d_min_acc_bp, n, "d_min_acc_bp"), _dev_ptr(d_batch_idx, n, "d_batch_idx"),
            _dev_ptr(d_out_variant, n, "d_out_variant"), _dev_ptr(d_out_tier, n, "d_out_tier"),
            _stream_ptr(stream)))

    def select_tiered_closest(self, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, d_out_tier,
                              d_out_closest, stream=None, n: Optional[int] = None) -> None:
        n = int(d_task.numel()) if n is None else int(n)
        _check(self._lib.infaas_sel_select_tiered_closest(
            self._h, n, _dev_ptr(d_task, n, "d_task"), _dev_ptr(d_slo_us, n, "d_slo_us"),
            _dev_ptr(d_min_acc_bp, n, "d_min_acc_bp"), _dev_ptr(d_batch_idx, n, "d_batch_idx"),
            _dev_ptr(d_out_variant, n, "d_out_variant"), _dev_ptr(d_out_tier, n, "d_out_tier"),
            _dev_ptr(d_out_closest, n, "d_out_closest"), _stream_ptr(stream)))

    def load_workers(self, worker_hw, worker_util, variant_hw, inst_variant, inst_worker, inst_load) -> None:
        """Host arrays: hardware code and utilisation of every worker [W], target hardware of every
        variant [V], and the running instances (variant row, worker, load) [I]."""
        worker_hw, worker_util, variant_hw = _host_i32(worker_hw), _host_i32(worker_util), _host_i32(variant_hw)
        inst_variant, inst_worker, inst_load = _host_i32(inst_variant), _host_i32(inst_worker), _host_i32(inst_load)
        assert worker_hw.shape == worker_util.shape and worker_hw.ndim == 1 and variant_hw.ndim == 1
        assert inst_variant.shape == inst_worker.shape == inst_load.shape and inst_variant.ndim == 1
        _check(self._lib.infaas_sel_load_workers(
            self._h, worker_hw.shape[0], worker_hw.ctypes.data_as(_I32P), worker_util.ctypes.data_as(_I32P),
            variant_hw.ctypes.data_as(_I32P), inst_variant.shape[0], inst_variant.ctypes.data_as(_I32P),
            inst_worker.ctypes.data_as(_I32P), inst_load.ctypes.data_as(_I32P)))

    def update_workers(self, d_worker_idx=None, d_worker_util=None, d_inst_idx=None, d_inst_load=None,
                       stream=None) -> None:
        """Device tensors; either pair may be left out."""
        n = int(d_worker_idx.numel()) if d_worker_idx is not None else 0
        m = int(d_inst_idx.numel()) if d_inst_idx is not None else 0
        _check(self._lib.infaas_sel_update_workers(
            self._h, n, _dev_ptr(d_worker_idx, n, "d_worker_idx") if n else None,
            _dev_ptr(d_worker_util, n, "d_worker_util") if n else None,
            m, _dev_ptr(d_inst_idx, m, "d_inst_idx") if m else None,
            _dev_ptr(d_inst_load, m, "d_inst_load") if m else None, _stream_ptr(stream)))

    def load_instance_states(self, inst_state) -> None:
        """Host array [I]: the state of every running instance, in the order of load_workers."""
        inst_state = _host_i32(inst_state)
        assert inst_state.ndim == 1
        _check(self._lib.infaas_sel_load_instance_states(self._h, inst_state.ctypes.data_as(_I32P)))

    def update_instance_states(self, d_inst_idx, d_state, stream=None, n: Optional[int] = None) -> None:
        n = int(d_inst_idx.numel()) if n is None else int(n)
        _check(self._lib.infaas_sel_update_instance_states(
            self._h, n, _dev_ptr(d_inst_idx, n, "d_inst_idx"), _dev_ptr(d_state, n, "d_state"),
            _stream_ptr(stream)))

    def select_workers(self, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, d_out_tier,
                       d_out_worker, stream=None, n: Optional[int] = None) -> None:
        n = int(d_task.numel()) if n is None else int(n)
        _check(self._lib.infaas_sel_select_workers(
            self._h, n, _dev_ptr(d_task, n, "d_task"), _dev_ptr(d_slo_us, n, "d_slo_us"),
            _dev_ptr(d_min_acc_bp, n, "d_min_acc_bp"), _dev_ptr(d_batch_idx, n, "d_batch_idx"),
            _dev_ptr(d_out_variant, n, "d_out_variant"), _dev_ptr(d_out_tier, n, "d_out_tier"),
            _dev_ptr(d_out_worker, n, "d_out_worker"), _stream_ptr(stream)))

    def select_workers_closest(self, d_task, d_slo_us, d_min_acc_bp, d_batch_idx, d_out_variant, d_out_tier,
                               d_out_worker, d_out_closest, stream=None, n: Optional[int] = None) -> None:
        n = int(d_task.numel()) if n is None else int(n)
        _check(self._lib.infaas_sel_select_workers_closest(
            self._h, n, _dev_ptr(d_task, n, "d_task"), _dev_ptr(d_slo_us, n, "d_slo_us"),
            _dev_ptr(d_min_acc_bp, n, "d_min_acc_bp"), _dev_ptr(d_batch_idx, n, "d_batch_idx"),
            _dev_ptr(d_out_variant, n, "d_out_variant"), _dev_ptr(d_out_tier, n, "d_out_tier"),
            _dev_ptr(d_out_worker, n, "d_out_worker"), _dev_ptr(d_out_closest, n, "d_out_closest"),
            _stream_ptr(stream)))

    def load_scaling(self, arch_id, sat_qps, hw_cost, load_us, lambda_per_s: int, slack_pct: int) -> None:
        """Host arrays [V]: model architecture, saturation throughput, hardware cost, loading latency."""
        arrs = [_host_i32(x) for x in (arch_id, sat_qps, hw_cost, load_us)]
        assert all(a.ndim == 1 and a.shape == arrs[0].shape for a in arrs)
        _check(self._lib.infaas_sel_load_scaling(self._h, *(a.ctypes.data_as(_I32P) for a in arrs),
                                                 int(lambda_per_s), int(slack_pct)))

    def scale(self, d_variant, d_instances, d_load_qps, d_slo_us, d_batch_idx, d_out_action, d_out_variant,
              d_out_instances, stream=None, n: Optional[int] = None, down: bool = False) -> None:
        n = int(d_variant.numel()) if n is None else int(n)
        _check((self._lib.infaas_sel_scale_down if down else self._lib.infaas_sel_scale)(
            self._h, n, _dev_ptr(d_variant, n, "d_variant"), _dev_ptr(d_instances, n, "d_instances"),
            _dev_ptr(d_load_qps, n, "d_load_qps"), _dev_ptr(d_slo_us, n, "d_slo_us"),
            _dev_ptr(d_batch_idx, n, "d_batch_idx"), _dev_ptr(d_out_action, n, "d_out_action"),
            _dev_ptr(d_out_variant, n, "d_out_variant"), _dev_ptr(d_out_instances, n, "d_out_instances"),
            _stream_ptr(stream)))

    def scale_down(self, *args, **kw) -> None:
        self.scale(*args, down=True, **kw)

    def destroy(self) -> None:
        if self._h:
            self._lib.infaas_sel_destroy(self._h)
            self._h = ctypes.c_void_p()

    # -- helpers -------------------------------------------------------------------
    def reserve(self, max_queries: int) -> None:
        _check(self._lib.infaas_sel_reserve(self._h, int(max_queries)))

    def read_load(self, num_variants: int, stream=None) -> np.ndarray:
        out = np.empty(num_variants, dtype=np.int32)
        _check(self._lib.infaas_sel_read_load(self._h, out.ctypes.data_as(_I32P),
                                              _stream_ptr(stream)))
        return out

    def set_timing(self, enabled: bool) -> None:
        _check(self._lib.infaas_sel_set_timing(self._h, 1 if enabled else 0))

    def get_timings(self) -> dict:
        t = _Timings()
        _check(self._lib.infaas_sel_get_timings(self._h, ctypes.byref(t)))
        return {name: dict(launches=int(t.launches[i]), total_ms=float(t.total_ms[i]))
                for i, name in enumerate(KERNEL_NAMES)}

    def info(self) -> dict:
        i = _Info()
        _check(self._lib.infaas_sel_get_info(self._h, ctypes.byref(i)))
        return {name: int(getattr(i, name)) for name, _ in _Info._fields_}

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
