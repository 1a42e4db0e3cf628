"""Build and call the C oracle (select_oracle.c) through ctypes.  Test infrastructure only.

Argument marshalling only: every array is checked to be C-contiguous int32 and
handed to the C functions as a plain pointer.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "select_oracle.c")
_LIB = os.path.join(_HERE, "libselect_oracle.so")

_I32P = ctypes.POINTER(ctypes.c_int32)


def build_oracle(src: str = _SRC, out: str = _LIB, force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, OpenMP for the outer query loop only)."""
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
        return out
    tmp = out + f".tmp{os.getpid()}"
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", tmp, src]
    subprocess.run(cmd, check=True)
    os.replace(tmp, out)
    return out


def _ptr(a: np.ndarray):
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"], "int32 C-contiguous array expected"
    return a.ctypes.data_as(_I32P)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


class Oracle:
    """Thin wrapper around one compiled oracle library."""

    def __init__(self, path: str):
        self.path = path
        lib = ctypes.CDLL(path)
        sel_args = [ctypes.c_int64, ctypes.c_int32, _I32P, _I32P, _I32P, _I32P, _I32P,
                    ctypes.c_int64, _I32P, _I32P, _I32P, _I32P, _I32P]
        for name in ("oracle_select", "oracle_select_literal"):
            fn = getattr(lib, name)
            fn.argtypes = sel_args
            fn.restype = ctypes.c_int
        for name in ("oracle_select_closest", "oracle_select_closest_literal"):
            fn = getattr(lib, name)
            fn.argtypes = sel_args + [_I32P]
            fn.restype = ctypes.c_int
        for name in ("oracle_select_tiered", "oracle_select_tiered_literal"):
            fn = getattr(lib, name)
            fn.argtypes = [ctypes.c_int64, ctypes.c_int32] + [_I32P] * 7 + [ctypes.c_int64] + [_I32P] * 6
            fn.restype = ctypes.c_int
        for name in ("oracle_select_case1", "oracle_select_case1_literal"):
            fn = getattr(lib, name)
            fn.argtypes = [ctypes.c_int64, ctypes.c_int32] + [_I32P] * 7 + [ctypes.c_int64] + [_I32P] * 7
            fn.restype = ctypes.c_int
        for name in ("oracle_select_workers", "oracle_select_workers_literal"):
            fn = getattr(lib, name)
            fn.argtypes = ([ctypes.c_int64, ctypes.c_int32] + [_I32P] * 8 + [ctypes.c_int64, _I32P, _I32P]
                           + [ctypes.c_int64, _I32P, _I32P, _I32P] + [ctypes.c_int64] + [_I32P] * 7)
            fn.restype = ctypes.c_int
        for name in ("oracle_update_worker_util", "oracle_update_instance_load"):
            fn = getattr(lib, name)
            fn.argtypes = [ctypes.c_int64, _I32P, ctypes.c_int64, _I32P, _I32P]
            fn.restype = None
        lib.oracle_derive_states.argtypes = [ctypes.c_int64, ctypes.c_int64, _I32P, _I32P, _I32P]
        lib.oracle_derive_states.restype = ctypes.c_int
        lib.oracle_select_instances.argtypes = ([ctypes.c_int64, ctypes.c_int32] + [_I32P] * 7
                                                + [ctypes.c_int64, _I32P, _I32P] + [ctypes.c_int64] + [_I32P] * 4
                                                + [ctypes.c_int32, ctypes.c_int64] + [_I32P] * 7)
        lib.oracle_select_instances.restype = ctypes.c_int
        lib.oracle_update_instance_state.argtypes = [ctypes.c_int64, _I32P, ctypes.c_int64, _I32P, _I32P]
        lib.oracle_update_instance_state.restype = None
        lib.oracle_scale.argtypes = ([ctypes.c_int64, ctypes.c_int32] + [_I32P] * 5 + [ctypes.c_int32, ctypes.c_int32]
                                     + [ctypes.c_int64] + [_I32P] * 8)
        lib.oracle_scale.restype = ctypes.c_int
        lib.oracle_scale_down.argtypes = lib.oracle_scale.argtypes
        lib.oracle_scale_down.restype = ctypes.c_int
        lib.oracle_update_state.argtypes = [ctypes.c_int64, _I32P, ctypes.c_int64, _I32P, _I32P]
        lib.oracle_update_state.restype = None
        lib.oracle_count_feasible.argtypes = [ctypes.c_int64, ctypes.c_int32, _I32P, _I32P, _I32P,
                                              _I32P, ctypes.c_int64, _I32P, _I32P, _I32P, _I32P,
                                              _I32P]
        lib.oracle_count_feasible.restype = ctypes.c_int
        lib.oracle_update_load.argtypes = [ctypes.c_int64, _I32P, ctypes.c_int64, _I32P, _I32P]
        lib.oracle_update_load.restype = None
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_threads.argtypes = [ctypes.c_int]
        lib.oracle_set_threads.restype = ctypes.c_int
        self._lib = lib

    def num_threads(self) -> int:
        return int(self._lib.oracle_num_threads())

    def set_threads(self, n: int) -> int:
        """Host threads for the grouped forms from now on; returns the number in use."""
        return int(self._lib.oracle_set_threads(int(n)))

    def _select(self, fn, task_id, acc_bp, lat_us, cost, queue_us, q_task, q_slo, q_min_acc, q_bidx):
        task_id, acc_bp, queue_us = _i32(task_id), _i32(acc_bp), _i32(queue_us)
        lat_us, cost = _i32(lat_us), _i32(cost)
        V = task_id.shape[0]
        assert lat_us.ndim == 2 and lat_us.shape[0] == V and cost.shape == lat_us.shape
        B = lat_us.shape[1]
        assert acc_bp.shape == (V,) and queue_us.shape == (V,)
        q_task, q_slo, q_min_acc, q_bidx = _i32(q_task), _i32(q_slo), _i32(q_min_acc), _i32(q_bidx)
        N = q_task.shape[0]
        assert q_slo.shape == (N,) and q_min_acc.shape == (N,) and q_bidx.shape == (N,)
        out = np.empty(N, dtype=np.int32)
        rc = fn(V, B, _ptr(task_id), _ptr(acc_bp), _ptr(lat_us), _ptr(cost), _ptr(queue_us),
                N, _ptr(q_task), _ptr(q_slo), _ptr(q_min_acc), _ptr(q_bidx), _ptr(out))
        if rc != 0:
            raise ValueError("oracle rejected its arguments")
        return out

    def select(self, task_id, acc_bp, lat_us, cost, queue_us, q_task, q_slo, q_min_acc, q_bidx):
        """Grouped brute force (multi-threaded over queries)."""
        return self._select(self._lib.oracle_select, task_id, acc_bp, lat_us, cost, queue_us,
                            q_task, q_slo, q_min_acc, q_bidx)

    def select_literal(self, task_id, acc_bp, lat_us, cost, queue_us, q_task, q_slo, q_min_acc,
                       q_bidx):
        """Literal O(N*V) scan in the caller's row order."""
        return self._select(self._lib.oracle_select_literal, task_id, acc_bp, lat_us, cost,
                            queue_us, q_task, q_slo, q_min_acc, q_bidx)

    def _closest(self, fn, task_id, acc_bp, lat_us, cost, queue_us, q_task, q_slo, q_min_acc, q_bidx):
        task_id, acc_bp, queue_us = _i32(task_id), _i32(acc_bp), _i32(queue_us)
        lat_us, cost = _i32(lat_us), _i32(cost)
        V, B = lat_us.shape
        assert cost.shape == lat_us.shape and acc_bp.shape == (V,) and queue_us.shape == (V,)
        q_task, q_slo, q_min_acc, q_bidx = _i32(q_task), _i32(q_slo), _i32(q_min_acc), _i32(q_bidx)
        N = q_task.shape[0]
        assert q_slo.shape == (N,) and q_min_acc.shape == (N,) and q_bidx.shape == (N,)
        out = np.empty(N, dtype=np.int32)
        closest = np.empty(N, dtype=np.int32)
        rc = fn(V, B, _ptr(task_id), _ptr(acc_bp), _ptr(lat_us), _ptr(cost), _ptr(queue_us),
                N, _ptr(q_task), _ptr(q_slo), _ptr(q_min_acc), _ptr(q_bidx), _ptr(out), _ptr(closest))
        if rc != 0:
            raise ValueError("oracle rejected its arguments")
        return out, closest

    def select_closest(self, task_id, acc_bp, lat_us, cost, queue_us, q_task, q_slo, q_min_acc, q_bidx):
        """(selected variant or -1, closest variant) per query; grouped, multi-threaded."""
        return self._closest(self._lib.oracle_select_closest, task_id, acc_bp, lat_us, cost, queue_us,
                             q_task, q_slo, q_min_acc, q_bidx)

    def select_closest_literal(self, task_id, acc_bp, lat_us, cost, queue_us, q_task, q_slo, q_min_acc,
                               q_bidx):
        """The same by the literal O(N*V) scan."""
        return self._closest(self._lib.oracle_select_closest_literal, task_id, acc_bp, lat_us, cost,
                             queue_us, q_task, q_slo, q_min_acc, q_bidx)

    def select_tiered(self, task_id, acc_bp, lat_us, cost, queue_us, state, load_us,
                      q_task, q_slo, q_min_acc, q_bidx, literal=False):
        """(variant or -1, tier 1 = Active / 2 = Inactive / 0 = none) per query."""
        task_id, acc_bp, queue_us = _i32(task_id), _i32(acc_bp), _i32(queue_us)
        lat_us, cost, state, load_us = _i32(lat_us), _i32(cost), _i32(state), _i32(load_us)
        V, B = lat_us.shape
        assert cost.shape == lat_us.shape
        for a in (task_id, acc_bp, queue_us, state, load_us):
            assert a.shape == (V,)
        q_task, q_slo, q_min_acc, q_bidx = _i32(q_task), _i32(q_slo), _i32(q_min_acc), _i32(q_bidx)
        N = q_task.shape[0]
        out = np.empty(N, dtype=np.int32)
        tier = np.empty(N, dtype=np.int32)
        fn = self._lib.oracle_select_tiered_literal if literal else self._lib.oracle_select_tiered
        rc = fn(V, B, _ptr(task_id), _ptr(acc_bp), _ptr(lat_us), _ptr(cost),
                                            _ptr(queue_us), _ptr(state), _ptr(load_us), N, _ptr(q_task),
                                            _ptr(q_slo), _ptr(q_min_acc), _ptr(q_bidx), _ptr(out), _ptr(tier))
        if rc != 0:
            raise ValueError("oracle rejected its arguments")
        return out, tier

    def select_case1(self, task_id, acc_bp, lat_us, cost, queue_us, state, load_us,
                     q_task, q_slo, q_min_acc, q_bidx, literal=False):
        """(variant or -1, tier, suggestion) per query: the state-aware selection and, where it
        finds nothing, the closest Active or Inactive variant."""
        task_id, acc_bp, queue_us = _i32(task_id), _i32(acc_bp), _i32(queue_us)
        lat_us, cost, state, load_us = _i32(lat_us), _i32(cost), _i32(state), _i32(load_us)
        V, B = lat_us.shape
        assert cost.shape == lat_us.shape
        for a in (task_id, acc_bp, queue_us, state, load_us):
            assert a.shape == (V,)
        q_task, q_slo, q_min_acc, q_bidx = _i32(q_task), _i32(q_slo), _i32(q_min_acc), _i32(q_bidx)
        N = q_task.shape[0]
        out, tier, closest = (np.empty(N, dtype=np.int32) for _ in range(3))
        fn = self._lib.oracle_select_case1_literal if literal else self._lib.oracle_select_case1
        rc = fn(V, B, _ptr(task_id), _ptr(acc_bp), _ptr(lat_us), _ptr(cost), _ptr(queue_us), _ptr(state),
                _ptr(load_us), N, _ptr(q_task), _ptr(q_slo), _ptr(q_min_acc), _ptr(q_bidx), _ptr(out), _ptr(tier),
                _ptr(closest))
        if rc != 0:
            raise ValueError("oracle rejected its arguments")
        return out, tier, closest

    def select_workers(self, task_id, acc_bp, lat_us, cost, queue_us, state, load_us, variant_hw,
                       worker_hw, worker_util, inst_variant, inst_worker, inst_load,
                       q_task, q_slo, q_min_acc, q_bidx, literal=False):
        """(variant or -1, tier, worker or -1) per query: the state-aware selection followed by
        the choice of the worker."""
        task_id, acc_bp, queue_us = _i32(task_id), _i32(acc_bp), _i32(queue_us)
        lat_us, cost, state, load_us = _i32(lat_us), _i32(cost), _i32(state), _i32(load_us)
        variant_hw, worker_hw, worker_util = _i32(variant_hw), _i32(worker_hw), _i32(worker_util)
        inst_variant, inst_worker, inst_load = _i32(inst_variant), _i32(inst_worker), _i32(inst_load)
        V, B = lat_us.shape
        assert cost.shape == lat_us.shape
        for a in (task_id, acc_bp, queue_us, state, load_us, variant_hw):
            assert a.shape == (V,)
        W, n_inst = worker_hw.shape[0], inst_variant.shape[0]
        assert worker_util.shape == (W,) and inst_worker.shape == (n_inst,) and inst_load.shape == (n_inst,)
        q_task, q_slo, q_min_acc, q_bidx = _i32(q_task), _i32(q_slo), _i32(q_min_acc), _i32(q_bidx)
        N = q_task.shape[0]
        out, tier, worker = (np.empty(N, dtype=np.int32) for _ in range(3))
        fn = self._lib.oracle_select_workers_literal if literal else self._lib.oracle_select_workers
        rc = fn(V, B, _ptr(task_id), _ptr(acc_bp), _ptr(lat_us), _ptr(cost), _ptr(queue_us), _ptr(state),
                _ptr(load_us), _ptr(variant_hw), W, _ptr(worker_hw), _ptr(worker_util),
                n_inst, _ptr(inst_variant), _ptr(inst_worker), _ptr(inst_load),
                N, _ptr(q_task), _ptr(q_slo), _ptr(q_min_acc), _ptr(q_bidx), _ptr(out), _ptr(tier), _ptr(worker))
        if rc != 0:
            raise ValueError("oracle rejected its arguments")
        return out, tier, worker

    def update_worker_util(self, worker_util: np.ndarray, worker_idx, new_util) -> None:
        """In place: worker_util[worker_idx[i]] = new_util[i], array order, invalid entries skipped."""
        assert worker_util.dtype == np.int32 and worker_util.flags["C_CONTIGUOUS"]
        worker_idx, new_util = _i32(worker_idx), _i32(new_util)
        self._lib.oracle_update_worker_util(worker_util.shape[0], _ptr(worker_util), worker_idx.shape[0],
                                            _ptr(worker_idx), _ptr(new_util))

    def update_instance_load(self, inst_load: np.ndarray, inst_idx, new_load) -> None:
        """In place: inst_load[inst_idx[i]] = new_load[i], array order, invalid entries skipped."""
        assert inst_load.dtype == np.int32 and inst_load.flags["C_CONTIGUOUS"]
        inst_idx, new_load = _i32(inst_idx), _i32(new_load)
        self._lib.oracle_update_instance_load(inst_load.shape[0], _ptr(inst_load), inst_idx.shape[0],
                                              _ptr(inst_idx), _ptr(new_load))

    def derive_states(self, num_variants, inst_variant, inst_state):
        """State of every variant from the states of its instances (Inactive without any)."""
        inst_variant, inst_state = _i32(inst_variant), _i32(inst_state)
        assert inst_variant.shape == inst_state.shape
        out = np.empty(num_variants, dtype=np.int32)
        if self._lib.oracle_derive_states(num_variants, inst_variant.shape[0], _ptr(inst_variant), _ptr(inst_state),
                                          _ptr(out)) != 0:
            raise ValueError("oracle rejected its arguments")
        return out

    def select_instances(self, task_id, acc_bp, lat_us, cost, queue_us, load_us, variant_hw,
                         worker_hw, worker_util, inst_variant, inst_worker, inst_load, inst_state,
                         q_task, q_slo, q_min_acc, q_bidx, literal=False):
        """(variant or -1, tier, worker or -1) per query with the state kept per running instance."""
        task_id, acc_bp, queue_us = _i32(task_id), _i32(acc_bp), _i32(queue_us)
        lat_us, cost, load_us = _i32(lat_us), _i32(cost), _i32(load_us)
        variant_hw, worker_hw, worker_util = _i32(variant_hw), _i32(worker_hw), _i32(worker_util)
        inst_variant, inst_worker = _i32(inst_variant), _i32(inst_worker)
        inst_load, inst_state = _i32(inst_load), _i32(inst_state)
        V, B = lat_us.shape
        assert cost.shape == lat_us.shape
        for a in (task_id, acc_bp, queue_us, load_us, variant_hw):
            assert a.shape == (V,)
        W, n_inst = worker_hw.shape[0], inst_variant.shape[0]
        assert worker_util.shape == (W,)
        for a in (inst_worker, inst_load, inst_state):
            assert a.shape == (n_inst,)
        q_task, q_slo, q_min_acc, q_bidx = _i32(q_task), _i32(q_slo), _i32(q_min_acc), _i32(q_bidx)
        N = q_task.shape[0]
        out, tier, worker = (np.empty(N, dtype=np.int32) for _ in range(3))
        rc = self._lib.oracle_select_instances(
            V, B, _ptr(task_id), _ptr(acc_bp), _ptr(lat_us), _ptr(cost), _ptr(queue_us), _ptr(load_us), _ptr(variant_hw),
            W, _ptr(worker_hw), _ptr(worker_util), n_inst, _ptr(inst_variant), _ptr(inst_worker), _ptr(inst_load),
            _ptr(inst_state), 1 if literal else 0, N, _ptr(q_task), _ptr(q_slo), _ptr(q_min_acc), _ptr(q_bidx),
            _ptr(out), _ptr(tier), _ptr(worker))
        if rc != 0:
            raise ValueError("oracle rejected its arguments")
        return out, tier, worker

    def get_variant(self, task_id, acc_bp, lat_us, cost, queue_us, state, load_us, variant_hw,
                    worker_hw, worker_util, inst_variant, inst_worker, inst_load,
                    q_task, q_slo, q_min_acc, q_bidx, inst_state=None, literal=False):
        """The whole of Case I (Section 4.1) per query: (variant or -1, tier, worker or -1, variant or
        suggestion).  Nothing is computed here: variant, tier and worker are those of select_workers
        (select_instances when the state is kept per instance: `state` is then ignored and the
        variants' states are the derived ones), the fourth array is that of select_case1 on the
        same states; both routines make the same state-aware selection, which is checked."""
        table = (task_id, acc_bp, lat_us, cost, queue_us)
        cluster = (worker_hw, worker_util, inst_variant, inst_worker, inst_load)
        queries = (q_task, q_slo, q_min_acc, q_bidx)
        if inst_state is None:
            out, tier, worker = self.select_workers(*table, state, load_us, variant_hw, *cluster, *queries,
                                                    literal=literal)
        else:
            out, tier, worker = self.select_instances(*table, load_us, variant_hw, *cluster, inst_state, *queries,
                                                      literal=literal)
            state = self.derive_states(_i32(task_id).shape[0], inst_variant, inst_state)
        out2, tier2, closest = self.select_case1(*table, state, load_us, *queries, literal=literal)
        if not (np.array_equal(out, out2) and np.array_equal(tier, tier2)):
            raise AssertionError("the two routines disagree on the state-aware selection")
        return out, tier, worker, closest

    def update_instance_state(self, inst_state: np.ndarray, inst_idx, new_state) -> None:
        """In place: inst_state[inst_idx[i]] = new_state[i], array order, invalid entries skipped."""
        assert inst_state.dtype == np.int32 and inst_state.flags["C_CONTIGUOUS"]
        inst_idx, new_state = _i32(inst_idx), _i32(new_state)
        self._lib.oracle_update_instance_state(inst_state.shape[0], _ptr(inst_state), inst_idx.shape[0],
                                               _ptr(inst_idx), _ptr(new_state))

    def scale(self, arch_id, sat_qps, hw_cost, load_us, lat_us, lambda_per_s, slack_pct,
              r_variant, r_instances, r_load_qps, r_slo, r_bidx, down=False):
        """Scaling decision per request: (action 0 none / 1 replicate / 2 upgrade / 3 impossible,
        variant to load or -1, instances of it to load).  down=True: the scaling-down decision,
        (action 0 keep / 1 remove / 2 downgrade, variant concerned or -1, instances to unload resp. load)."""
        arch_id, sat_qps, hw_cost, load_us = _i32(arch_id), _i32(sat_qps), _i32(hw_cost), _i32(load_us)
        lat_us = _i32(lat_us)
        V, B = lat_us.shape
        for a in (arch_id, sat_qps, hw_cost, load_us):
            assert a.shape == (V,)
        r_variant, r_instances, r_load_qps = _i32(r_variant), _i32(r_instances), _i32(r_load_qps)
        r_slo, r_bidx = _i32(r_slo), _i32(r_bidx)
        R = r_variant.shape[0]
        for a in (r_instances, r_load_qps, r_slo, r_bidx):
            assert a.shape == (R,)
        action, variant, inst = (np.empty(R, dtype=np.int32) for _ in range(3))
        routine = self._lib.oracle_scale_down if down else self._lib.oracle_scale
        rc = routine(V, B, _ptr(arch_id), _ptr(sat_qps), _ptr(hw_cost), _ptr(load_us), _ptr(lat_us),
                     int(lambda_per_s), int(slack_pct), R, _ptr(r_variant), _ptr(r_instances),
                     _ptr(r_load_qps), _ptr(r_slo), _ptr(r_bidx), _ptr(action), _ptr(variant), _ptr(inst))
        if rc != 0:
            raise ValueError("oracle rejected its arguments")
        return action, variant, inst

    def scale_down(self, *args):
        """Section 4.2.2, scaling down: see scale(..., down=True)."""
        return self.scale(*args, down=True)

    def update_state(self, state: np.ndarray, variant_idx, new_state) -> None:
        """In place: state[variant_idx[i]] = new_state[i], array order."""
        assert state.dtype == np.int32 and state.flags["C_CONTIGUOUS"]
        variant_idx, new_state = _i32(variant_idx), _i32(new_state)
        self._lib.oracle_update_state(state.shape[0], _ptr(state), variant_idx.shape[0],
                                      _ptr(variant_idx), _ptr(new_state))

    def count_feasible(self, task_id, acc_bp, lat_us, queue_us, q_task, q_slo, q_min_acc, q_bidx):
        task_id, acc_bp, queue_us, lat_us = _i32(task_id), _i32(acc_bp), _i32(queue_us), _i32(lat_us)
        V, B = lat_us.shape
        q_task, q_slo, q_min_acc, q_bidx = _i32(q_task), _i32(q_slo), _i32(q_min_acc), _i32(q_bidx)
        N = q_task.shape[0]
        out = np.empty(N, dtype=np.int32)
        rc = self._lib.oracle_count_feasible(V, B, _ptr(task_id), _ptr(acc_bp), _ptr(lat_us),
                                             _ptr(queue_us), N, _ptr(q_task), _ptr(q_slo),
                                             _ptr(q_min_acc), _ptr(q_bidx), _ptr(out))
        if rc != 0:
            raise ValueError("oracle rejected its arguments")
        return out

    def update_load(self, queue_us: np.ndarray, variant_idx, new_queue_us) -> None:
        """In place: queue_us[variant_idx[i]] = new_queue_us[i], array order."""
        assert queue_us.dtype == np.int32 and queue_us.flags["C_CONTIGUOUS"]
        variant_idx, new_queue_us = _i32(variant_idx), _i32(new_queue_us)
        assert variant_idx.shape == new_queue_us.shape
        self._lib.oracle_update_load(queue_us.shape[0], _ptr(queue_us), variant_idx.shape[0],
                                     _ptr(variant_idx), _ptr(new_queue_us))


_cached: Optional[Oracle] = None


def load_oracle() -> Oracle:
    """The oracle built from the committed source (compiled on first use)."""
    global _cached
    if _cached is None:
        _cached = Oracle(build_oracle(force=False))
    return _cached
