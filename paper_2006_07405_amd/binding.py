"""Thin ctypes binding of liba2sgd.so: the same names as the C ABI in include/a2sgd.h, argument marshalling only.

Tensors are torch CUDA tensors used as plain device memory (data_ptr) and the current torch stream supplies
the hipStream_t.  Every step of the path runs inside the library's kernels.  There is no fallback: if the
shared library is missing or fails to load, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liba2sgd.so")

A2SGD_MAX_WORKERS = 64
(A2SGD_OK, A2SGD_ERR_INVALID_ARG, A2SGD_ERR_ALIGNMENT, A2SGD_ERR_DEVICE, A2SGD_ERR_NOMEM, A2SGD_ERR_WORKSPACE_TOO_SMALL,
 A2SGD_ERR_WORKSPACE_STATE, A2SGD_ERR_SCRATCH_LIMIT) = range(8)
A2SGD_STATIC_SCRATCH_BYTES = 256 * 1024
A2SGD_MODE_RETAINED_ERROR, A2SGD_MODE_ALG1_LITERAL = 0, 1


class a2sgd_config_t(C.Structure):
    _fields_ = [("n", C.c_uint64), ("num_workers", C.c_uint32), ("mode", C.c_int32),
                ("blocks_per_worker", C.c_uint32), ("num_segments", C.c_uint32),
                ("seg_length", C.POINTER(C.c_uint64)), ("seg_offset", C.POINTER(C.c_uint64)),
                ("pooled_means", C.c_uint32), ("device", C.c_int32)]


class a2sgd_worker_stats_t(C.Structure):
    _fields_ = [("mu_pos", C.c_float), ("mu_neg", C.c_float), ("n_pos", C.c_uint64), ("n_neg", C.c_uint64),
                ("n_zero", C.c_uint64), ("n_nan", C.c_uint64)]


class a2sgd_global_stats_t(C.Structure):
    _fields_ = [("gmu_pos", C.c_float), ("gmu_neg", C.c_float)]


class a2sgd_device_info_t(C.Structure):
    _fields_ = [("compute_units", C.c_uint32), ("memory_clock_khz", C.c_uint32), ("memory_bus_bits", C.c_uint32),
                ("reserved", C.c_uint32), ("total_memory_bytes", C.c_uint64),
                ("l2_bytes", C.c_uint64)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, u64p = C.c_void_p, C.POINTER(C.c_uint64)
    tab = C.POINTER(C.c_void_p)
    L.a2sgd_plan.argtypes = [C.POINTER(a2sgd_config_t), C.POINTER(vp)]
    L.a2sgd_plan_destroy.argtypes = [vp]
    L.a2sgd_workspace_bytes.argtypes = [vp]
    L.a2sgd_workspace_bytes.restype = C.c_size_t
    L.a2sgd_plan_blocks_per_worker.argtypes = [vp]
    L.a2sgd_plan_blocks_per_worker.restype = C.c_uint32
    L.a2sgd_plan_single_launch_cell.argtypes = [vp]
    L.a2sgd_plan_single_launch_cell.restype = C.c_int32
    L.a2sgd_workspace_check.argtypes = [vp, vp, C.c_size_t]
    L.a2sgd_workspace_check.restype = C.c_int
    L.a2sgd_local_averages.argtypes = [vp, tab, tab, vp, vp]
    L.a2sgd_global_average.argtypes = [vp, vp, vp]
    L.a2sgd_apply_and_update_error.argtypes = [vp, tab, tab, vp, C.c_float, vp, vp]
    L.a2sgd_step.argtypes = [vp, tab, tab, vp, C.c_float, vp, vp]
    L.a2sgd_step_static.argtypes = [vp, tab, tab, vp, C.c_float, vp]
    L.a2sgd_step_static.restype = C.c_int
    L.a2sgd_read_stats.argtypes = [vp, vp, vp, C.POINTER(a2sgd_worker_stats_t), C.POINTER(a2sgd_global_stats_t)]
    L.a2sgd_export_mask.argtypes = [vp, tab, tab, vp, vp]
    L.a2sgd_dense_step.argtypes = [vp, tab, vp, C.c_float, vp]
    L.a2sgd_apply_and_update_error_replicas.argtypes = [vp, tab, tab, tab, C.c_float, vp, vp]
    L.a2sgd_step_replicas.argtypes = [vp, tab, tab, tab, C.c_float, vp, vp]
    L.a2sgd_dense_step_replicas.argtypes = [vp, tab, tab, C.c_float, vp]
    L.a2sgd_replica_drift.argtypes = [vp, tab, vp, vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    L.a2sgd_lazy_reset.argtypes = [vp, vp, vp]
    L.a2sgd_lazy_step.argtypes = [vp, tab, tab, vp, C.c_float, vp, vp]
    L.a2sgd_lazy_local_averages.argtypes = [vp, tab, tab, vp, vp]
    L.a2sgd_lazy_apply.argtypes = [vp, tab, vp, C.c_float, vp, vp]
    L.a2sgd_lazy_materialize.argtypes = [vp, tab, vp, vp]
    L.a2sgd_selftest_barrier.argtypes = [vp, vp]
    L.a2sgd_selftest_barrier.restype = C.c_int
    L.a2sgd_workspace_init.argtypes = [vp, vp, vp]
    L.a2sgd_workspace_init.restype = C.c_int
    L.a2sgd_read_segment_stats.argtypes = [vp, vp, vp, C.POINTER(a2sgd_worker_stats_t),
                                           C.POINTER(a2sgd_global_stats_t)]
    L.a2sgd_read_segment_stats.restype = C.c_int
    L.a2sgd_device_info.argtypes = [C.POINTER(a2sgd_device_info_t)]
    L.a2sgd_export_local_means.argtypes = [vp, vp, vp, vp]
    L.a2sgd_import_global_means.argtypes = [vp, vp, vp, vp]
    L.a2sgd_status_string.argtypes = [C.c_int]
    L.a2sgd_status_string.restype = C.c_char_p
    for name in ("a2sgd_plan", "a2sgd_plan_destroy", "a2sgd_local_averages", "a2sgd_global_average",
                 "a2sgd_apply_and_update_error", "a2sgd_step", "a2sgd_read_stats", "a2sgd_export_mask",
                 "a2sgd_dense_step", "a2sgd_apply_and_update_error_replicas", "a2sgd_step_replicas",
                 "a2sgd_dense_step_replicas", "a2sgd_replica_drift", "a2sgd_lazy_reset", "a2sgd_lazy_step",
                 "a2sgd_lazy_materialize"):
        getattr(L, name).restype = C.c_int
    return L


raw = _load()  # the bare ctypes library, for tests that pass hand-made pointers


class A2sgdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {raw.a2sgd_status_string(status).decode()} (status {status})")


def _check(status: int, where: str) -> None:
    if status != A2SGD_OK:
        raise A2sgdError(status, where)


class Plan:
    """Owns an a2sgd_plan_t*; remembers n and P so the binding can check tensor shapes before marshalling."""

    def __init__(self, handle: int, n: int, num_workers: int, mode: int, num_segments: int = 0):
        self.handle, self.n, self.num_workers, self.mode = handle, n, num_workers, mode
        self.num_segments = num_segments
        self.workspace_bytes = int(raw.a2sgd_workspace_bytes(handle))  # fixed by the plan

    def __del__(self):
        if getattr(self, "handle", None):
            raw.a2sgd_plan_destroy(self.handle)
            self.handle = None


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev_ptr(t: torch.Tensor, numel: Optional[int], dtype, what: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{what}: expected a contiguous CUDA tensor of {dtype}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"{what}: {t.numel()} elements, the plan needs {numel}")
    return t.data_ptr()


def _table(plan: Plan, ts: Optional[Sequence[torch.Tensor]], what: str):
    if ts is None:
        return None
    if len(ts) != plan.num_workers:
        raise ValueError(f"{what}: {len(ts)} buffers for a plan of {plan.num_workers} workers")
    return (C.c_void_p * plan.num_workers)(*[_dev_ptr(t, plan.n, torch.float32, f"{what}[{i}]")
                                             for i, t in enumerate(ts)])


def _workspace(plan: Plan, ws: torch.Tensor) -> int:
    if not (isinstance(ws, torch.Tensor) and ws.is_cuda and ws.is_contiguous()):
        raise TypeError("workspace: expected a contiguous CUDA tensor")
    _check(raw.a2sgd_workspace_check(plan.handle, ws.data_ptr(), ws.numel() * ws.element_size()), "workspace")
    return ws.data_ptr()


def a2sgd_workspace_check(plan: Plan, workspace: torch.Tensor) -> None:
    """Raises A2sgdError (A2SGD_ERR_WORKSPACE_TOO_SMALL, ...) unless the tensor can serve as the plan's workspace."""
    _workspace(plan, workspace)


def a2sgd_plan(n: int, num_workers: int, mode: int = A2SGD_MODE_RETAINED_ERROR, blocks_per_worker: int = 0,
               seg_lengths: Optional[Sequence[int]] = None, seg_offsets: Optional[Sequence[int]] = None,
               pooled_means: bool = False, device: int = -1) -> Plan:
    """seg_lengths: tensor sizes in address order; None = the whole range [0, n) with whole-model means.
    seg_offsets: their start indices (None = packed back to back from 0, sizes summing to n); elements outside every
    tensor are padding.  pooled_means: one pair of means per worker over all tensors instead of one per tensor.
    device: HIP device index that every launching call must find current, or -1 for no check."""
    S = len(seg_lengths) if seg_lengths is not None else 0
    arr = (C.c_uint64 * S)(*[int(x) for x in seg_lengths]) if S else None
    if seg_offsets is not None and len(seg_offsets) != S:
        raise ValueError("seg_offsets: one start index per tensor")
    off = (C.c_uint64 * S)(*[int(x) for x in seg_offsets]) if (S and seg_offsets is not None) else None
    cfg = a2sgd_config_t(n, num_workers, mode, blocks_per_worker, S, arr, off, 1 if pooled_means else 0, device)
    h = C.c_void_p()
    _check(raw.a2sgd_plan(C.byref(cfg), C.byref(h)), "a2sgd_plan")
    return Plan(h.value, n, num_workers, mode, S)


def a2sgd_workspace_bytes(plan: Plan) -> int:
    return int(raw.a2sgd_workspace_bytes(plan.handle))


def a2sgd_device_info() -> dict:
    info = a2sgd_device_info_t()
    _check(raw.a2sgd_device_info(C.byref(info)), "a2sgd_device_info")
    return {name: getattr(info, name) for name, _ in a2sgd_device_info_t._fields_ if name != "reserved"}


def a2sgd_plan_blocks_per_worker(plan: Plan) -> int:
    return int(raw.a2sgd_plan_blocks_per_worker(plan.handle))


def a2sgd_plan_single_launch_cell(plan: Plan) -> int:
    return int(raw.a2sgd_plan_single_launch_cell(plan.handle))


def alloc_workspace(plan: Plan, device="cuda") -> torch.Tensor:
    """Convenience for callers that let torch own the memory: a device buffer of the right size, with the plan's
    segment tables uploaded when it has any (a2sgd_workspace_init); otherwise uninitialised."""
    ws = torch.empty((a2sgd_workspace_bytes(plan) + 7) // 8, dtype=torch.int64, device=device)
    if plan.num_segments:
        a2sgd_workspace_init(plan, ws)
    return ws


def a2sgd_workspace_init(plan: Plan, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_workspace_init(plan.handle, _workspace(plan, workspace), _stream(stream)), "a2sgd_workspace_init")


def a2sgd_read_segment_stats(plan: Plan, workspace: torch.Tensor, stream=None):
    """Returns (stats[p][s] as WorkerStats, [(gmu_pos, gmu_neg)] * S).  Synchronises the stream."""
    P, S = plan.num_workers, plan.num_segments
    ws = (a2sgd_worker_stats_t * (P * S))()
    gs = (a2sgd_global_stats_t * S)()
    _check(raw.a2sgd_read_segment_stats(plan.handle, _workspace(plan, workspace), _stream(stream), ws, gs),
           "a2sgd_read_segment_stats")
    stats = [[WorkerStats(ws[p * S + s].mu_pos, ws[p * S + s].mu_neg, ws[p * S + s].n_pos, ws[p * S + s].n_neg,
                          ws[p * S + s].n_zero, ws[p * S + s].n_nan) for s in range(S)] for p in range(P)]
    return stats, [(x.gmu_pos, x.gmu_neg) for x in gs]


def a2sgd_local_averages(plan: Plan, g, e, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_local_averages(plan.handle, _table(plan, g, "g"), _table(plan, e, "e"),
                                    _workspace(plan, workspace), _stream(stream)), "a2sgd_local_averages")


def a2sgd_global_average(plan: Plan, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_global_average(plan.handle, _workspace(plan, workspace), _stream(stream)),
           "a2sgd_global_average")


def a2sgd_export_local_means(plan: Plan, workspace: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    """out: a CUDA float32 tensor of 2 * P elements; receives (mu_pos, mu_neg) of every worker of this plan."""
    _check(raw.a2sgd_export_local_means(plan.handle, _workspace(plan, workspace),
                                        _dev_ptr(out, 2 * plan.num_workers, torch.float32, "out"), _stream(stream)),
           "a2sgd_export_local_means")


def a2sgd_import_global_means(plan: Plan, workspace: torch.Tensor, gmu: torch.Tensor, stream=None) -> None:
    """gmu: a CUDA float32 tensor of 2 elements, (gmu_pos, gmu_neg) averaged over all workers of the job."""
    _check(raw.a2sgd_import_global_means(plan.handle, _workspace(plan, workspace),
                                         _dev_ptr(gmu, 2, torch.float32, "gmu"), _stream(stream)),
           "a2sgd_import_global_means")


def a2sgd_apply_and_update_error(plan: Plan, g, e, w: torch.Tensor, eta: float, workspace: torch.Tensor,
                                 stream=None) -> None:
    _check(raw.a2sgd_apply_and_update_error(plan.handle, _table(plan, g, "g"), _table(plan, e, "e"),
                                            _dev_ptr(w, plan.n, torch.float32, "w"), C.c_float(eta),
                                            _workspace(plan, workspace), _stream(stream)),
           "a2sgd_apply_and_update_error")


def a2sgd_step(plan: Plan, g, e, w: torch.Tensor, eta: float, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_step(plan.handle, _table(plan, g, "g"), _table(plan, e, "e"),
                          _dev_ptr(w, plan.n, torch.float32, "w"), C.c_float(eta), _workspace(plan, workspace),
                          _stream(stream)), "a2sgd_step")


def a2sgd_step_static(plan: Plan, g, e, w: torch.Tensor, eta: float, stream=None) -> None:
    """The three passes of one step on the library's built-in scratch array: no workspace, no allocation."""
    _check(raw.a2sgd_step_static(plan.handle, _table(plan, g, "g"), _table(plan, e, "e"),
                                 _dev_ptr(w, plan.n, torch.float32, "w"), C.c_float(eta), _stream(stream)),
           "a2sgd_step_static")


@dataclass
class WorkerStats:
    mu_pos: float
    mu_neg: float
    n_pos: int
    n_neg: int
    n_zero: int
    n_nan: int


def a2sgd_read_stats(plan: Plan, workspace: torch.Tensor, stream=None):
    """Returns ([WorkerStats] * P, (gmu_pos, gmu_neg)).  Synchronises the stream."""
    ws = (a2sgd_worker_stats_t * plan.num_workers)()
    gs = a2sgd_global_stats_t()
    _check(raw.a2sgd_read_stats(plan.handle, _workspace(plan, workspace), _stream(stream), ws, C.byref(gs)),
           "a2sgd_read_stats")
    return ([WorkerStats(s.mu_pos, s.mu_neg, s.n_pos, s.n_neg, s.n_zero, s.n_nan) for s in ws],
            (gs.gmu_pos, gs.gmu_neg))


def a2sgd_export_mask(plan: Plan, g, e, mask: torch.Tensor, stream=None) -> None:
    words = plan.num_workers * ((plan.n + 63) // 64)
    _check(raw.a2sgd_export_mask(plan.handle, _table(plan, g, "g"), _table(plan, e, "e"),
                                 _dev_ptr(mask, words, torch.int64, "mask"), _stream(stream)), "a2sgd_export_mask")


def a2sgd_dense_step(plan: Plan, g, w: torch.Tensor, eta: float, stream=None) -> None:
    _check(raw.a2sgd_dense_step(plan.handle, _table(plan, g, "g"), _dev_ptr(w, plan.n, torch.float32, "w"),
                                C.c_float(eta), _stream(stream)), "a2sgd_dense_step")


def a2sgd_apply_and_update_error_replicas(plan: Plan, g, e, w, eta: float, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_apply_and_update_error_replicas(plan.handle, _table(plan, g, "g"), _table(plan, e, "e"),
                                                     _table(plan, w, "w"), C.c_float(eta),
                                                     _workspace(plan, workspace), _stream(stream)),
           "a2sgd_apply_and_update_error_replicas")


def a2sgd_step_replicas(plan: Plan, g, e, w, eta: float, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_step_replicas(plan.handle, _table(plan, g, "g"), _table(plan, e, "e"), _table(plan, w, "w"),
                                   C.c_float(eta), _workspace(plan, workspace), _stream(stream)), "a2sgd_step_replicas")


def a2sgd_dense_step_replicas(plan: Plan, g, w, eta: float, stream=None) -> None:
    _check(raw.a2sgd_dense_step_replicas(plan.handle, _table(plan, g, "g"), _table(plan, w, "w"), C.c_float(eta),
                                         _stream(stream)), "a2sgd_dense_step_replicas")


def a2sgd_replica_drift(plan: Plan, w, workspace: torch.Tensor, stream=None):
    """Returns (max_abs[P], rms[P]) of w^p - mean_p w^p.  Synchronises the stream."""
    mx = (C.c_double * plan.num_workers)()
    rms = (C.c_double * plan.num_workers)()
    _check(raw.a2sgd_replica_drift(plan.handle, _table(plan, w, "w"), _workspace(plan, workspace), _stream(stream),
                                   mx, rms), "a2sgd_replica_drift")
    return list(mx), list(rms)


def a2sgd_lazy_reset(plan: Plan, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_lazy_reset(plan.handle, _workspace(plan, workspace), _stream(stream)), "a2sgd_lazy_reset")


def a2sgd_lazy_step(plan: Plan, g, s, w: torch.Tensor, eta: float, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_lazy_step(plan.handle, _table(plan, g, "g"), _table(plan, s, "s"),
                               _dev_ptr(w, plan.n, torch.float32, "w"), C.c_float(eta), _workspace(plan, workspace),
                               _stream(stream)), "a2sgd_lazy_step")


def a2sgd_lazy_local_averages(plan: Plan, g, s, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_lazy_local_averages(plan.handle, _table(plan, g, "g"), _table(plan, s, "s"),
                                         _workspace(plan, workspace), _stream(stream)), "a2sgd_lazy_local_averages")


def a2sgd_lazy_apply(plan: Plan, s, w: torch.Tensor, eta: float, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_lazy_apply(plan.handle, _table(plan, s, "s"), _dev_ptr(w, plan.n, torch.float32, "w"),
                                C.c_float(eta), _workspace(plan, workspace), _stream(stream)), "a2sgd_lazy_apply")


def a2sgd_lazy_materialize(plan: Plan, s, workspace: torch.Tensor, stream=None) -> None:
    _check(raw.a2sgd_lazy_materialize(plan.handle, _table(plan, s, "s"), _workspace(plan, workspace),
                                      _stream(stream)), "a2sgd_lazy_materialize")


def a2sgd_selftest_barrier(scratch: torch.Tensor, stream=None) -> None:
    if not (isinstance(scratch, torch.Tensor) and scratch.is_cuda and scratch.numel() * scratch.element_size() >= 4096):
        raise ValueError("scratch: at least 4 KiB of device memory")
    _check(raw.a2sgd_selftest_barrier(scratch.data_ptr(), _stream(stream)), "a2sgd_selftest_barrier")
