"""TEST INFRASTRUCTURE — ctypes front end of the plain CPU oracle in a2sgd_oracle.c.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module; the product never
does, and this module imports nothing of the product.  All arithmetic lives in the C file; this file only
marshals numpy arrays, and strings the C calls together in the order of Algorithm 1 (lines 3-7).
"""
from __future__ import annotations

import contextlib
import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "a2sgd_oracle.c")
_LIB = os.path.join(_HERE, "liba2sgd_oracle.so")

RETAINED_ERROR = 0
ALG1_LITERAL = 1


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off and no fast-math keep every operation IEEE-exact."""
    if force or not os.path.exists(_LIB):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", "-Wall",
                               "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class Acc(C.Structure):
    _fields_ = [("s_pos", C.c_longdouble), ("s_neg", C.c_longdouble),
                ("n_pos", C.c_uint64), ("n_neg", C.c_uint64), ("n_zero", C.c_uint64), ("n_nan", C.c_uint64)]


_lib = None
_FP = C.POINTER(C.c_float)
_FPP = C.POINTER(_FP)
_U8P = C.POINTER(C.c_uint8)
_U8PP = C.POINTER(_U8P)


def _bind(path: str):
    L = C.CDLL(path)
    L.a2sgd_oracle_acc_init.argtypes = [C.POINTER(Acc)]
    L.a2sgd_oracle_acc_init.restype = None
    L.a2sgd_oracle_accumulate.argtypes = [_FP, _FP, C.c_uint64, C.POINTER(Acc)]
    L.a2sgd_oracle_accumulate.restype = None
    L.a2sgd_oracle_local_means.argtypes = [C.POINTER(Acc), _FP, _FP]
    L.a2sgd_oracle_local_means.restype = None
    L.a2sgd_oracle_global_means.argtypes = [_FP, _FP, C.c_uint32, _FP, _FP]
    L.a2sgd_oracle_global_means.restype = None
    L.a2sgd_oracle_apply_chunk.argtypes = [_FPP, _FPP, C.c_uint32, C.c_uint64, _FP, _FP, C.c_float, C.c_float,
                                           C.c_float, C.c_int, _FPP, _FP, _FP, _U8PP]
    L.a2sgd_oracle_apply_chunk.restype = None
    L.a2sgd_oracle_dense_step.argtypes = [_FPP, C.c_uint32, C.c_uint64, C.c_float, _FP, _FP]
    L.a2sgd_oracle_dense_step.restype = None
    L.a2sgd_oracle_apply_chunk_replicas.argtypes = [_FPP, _FPP, C.c_uint32, C.c_uint64, _FP, _FP, C.c_float,
                                                    C.c_float, C.c_float, C.c_int, _FPP, _FPP, _FPP]
    L.a2sgd_oracle_apply_chunk_replicas.restype = None
    L.a2sgd_oracle_dense_step_replicas.argtypes = [_FPP, C.c_uint32, C.c_uint64, C.c_float, _FPP, _FPP]
    L.a2sgd_oracle_dense_step_replicas.restype = None
    L.a2sgd_oracle_replica_drift.argtypes = [_FPP, C.c_uint32, C.c_uint64, C.POINTER(C.c_double),
                                             C.POINTER(C.c_longdouble)]
    L.a2sgd_oracle_replica_drift.restype = None
    return L


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = _bind(_LIB)
    return _lib


@contextlib.contextmanager
def use_library(path: str):
    """Route every call through another build of the C file (mutation tests plant a mistake in a copy of
    the source, compile it, and check that the pins notice)."""
    global _lib
    saved = _lib
    _lib = _bind(path)
    try:
        yield
    finally:
        _lib = saved


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    assert a.ndim == 1
    return a


def _fp(a: Optional[np.ndarray]):
    return a.ctypes.data_as(_FP) if a is not None else _FP()


def _fpp(arrs: Sequence[Optional[np.ndarray]]):
    return (_FP * len(arrs))(*[_fp(a) for a in arrs])


@dataclass
class WorkerStats:
    mu_pos: float  # fp32 value, held as a Python float
    mu_neg: float
    n_pos: int
    n_neg: int
    n_zero: int
    n_nan: int


@dataclass
class StepResult:
    workers: List[WorkerStats]
    gmu_pos: float
    gmu_neg: float
    e_new: List[np.ndarray]
    w_new: np.ndarray
    mask: List[np.ndarray]  # uint8, 1 where v >= 0


class LocalAccumulator:
    """Pass A for one worker: feed chunks in index order, then read the local means."""

    def __init__(self):
        self.acc = Acc()
        lib().a2sgd_oracle_acc_init(C.byref(self.acc))

    def feed(self, g: np.ndarray, e: Optional[np.ndarray]) -> None:
        g = _f32(g)
        e = _f32(e) if e is not None else None
        assert e is None or e.shape == g.shape
        lib().a2sgd_oracle_accumulate(_fp(g), _fp(e), g.shape[0], C.byref(self.acc))

    def stats(self) -> WorkerStats:
        mp, mn = C.c_float(), C.c_float()
        lib().a2sgd_oracle_local_means(C.byref(self.acc), C.byref(mp), C.byref(mn))
        a = self.acc
        return WorkerStats(mp.value, mn.value, a.n_pos, a.n_neg, a.n_zero, a.n_nan)


def global_means(workers: Sequence[WorkerStats]):
    P = len(workers)
    mp = np.array([w.mu_pos for w in workers], dtype=np.float32)
    mn = np.array([w.mu_neg for w in workers], dtype=np.float32)
    gp, gn = C.c_float(), C.c_float()
    lib().a2sgd_oracle_global_means(_fp(mp), _fp(mn), P, C.byref(gp), C.byref(gn))
    return gp.value, gn.value


def apply_chunk(g: Sequence[np.ndarray], e: Optional[Sequence[Optional[np.ndarray]]], w: np.ndarray,
                workers: Sequence[WorkerStats], gmu_pos: float, gmu_neg: float, eta: float, mode: int):
    """Pass B on one chunk (same index range of every worker).  Returns (e_new list, w_new, mask list)."""
    P = len(g)
    g = [_f32(x) for x in g]
    m = g[0].shape[0]
    e_arr = [(_f32(x) if x is not None else None) for x in e] if e is not None else None
    w = _f32(w)
    assert all(x.shape[0] == m for x in g) and w.shape[0] == m
    e_new = [np.empty(m, dtype=np.float32) for _ in range(P)]
    mask = [np.empty(m, dtype=np.uint8) for _ in range(P)]
    w_new = np.empty(m, dtype=np.float32)
    mp = np.array([s.mu_pos for s in workers], dtype=np.float32)
    mn = np.array([s.mu_neg for s in workers], dtype=np.float32)
    maskp = (_U8P * P)(*[x.ctypes.data_as(_U8P) for x in mask])
    lib().a2sgd_oracle_apply_chunk(_fpp(g), _fpp(e_arr) if e_arr is not None else _FPP(), P, m, _fp(mp), _fp(mn),
                                   C.c_float(gmu_pos), C.c_float(gmu_neg), C.c_float(eta), int(mode),
                                   _fpp(e_new), _fp(w), _fp(w_new), maskp)
    return e_new, w_new, mask


def step(g: Sequence[np.ndarray], e: Optional[Sequence[Optional[np.ndarray]]], w: np.ndarray, eta: float,
         mode: int = RETAINED_ERROR, chunk: int = 1 << 22) -> StepResult:
    """One whole A2SGD step over in-memory arrays, processed chunk by chunk as the streamed form would."""
    P = len(g)
    n = int(np.asarray(g[0]).shape[0])
    workers = []
    for p in range(P):
        acc = LocalAccumulator()
        for lo in range(0, n, chunk):
            hi = min(n, lo + chunk)
            acc.feed(g[p][lo:hi], e[p][lo:hi] if (e is not None and e[p] is not None) else None)
        workers.append(acc.stats())
    gp, gn = global_means(workers)
    e_new = [np.empty(n, dtype=np.float32) for _ in range(P)]
    mask = [np.empty(n, dtype=np.uint8) for _ in range(P)]
    w_new = np.empty(n, dtype=np.float32)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        ec = [(x[lo:hi] if x is not None else None) for x in e] if e is not None else None
        en, wn, mk = apply_chunk([x[lo:hi] for x in g], ec, w[lo:hi], workers, gp, gn, eta, mode)
        for p in range(P):
            e_new[p][lo:hi] = en[p]
            mask[p][lo:hi] = mk[p]
        w_new[lo:hi] = wn
    return StepResult(workers, gp, gn, e_new, w_new, mask)


def dense_step(g: Sequence[np.ndarray], w: np.ndarray, eta: float) -> np.ndarray:
    """w - eta * mean_p g^p  (Eq. 1; Algorithm 1 lines 9-10)."""
    g = [_f32(x) for x in g]
    w = _f32(w)
    out = np.empty_like(w)
    lib().a2sgd_oracle_dense_step(_fpp(g), len(g), w.shape[0], C.c_float(eta), _fp(w), _fp(out))
    return out


def local_stats(g: Sequence[np.ndarray], e: Optional[Sequence[Optional[np.ndarray]]], chunk: int = 1 << 22):
    """Pass A for every worker of in-memory arrays: ([WorkerStats] * P, (gmu_pos, gmu_neg))."""
    workers = []
    n = int(np.asarray(g[0]).shape[0])
    for p in range(len(g)):
        acc = LocalAccumulator()
        for lo in range(0, n, chunk):
            hi = min(n, lo + chunk)
            acc.feed(g[p][lo:hi], e[p][lo:hi] if (e is not None and e[p] is not None) else None)
        workers.append(acc.stats())
    return workers, global_means(workers)


def step_replicas(g: Sequence[np.ndarray], e: Optional[Sequence[Optional[np.ndarray]]], w: Sequence[np.ndarray],
                  eta: float, mode: int = RETAINED_ERROR):
    """One step with one weight vector per worker (Algorithm 1 line 7 as printed).  Returns
    (workers, (gmu_pos, gmu_neg), e_new list, w_new list)."""
    P = len(g)
    g = [_f32(x) for x in g]
    m = g[0].shape[0]
    e_arr = [(_f32(x) if x is not None else None) for x in e] if e is not None else None
    w = [_f32(x) for x in w]
    workers, (gp, gn) = local_stats(g, e_arr)
    e_new = [np.empty(m, dtype=np.float32) for _ in range(P)]
    w_new = [np.empty(m, dtype=np.float32) for _ in range(P)]
    mp = np.array([s.mu_pos for s in workers], dtype=np.float32)
    mn = np.array([s.mu_neg for s in workers], dtype=np.float32)
    lib().a2sgd_oracle_apply_chunk_replicas(_fpp(g), _fpp(e_arr) if e_arr is not None else _FPP(), P, m, _fp(mp),
                                            _fp(mn), C.c_float(gp), C.c_float(gn), C.c_float(eta), int(mode),
                                            _fpp(e_new), _fpp(w), _fpp(w_new))
    return workers, (gp, gn), e_new, w_new


def dense_step_replicas(g: Sequence[np.ndarray], w: Sequence[np.ndarray], eta: float) -> List[np.ndarray]:
    g = [_f32(x) for x in g]
    w = [_f32(x) for x in w]
    out = [np.empty_like(x) for x in w]
    lib().a2sgd_oracle_dense_step_replicas(_fpp(g), len(g), g[0].shape[0], C.c_float(eta), _fpp(w), _fpp(out))
    return out


def replica_drift(w: Sequence[np.ndarray]):
    """(max_abs[P], rms[P]) of w[p] - mean_p w[p]."""
    w = [_f32(x) for x in w]
    P, m = len(w), w[0].shape[0]
    mx = (C.c_double * P)(*([0.0] * P))
    sq = (C.c_longdouble * P)(*([0.0] * P))
    lib().a2sgd_oracle_replica_drift(_fpp(w), P, m, mx, sq)
    return [float(x) for x in mx], [float(np.sqrt(float(x) / m)) for x in sq]


def step_segmented(g: Sequence[np.ndarray], e: Optional[Sequence[Optional[np.ndarray]]], w: np.ndarray, eta: float,
                   mode: int, seg_lengths: Sequence[int], seg_offsets: Optional[Sequence[int]] = None,
                   pooled: bool = False):
    """The step on buffers that consist of tensors (and possibly padding between them).

    pooled = False: the whole-model step applied to each tensor on its own, i.e. one pair of local means per worker
    AND tensor, averaged over the workers per tensor (the paper's operator of Eq. 2 and Algorithm 1 lines 3-7 with v
    restricted to one tensor).  pooled = True: the whole-model step applied to the tensors laid end to end, i.e.
    the paper's method on the model that the buffers hold, padding left out.  seg_lengths are the tensor sizes in
    address order, seg_offsets their start indices (None: packed back to back from 0, covering [0, n)).  Elements
    outside every tensor come back unchanged.  Returns (list of StepResult per tensor, or one-element list when
    pooled; e_new list; w_new)."""
    P = len(g)
    n = int(np.asarray(w).shape[0])
    lengths = [int(x) for x in seg_lengths]
    if seg_offsets is None:
        offsets = [int(x) for x in np.concatenate([[0], np.cumsum(lengths)[:-1]])]
        assert sum(lengths) == n
    else:
        offsets = [int(x) for x in seg_offsets]
    assert all(x > 0 for x in lengths) and all(offsets[k] + lengths[k] <= (offsets[k + 1] if k + 1 < len(offsets) else n)
                                              for k in range(len(offsets)))
    e_new = [np.array(x, dtype=np.float32, copy=True) if x is not None else np.zeros(n, np.float32) for x in e] \
        if e is not None else [np.zeros(n, np.float32) for _ in range(P)]
    w_new = np.array(w, dtype=np.float32, copy=True)
    ranges = [(o, o + l) for o, l in zip(offsets, lengths)]
    if pooled:
        cat = lambda x: np.concatenate([x[lo:hi] for lo, hi in ranges])
        r = step([cat(x) for x in g], [cat(x) for x in e] if e is not None else None, cat(w), eta, mode)
        pos = 0
        for lo, hi in ranges:
            for p in range(P):
                e_new[p][lo:hi] = r.e_new[p][pos:pos + hi - lo]
            w_new[lo:hi] = r.w_new[pos:pos + hi - lo]
            pos += hi - lo
        return [r], e_new, w_new
    per_seg = []
    for lo, hi in ranges:
        es = [x[lo:hi] for x in e] if e is not None else None
        r = step([x[lo:hi] for x in g], es, w[lo:hi], eta, mode)
        for p in range(P):
            e_new[p][lo:hi] = r.e_new[p]
        w_new[lo:hi] = r.w_new
        per_seg.append(r)
    return per_seg, e_new, w_new


def step_replicas_segmented(g: Sequence[np.ndarray], e: Optional[Sequence[Optional[np.ndarray]]], w: Sequence[np.ndarray],
                            eta: float, mode: int, seg_lengths: Sequence[int],
                            seg_offsets: Optional[Sequence[int]] = None, pooled: bool = False):
    """step_replicas on buffers that consist of tensors: one weight vector per worker, each tensor with its own means
    (pooled: one pair per worker over the tensors laid end to end).  The same slicing as step_segmented; elements
    outside every tensor come back unchanged.  Returns (e_new list, w_new list)."""
    P = len(g)
    n = int(np.asarray(w[0]).shape[0])
    lengths = [int(x) for x in seg_lengths]
    offsets = [int(x) for x in (seg_offsets if seg_offsets is not None else np.concatenate([[0], np.cumsum(lengths)[:-1]]))]
    ranges = [(o, o + l) for o, l in zip(offsets, lengths)]
    e_new = [np.array(x, dtype=np.float32, copy=True) for x in e] if e is not None else [np.zeros(n, np.float32) for _ in range(P)]
    w_new = [np.array(x, dtype=np.float32, copy=True) for x in w]
    if pooled:
        cat = lambda x: np.concatenate([x[lo:hi] for lo, hi in ranges])
        _, _, en, wn = step_replicas([cat(x) for x in g], [cat(x) for x in e] if e is not None else None,
                                     [cat(x) for x in w], eta, mode)
        pos = 0
        for lo, hi in ranges:
            for p in range(P):
                e_new[p][lo:hi] = en[p][pos:pos + hi - lo]
                w_new[p][lo:hi] = wn[p][pos:pos + hi - lo]
            pos += hi - lo
        return e_new, w_new
    for lo, hi in ranges:
        _, _, en, wn = step_replicas([x[lo:hi] for x in g], [x[lo:hi] for x in e] if e is not None else None,
                                     [x[lo:hi] for x in w], eta, mode)
        for p in range(P):
            e_new[p][lo:hi] = en[p]
            w_new[p][lo:hi] = wn[p]
    return e_new, w_new
