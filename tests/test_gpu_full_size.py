"""GPU parity at the full size of benchmark configurations 2-5 (config 1 runs its 10 steps in test_gpu_parity.py),
in the launch configuration bench.py times (the plan's own choice of geometry), every element of every output.

Inputs are generated on the GPU from the workload's seeds.  Both passes of the oracle stream: pass A (sums and
counts, which must be exact) takes every element of every worker in index order; pass B recomputes e and w chunk by
chunk, all chunks, on a pool of host threads (the oracle's C calls release the interpreter lock), and each chunk is
compared with the same index range of the GPU's outputs as soon as it is computed, so the host never holds more
than a few chunks of a 54 GB workload.  Copies of e and w from before the step stay on the GPU for that, since
the step updates them in place.

The single-step cases take the seeded synthetic error of the workload as `e` (a carried error would have to come
from one of the two implementations under comparison); the multi-step cases start from e = 0, as the benchmark
does, and each side carries its own state.
"""
import queue
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

import workloads
from oracle import a2sgd_oracle as O
from tests.helpers import assert_array_close, assert_chunk_close, compare_stats

pytestmark = pytest.mark.gpu
f32 = np.float32
THREADS = 16  # the GPU machine's share of host cores
CHUNK = 1 << 21


@pytest.fixture(scope="module")
def A():
    import paper_2006_07405_amd as A
    assert torch.cuda.is_available()
    return A


class Stage:
    """Pinned host buffers of one pool thread and a stream of its own for the device-to-host copies."""

    def __init__(self, count, chunk):
        self.buf = [torch.empty(chunk, dtype=torch.float32, pin_memory=True) for _ in range(count)]
        self.stream = torch.cuda.Stream()

    def fetch(self, slices):
        """Device slices (all of one length) -> numpy views of this stage's buffers."""
        m = slices[0].numel()
        with torch.cuda.stream(self.stream):
            for b, s in zip(self.buf, slices):
                b[:m].copy_(s, non_blocking=True)
        self.stream.synchronize()
        return [b[:m].numpy() for b in self.buf[:len(slices)]]


class Stages:
    def __init__(self, count, chunk=CHUNK, threads=THREADS):
        self.chunk, self.threads = chunk, threads
        self.free = queue.SimpleQueue()
        for _ in range(threads):
            self.free.put(Stage(count, chunk))

    def run(self, n, task):
        """task(stage, lo, hi) for every chunk of [0, n), on the pool; the first failure is raised."""
        def one(lo):
            st = self.free.get()
            try:
                task(st, lo, min(n, lo + self.chunk))
            finally:
                self.free.put(st)

        torch.cuda.synchronize()  # what the tasks read was written on the default stream
        with ThreadPoolExecutor(self.threads) as pool:
            list(pool.map(one, range(0, n, self.chunk)))


def oracle_pass_a(g, e, n, P, stages):
    """Sums and counts of every worker over every element: one oracle accumulator per worker, fed in index order by
    one thread per worker.  g: device tensors; e: device tensors, host arrays, or None (v = g)."""
    accs = [O.LocalAccumulator() for _ in range(P)]
    torch.cuda.synchronize()

    def worker(p):
        st = stages.free.get()
        try:
            for lo in range(0, n, stages.chunk):
                hi = min(n, lo + stages.chunk)
                if e is None:
                    accs[p].feed(st.fetch([g[p][lo:hi]])[0], None)
                elif isinstance(e[p], np.ndarray):
                    accs[p].feed(st.fetch([g[p][lo:hi]])[0], e[p][lo:hi])
                else:
                    gh, eh = st.fetch([g[p][lo:hi], e[p][lo:hi]])
                    accs[p].feed(gh, eh)
        finally:
            stages.free.put(st)

    with ThreadPoolExecutor(min(P, stages.threads)) as pool:
        list(pool.map(worker, range(P)))
    return [a.stats() for a in accs]


@pytest.mark.parametrize("k,lazy", [(2, False), (3, False), (4, False), (5, False), (4, True), (5, True)])
def test_full_size_config(A, k, lazy):
    """One step at full size from a nonzero error, every element of e and w against the oracle.  lazy = the same
    step through a2sgd_lazy_step (the buffers then hold v) followed by a2sgd_lazy_materialize, after which they hold
    the same new errors as the eager step leaves."""
    run_full_size(A, workloads.FULL[k](), (lazy,), k)


def run_full_size(A, wl, variants, k):
    """variants: which steps to run from the same inputs, False = eager, True = lazy; the oracle's first pass is taken
    once."""
    t0 = time.time()
    n, P = wl.n, wl.num_workers
    print(f"config {k} lazy={variants}: n={n} P={P}", flush=True)
    g = [wl.gradient(p, 0, device="cuda") for p in range(P)]
    e0 = [wl.synthetic_error(p, device="cuda") for p in range(P)]
    w0 = wl.weights(device="cuda")
    stages = Stages(3 * P + 2)
    print(f"  generated in {time.time() - t0:.1f}s", flush=True)

    t1 = time.time()
    stats_ref = oracle_pass_a(g, e0, n, P, stages)
    gp, gn = O.global_means(stats_ref)
    print(f"  oracle pass A in {time.time() - t1:.1f}s", flush=True)

    plan = A.a2sgd_plan(n, P, 0)
    ws = A.alloc_workspace(plan)
    for lazy in variants:
        e, w = [x.clone() for x in e0], w0.clone()
        if lazy:
            A.a2sgd_lazy_reset(plan, ws)
            A.a2sgd_lazy_step(plan, g, e, w, wl.eta, ws)
            A.a2sgd_lazy_materialize(plan, e, ws)
        else:
            A.a2sgd_step(plan, g, e, w, wl.eta, ws)
        stats, gmu = A.a2sgd_read_stats(plan, ws)
        compare_stats(stats, gmu, O.StepResult(stats_ref, gp, gn, [], np.empty(0, f32), []))
        for p in range(P):
            assert stats[p].n_pos + stats[p].n_neg == n and stats[p].n_nan == 0

        t2 = time.time()

        def pass_b(st, lo, hi):
            h = st.fetch([x[lo:hi] for x in g] + [x[lo:hi] for x in e0] + [w0[lo:hi]] + [x[lo:hi] for x in e] + [w[lo:hi]])
            e_ref, w_ref, _ = O.apply_chunk(h[:P], h[P:2 * P], h[2 * P], stats_ref, gp, gn, wl.eta, O.RETAINED_ERROR)
            for p in range(P):
                assert_chunk_close(h[2 * P + 1 + p], e_ref[p], f"config {k} lazy={lazy} e[{p}][{lo}:{hi}]")
            assert_chunk_close(h[3 * P + 1], w_ref, f"config {k} lazy={lazy} w[{lo}:{hi}]")

        stages.run(n, pass_b)
        print(f"  lazy={lazy}: oracle pass B on all {-(-n // CHUNK)} chunks in {time.time() - t2:.1f}s", flush=True)
        del e, w
    print(f"  total {time.time() - t0:.1f}s", flush=True)


def test_more_than_two_to_the_32_elements(A):
    """One worker with 2^32 + 4099 parameters (17 GB per buffer): element indices beyond 32 bits in every pass, a
    ragged last workgroup and a scalar tail up there.  The eager and the lazy step from the same inputs, every element
    of e and w against the oracle, as above."""
    run_full_size(A, workloads.config1(n=(1 << 32) + 4099, num_workers=1), (False, True), "flat 2^32+4099")


def test_config5_two_steps_from_zero_error_as_the_benchmark_runs_them(A):
    """The benchmark's own sequence at the size it is quoted on: e = 0, one step, then a second step on the carried
    state with the same gradients; the GPU and the oracle each carry their own e and w (the oracle's 30 GB live in
    host memory).  Counts equal and means within tolerance at both steps, every element of e and w within tolerance
    after each."""
    t0 = time.time()
    wl = workloads.FULL[5]()
    n, P = wl.n, wl.num_workers
    g = [wl.gradient(p, 0, device="cuda") for p in range(P)]
    e = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(P)]
    w = wl.weights(device="cuda")
    e_o = [np.zeros(n, f32) for _ in range(P)]
    w_o = w.cpu().numpy()
    stages = Stages(2 * P + 1)
    plan = A.a2sgd_plan(n, P, 0)
    ws = A.alloc_workspace(plan)
    print(f"config 5 two steps: generated in {time.time() - t0:.1f}s", flush=True)
    for t in range(2):
        t1 = time.time()
        stats_ref = oracle_pass_a(g, e_o, n, P, stages)
        gp, gn = O.global_means(stats_ref)
        # the three calls, as bench.py issues them
        A.a2sgd_local_averages(plan, g, e, ws)
        A.a2sgd_global_average(plan, ws)
        A.a2sgd_apply_and_update_error(plan, g, e, w, wl.eta, ws)
        stats, gmu = A.a2sgd_read_stats(plan, ws)
        compare_stats(stats, gmu, O.StepResult(stats_ref, gp, gn, [], np.empty(0, f32), []))

        def pass_b(st, lo, hi):
            h = st.fetch([x[lo:hi] for x in g] + [x[lo:hi] for x in e] + [w[lo:hi]])
            e_ref, w_ref, _ = O.apply_chunk(h[:P], [x[lo:hi] for x in e_o], w_o[lo:hi], stats_ref, gp, gn, wl.eta,
                                            O.RETAINED_ERROR)
            for p in range(P):
                assert_chunk_close(h[P + p], e_ref[p], f"step {t} e[{p}][{lo}:{hi}]")
                e_o[p][lo:hi] = e_ref[p]
            assert_chunk_close(h[2 * P], w_ref, f"step {t} w[{lo}:{hi}]")
            w_o[lo:hi] = w_ref

        stages.run(n, pass_b)
        print(f"  step {t}: counts equal, every element of e and w within tolerance, {time.time() - t1:.1f}s", flush=True)


@pytest.mark.parametrize("lazy", [False, True])
def test_config5_full_size_per_tensor(A, lazy):
    """The headline size with one pair of means per worker and tensor (557 tensors), as `bench.py --per-tensor` runs
    it: one step from a nonzero error, counts equal for every worker and tensor, every element of e and w against the
    oracle applied tensor by tensor.  lazy = through a2sgd_lazy_step and a2sgd_lazy_materialize (the one-shot
    reduction by blocks of 2048 elements, the apply pass from the stored sign bits)."""
    wl = workloads.FULL[5]()
    run_full_size_per_tensor(A, wl, [numel for _, numel in wl.tensors], (lazy,))


def test_tensor_boundaries_beyond_two_to_the_32(A):
    """One worker, 2^32 + 4099 parameters in three tensors whose boundaries lie just below and just above element
    2^32 (neither on a float4 group): the per-tensor passes, eager and lazy, with element indices beyond 32 bits."""
    n = (1 << 32) + 4099
    run_full_size_per_tensor(A, workloads.config1(n=n, num_workers=1), [(1 << 32) - 1001, 3003, n - (1 << 32) - 2002],
                             (False, True))


def run_full_size_per_tensor(A, wl, seg, variants):
    t0 = time.time()
    n, P = wl.n, wl.num_workers
    S = len(seg)
    bounds = np.concatenate([[0], np.cumsum(seg)]).astype(np.int64)
    assert bounds[-1] == n
    g = [wl.gradient(p, 0, device="cuda") for p in range(P)]
    e0 = [wl.synthetic_error(p, device="cuda") for p in range(P)]
    w0 = wl.weights(device="cuda")
    stages = Stages(3 * P + 2)
    print(f"per tensor lazy={variants}: n={n} P={P}, {S} tensors, generated in {time.time() - t0:.1f}s", flush=True)

    def pieces(lo, hi):
        """(tensor, a, b): the parts of the tensors that lie in [lo, hi)."""
        k = int(np.searchsorted(bounds, lo, side="right")) - 1
        while k < S and bounds[k] < hi:
            yield k, max(lo, int(bounds[k])), min(hi, int(bounds[k + 1]))
            k += 1

    t1 = time.time()
    accs = [[O.LocalAccumulator() for _ in range(S)] for _ in range(P)]
    torch.cuda.synchronize()

    def pass_a(p):  # one thread per worker, every tensor fed in index order
        st = stages.free.get()
        try:
            for lo in range(0, n, stages.chunk):
                hi = min(n, lo + stages.chunk)
                gh, eh = st.fetch([g[p][lo:hi], e0[p][lo:hi]])
                for k, a, b in pieces(lo, hi):
                    accs[p][k].feed(gh[a - lo:b - lo], eh[a - lo:b - lo])
        finally:
            stages.free.put(st)

    with ThreadPoolExecutor(P) as pool:
        list(pool.map(pass_a, range(P)))
    stats_ref = [[accs[p][k].stats() for p in range(P)] for k in range(S)]
    gmu_ref = [O.global_means(stats_ref[k]) for k in range(S)]
    print(f"  oracle pass A in {time.time() - t1:.1f}s", flush=True)

    plan = A.a2sgd_plan(n, P, 0, 0, seg_lengths=seg)
    ws = A.alloc_workspace(plan)
    for lazy in variants:
        e, w = [x.clone() for x in e0], w0.clone()
        if lazy:
            A.a2sgd_lazy_reset(plan, ws)
            A.a2sgd_lazy_step(plan, g, e, w, wl.eta, ws)
            A.a2sgd_lazy_materialize(plan, e, ws)
        else:
            A.a2sgd_local_averages(plan, g, e, ws)
            A.a2sgd_global_average(plan, ws)
            A.a2sgd_apply_and_update_error(plan, g, e, w, wl.eta, ws)
        stats, gmu = A.a2sgd_read_segment_stats(plan, ws)
        for k in range(S):
            for p in range(P):
                a, b = stats[p][k], stats_ref[k][p]
                assert (a.n_pos, a.n_neg, a.n_zero, a.n_nan) == (b.n_pos, b.n_neg, b.n_zero, b.n_nan), f"tensor {k} worker {p}"
                assert abs(a.mu_pos - b.mu_pos) <= 1e-5 * abs(b.mu_pos) and abs(a.mu_neg - b.mu_neg) <= 1e-5 * abs(b.mu_neg)
            assert abs(gmu[k][0] - gmu_ref[k][0]) <= 1e-5 * abs(gmu_ref[k][0])
            assert abs(gmu[k][1] - gmu_ref[k][1]) <= 1e-5 * abs(gmu_ref[k][1])

        t2 = time.time()

        def pass_b(st, lo, hi):
            h = st.fetch([x[lo:hi] for x in g] + [x[lo:hi] for x in e0] + [w0[lo:hi]] + [x[lo:hi] for x in e] + [w[lo:hi]])
            for k, a, b in pieces(lo, hi):
                sl = slice(a - lo, b - lo)
                e_ref, w_ref, _ = O.apply_chunk([x[sl] for x in h[:P]], [x[sl] for x in h[P:2 * P]], h[2 * P][sl],
                                                stats_ref[k], gmu_ref[k][0], gmu_ref[k][1], wl.eta, O.RETAINED_ERROR)
                for p in range(P):
                    assert_chunk_close(h[2 * P + 1 + p][sl], e_ref[p], f"lazy={lazy} tensor {k} e[{p}][{a}:{b}]")
                assert_chunk_close(h[3 * P + 1][sl], w_ref, f"lazy={lazy} tensor {k} w[{a}:{b}]")

        stages.run(n, pass_b)
        print(f"  lazy={lazy}: oracle pass B on all {-(-n // CHUNK)} chunks in {time.time() - t2:.1f}s, total {time.time() - t0:.1f}s", flush=True)
        del e, w


def oracle_step_threaded(g, e, w, eta, chunk=1 << 22, threads=THREADS):
    """One whole oracle step on host arrays, the oracle's own calls spread over host threads: one accumulator per
    worker fed in index order, then the elementwise pass chunk by chunk.  Returns (stats, gmu, e_new, w_new)."""
    P, n = len(g), int(w.shape[0])

    def pass_a(p):
        acc = O.LocalAccumulator()
        for lo in range(0, n, chunk):
            acc.feed(g[p][lo:lo + chunk], e[p][lo:lo + chunk])
        return acc.stats()

    e_new = [np.empty(n, f32) for _ in range(P)]
    w_new = np.empty(n, f32)
    with ThreadPoolExecutor(max_workers=threads) as pool:
        stats = list(pool.map(pass_a, range(P)))
        gp, gn = O.global_means(stats)

        def pass_b(lo):
            hi = min(n, lo + chunk)
            en, wn, _ = O.apply_chunk([x[lo:hi] for x in g], [x[lo:hi] for x in e], w[lo:hi], stats, gp, gn, eta,
                                      O.RETAINED_ERROR)
            for p in range(P):
                e_new[p][lo:hi] = en[p]
            w_new[lo:hi] = wn

        list(pool.map(pass_b, range(0, n, chunk)))
    return stats, (gp, gn), e_new, w_new


@pytest.mark.parametrize("k", [2, 3, 4])
def test_full_size_four_steps_free_running(A, k):
    """Four steps at full size with fresh gradients, each side carrying its own error and weights from e = 0 (the
    workload's start): counts equal and means within tolerance at every step, every element of e and w within
    tolerance at the end."""
    t0 = time.time()
    wl = workloads.FULL[k]()
    n, P = wl.n, wl.num_workers
    e_d = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(P)]
    w_d = wl.weights(device="cuda")
    e_o = [np.zeros(n, f32) for _ in range(P)]
    w_o = w_d.cpu().numpy()
    plan = A.a2sgd_plan(n, P, 0)
    ws = A.alloc_workspace(plan)
    g_d = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(P)]
    for t in range(4):
        for p in range(P):
            wl.gradient(p, t, out=g_d[p])
        g_h = [x.cpu().numpy() for x in g_d]
        A.a2sgd_step(plan, g_d, e_d, w_d, wl.eta, ws)
        stats, gmu = A.a2sgd_read_stats(plan, ws)
        stats_ref, gmu_ref, e_o, w_o = oracle_step_threaded(g_h, e_o, w_o, wl.eta)
        compare_stats(stats, gmu, O.StepResult(stats_ref, gmu_ref[0], gmu_ref[1], [], np.empty(0, f32), []))
        print(f"  config {k} step {t}: counts equal, {time.time() - t0:.1f}s", flush=True)
    for p in range(P):
        assert_array_close(e_d[p].cpu().numpy(), e_o[p], f"config {k} e[{p}] after 4 steps")
    assert_array_close(w_d.cpu().numpy(), w_o, f"config {k} w after 4 steps")
