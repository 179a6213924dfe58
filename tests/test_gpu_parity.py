"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Element-by-element at sizes the oracle finishes quickly (these span several tiles of the reduction and ragged
tails of every kind); the five benchmark configurations at full size live in test_gpu_full_size.py.
"""
import os

import numpy as np
import pytest
import torch

import workloads
from oracle import a2sgd_oracle as O
from tests.helpers import (assert_array_close, check_against_oracle, compare_stats, dev, gpu_step)

pytestmark = pytest.mark.gpu
f32 = np.float32
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example.txt")


@pytest.fixture(scope="module")
def A():
    import paper_2006_07405_amd as A
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    assert os.path.exists(A.LIB_PATH)
    return A


def make_case(seed, n, P, scale=1e-3, zeros=True):
    rng = np.random.default_rng(seed)
    g = [(rng.standard_normal(n) * scale).astype(f32) for _ in range(P)]
    e = [(rng.standard_normal(n) * scale * 0.5).astype(f32) for _ in range(P)]
    if zeros and n >= 8:
        for p in range(P):
            idx = rng.integers(0, n, max(1, n // 50))
            g[p][idx] = 0.0
            e[p][idx] = 0.0
    w = (rng.standard_normal(n) * 0.02).astype(f32)
    return g, e, w


# a tile of the reduction is 4096 elements, a block of the apply pass covers 1024
SIZES = [1, 2, 3, 4, 5, 7, 8, 63, 64, 65, 255, 256, 257, 1023, 1024, 1025, 1027, 4095, 4096, 4097, 4099, 8191,
         12289, 40961, 65539, 300_001]


@pytest.mark.parametrize("n", SIZES)
def test_sizes_and_tails(A, n):
    for P, mode in ((1, 0), (3, 0), (4, 1)):
        print(f"case n={n} P={P} mode={mode}", flush=True)
        g, e, w = make_case(n * 31 + P, n, P)
        check_against_oracle(A, g, e, w, 0.1, mode)


@pytest.mark.parametrize("P", [1, 2, 3, 4, 5, 7, 8, 9, 16, 17, 33, 64])
def test_worker_counts(A, P):
    print(f"case P={P}", flush=True)
    g, e, w = make_case(1000 + P, 20_003, P)
    check_against_oracle(A, g, e, w, 0.05, 0)
    check_against_oracle(A, g, e, w, 0.05, 1, split_calls=False)


@pytest.mark.parametrize("n", [1, 3, 4, 5, 255, 1023, 1024, 1025, 4099, 65_539, 524_288, 1_048_577, 3_000_001])
def test_single_launch_step(A, n):
    """a2sgd_step on cache-resident sizes takes the single-launch route (one cooperative kernel)."""
    for P, mode, with_e in ((1, 0, True), (4, 0, True), (5, 1, True), (3, 1, False)):
        print(f"case n={n} P={P} mode={mode} e={with_e}", flush=True)
        g, e, w = make_case(n * 7 + P, n, P)
        check_against_oracle(A, g, e if with_e else None, w, 0.1, mode, split_calls=False, want_mask=False)


def test_single_launch_step_many_workers(A):
    for P in (16, 33, 64):
        g, e, w = make_case(P, 50_003, P)
        check_against_oracle(A, g, e, w, 0.1, 0, split_calls=False, want_mask=False)
    g, e, w = make_case(5, 10_007, 2)
    g[1][[0, 77, 10_006]] = np.nan
    check_against_oracle(A, g, e, w, 0.1, 0, split_calls=False, want_mask=False)
    # both routes give the same counts and means on the same inputs
    g, e, w = make_case(6, 700_001, 4)
    a = gpu_step(A, g, e, w, 0.1, 0, split_calls=True)
    b = gpu_step(A, g, e, w, 0.1, 0, split_calls=False)
    assert [(s.n_pos, s.n_neg, s.n_zero) for s in a[0]] == [(s.n_pos, s.n_neg, s.n_zero) for s in b[0]]
    assert all(abs(x.mu_pos - y.mu_pos) <= 1e-6 * y.mu_pos for x, y in zip(a[0], b[0]))


def test_literal_mode_without_error_buffer(A):
    g, _, w = make_case(5, 70_001, 4)
    (stats, gmu, e_new, w_new, _), ref = check_against_oracle(A, g, None, w, 0.1, 1)
    assert e_new is None
    # P = 1: Theorem 1's net gain vanishes and the step is plain SGD, w - eta*g
    g1, _, w1 = make_case(6, 33_333, 1)
    _, _, _, w_new, _ = gpu_step(A, g1, None, w1, 0.25, 1)
    ref = w1.astype(np.float64) - 0.25 * g1[0].astype(np.float64)
    assert np.max(np.abs(w_new - ref)) <= 2e-8


def test_worked_example(A):
    G = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            G[k.strip()] = [float(t) for t in v.split()]
    w = np.zeros(6, f32)
    e = [np.zeros(6, f32), np.zeros(6, f32)]
    for s in ("step1", "step2"):
        g = [np.array(G[f"{s}.gA"], f32), np.array(G[f"{s}.gB"], f32)]
        stats, gmu, e, w, mask = gpu_step(A, g, e, w, 0.5, 0, want_mask=True)
        for name, st in zip("AB", stats):
            assert (st.n_pos, st.n_neg, st.n_zero) == tuple(G[f"{s}.{name}.{k}"][0] for k in ("n_pos", "n_neg", "n_zero"))
            assert (st.mu_pos, st.mu_neg) == (G[f"{s}.{name}.mu_pos"][0], G[f"{s}.{name}.mu_neg"][0])
        assert gmu == (G[f"{s}.gmu_pos"][0], G[f"{s}.gmu_neg"][0])
        assert np.array_equal(e[0], np.array(G[f"{s}.eA"], f32)) and np.array_equal(e[1], np.array(G[f"{s}.eB"], f32))
        assert list(mask[0]) == G[f"{s}.maskA"] and list(mask[1]) == G[f"{s}.maskB"]
        assert np.array_equal(w, np.array(G[f"{s}.w"], f32))
    g = [np.array(G["step1.gA"], f32), np.array(G["step1.gB"], f32)]
    _, _, _, w, _ = gpu_step(A, g, None, np.zeros(6, f32), 0.5, 1)
    assert np.array_equal(w, np.array(G["step1.literal.w"], f32))


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_small_variants_of_the_five_configs(A, k):
    wl = workloads.small(k)
    P = wl.num_workers
    g = [wl.gradient(p).numpy() for p in range(P)]
    e = [wl.synthetic_error(p).numpy() for p in range(P)]
    w = wl.weights().numpy()
    check_against_oracle(A, g, e, w, wl.eta, 0)
    check_against_oracle(A, g, [np.zeros_like(x) for x in g], w, wl.eta, 0)  # the configs start from e = 0
    check_against_oracle(A, g, e, w, wl.eta, 1)


def test_edge_cases(A):
    z4 = np.zeros(4, f32)
    # all entries >= 0: the negative group is empty, its mean is 0
    (st, gmu, e_new, w_new, _), _ = check_against_oracle(A, [np.array([1, 2, 3, 0], f32)], [z4], z4, 1.0, 0)
    assert (st[0].n_pos, st[0].n_neg, st[0].mu_pos, st[0].mu_neg) == (4, 0, 1.5, 0.0)
    assert np.array_equal(e_new[0], np.array([-0.5, 0.5, 1.5, -1.5], f32))
    # all entries < 0
    (st, gmu, e_new, w_new, _), _ = check_against_oracle(A, [np.array([-1, -2, -3, -2], f32)], [z4], z4, 1.0, 0)
    assert (st[0].n_pos, st[0].n_neg, st[0].mu_pos, st[0].mu_neg) == (0, 4, 0.0, 2.0)
    assert np.array_equal(w_new, np.array([2, 2, 2, 2], f32))
    # one worker all positive, the other all negative: empty groups enter the global mean as 0
    (st, gmu, _, w_new, _), _ = check_against_oracle(
        A, [np.array([1, 2, 3, 0], f32), np.array([-1, -2, -3, -2], f32)], [z4, z4], z4, 1.0, 0)
    assert gmu == (0.75, 1.0) and np.array_equal(w_new, np.full(4, 0.125, f32))
    # all zeros, including -0.0
    v = np.array([0.0, -0.0, 0.0, -0.0, 0.0], f32)
    (st, _, e_new, _, mask), _ = check_against_oracle(A, [v], [np.zeros(5, f32)], np.ones(5, f32), 1.0, 0)
    assert (st[0].n_pos, st[0].n_zero, st[0].n_neg) == (5, 5, 0) and list(mask[0]) == [1] * 5
    # g and e cancel exactly: v = +0 belongs to the ">= 0" group
    g = np.array([1.5, -2.5, 3.0], f32)
    (st, _, _, _, _), _ = check_against_oracle(A, [g], [-g], np.zeros(3, f32), 1.0, 0)
    assert st[0].n_pos == 3 and st[0].n_zero == 3
    # denormals keep their sign group (no flush to zero)
    d = np.array([1e-45, -1e-45, 1e-40, -1e-40, 0.0, 3e-39, -3e-39], f32)
    (st, _, _, _, _), _ = check_against_oracle(A, [d], [np.zeros(7, f32)], np.zeros(7, f32), 1.0, 0)
    assert (st[0].n_pos, st[0].n_neg, st[0].n_zero) == (4, 3, 1)
    # a two-valued vector is encoded without loss
    v = np.array([0.375, -1.25] * 3000 + [0.375], f32)
    (_, _, e_new, _, _), _ = check_against_oracle(A, [v], [np.zeros_like(v)], np.zeros_like(v), 1.0, 0)
    assert not e_new[0].any()
    # huge and tiny magnitudes together: fp64 sums do not lose the tiny group
    v = np.array([1e30, 2e30, -1e-30, -3e-30] * 1000, f32)
    check_against_oracle(A, [v], [np.zeros_like(v)], np.zeros_like(v), 1e-30, 0)


def test_nan_is_in_neither_group(A):
    g, e, w = make_case(77, 10_007, 2)
    g[0][[3, 5000, 10_006]] = np.nan
    (st, _, e_new, w_new, _), _ = check_against_oracle(A, g, e, w, 0.1, 0)
    assert st[0].n_nan == 3 and st[1].n_nan == 0 and st[0].n_pos + st[0].n_neg + 3 == 10_007
    assert np.isnan(w_new).sum() == 3 and np.isnan(e_new[0]).sum() == 3 and not np.isnan(e_new[1]).any()
    check_against_oracle(A, g, e, w, 0.1, 1)


def test_deterministic_and_block_count_independent(A):
    g, e, w = make_case(99, 500_009, 4)
    a = gpu_step(A, g, e, w, 0.1, 0)
    b = gpu_step(A, g, e, w, 0.1, 0)
    assert [vars(s) for s in a[0]] == [vars(s) for s in b[0]] and a[1] == b[1]
    assert all(np.array_equal(x.view(np.uint32), y.view(np.uint32)) for x, y in zip(a[2], b[2]))
    assert np.array_equal(a[3].view(np.uint32), b[3].view(np.uint32))
    ref = O.step(g, e, w, 0.1, 0)
    for bpw in (1, 2, 3, 17, 128, 1000, 4096):
        print(f"case blocks_per_worker={bpw}", flush=True)
        st, gmu, e_new, w_new, _ = gpu_step(A, g, e, w, 0.1, 0, blocks_per_worker=bpw)
        compare_stats(st, gmu, ref)
        assert_array_close(w_new, ref.w_new, "w")


def test_power_of_two_scaling_is_bitwise(A):
    """g, e times 2^k and eta times 2^-k: means and errors scale exactly; counts and new weights are unchanged."""
    g, e, w = make_case(123, 200_003, 3)
    k = 6
    a = gpu_step(A, g, e, w, 0.125, 0)
    b = gpu_step(A, [x * f32(2.0 ** k) for x in g], [x * f32(2.0 ** k) for x in e], w, 0.125 * 2.0 ** -k, 0)
    for sa, sb in zip(a[0], b[0]):
        assert (sb.mu_pos, sb.mu_neg) == (sa.mu_pos * 2 ** k, sa.mu_neg * 2 ** k)
        assert (sb.n_pos, sb.n_neg, sb.n_zero) == (sa.n_pos, sa.n_neg, sa.n_zero)
    assert all(np.array_equal(x * f32(2.0 ** k), y) for x, y in zip(a[2], b[2]))
    assert np.array_equal(a[3], b[3])


def test_config1_ten_steps_teacher_forced_and_free_running(A):
    """Config 1 at full size (n = 1,048,576, P = 4, 10 steps, fresh gradients each step).  Teacher-forced: both
    sides start every step from the oracle's state.  Free-running: each side carries its own state."""
    wl = workloads.config1()
    n, P = wl.n, wl.num_workers
    plan = A.a2sgd_plan(n, P, 0)
    ws = A.alloc_workspace(plan)
    w_o = wl.weights().numpy()
    e_o = [np.zeros(n, f32) for _ in range(P)]
    w_f = dev(w_o)
    e_f = [dev(x) for x in e_o]
    flips = 0
    for t in range(wl.steps):
        print(f"step {t}", flush=True)
        g = [wl.gradient(p, t).numpy() for p in range(P)]
        gd = [dev(x) for x in g]
        ref = O.step(g, e_o, w_o, wl.eta, 0)
        # teacher-forced
        e_t = [dev(x) for x in e_o]
        w_t = dev(w_o)
        A.a2sgd_step(plan, gd, e_t, w_t, wl.eta, ws)
        st, gmu = A.a2sgd_read_stats(plan, ws)
        compare_stats(st, gmu, ref)
        for p in range(P):
            assert_array_close(e_t[p].cpu().numpy(), ref.e_new[p], f"step {t} e[{p}]")
        assert_array_close(w_t.cpu().numpy(), ref.w_new, f"step {t} w")
        # free-running
        A.a2sgd_step(plan, gd, e_f, w_f, wl.eta, ws)
        st_f, gmu_f = A.a2sgd_read_stats(plan, ws)
        for p in range(P):
            flips += abs(st_f[p].n_pos - ref.workers[p].n_pos)
        e_o, w_o = ref.e_new, ref.w_new
    for p in range(P):
        assert_array_close(e_f[p].cpu().numpy(), e_o[p], f"free-running e[{p}] after 10 steps")
    assert_array_close(w_f.cpu().numpy(), w_o, "free-running w after 10 steps")
    assert flips == 0, f"{flips} sign-group flips between the free-running GPU state and the oracle"


def test_checkpoint_resume_is_bitwise(A):
    """State = (w, e^p): 6 steps in one go equal 3 steps, a copy of the state out and back in, and 3 more."""
    wl = workloads.config1(n=262_147, num_workers=3)
    n, P = wl.n, wl.num_workers
    plan = A.a2sgd_plan(n, P, 0)
    ws = A.alloc_workspace(plan)
    grads = [[wl.gradient(p, t, device="cuda") for p in range(P)] for t in range(6)]
    w1 = wl.weights(device="cuda")
    e1 = [torch.zeros(n, device="cuda") for _ in range(P)]
    for t in range(6):
        A.a2sgd_step(plan, grads[t], e1, w1, wl.eta, ws)
    w2 = wl.weights(device="cuda")
    e2 = [torch.zeros(n, device="cuda") for _ in range(P)]
    for t in range(3):
        A.a2sgd_step(plan, grads[t], e2, w2, wl.eta, ws)
    saved = ([x.cpu() for x in e2], w2.cpu())
    plan2 = A.a2sgd_plan(n, P, 0)
    ws2 = A.alloc_workspace(plan2)
    e3 = [x.cuda() for x in saved[0]]
    w3 = saved[1].cuda()
    for t in range(3, 6):
        A.a2sgd_step(plan2, grads[t], e3, w3, wl.eta, ws2)
    assert torch.equal(w1, w3) and all(torch.equal(a, b) for a, b in zip(e1, e3))


def test_dense_step(A):
    for n, P in ((1, 1), (5, 3), (4099, 4), (300_001, 8), (65_536, 5)):
        g, _, w = make_case(n + P, n, P)
        plan = A.a2sgd_plan(n, P)
        gd = [dev(x) for x in g]
        wd = dev(w)
        A.a2sgd_dense_step(plan, gd, wd, 0.1)
        assert_array_close(wd.cpu().numpy(), O.dense_step(g, w, 0.1), f"dense n={n} P={P}")


@pytest.mark.parametrize("n,P", [(8_000_003, 3), (3_500_003, 7), (2_100_001, 12), (1_700_003, 15), (1_000_001, 33),
                                 (420_001, 64)])
def test_streaming_path_with_worker_counts_that_leave_a_short_group(A, n, P):
    """Footprints above the cache limit take the streaming kernels (non-temporal loads, write-through stores, capped
    residency); these P are not multiples of the group size, so the last group of workers is a short one.  Eager
    step in both modes, the dense step, the replica step and the lazy step (literal mode reads v in groups too)."""
    assert (2 * P + 1) * 4 * n > 192 << 20
    g, e, w = make_case(n + P, n, P)
    for mode in (0, 1):
        check_against_oracle(A, g, e, w, 0.1, mode, want_mask=False)
    plan = A.a2sgd_plan(n, P, 1)
    ws = A.alloc_workspace(plan)
    gd = [dev(x) for x in g]
    wd = dev(w)
    A.a2sgd_dense_step(plan, gd, wd, 0.1)
    assert_array_close(wd.cpu().numpy(), O.dense_step(g, w, 0.1), "dense w")
    # replicas (all starting from w) in literal mode, then the dense step on replicas
    ed, wr = [dev(x) for x in e], [dev(w) for _ in range(P)]
    A.a2sgd_step_replicas(plan, gd, ed, wr, 0.1, ws)
    _, _, e_ref, w_ref = O.step_replicas(g, e, [w] * P, 0.1, 1)
    for p in range(P):
        assert_array_close(ed[p].cpu().numpy(), e_ref[p], f"replica e[{p}]")
        assert_array_close(wr[p].cpu().numpy(), w_ref[p], f"replica w[{p}]")
    A.a2sgd_dense_step_replicas(plan, gd, wr, 0.05)
    ref = O.dense_step_replicas(g, w_ref, 0.05)
    for p in range(P):
        assert_array_close(wr[p].cpu().numpy(), ref[p], f"dense replica w[{p}]")
    # lazy step, literal mode, from the same inputs
    s, wl_ = [dev(x) for x in e], dev(w)
    A.a2sgd_lazy_reset(plan, ws)
    A.a2sgd_lazy_step(plan, gd, s, wl_, 0.1, ws)
    A.a2sgd_lazy_materialize(plan, s, ws)
    ref1 = O.step(g, e, w, 0.1, 1)
    assert_array_close(wl_.cpu().numpy(), ref1.w_new, "lazy w")
    for p in range(P):
        assert_array_close(s[p].cpu().numpy(), ref1.e_new[p], f"lazy e[{p}]")


@pytest.mark.parametrize("n,P", [(3_200_003, 8), (3_145_728, 8), (1_600_002, 16), (1_574_913, 17), (420_001, 64)])
def test_two_kernel_apply_pass(A, n, P):
    """From 8 workers on, streaming plans in retained-error mode write the errors back and update the weights in two
    kernels, the second working from stored sign bits.  Against the oracle on sizes with every kind of tail (n % 4,
    part of a 2048-element workgroup, a whole number of them), with exact zeros in g and e so that v = 0 occurs; then with a
    few NaNs in g, which have no sign bit and take the pass's other branch; over two steps on carried state."""
    assert (2 * P + 1) * 4 * n > 192 << 20
    g, e, w = make_case(n * 7 + P, n, P)
    plan = A.a2sgd_plan(n, P, 0)
    ws = A.alloc_workspace(plan)
    for with_nan in (False, True):
        print(f"case n={n} P={P} nan={with_nan}", flush=True)
        if with_nan:
            rng = np.random.default_rng(n)
            for p in (0, P - 1):
                g[p][rng.integers(0, n, 5)] = np.nan
            g[1][n - 1] = np.nan  # in the scalar tail when n % 4 != 0
        gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
        e_o, w_o = e, w
        for t in range(2):
            A.a2sgd_local_averages(plan, gd, ed, ws)
            A.a2sgd_global_average(plan, ws)
            A.a2sgd_apply_and_update_error(plan, gd, ed, wd, 0.1, ws)
            stats, gmu = A.a2sgd_read_stats(plan, ws)
            ref = O.step(g, e_o, w_o, 0.1, 0)
            compare_stats(stats, gmu, ref)
            e_o, w_o = ref.e_new, ref.w_new
            for p in range(P):
                assert_array_close(ed[p].cpu().numpy(), e_o[p], f"step {t} e[{p}]")
            assert_array_close(wd.cpu().numpy(), w_o, f"step {t} w")
        for p in range(P):
            assert np.array_equal(gd[p].cpu().numpy().view(np.uint32), g[p].view(np.uint32))  # g is read-only


def test_runs_on_a_side_stream_and_respects_stream_order(A):
    g, e, w = make_case(4242, 1_000_003, 4)
    ref = O.step(g, e, w, 0.1, 0)
    s = torch.cuda.Stream()
    plan = A.a2sgd_plan(len(w), 4)
    with torch.cuda.stream(s):
        ws = A.alloc_workspace(plan)
        gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
        A.a2sgd_step(plan, gd, ed, wd, 0.1, ws)  # picks up the current torch stream
        st, gmu = A.a2sgd_read_stats(plan, ws)
    s.synchronize()
    compare_stats(st, gmu, ref)
    assert_array_close(wd.cpu().numpy(), ref.w_new, "w")


@pytest.mark.parametrize("n,P", [(1, 1), (5, 2), (1023, 3), (4099, 4), (65_539, 5), (300_001, 8), (70_001, 17)])
def test_replicas(A, n, P):
    """One weight vector per worker (Algorithm 1 line 7 as printed), the final synchronisation on replicas and the
    drift diagnostic, against the oracle; and the mean of the replicas against the shared-weight path."""
    g, e, w = make_case(n * 3 + P, n, P)
    rng = np.random.default_rng(n + P)
    wr = [(w + (rng.standard_normal(n) * 1e-3).astype(f32)) for _ in range(P)]
    for mode in (0, 1):
        plan = A.a2sgd_plan(n, P, mode)
        ws = A.alloc_workspace(plan)
        gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], [dev(x) for x in wr]
        A.a2sgd_step_replicas(plan, gd, ed, wd, 0.1, ws)
        stats, gmu = A.a2sgd_read_stats(plan, ws)
        workers, gmu_ref, e_ref, w_ref = O.step_replicas(g, e, wr, 0.1, mode)
        compare_stats(stats, gmu, O.StepResult(workers, gmu_ref[0], gmu_ref[1], [], np.empty(0, f32), []))
        for p in range(P):
            assert_array_close(ed[p].cpu().numpy(), e_ref[p], f"e[{p}]")
            assert_array_close(wd[p].cpu().numpy(), w_ref[p], f"w[{p}]")
        # the replica mean moves like the single weight vector of the shared path
        w_mean0 = np.mean(np.stack(wr).astype(np.float64), axis=0).astype(f32)
        _, _, _, w_shared, _ = gpu_step(A, g, e, w_mean0, 0.1, mode)
        got = np.mean(np.stack([x.cpu().numpy() for x in wd]).astype(np.float64), axis=0)
        assert np.allclose(got - w_mean0, w_shared.astype(np.float64) - w_mean0, rtol=0, atol=3e-8)
        # drift diagnostic
        mx, rms = A.a2sgd_replica_drift(plan, wd, ws)
        mx_ref, rms_ref = O.replica_drift([x.cpu().numpy() for x in wd])
        assert np.allclose(mx, mx_ref, rtol=1e-12, atol=0) and np.allclose(rms, rms_ref, rtol=1e-9, atol=1e-300)
        # final synchronisation (Algorithm 1 lines 9-10) applied to every replica
        before = [x.cpu().numpy() for x in wd]
        A.a2sgd_dense_step_replicas(plan, gd, wd, 0.05)
        ref = O.dense_step_replicas(g, before, 0.05)
        for p in range(P):
            assert_array_close(wd[p].cpu().numpy(), ref[p], f"dense w[{p}]")


@pytest.mark.parametrize("n,P,mode,with_e", [(3_100_003, 8, 0, True), (3_100_001, 8, 1, True), (800_002, 33, 1, False),
                                              (400_003, 64, 0, True), (1_700_000, 15, 1, True)])
def test_replicas_streaming_one_worker_per_workgroup(A, n, P, mode, with_e):
    """From 8 workers on the streaming replica pass gives every workgroup one worker's g, e and w^p: against the
    oracle at sizes with a ragged last workgroup and a scalar tail, both modes, with and without an error buffer."""
    assert (2 * P + 1) * 4 * n > 192 << 20
    g, e, w = make_case(n + P, n, P)
    rng = np.random.default_rng(n + P)
    wr = [(w + (rng.standard_normal(n) * 1e-3).astype(f32)) for _ in range(P)]
    plan = A.a2sgd_plan(n, P, mode)
    ws = A.alloc_workspace(plan)
    gd, wd = [dev(x) for x in g], [dev(x) for x in wr]
    ed = [dev(x) for x in e] if with_e else None
    A.a2sgd_step_replicas(plan, gd, ed, wd, 0.1, ws)
    stats, gmu = A.a2sgd_read_stats(plan, ws)
    workers, gmu_ref, e_ref, w_ref = O.step_replicas(g, e if with_e else None, wr, 0.1, mode)
    compare_stats(stats, gmu, O.StepResult(workers, gmu_ref[0], gmu_ref[1], [], np.empty(0, f32), []))
    for p in range(P):
        if with_e:
            assert_array_close(ed[p].cpu().numpy(), e_ref[p], f"e[{p}]")
        assert_array_close(wd[p].cpu().numpy(), w_ref[p], f"w[{p}]")
        assert np.array_equal(gd[p].cpu().numpy().view(np.uint32), g[p].view(np.uint32)), "g is read-only"


def test_replicas_full_size_config2(A):
    """Config 2 shape (25.6 M parameters, 8 workers) on device-generated inputs: the replica mean against the
    shared path, elementwise, and identical errors."""
    wl = workloads.config2()
    n, P = wl.n, wl.num_workers
    plan = A.a2sgd_plan(n, P, 0)
    ws = A.alloc_workspace(plan)
    g = [wl.gradient(p, 0, device="cuda") for p in range(P)]
    e1 = [wl.synthetic_error(p, device="cuda") for p in range(P)]
    e2 = [x.clone() for x in e1]
    w = wl.weights(device="cuda")
    wr = [w.clone() for _ in range(P)]
    A.a2sgd_step(plan, g, e1, w, wl.eta, ws)
    A.a2sgd_step_replicas(plan, g, e2, wr, wl.eta, ws)
    assert all(torch.equal(a, b) for a, b in zip(e1, e2))
    mean = torch.stack([x.double() for x in wr]).mean(dim=0)
    assert float((mean - w.double()).abs().max()) <= 1e-8
    mx, rms = A.a2sgd_replica_drift(plan, wr, ws)
    assert all(0 < r < m < 1e-2 for m, r in zip(mx, rms))


@pytest.mark.parametrize("n,P,mode", [(1, 1, 0), (7, 2, 0), (4099, 3, 1), (65_539, 4, 0), (300_001, 8, 1), (50_001, 17, 0),
                                      (2_000_003, 4, 0), (2047, 2, 0), (3 * 2048, 2, 1), (12_000_017, 2, 0)])
def test_lazy_error_state(A, n, P, mode):
    """Five steps on the lazy state (buffers hold v, the error is formed on the next read) against five eager
    steps of the oracle and of the GPU: same w and statistics at every step, same errors once materialised.  The
    sizes include less than one workgroup of the reduction pass (2048 elements), a whole number of them, and one
    whose records need more than one workgroup of the fold pass (and whose footprint takes the streaming path)."""
    wl = workloads.config1(n=n, num_workers=P)
    rng = np.random.default_rng(n)
    e0 = [(rng.standard_normal(n) * 4e-4).astype(f32) for _ in range(P)]  # start from a nonzero true error
    w0 = wl.weights().numpy()
    plan = A.a2sgd_plan(n, P, mode)
    ws_l, ws_e = A.alloc_workspace(plan), A.alloc_workspace(plan)
    s = [dev(x) for x in e0]
    w_l = dev(w0)
    e_g = [dev(x) for x in e0]
    w_g = dev(w0)
    e_o, w_o = [x.copy() for x in e0], w0.copy()
    A.a2sgd_lazy_reset(plan, ws_l)
    ulp_w = float(np.spacing(f32(np.abs(w0).max() + 1e-3)))
    for t in range(5):
        g = [wl.gradient(p, t).numpy() for p in range(P)]
        gd = [dev(x) for x in g]
        ref = O.step(g, e_o, w_o, wl.eta, mode)
        A.a2sgd_lazy_step(plan, gd, s, w_l, wl.eta, ws_l)
        st, gmu = A.a2sgd_read_stats(plan, ws_l)
        compare_stats(st, gmu, ref)
        assert_array_close(w_l.cpu().numpy(), ref.w_new, f"step {t} w (lazy)")
        # the eager GPU path from the same state: same counts; the sums are grouped differently, so the means may
        # differ in the last bit once in a long while, and in retained-error mode the lazy update is formed from
        # the number of workers in the positive group instead of worker by worker: the weights agree to an ulp
        A.a2sgd_local_averages(plan, gd, e_g, ws_e)
        A.a2sgd_global_average(plan, ws_e)
        A.a2sgd_apply_and_update_error(plan, gd, e_g, w_g, wl.eta, ws_e)
        st_e, _ = A.a2sgd_read_stats(plan, ws_e)
        assert [(a.n_pos, a.n_neg, a.n_zero) for a in st] == [(a.n_pos, a.n_neg, a.n_zero) for a in st_e]
        assert float((w_l - w_g).abs().max()) <= ulp_w, f"step {t}: lazy and eager weights differ"
        e_o, w_o = ref.e_new, ref.w_new
    A.a2sgd_lazy_materialize(plan, s, ws_l)
    for p in range(P):
        assert_array_close(s[p].cpu().numpy(), e_o[p], f"materialised e[{p}]")
        assert float((s[p] - e_g[p]).abs().max()) <= 1e-9, f"materialised error of worker {p} differs from the eager path's"
    # after materialising, the buffers are true errors again: one more lazy step and one more eager step agree
    g = [wl.gradient(p, 5, device="cuda") for p in range(P)]
    A.a2sgd_lazy_step(plan, g, s, w_l, wl.eta, ws_l)
    A.a2sgd_local_averages(plan, g, e_g, ws_e)
    A.a2sgd_global_average(plan, ws_e)
    A.a2sgd_apply_and_update_error(plan, g, e_g, w_g, wl.eta, ws_e)
    assert float((w_l - w_g).abs().max()) <= 1e-9


@pytest.mark.parametrize("n,P,calls", [(1_048_576, 4, "step"), (1_048_576, 4, "three"), (14_000_003, 4, "three"),
                                       (300_001, 3, "lazy")])
def test_step_captured_in_a_hip_graph(A, n, P, calls):
    """The step calls only enqueue kernels (no allocation, no copy, no host wait), so a stream capture records them.
    Three replays, with the program's own eager work and synchronisations between them, must leave exactly what
    three eager steps leave (the eager steps are the ones the other tests check against the oracle)."""
    wl = workloads.config1(n=n, num_workers=P)
    g = [wl.gradient(p, 0, device="cuda") for p in range(P)]
    e0 = [wl.synthetic_error(p, device="cuda") for p in range(P)]
    w0 = wl.weights(device="cuda")
    plan = A.a2sgd_plan(n, P, 0)

    def one_step(e, w, ws):
        if calls == "step":  # one launch at this size
            A.a2sgd_step(plan, g, e, w, wl.eta, ws)
        elif calls == "lazy":
            A.a2sgd_lazy_step(plan, g, e, w, wl.eta, ws)
        else:
            A.a2sgd_local_averages(plan, g, e, ws)
            A.a2sgd_global_average(plan, ws)
            A.a2sgd_apply_and_update_error(plan, g, e, w, wl.eta, ws)

    ws_ref = A.alloc_workspace(plan)
    e_ref, w_ref = [x.clone() for x in e0], w0.clone()
    if calls == "lazy":
        A.a2sgd_lazy_reset(plan, ws_ref)
    expected = []
    for _ in range(3):
        one_step(e_ref, w_ref, ws_ref)
        expected.append(([x.clone() for x in e_ref], w_ref.clone()))
    torch.cuda.synchronize()

    ws = A.alloc_workspace(plan)
    e, w = [x.clone() for x in e0], w0.clone()
    if calls == "lazy":
        A.a2sgd_lazy_reset(plan, ws)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        one_step(e, w, ws)
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        busy = (w0 * 2.0).sum().item()  # unrelated eager work and a host wait between replays
        assert np.isfinite(busy)
        for p in range(P):
            assert torch.equal(e[p], expected[k][0][p]), f"replay {k}: buffer of worker {p} differs from eager"
        assert torch.equal(w, expected[k][1]), f"replay {k}: w differs from eager"


def test_random_shapes_against_the_oracle(A):
    """Seeded random draws of (n, P, mode, e present, blocks per worker, which calls): the combinations nobody
    thought of.  Sizes are skewed towards the small and ragged, where the bounds logic lives."""
    rng = np.random.default_rng(20260607)
    for case in range(60):
        P = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 11, 13, 16, 17, 31, 32, 33, 47, 63, 64]))
        n = int(rng.choice([rng.integers(1, 70), rng.integers(70, 5000), rng.integers(5000, 2_000_000 // P + 5001)]))
        mode = int(rng.integers(0, 2))
        with_e = bool(mode == 0 or rng.integers(0, 2))
        bpw = int(rng.choice([0, 0, 1, 3, 64, 1000]))
        path = str(rng.choice(["three", "step", "lazy", "replicas"]))
        print(f"case {case}: n={n} P={P} mode={mode} e={with_e} blocks_per_worker={bpw} path={path}", flush=True)
        g, e, w = make_case(case, n, P)
        if path in ("three", "step"):
            check_against_oracle(A, g, e if with_e else None, w, 0.1, mode, blocks_per_worker=bpw,
                                 split_calls=(path == "three"))
            continue
        plan = A.a2sgd_plan(n, P, mode, bpw)
        ws = A.alloc_workspace(plan)
        gd, ed = [dev(x) for x in g], [dev(x) for x in e]
        if path == "lazy":
            wd = dev(w)
            A.a2sgd_lazy_reset(plan, ws)
            A.a2sgd_lazy_step(plan, gd, ed, wd, 0.1, ws)
            stats, gmu = A.a2sgd_read_stats(plan, ws)
            A.a2sgd_lazy_materialize(plan, ed, ws)
            ref = O.step(g, e, w, 0.1, mode)
            compare_stats(stats, gmu, ref)
            assert_array_close(wd.cpu().numpy(), ref.w_new, "lazy w")
            for p in range(P):
                assert_array_close(ed[p].cpu().numpy(), ref.e_new[p], f"lazy e[{p}]")
        else:
            wr = [dev(w + f32(1e-3) * f32(p)) for p in range(P)]
            A.a2sgd_step_replicas(plan, gd, ed, wr, 0.1, ws)
            _, _, e_ref, w_ref = O.step_replicas(g, e, [w + f32(1e-3) * f32(p) for p in range(P)], 0.1, mode)
            for p in range(P):
                assert_array_close(ed[p].cpu().numpy(), e_ref[p], f"replica e[{p}]")
                assert_array_close(wr[p].cpu().numpy(), w_ref[p], f"replica w[{p}]")


def test_buffers_at_the_minimum_alignment(A):
    """g, e and w as views that start 16 bytes (and for one buffer 48 bytes) into larger allocations: 16 bytes is
    all the interface asks for.  Eager three calls, single launch, lazy step."""
    n, P = 70_003, 3
    g, e, w = make_case(5, n, P)
    ref = O.step(g, e, w, 0.1, 0)

    def view(a, off):
        big = torch.zeros(n + 64, dtype=torch.float32, device="cuda")
        v = big[off:off + n]
        v.copy_(torch.from_numpy(a))
        assert v.data_ptr() % 16 == 0 and v.data_ptr() % 64 != 0
        return v

    for path in ("three", "step", "lazy"):
        gd = [view(x, 4) for x in g]
        ed = [view(x, 12 if p == 1 else 4) for p, x in enumerate(e)]
        wd = view(w, 4)
        plan = A.a2sgd_plan(n, P, 0)
        ws_big = torch.zeros(A.a2sgd_workspace_bytes(plan) // 8 + 8, dtype=torch.int64, device="cuda")
        ws = ws_big[2:]  # 16 bytes in
        if path == "three":
            A.a2sgd_local_averages(plan, gd, ed, ws)
            A.a2sgd_global_average(plan, ws)
            A.a2sgd_apply_and_update_error(plan, gd, ed, wd, 0.1, ws)
        elif path == "step":
            A.a2sgd_step(plan, gd, ed, wd, 0.1, ws)
        else:
            A.a2sgd_lazy_reset(plan, ws)
            A.a2sgd_lazy_step(plan, gd, ed, wd, 0.1, ws)
            A.a2sgd_lazy_materialize(plan, ed, ws)
        stats, gmu = A.a2sgd_read_stats(plan, ws)
        compare_stats(stats, gmu, ref)
        assert_array_close(wd.cpu().numpy(), ref.w_new, f"{path}: w")
        for p in range(P):
            assert_array_close(ed[p].cpu().numpy(), ref.e_new[p], f"{path}: e[{p}]")


@pytest.mark.parametrize("n,P,mode,three", [(100_003, 3, 0, 0), (100_003, 3, 1, 1), (6_000_001, 4, 0, 0),
                                            (100_003, 3, 0, 2), (6_000_001, 8, 0, 2)])
def test_c_client_without_python_in_the_path(A, tmp_path, n, P, mode, three):
    """tests/c_client/client.cpp calls the C ABI with memory from hipMalloc and a stream of its own; this test only
    writes its input file and reads its output file.  Sizes: a single-launch step, the three calls, a streaming size;
    the last two go through the entry point that allocates nothing (no statistics to read back there)."""
    import subprocess
    client = os.path.join(os.path.dirname(__file__), "c_client", "client")
    if not os.path.exists(client):
        pytest.skip("tests/c_client/client is not built (build() compiles it)")
    g, e, w = make_case(n + mode, n, P)
    fin, fout = tmp_path / "in.bin", tmp_path / "out.bin"
    np.concatenate(g + e + [w]).astype(f32).tofile(fin)
    subprocess.run([client, str(fin), str(fout), str(n), str(P), str(mode), "0.1", str(three)], check=True, timeout=120)
    raw = np.fromfile(fout, dtype=np.uint8)
    rec = np.dtype([("mu_pos", f32), ("mu_neg", f32), ("n_pos", np.uint64), ("n_neg", np.uint64),
                    ("n_zero", np.uint64), ("n_nan", np.uint64)])
    stats = raw[:40 * P].view(rec)
    gmu = raw[40 * P:40 * P + 8].view(f32)
    body = raw[40 * P + 8:].view(f32)
    assert body.size == (P + 1) * n
    ref = O.step(g, e, w, 0.1, mode)
    for p in range(P):
        assert_array_close(body[p * n:(p + 1) * n], ref.e_new[p], f"e[{p}]")
    assert_array_close(body[P * n:], ref.w_new, "w")
    if three == 2:
        return
    for p in range(P):
        r = ref.workers[p]
        assert (int(stats[p]["n_pos"]), int(stats[p]["n_neg"]), int(stats[p]["n_zero"]), int(stats[p]["n_nan"])) == \
            (r.n_pos, r.n_neg, r.n_zero, r.n_nan)
        assert abs(float(stats[p]["mu_pos"]) - r.mu_pos) <= 1e-5 * abs(r.mu_pos)
        assert abs(float(stats[p]["mu_neg"]) - r.mu_neg) <= 1e-5 * abs(r.mu_neg)
    assert abs(float(gmu[0]) - ref.gmu_pos) <= 1e-5 * abs(ref.gmu_pos) and abs(float(gmu[1]) - ref.gmu_neg) <= 1e-5 * abs(ref.gmu_neg)


@pytest.mark.parametrize("ranks,per_rank,n,mode", [(4, 1, 70_003, 0), (3, 1, 4099, 1), (2, 2, 300_001, 0),
                                                     (4, 1, 14_000_003, 0)])
def test_line_5_done_by_the_caller_as_on_several_gpus(A, ranks, per_rank, n, mode):
    """The multi-GPU shape on one GPU: every "rank" has a plan, a workspace and a weight replica of its own for its
    per_rank workers; the ranks exchange only their local pairs, here through a device-side average that stands in
    for the all-reduce (summed in rank order in fp64, one rounding, as Algorithm 1 line 5 is defined).  With one
    worker per rank this is Algorithm 1 as each worker runs it: checked against the oracle's per-replica step;
    with several workers per rank each rank's w is the mean of its own workers' updates."""
    P = ranks * per_rank
    g, e, w = make_case(n + P, n, P)
    plans = [A.a2sgd_plan(n, per_rank, mode) for _ in range(ranks)]
    wss = [A.alloc_workspace(pl) for pl in plans]
    gd, ed = [dev(x) for x in g], [dev(x) for x in e]
    wd = [dev(w) for _ in range(ranks)]
    pairs = torch.empty(ranks, 2 * per_rank, dtype=torch.float32, device="cuda")
    for r in range(ranks):
        sl = slice(r * per_rank, (r + 1) * per_rank)
        A.a2sgd_local_averages(plans[r], gd[sl], ed[sl], wss[r])
        A.a2sgd_export_local_means(plans[r], wss[r], pairs[r])
    allp = pairs.view(P, 2).double()
    gmu = (allp.sum(dim=0) / P).float().contiguous()  # the stand-in for the all-reduce (average) of 2 floats
    for r in range(ranks):
        sl = slice(r * per_rank, (r + 1) * per_rank)
        A.a2sgd_import_global_means(plans[r], wss[r], gmu)
        A.a2sgd_apply_and_update_error(plans[r], gd[sl], ed[sl], wd[r], 0.1, wss[r])
    # the same exchange on the lazy state (fresh buffers; materialised afterwards): same weights, same errors
    sd = [dev(x) for x in e]
    wl_ = [dev(w) for _ in range(ranks)]
    wsl = [A.alloc_workspace(pl) for pl in plans]
    pairs_l = torch.empty_like(pairs)
    for r in range(ranks):
        sl = slice(r * per_rank, (r + 1) * per_rank)
        A.a2sgd_lazy_reset(plans[r], wsl[r])
        A.a2sgd_lazy_local_averages(plans[r], gd[sl], sd[sl], wsl[r])
        A.a2sgd_export_local_means(plans[r], wsl[r], pairs_l[r])
    gmu_l = (pairs_l.view(P, 2).double().sum(dim=0) / P).float().contiguous()
    for r in range(ranks):
        sl = slice(r * per_rank, (r + 1) * per_rank)
        A.a2sgd_import_global_means(plans[r], wsl[r], gmu_l)
        A.a2sgd_lazy_apply(plans[r], sd[sl], wl_[r], 0.1, wsl[r])
        A.a2sgd_lazy_materialize(plans[r], sd[sl], wsl[r])
    workers, gmu_ref, e_ref, w_ref = O.step_replicas(g, e, [w] * P, 0.1, mode)
    for r in range(ranks):
        mine = np.mean(np.stack([w_ref[r * per_rank + q].astype(np.float64) for q in range(per_rank)]), axis=0)
        assert_array_close(wl_[r].cpu().numpy(), mine.astype(f32), f"lazy w of rank {r}")
        for q in range(per_rank):
            assert_array_close(sd[r * per_rank + q].cpu().numpy(), e_ref[r * per_rank + q], f"lazy e[{r * per_rank + q}]")
    assert abs(float(gmu[0]) - gmu_ref[0]) <= 1e-5 * abs(gmu_ref[0]) and abs(float(gmu[1]) - gmu_ref[1]) <= 1e-5 * abs(gmu_ref[1])
    for r in range(ranks):
        st, gm = A.a2sgd_read_stats(plans[r], wss[r])
        for q in range(per_rank):
            p = r * per_rank + q
            assert (st[q].n_pos, st[q].n_neg, st[q].n_zero) == (workers[p].n_pos, workers[p].n_neg, workers[p].n_zero)
            assert_array_close(ed[p].cpu().numpy(), e_ref[p], f"e[{p}]")
        assert gm == (float(gmu[0]), float(gmu[1]))
        mine = np.mean(np.stack([w_ref[r * per_rank + q].astype(np.float64) for q in range(per_rank)]), axis=0)
        assert_array_close(wd[r].cpu().numpy(), mine.astype(f32), f"w of rank {r}")


def test_device_info(A):
    info = A.a2sgd_device_info()
    assert info["compute_units"] >= 64 and info["total_memory_bytes"] > 64 << 30
    assert info["memory_bus_bits"] >= 1024 and info["memory_clock_khz"] > 100_000 and info["l2_bytes"] > 0


def test_grid_barrier_gives_up_instead_of_hanging(A):
    """The bounded wait of the single-launch step's barrier, forced from the host on a spare cell: all workgroups
    pass a complete barrier; all give up, and exit, when one arrival is missing.  Steps still work afterwards."""
    scratch = torch.empty(4096, dtype=torch.uint8, device="cuda")
    A.a2sgd_selftest_barrier(scratch)
    A.a2sgd_selftest_barrier(scratch)  # the spare cell was cleared: the test can run again
    g, e, w = make_case(8, 100_003, 4)
    check_against_oracle(A, g, e, w, 0.1, 0, split_calls=False, want_mask=False)
