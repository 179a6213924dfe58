"""GPU tests of what the boundary promises beyond the arithmetic: grid-barrier cells owned by live plans (two
single-launch steps at once on two streams), plans bound to a device, a tensor plan on a workspace that was never
initialised, the sign words that the lazy state stores (bit for bit against the oracle's mask), and the streaming
stores of the kernels that the other files do not reach at large worker counts."""
import gc

import numpy as np
import pytest
import torch

import workloads
from oracle import a2sgd_oracle as O
from tests.helpers import stored_sign_bits, assert_array_close, compare_stats, dev
from tests.test_gpu_parity import make_case

pytestmark = pytest.mark.gpu
f32 = np.float32


@pytest.fixture(scope="module")
def A():
    import paper_2006_07405_amd as A
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return A


@pytest.mark.parametrize("n,P", [(1_048_576, 4), (1_048_576, 8)])
def test_two_single_launch_steps_at_once_on_two_streams(A, n, P):
    """Two plans made 64 plans apart (the distance at which cells used to repeat), each with its own cell, run their
    single-launch steps on two streams at the same time for several steps; both must match the oracle.  Both grids
    have 256 workgroups: the device must hold the two together (two workgroups per compute unit at every P)."""
    gc.collect()
    first = A.a2sgd_plan(n, P, 0)
    fillers = [A.a2sgd_plan(4096, 1, 0) for _ in range(63)]
    del fillers[1:]  # 62 cells free again; the next plan gets the lowest free one, not first's
    second = A.a2sgd_plan(n, P, 0)
    cells = (A.a2sgd_plan_single_launch_cell(first), A.a2sgd_plan_single_launch_cell(second))
    print(f"cells {cells}", flush=True)
    assert cells[0] >= 0 and cells[1] >= 0 and cells[0] != cells[1]
    plans = (first, second)
    cases = [make_case(100 + k, n, P) for k in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ws = [A.alloc_workspace(pl) for pl in plans]
    gd = [[dev(x) for x in c[0]] for c in cases]
    ed = [[dev(x) for x in c[1]] for c in cases]
    wd = [dev(c[2]) for c in cases]
    torch.cuda.synchronize()
    steps = 6
    for _ in range(steps):
        for k in range(2):
            with torch.cuda.stream(streams[k]):
                A.a2sgd_step(plans[k], gd[k], ed[k], wd[k], 0.1, ws[k])
    for k in range(2):
        streams[k].synchronize()
    for k in range(2):
        g, e, w = cases[k]
        for _ in range(steps):
            ref = O.step(g, e, w, 0.1, 0)
            e, w = ref.e_new, ref.w_new
        with torch.cuda.stream(streams[k]):
            stats, gmu = A.a2sgd_read_stats(plans[k], ws[k])
        compare_stats(stats, gmu, ref)
        for p in range(P):
            assert_array_close(ed[k][p].cpu().numpy(), e[p], f"plan {k} e[{p}] after {steps} steps")
        assert_array_close(wd[k].cpu().numpy(), w, f"plan {k} w after {steps} steps")


def test_plan_bound_to_a_device(A):
    """A plan made for device 0 runs here; one made for device 1 refuses every launching call on this one-GPU machine
    before anything is enqueued: outputs stay as they were."""
    n, P = 70_001, 3
    g, e, w = make_case(5, n, P)
    gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
    good = A.a2sgd_plan(n, P, 0, device=0)
    ws = A.alloc_workspace(good)
    other = A.a2sgd_plan(n, P, 0, device=1)
    for call in (lambda: A.a2sgd_step(other, gd, ed, wd, 0.1, ws),
                 lambda: A.a2sgd_local_averages(other, gd, ed, ws),
                 lambda: A.a2sgd_global_average(other, ws),
                 lambda: A.a2sgd_apply_and_update_error(other, gd, ed, wd, 0.1, ws),
                 lambda: A.a2sgd_dense_step(other, gd, wd, 0.1),
                 lambda: A.a2sgd_lazy_reset(other, ws),
                 lambda: A.a2sgd_lazy_step(other, gd, ed, wd, 0.1, ws)):
        with pytest.raises(A.A2sgdError) as ei:
            call()
        assert ei.value.status == A.A2SGD_ERR_DEVICE
    torch.cuda.synchronize()
    assert np.array_equal(wd.cpu().numpy(), w) and all(np.array_equal(ed[p].cpu().numpy(), e[p]) for p in range(P))
    A.a2sgd_step(good, gd, ed, wd, 0.1, ws)
    ref = O.step(g, e, w, 0.1, 0)
    assert_array_close(wd.cpu().numpy(), ref.w_new, "w")


def test_tensor_plan_on_a_workspace_that_was_not_initialised(A):
    """Forgetting a2sgd_workspace_init (or initialising for another plan) must not index through garbage tables: the
    step computes nothing, leaves e and w as they were, and the stats call says why.  After the init it works."""
    seg = [1000, 70_001, 3, 29_000]
    n, P = sum(seg), 3
    g, e, w = make_case(21, n, P)
    plan = A.a2sgd_plan(n, P, 0, seg_lengths=seg)
    other = A.a2sgd_plan(n, P, 0, seg_lengths=[seg[0] + 1, seg[1] - 1] + seg[2:])
    nbytes = A.a2sgd_workspace_bytes(plan)
    assert A.a2sgd_workspace_bytes(other) == nbytes
    rng = np.random.default_rng(3)
    for fill in ("zeros", "noise", "other plan"):
        print(f"case {fill}", flush=True)
        if fill == "noise":  # small garbage where the tables live: as indices they would point anywhere in the tables
            ws = torch.from_numpy(rng.integers(0, 1 << 12, (nbytes + 7) // 8, dtype=np.int64)).cuda()
        else:
            ws = torch.zeros((nbytes + 7) // 8, dtype=torch.int64, device="cuda")
        if fill == "other plan":
            A.a2sgd_workspace_init(other, ws)
        gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
        A.a2sgd_step(plan, gd, ed, wd, 0.1, ws)
        with pytest.raises(A.A2sgdError) as ei:
            A.a2sgd_read_segment_stats(plan, ws)
        assert ei.value.status == A.A2SGD_ERR_WORKSPACE_STATE
        assert np.array_equal(wd.cpu().numpy(), w) and all(np.array_equal(ed[p].cpu().numpy(), e[p]) for p in range(P))
        A.a2sgd_workspace_init(plan, ws)
        A.a2sgd_step(plan, gd, ed, wd, 0.1, ws)
        A.a2sgd_read_segment_stats(plan, ws)
        _, e_ref, w_ref = O.step_segmented(g, e, w, 0.1, 0, seg)
        assert_array_close(wd.cpu().numpy(), w_ref, "w")
        for p in range(P):
            assert_array_close(ed[p].cpu().numpy(), e_ref[p], f"e[{p}]")
    # pooled means report through a2sgd_read_stats
    pooled = A.a2sgd_plan(n, P, 0, seg_lengths=seg, pooled_means=True)
    ws = torch.zeros((A.a2sgd_workspace_bytes(pooled) + 7) // 8, dtype=torch.int64, device="cuda")
    gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
    A.a2sgd_step(pooled, gd, ed, wd, 0.1, ws)
    with pytest.raises(A.A2sgdError) as ei:
        A.a2sgd_read_stats(pooled, ws)
    assert ei.value.status == A.A2SGD_ERR_WORKSPACE_STATE
    with pytest.raises(A.A2sgdError) as ei:
        A.a2sgd_step(plan, gd, ed, wd, 0.1, ws[:16])
    assert ei.value.status == A.A2SGD_ERR_WORKSPACE_TOO_SMALL


SIGN_SIZES = [1, 2, 3, 4, 5, 7, 8, 255, 256, 257, 1023, 2044, 2047, 2048, 2049, 2051, 2052, 4095, 4096, 4097, 4099,
              65_539]


@pytest.mark.parametrize("n,P", [(n, 3) for n in SIGN_SIZES] + [(3_500_003, 7)])
def test_stored_sign_words_equal_the_oracle_mask(A, n, P):
    """pos(v) of Eq. 2 as the library stores it (the only mask it keeps): every bit of the sign words after each of
    two lazy reductions against the oracle's mask of the same step; bits of float4 groups past the end are 0.  The
    last n % 4 elements have no stored bit (the apply pass reads their v)."""
    if P == 7:
        assert (2 * P + 1) * 4 * n > 192 << 20  # the streaming instantiation
    wl = workloads.config1(n=n, num_workers=P)
    rng = np.random.default_rng(n)
    e0 = [(rng.standard_normal(n) * 4e-4).astype(f32) for _ in range(P)]
    w0 = wl.weights().numpy()
    plan = A.a2sgd_plan(n, P, 0)
    ws = A.alloc_workspace(plan)
    ws.fill_(-1)  # stale ones everywhere: whatever is 0 afterwards was written
    s, wd = [dev(x) for x in e0], dev(w0)
    e_o, w_o = [x.copy() for x in e0], w0.copy()
    A.a2sgd_lazy_reset(plan, ws)
    covered = (n >> 2) << 2
    for t in range(2):
        g = [wl.gradient(p, t).numpy() for p in range(P)]
        gd = [dev(x) for x in g]
        ref = O.step(g, e_o, w_o, wl.eta, 0)
        A.a2sgd_lazy_local_averages(plan, gd, s, ws)
        torch.cuda.synchronize()
        bits = stored_sign_bits(A, plan, ws, n, P)
        for p in range(P):
            assert np.array_equal(bits[p, :covered], ref.mask[p][:covered]), f"step {t} worker {p}: stored signs differ"
            assert not bits[p, covered:].any(), f"step {t} worker {p}: bits past the last float4 group are set"
        A.a2sgd_global_average(plan, ws)
        A.a2sgd_lazy_apply(plan, s, wd, wl.eta, ws)
        st, gmu = A.a2sgd_read_stats(plan, ws)
        compare_stats(st, gmu, ref)
        assert_array_close(wd.cpu().numpy(), ref.w_new, f"step {t} w")
        e_o, w_o = ref.e_new, ref.w_new


def test_dense_step_on_replicas_streaming_with_64_workers(A):
    """The final synchronisation on replicas with streaming stores and the most workers the library takes."""
    n, P = 400_003, 64
    assert (2 * P + 1) * 4 * n > 192 << 20
    rng = np.random.default_rng(64)
    g = [(rng.standard_normal(n) * 1e-3).astype(f32) for _ in range(P)]
    w0 = (rng.standard_normal(n) * 0.02).astype(f32)
    wr = [(w0 + (rng.standard_normal(n) * 1e-3).astype(f32)) for _ in range(P)]
    plan = A.a2sgd_plan(n, P, 0)
    gd, wd = [dev(x) for x in g], [dev(x) for x in wr]
    A.a2sgd_dense_step_replicas(plan, gd, wd, 0.05)
    ref = O.dense_step_replicas(g, wr, 0.05)
    for p in range(P):
        assert_array_close(wd[p].cpu().numpy(), ref[p], f"dense w[{p}]")
    for p in range(P):
        assert np.array_equal(gd[p].cpu().numpy(), g[p])
