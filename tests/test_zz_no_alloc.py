"""a2sgd_step_static, the step for callers that cannot allocate: its outputs against those of the existing entry
points on the same inputs, on two calls in a row, the second with a smaller input (the built-in scratch array keeps
what the first call left).  Collected last, so that a failure here hides no other test."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import a2sgd_oracle as O
from tests.helpers import assert_array_close, dev

pytestmark = pytest.mark.gpu
f32 = np.float32


@pytest.fixture(scope="module")
def A():
    import paper_2006_07405_amd as A
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return A


def make_case(seed, n, P):
    rng = np.random.default_rng(seed)
    g = [(rng.standard_normal(n) * 1e-3).astype(f32) for _ in range(P)]
    e = [(rng.standard_normal(n) * 5e-4).astype(f32) for _ in range(P)]
    w = (rng.standard_normal(n) * 0.02).astype(f32)
    return g, e, w


def run_three_calls(A, plan, g, e, w, eta):
    ws = A.alloc_workspace(plan)
    gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
    A.a2sgd_local_averages(plan, gd, ed, ws)
    A.a2sgd_global_average(plan, ws)
    A.a2sgd_apply_and_update_error(plan, gd, ed, wd, eta, ws)
    torch.cuda.synchronize()
    return [x.cpu().numpy() for x in ed], wd.cpu().numpy()


def run_step(A, plan, g, e, w, eta):
    ws = A.alloc_workspace(plan)
    gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
    A.a2sgd_step(plan, gd, ed, wd, eta, ws)
    torch.cuda.synchronize()
    return [x.cpu().numpy() for x in ed], wd.cpu().numpy()


@pytest.mark.parametrize("mode", [0, 1])
def test_two_calls_in_a_row_the_second_smaller(A, mode):
    # first a model that takes the streaming kernels and 128 partial records per worker, then a small one
    for seed, (n, P) in enumerate([(6_300_003, 4), (70_001, 3)]):
        print(f"case mode={mode} n={n} P={P}", flush=True)
        g, e, w = make_case(40 + seed, n, P)
        plan = A.a2sgd_plan(n, P, mode)
        gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        A.a2sgd_step_static(plan, gd, ed, wd, 0.1)
        torch.cuda.synchronize()
        if seed == 1:  # (the process's first call into the library may make the runtime load its code object)
            assert torch.cuda.mem_get_info()[0] == free_before, "the call changed the amount of free device memory"
        e_got, w_got = [x.cpu().numpy() for x in ed], wd.cpu().numpy()
        # the same kernels on a caller's workspace: bit for bit
        e_three, w_three = run_three_calls(A, plan, g, e, w, 0.1)
        assert np.array_equal(w_got.view(np.uint32), w_three.view(np.uint32))
        for p in range(P):
            assert np.array_equal(e_got[p].view(np.uint32), e_three[p].view(np.uint32))
        # a2sgd_step (the single launch for the small model): within the tolerance of every parity test
        e_step, w_step = run_step(A, plan, g, e, w, 0.1)
        assert_array_close(w_got, w_step, "w against a2sgd_step")
        for p in range(P):
            assert_array_close(e_got[p], e_step[p], f"e[{p}] against a2sgd_step")
        # and the oracle
        ref = O.step(g, e, w, 0.1, mode)
        assert_array_close(w_got, ref.w_new, "w against the oracle")
        for p in range(P):
            assert_array_close(e_got[p], ref.e_new[p], f"e[{p}] against the oracle")
        for p in range(P):  # g is read-only
            assert np.array_equal(gd[p].cpu().numpy(), g[p])


def test_carried_state_over_several_calls_and_literal_mode_without_e(A):
    n, P = 300_001, 5
    g, e, w = make_case(7, n, P)
    plan = A.a2sgd_plan(n, P, 0)
    gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
    e_o, w_o = e, w
    for t in range(3):
        A.a2sgd_step_static(plan, gd, ed, wd, 0.05)
        ref = O.step(g, e_o, w_o, 0.05, 0)
        e_o, w_o = ref.e_new, ref.w_new
    assert_array_close(wd.cpu().numpy(), w_o, "w after 3 calls")
    for p in range(P):
        assert_array_close(ed[p].cpu().numpy(), e_o[p], f"e[{p}] after 3 calls")
    lit = A.a2sgd_plan(n, P, 1)
    wd = dev(w)
    A.a2sgd_step_static(lit, gd, None, wd, 0.05)
    assert_array_close(wd.cpu().numpy(), O.step(g, None, w, 0.05, 1).w_new, "literal mode, e = NULL")


def test_captured_in_a_hip_graph(A):
    """One of the callers the entry point is for: code under stream capture.  After one eager call (which looks the
    array's address up), the call is captured and replayed three times with eager work and host waits between the
    replays; every replay must leave what an eager call leaves."""
    n, P = 2_000_003, 4
    g, e, w = make_case(11, n, P)
    plan = A.a2sgd_plan(n, P, 0)
    gd = [dev(x) for x in g]
    e_ref, w_ref = [dev(x) for x in e], dev(w)
    expected = []
    for _ in range(3):
        A.a2sgd_step_static(plan, gd, e_ref, w_ref, 0.1)
        expected.append(([x.clone() for x in e_ref], w_ref.clone()))
    ed, wd = [dev(x) for x in e], dev(w)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        A.a2sgd_step_static(plan, gd, ed, wd, 0.1)
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        busy = (w_ref * 2.0).sum().item()  # unrelated eager work and a host wait between replays
        assert busy == busy
        assert torch.equal(wd, expected[k][1]), f"replay {k}: w differs from the eager call"
        assert all(torch.equal(a, b) for a, b in zip(ed, expected[k][0])), f"replay {k}: e differs from the eager call"


def test_limits_and_argument_errors(A):
    n, P = 1_000_000, 2
    g, e, w = make_case(9, n, P)
    gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
    # 40 bytes per record: 4096 + 40 * P * B must fit 256 KiB
    fits = A.a2sgd_plan(n, P, 0, blocks_per_worker=(A.A2SGD_STATIC_SCRATCH_BYTES - 4096) // (40 * P))
    A.a2sgd_step_static(fits, gd, ed, wd, 0.1)
    ref = O.step(g, e, w, 0.1, 0)
    assert_array_close(wd.cpu().numpy(), ref.w_new, "w with the largest grid that fits")
    before = wd.clone()
    too_big = A.a2sgd_plan(n, P, 0, blocks_per_worker=(A.A2SGD_STATIC_SCRATCH_BYTES - 4096) // (40 * P) + 1)
    with pytest.raises(A.A2sgdError) as ei:
        A.a2sgd_step_static(too_big, gd, ed, wd, 0.1)
    assert ei.value.status == A.A2SGD_ERR_SCRATCH_LIMIT
    tensors = A.a2sgd_plan(n, P, 0, seg_lengths=[n // 2, n - n // 2])
    with pytest.raises(A.A2sgdError) as ei:
        A.a2sgd_step_static(tensors, gd, ed, wd, 0.1)
    assert ei.value.status == A.A2SGD_ERR_INVALID_ARG
    R, h = A.raw, fits.handle
    tab = (C.c_void_p * P)(*[x.data_ptr() for x in gd])
    etab = (C.c_void_p * P)(*[x.data_ptr() for x in ed])
    assert R.a2sgd_step_static(None, tab, etab, wd.data_ptr(), 0.1, None) == A.A2SGD_ERR_INVALID_ARG
    assert R.a2sgd_step_static(h, tab, None, wd.data_ptr(), 0.1, None) == A.A2SGD_ERR_INVALID_ARG  # retained mode needs e
    assert R.a2sgd_step_static(h, tab, etab, None, 0.1, None) == A.A2SGD_ERR_INVALID_ARG
    assert R.a2sgd_step_static(h, tab, etab, wd.data_ptr() + 4, 0.1, None) == A.A2SGD_ERR_ALIGNMENT
    assert R.a2sgd_step_static(h, tab, tab, wd.data_ptr(), 0.1, None) == A.A2SGD_ERR_INVALID_ARG  # e^p is g^p
    torch.cuda.synchronize()
    assert torch.equal(wd, before), "a refused call must not have enqueued anything"
