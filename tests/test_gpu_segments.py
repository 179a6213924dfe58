"""GPU parity of the per-tensor variant: one pair of means per worker and tensor.  The oracle is the whole-model
oracle applied to every tensor's slice (oracle.step_segmented)."""
import numpy as np
import pytest
import torch

import workloads
from oracle import a2sgd_oracle as O
from tests.helpers import assert_array_close, close, compare_stats, dev, stored_sign_bits

pytestmark = pytest.mark.gpu
f32 = np.float32


@pytest.fixture(scope="module")
def A():
    import paper_2006_07405_amd as A
    assert torch.cuda.is_available()
    return A


def run_case(A, g, e, w, eta, mode, seg, split_calls=True):
    P, n = len(g), int(w.shape[0])
    plan = A.a2sgd_plan(n, P, mode, 0, seg_lengths=seg)
    ws = A.alloc_workspace(plan)
    gd = [dev(x) for x in g]
    ed = [dev(x) for x in e] if e is not None else None
    wd = dev(w)
    if split_calls:
        A.a2sgd_local_averages(plan, gd, ed, ws)
        A.a2sgd_global_average(plan, ws)
        A.a2sgd_apply_and_update_error(plan, gd, ed, wd, eta, ws)
    else:
        A.a2sgd_step(plan, gd, ed, wd, eta, ws)
    stats, gmu = A.a2sgd_read_segment_stats(plan, ws)
    per_seg, e_ref, w_ref = O.step_segmented(g, e, w, eta, mode, seg)
    for s, r in enumerate(per_seg):
        for p in range(P):
            a, b = stats[p][s], r.workers[p]
            assert (a.n_pos, a.n_neg, a.n_zero, a.n_nan) == (b.n_pos, b.n_neg, b.n_zero, b.n_nan), f"segment {s} worker {p}"
            close(a.mu_pos, b.mu_pos, f"segment {s} worker {p} mu_pos")
            close(a.mu_neg, b.mu_neg, f"segment {s} worker {p} mu_neg")
        close(gmu[s][0], r.gmu_pos, f"segment {s} gmu_pos")
        close(gmu[s][1], r.gmu_neg, f"segment {s} gmu_neg")
    # tolerance per tensor: the rms that scales it is the tensor's own
    off = 0
    for s, length in enumerate(seg):
        lo, hi = off, off + length
        if ed is not None:
            for p in range(P):
                assert_array_close(ed[p][lo:hi].cpu().numpy(), e_ref[p][lo:hi], f"e[{p}] segment {s}")
        assert_array_close(wd[lo:hi].cpu().numpy(), w_ref[lo:hi], f"w segment {s}")
        off = hi
    return stats, gmu


def make_case(seed, n, P, scales):
    """Per-segment scales make a wrong segment assignment visible at once."""
    rng = np.random.default_rng(seed)
    g = [(rng.standard_normal(n)).astype(f32) * scales for _ in range(P)]
    e = [(rng.standard_normal(n) * 0.5).astype(f32) * scales for _ in range(P)]
    w = (rng.standard_normal(n) * 0.02).astype(f32)
    return [x.astype(f32) for x in g], [x.astype(f32) for x in e], w


def scales_for(seg, seed):
    rng = np.random.default_rng(seed)
    return np.concatenate([np.full(L, 10.0 ** rng.uniform(-5, -2), dtype=f32) for L in seg])


LAYOUTS = [
    [1, 1],
    [3, 2],
    [1, 2, 3, 4, 5, 6, 7],
    [255, 1, 256, 3, 257],
    [4096, 1, 4095, 2, 4097],
    [65_536, 65_537, 65_535, 1, 131_073],
    [5] * 300,
    [1000, 1] * 50 + [70_001],
    [300_001, 7, 200_000],
]


@pytest.mark.parametrize("seg", LAYOUTS, ids=[f"layout{i}" for i in range(len(LAYOUTS))])
def test_segment_layouts(A, seg):
    n = sum(seg)
    for P, mode, with_e, split in ((1, 0, True, True), (3, 0, True, False), (4, 1, True, True), (5, 1, False, False),
                                   (9, 0, True, True)):
        print(f"case S={len(seg)} n={n} P={P} mode={mode} e={with_e}", flush=True)
        g, e, w = make_case(n + P, n, P, scales_for(seg, n))
        run_case(A, g, e if with_e else None, w, 0.1, mode, seg, split_calls=split)


def run_padded_case(A, seed, n, P, mode, lengths, offsets, pooled, with_e=True):
    """Tensors at `offsets` inside buffers of n elements; everything outside them is padding, filled with NaN in g,
    e and w: it must come back bit for bit and must not enter any count or sum."""
    rng = np.random.default_rng(seed)
    member = np.zeros(n, bool)
    scale = np.ones(n, f32)
    for k, (o, l) in enumerate(zip(offsets, lengths)):
        member[o:o + l] = True
        scale[o:o + l] = 10.0 ** rng.uniform(-5, -2)
    g = [(rng.standard_normal(n).astype(f32) * scale) for _ in range(P)]
    e = [(rng.standard_normal(n).astype(f32) * scale * f32(0.5)) for _ in range(P)]
    w = (rng.standard_normal(n) * 0.02).astype(f32)
    for x in g + e + [w]:
        x[~member] = np.nan
    plan = A.a2sgd_plan(n, P, mode, 0, seg_lengths=lengths, seg_offsets=offsets, pooled_means=pooled)
    ws = A.alloc_workspace(plan)
    gd = [dev(x) for x in g]
    ed = [dev(x) for x in e] if with_e else None
    wd = dev(w)
    A.a2sgd_step(plan, gd, ed, wd, 0.1, ws)
    res, e_ref, w_ref = O.step_segmented(g, e if with_e else None, w, 0.1, mode, lengths, offsets, pooled)
    stats, gmu = A.a2sgd_read_segment_stats(plan, ws)
    for s in range(len(lengths)):
        r = res[0] if pooled else res[s]
        for p in range(P):
            a, b = stats[p][s], r.workers[p]
            assert (a.n_pos, a.n_neg, a.n_zero, a.n_nan) == (b.n_pos, b.n_neg, b.n_zero, b.n_nan), f"tensor {s} worker {p}"
            close(a.mu_pos, b.mu_pos, f"tensor {s} worker {p} mu_pos")
            close(a.mu_neg, b.mu_neg, f"tensor {s} worker {p} mu_neg")
        close(gmu[s][0], r.gmu_pos, f"tensor {s} gmu_pos")
        close(gmu[s][1], r.gmu_neg, f"tensor {s} gmu_neg")
    if pooled:
        st, gm = A.a2sgd_read_stats(plan, ws)
        compare_stats(st, gm, res[0])
    w_got = wd.cpu().numpy()
    assert np.isnan(w_got[~member]).all(), "padding of w was written"
    for o, l in zip(offsets, lengths):
        assert_array_close(w_got[o:o + l], w_ref[o:o + l], f"w tensor at {o}")
    if with_e:
        for p in range(P):
            e_got = ed[p].cpu().numpy()
            assert np.isnan(e_got[~member]).all(), "padding of e was written"
            for o, l in zip(offsets, lengths):
                assert_array_close(e_got[o:o + l], e_ref[p][o:o + l], f"e[{p}] tensor at {o}")


PADDED = [  # (n, lengths, offsets)
    (10, [3], [4]),
    (64, [1, 1, 1], [0, 2, 63]),
    (1000, [5, 250, 3, 100], [1, 7, 300, 900]),
    (5000, [255, 1, 256, 3, 257, 1024], [3, 258, 259, 1027, 1030, 2000]),
    (70_000, [4096, 1, 4095, 30_000], [4, 4100, 8192, 20_001]),
    (400_000, [65_536, 65_537, 131_073], [0, 65_536, 200_003]),
    (300_000, [299_000], [1000]),
]


@pytest.mark.parametrize("case", PADDED, ids=[f"padded{i}" for i in range(len(PADDED))])
def test_tensors_with_padding(A, case):
    n, lengths, offsets = case
    for P, mode, pooled, with_e in ((1, 0, False, True), (3, 0, True, True), (4, 1, False, True), (5, 1, True, False),
                                    (9, 0, True, True)):
        print(f"case n={n} S={len(lengths)} P={P} mode={mode} pooled={pooled} e={with_e}", flush=True)
        run_padded_case(A, n + P, n, P, mode, lengths, offsets, pooled, with_e)


def test_pooled_means_on_packed_tensors_equal_the_whole_model_step(A):
    """Without padding, pooled means are the paper's whole-model means: same counts as the plain plan, means equal
    to the tolerance of the sums' grouping, same e and w."""
    seg = [1000, 1, 70_001, 4096, 300_000]
    n, P = sum(seg), 4
    g, e, w = make_case(n, n, P, scales_for(seg, 3))
    ref = O.step(g, e, w, 0.1, 0)
    plan = A.a2sgd_plan(n, P, 0, 0, seg_lengths=seg, pooled_means=True)
    ws = A.alloc_workspace(plan)
    gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
    A.a2sgd_local_averages(plan, gd, ed, ws)
    A.a2sgd_global_average(plan, ws)
    A.a2sgd_apply_and_update_error(plan, gd, ed, wd, 0.1, ws)
    st, gm = A.a2sgd_read_stats(plan, ws)
    compare_stats(st, gm, ref)
    assert_array_close(wd.cpu().numpy(), ref.w_new, "w")
    for p in range(P):
        assert_array_close(ed[p].cpu().numpy(), ref.e_new[p], f"e[{p}]")


def test_streaming_size_with_padding(A):
    seg = [1_000_003, 5, 777_777, 64, 1_300_001]
    off = [7, 1_000_013, 1_000_020, 1_800_000, 1_800_257]
    n = 3_500_003
    run_padded_case(A, 11, n, 7, 0, seg, off, pooled=False)
    run_padded_case(A, 12, n, 7, 0, seg, off, pooled=True)
    # from 8 workers on the apply pass is two kernels (errors and sign bits, then the weights from the sign bits)
    run_padded_case(A, 13, n, 8, 0, seg, off, pooled=False)
    run_padded_case(A, 14, n, 9, 0, seg, off, pooled=True)


def test_two_kernel_apply_on_a_tensor_plan_with_nans(A):
    """The per-tensor apply pass in its two-kernel form (8 workers, streaming size) when some gradients are NaN: a
    NaN has no sign bit; its element of e and w becomes NaN and nothing else changes.  Two steps on carried state."""
    seg = [1_000_003, 5, 777_777, 64, 1_300_001, 131_072, 2, 291_079]
    n, P = sum(seg), 8
    assert (2 * P + 1) * 4 * n > 192 << 20
    g, e, w = make_case(n, n, P, scales_for(seg, 5))
    rng = np.random.default_rng(8)
    for p in (0, 3, P - 1):
        g[p][rng.integers(0, n, 6)] = np.nan
    g[2][n - 1] = np.nan   # the scalar tail
    g[5][1_000_003] = np.nan  # a tensor of five elements
    plan = A.a2sgd_plan(n, P, 0, 0, seg_lengths=seg)
    ws = A.alloc_workspace(plan)
    gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
    e_o, w_o = e, w
    for t in range(2):
        A.a2sgd_local_averages(plan, gd, ed, ws)
        A.a2sgd_global_average(plan, ws)
        A.a2sgd_apply_and_update_error(plan, gd, ed, wd, 0.1, ws)
        stats, gmu = A.a2sgd_read_segment_stats(plan, ws)
        res, e_o, w_o = O.step_segmented(g, e_o, w_o, 0.1, 0, seg)
        assert sum(stats[p][k].n_nan for p in range(P) for k in range(len(seg))) == sum(r.workers[p].n_nan for r in res for p in range(P)) > 0
        off = 0
        for k, length in enumerate(seg):
            for p in range(P):
                a, b = stats[p][k], res[k].workers[p]
                assert (a.n_pos, a.n_neg, a.n_zero, a.n_nan) == (b.n_pos, b.n_neg, b.n_zero, b.n_nan)
                assert_array_close(ed[p][off:off + length].cpu().numpy(), e_o[p][off:off + length], f"step {t} e[{p}] tensor {k}")
            assert_array_close(wd[off:off + length].cpu().numpy(), w_o[off:off + length], f"step {t} w tensor {k}")
            off += length


@pytest.mark.parametrize("P,mode", [(7, 0), (12, 1), (16, 0), (33, 1), (9, 0), (33, 0)])
def test_streaming_size_with_a_short_group_of_workers(A, P, mode):
    """A footprint above the cache limit (streaming kernels) with tensor boundaries of every alignment and a worker
    count that is not a multiple of the group size; 16 and 33 workers take the widest groups of the apply pass, two
    and five of them, with streaming stores."""
    seg = [1_000_003, 5, 777_777, 64, 1_300_001, 131_072, 2, 291_079]
    if P >= 16:
        seg = [600_003, 5, 477_777, 64, 500_001, 131_072, 2, 91_079]
    n = sum(seg)
    assert (2 * P + 1) * 4 * n > 192 << 20
    g, e, w = make_case(n + P, n, P, scales_for(seg, P))
    run_case(A, g, e, w, 0.1, mode, seg)


@pytest.mark.parametrize("k", [2, 3, 4, 5])
def test_small_model_shapes(A, k):
    wl = workloads.small(k)
    P = wl.num_workers
    seg = [numel for _, numel in wl.tensors]
    g = [wl.gradient(p).numpy() for p in range(P)]
    e = [wl.synthetic_error(p).numpy() for p in range(P)]
    w = wl.weights().numpy()
    run_case(A, g, e, w, wl.eta, 0, seg)


def test_empty_groups_and_nan_per_segment(A):
    seg = [4, 4, 5]
    g = [np.array([1, 2, 3, 0, -1, -2, -3, -2, 1, -1, np.nan, 2, -2], f32)]
    e = [np.zeros(13, f32)]
    stats, gmu = run_case(A, g, e, np.zeros(13, f32), 1.0, 0, seg)
    assert (stats[0][0].n_neg, stats[0][0].mu_neg, stats[0][1].n_pos, stats[0][1].mu_pos) == (0, 0.0, 0, 0.0)
    assert stats[0][2].n_nan == 1 and stats[0][2].n_pos == 2 and stats[0][2].n_neg == 2


def test_one_tensor_is_the_whole_model_method(A):
    """One tensor that covers the buffers: the tensor path must give what the whole-model oracle gives."""
    n = 50_001
    g, e, w = make_case(3, n, 3, np.full(n, 1e-3, f32))
    stats, gmu = run_case(A, g, e, w, 0.1, 0, [n])
    ref = O.step(g, e, w, 0.1, 0)
    compare_stats([row[0] for row in stats], gmu[0], ref)


def test_config2_full_size_per_tensor(A):
    """ResNet-50 shape, 161 tensors, 25.6 M parameters, 8 workers, inputs generated on the device: every tensor's
    counts and means against the oracle, e and w on the first and last tensors and on the largest one."""
    wl = workloads.config2()
    n, P = wl.n, wl.num_workers
    seg = [numel for _, numel in wl.tensors]
    plan = A.a2sgd_plan(n, P, 0, 0, seg_lengths=seg)
    ws = A.alloc_workspace(plan)
    g = [wl.gradient(p, 0, device="cuda") for p in range(P)]
    e = [wl.synthetic_error(p, device="cuda") for p in range(P)]
    w = wl.weights(device="cuda")
    gh, eh, wh = [x.cpu().numpy() for x in g], [x.cpu().numpy() for x in e], w.cpu().numpy()
    A.a2sgd_step(plan, g, e, w, wl.eta, ws)
    stats, gmu = A.a2sgd_read_segment_stats(plan, ws)
    per_seg, e_ref, w_ref = O.step_segmented(gh, eh, wh, wl.eta, 0, seg)
    offs = np.concatenate([[0], np.cumsum(seg)])
    for s, r in enumerate(per_seg):
        for p in range(P):
            a, b = stats[p][s], r.workers[p]
            assert (a.n_pos, a.n_neg, a.n_zero, a.n_nan) == (b.n_pos, b.n_neg, b.n_zero, b.n_nan)
            close(a.mu_pos, b.mu_pos, f"tensor {s} worker {p} mu_pos")
            close(a.mu_neg, b.mu_neg, f"tensor {s} worker {p} mu_neg")
        close(gmu[s][0], r.gmu_pos, f"tensor {s}")
        close(gmu[s][1], r.gmu_neg, f"tensor {s}")
    for s in sorted(set([0, 1, 2, len(seg) - 2, len(seg) - 1, int(np.argmax(seg))] + list(range(3, len(seg), 13)))):
        lo, hi = int(offs[s]), int(offs[s + 1])
        for p in range(P):
            assert_array_close(e[p][lo:hi].cpu().numpy(), e_ref[p][lo:hi], f"e[{p}] tensor {s}")
        assert_array_close(w[lo:hi].cpu().numpy(), w_ref[lo:hi], f"w tensor {s}")


# ---- one weight vector per worker, and the lazy error state, on plans with tensors ----------------------------------

def run_replica_case(A, seed, n, P, mode, lengths, offsets=None, pooled=False):
    """a2sgd_step_replicas and a2sgd_dense_step_replicas on a plan with tensors against the oracle's per-replica step
    applied tensor by tensor; padding (NaN in every buffer) must come back untouched."""
    rng = np.random.default_rng(seed)
    offs = offsets if offsets is not None else list(np.concatenate([[0], np.cumsum(lengths)[:-1]]))
    member = np.zeros(n, bool)
    scale = np.ones(n, f32)
    for o, l in zip(offs, lengths):
        member[o:o + l] = True
        scale[o:o + l] = 10.0 ** rng.uniform(-5, -2)
    g = [(rng.standard_normal(n).astype(f32) * scale) for _ in range(P)]
    e = [(rng.standard_normal(n).astype(f32) * scale * f32(0.5)) for _ in range(P)]
    w = [(rng.standard_normal(n) * 0.02).astype(f32) for _ in range(P)]
    for x in g + e + w:
        x[~member] = np.nan
    plan = A.a2sgd_plan(n, P, mode, 0, seg_lengths=lengths, seg_offsets=offsets, pooled_means=pooled)
    ws = A.alloc_workspace(plan)
    gd, ed, wd = [dev(x) for x in g], [dev(x) for x in e], [dev(x) for x in w]
    A.a2sgd_step_replicas(plan, gd, ed, wd, 0.1, ws)
    e_ref, w_ref = O.step_replicas_segmented(g, e, w, 0.1, mode, lengths, offsets, pooled)
    for p in range(P):
        e_got, w_got = ed[p].cpu().numpy(), wd[p].cpu().numpy()
        assert np.isnan(e_got[~member]).all() and np.isnan(w_got[~member]).all(), "padding was written"
        for o, l in zip(offs, lengths):
            assert_array_close(e_got[o:o + l], e_ref[p][o:o + l], f"e[{p}] tensor at {o}")
            assert_array_close(w_got[o:o + l], w_ref[p][o:o + l], f"w[{p}] tensor at {o}")


@pytest.mark.parametrize("seg", LAYOUTS, ids=[f"layout{i}" for i in range(len(LAYOUTS))])
def test_replicas_on_tensor_plans(A, seg):
    n = sum(seg)
    for P, mode in ((1, 0), (3, 1), (4, 0), (9, 1)):
        print(f"case S={len(seg)} n={n} P={P} mode={mode}", flush=True)
        run_replica_case(A, n + P, n, P, mode, seg)


@pytest.mark.parametrize("case", PADDED, ids=[f"padded{i}" for i in range(len(PADDED))])
def test_replicas_on_tensor_plans_with_padding(A, case):
    n, lengths, offsets = case
    for P, mode, pooled in ((2, 0, False), (3, 1, True), (5, 0, True)):
        print(f"case n={n} S={len(lengths)} P={P} mode={mode} pooled={pooled}", flush=True)
        run_replica_case(A, n + P, n, P, mode, lengths, offsets, pooled)


def test_replicas_on_a_tensor_plan_streaming(A):
    seg = [1_000_003, 5, 777_777, 64, 1_300_001, 131_072, 2, 291_079]
    assert (2 * 7 + 1) * 4 * sum(seg) > 192 << 20
    run_replica_case(A, 77, sum(seg), 7, 0, seg)


@pytest.mark.parametrize("P,mode,padded,pooled", [(8, 0, False, False), (9, 1, True, False), (16, 0, True, True),
                                                  (33, 1, False, False)])
def test_replicas_on_a_tensor_plan_streaming_one_worker_per_workgroup(A, P, mode, padded, pooled):
    """From 8 workers on the streaming replica pass of a plan with tensors gives every workgroup one worker's g, e
    and w^p: tensor boundaries of every alignment inside a workgroup's two lookup chunks, with and without padding
    between the tensors (NaN there, which must come back untouched)."""
    seg = [1_000_003, 5, 777_777, 64, 1_300_001, 131_072, 2, 291_079] if P < 16 else \
        [600_003, 5, 477_777, 64, 500_001, 131_072, 2, 91_079]
    offsets, n = None, sum(seg)
    if padded:
        offsets, pos = [], 3
        for k, length in enumerate(seg):
            offsets.append(pos)
            pos += length + (0, 1, 255, 1027)[k % 4]
        n = pos + 6
    assert (2 * P + 1) * 4 * n > 192 << 20
    run_replica_case(A, 90 + P, n, P, mode, seg, offsets, pooled)


def run_lazy_case(A, seed, n, P, mode, lengths, offsets=None, pooled=False, steps=4):
    """Steps on the lazy state of a plan with tensors (the buffers hold v, every tensor's pending error is formed with
    that tensor's carried means) against eager steps of the per-tensor oracle: same statistics and w at every step,
    same errors once materialised; padding untouched."""
    rng = np.random.default_rng(seed)
    offs = offsets if offsets is not None else list(np.concatenate([[0], np.cumsum(lengths)[:-1]]))
    member = np.zeros(n, bool)
    scale = np.ones(n, f32)
    for o, l in zip(offs, lengths):
        member[o:o + l] = True
        scale[o:o + l] = 10.0 ** rng.uniform(-5, -2)
    e0 = [(rng.standard_normal(n).astype(f32) * scale * f32(0.5)) for _ in range(P)]
    w0 = (rng.standard_normal(n) * 0.02).astype(f32)
    for x in e0 + [w0]:
        x[~member] = np.nan
    plan = A.a2sgd_plan(n, P, mode, 0, seg_lengths=lengths, seg_offsets=offsets, pooled_means=pooled)
    ws = A.alloc_workspace(plan)
    s, wd = [dev(x) for x in e0], dev(w0)
    e_o, w_o = [x.copy() for x in e0], w0.copy()
    A.a2sgd_lazy_reset(plan, ws)
    for t in range(steps):
        g = [(rng.standard_normal(n).astype(f32) * scale) for _ in range(P)]
        for x in g:
            x[~member] = np.nan
        gd = [dev(x) for x in g]
        res, e_o, w_o = O.step_segmented(g, e_o, w_o, 0.1, mode, lengths, offsets, pooled)
        A.a2sgd_lazy_step(plan, gd, s, wd, 0.1, ws)
        stats, gmu = A.a2sgd_read_segment_stats(plan, ws)
        for k in range(len(lengths)):
            r = res[0] if pooled else res[k]
            for p in range(P):
                a, b = stats[p][k], r.workers[p]
                assert (a.n_pos, a.n_neg, a.n_zero, a.n_nan) == (b.n_pos, b.n_neg, b.n_zero, b.n_nan), f"step {t} tensor {k} worker {p}"
                close(a.mu_pos, b.mu_pos, f"step {t} tensor {k} worker {p} mu_pos")
                close(a.mu_neg, b.mu_neg, f"step {t} tensor {k} worker {p} mu_neg")
            close(gmu[k][0], r.gmu_pos, f"step {t} tensor {k} gmu_pos")
            close(gmu[k][1], r.gmu_neg, f"step {t} tensor {k} gmu_neg")
        w_got = wd.cpu().numpy()
        assert np.isnan(w_got[~member]).all(), "padding of w was written"
        for o, l in zip(offs, lengths):
            assert_array_close(w_got[o:o + l], w_o[o:o + l], f"step {t} w tensor at {o}")
    A.a2sgd_lazy_materialize(plan, s, ws)
    for p in range(P):
        e_got = s[p].cpu().numpy()
        assert np.isnan(e_got[~member]).all(), "padding of the state was written"
        for o, l in zip(offs, lengths):
            assert_array_close(e_got[o:o + l], e_o[p][o:o + l], f"materialised e[{p}] tensor at {o}")
    # the buffers are true errors again: an eager step goes on from them
    g = [(rng.standard_normal(n).astype(f32) * scale) for _ in range(P)]
    for x in g:
        x[~member] = np.nan
    A.a2sgd_step(plan, [dev(x) for x in g], s, wd, 0.1, ws)
    _, e_o, w_o = O.step_segmented(g, e_o, w_o, 0.1, mode, lengths, offsets, pooled)
    for o, l in zip(offs, lengths):
        assert_array_close(wd.cpu().numpy()[o:o + l], w_o[o:o + l], f"eager step after materialise, w tensor at {o}")


# The lazy state's reduction goes by blocks of 2048 elements: tensors that start and end on block boundaries, a tensor
# inside one block next to such tensors, and a tensor with more whole blocks than one fold of the block records takes.
LAZY_LAYOUTS = LAYOUTS + [
    [2048, 4096, 100, 1948, 3 * 2048 + 1],
    [2048] * 5,
    [2047, 2049, 2048, 1, 4095],
    [2048 * 1100 + 5, 3],
    [7, 2048 * 2050 + 2041, 2048, 9],
]


@pytest.mark.parametrize("seg", LAZY_LAYOUTS, ids=[f"layout{i}" for i in range(len(LAZY_LAYOUTS))])
def test_lazy_state_on_tensor_plans(A, seg):
    n = sum(seg)
    for P, mode in ((1, 0), (3, 1), (4, 0), (9, 0)):
        print(f"case S={len(seg)} n={n} P={P} mode={mode}", flush=True)
        run_lazy_case(A, n + P, n, P, mode, seg)


@pytest.mark.parametrize("case", PADDED, ids=[f"padded{i}" for i in range(len(PADDED))])
def test_lazy_state_on_tensor_plans_with_padding(A, case):
    n, lengths, offsets = case
    for P, mode, pooled in ((2, 0, False), (3, 1, True), (5, 0, True)):
        print(f"case n={n} S={len(lengths)} P={P} mode={mode} pooled={pooled}", flush=True)
        run_lazy_case(A, n + P, n, P, mode, lengths, offsets, pooled, steps=3)


def test_lazy_state_on_a_tensor_plan_streaming(A):
    seg = [1_000_003, 5, 777_777, 64, 1_300_001, 131_072, 2, 291_079]
    assert (2 * 7 + 1) * 4 * sum(seg) > 192 << 20
    run_lazy_case(A, 78, sum(seg), 7, 0, seg, steps=2)
    run_lazy_case(A, 79, sum(seg), 7, 1, seg, steps=2)
    # the widest groups of the sign-reading apply pass: 16 workers at a time, then a short group
    seg = [600_003, 5, 477_777, 64, 500_001, 131_072, 2, 91_079]
    for P in (16, 33):
        assert (2 * P + 1) * 4 * sum(seg) > 192 << 20
        run_lazy_case(A, 80 + P, sum(seg), P, 0, seg, steps=2)


def test_lazy_state_on_a_tensor_plan_with_nans(A):
    """Retained-error mode on the lazy state of a plan with tensors when some gradients are NaN: a NaN has no sign bit
    in the stored words; its element of the state and of w becomes NaN, its tensor counts it, nothing else changes."""
    seg = [1_000_003, 5, 777_777, 64, 1_300_001, 131_072, 2, 291_079]
    n, P = sum(seg), 7
    assert (2 * P + 1) * 4 * n > 192 << 20
    g, e, w = make_case(n, n, P, scales_for(seg, 6))
    rng = np.random.default_rng(9)
    for p in (0, 3, P - 1):
        g[p][rng.integers(0, n, 6)] = np.nan
    g[2][n - 1] = np.nan   # the scalar tail
    g[5][1_000_003] = np.nan  # a tensor of five elements
    plan = A.a2sgd_plan(n, P, 0, 0, seg_lengths=seg)
    ws = A.alloc_workspace(plan)
    gd, s, wd = [dev(x) for x in g], [dev(x) for x in e], dev(w)
    e_o, w_o = e, w
    A.a2sgd_lazy_reset(plan, ws)
    for t in range(2):
        A.a2sgd_lazy_step(plan, gd, s, wd, 0.1, ws)
        stats, gmu = A.a2sgd_read_segment_stats(plan, ws)
        res, e_o, w_o = O.step_segmented(g, e_o, w_o, 0.1, 0, seg)
        assert sum(r.workers[p].n_nan for r in res for p in range(P)) > 0
        off = 0
        for k, length in enumerate(seg):
            for p in range(P):
                a, b = stats[p][k], res[k].workers[p]
                assert (a.n_pos, a.n_neg, a.n_zero, a.n_nan) == (b.n_pos, b.n_neg, b.n_zero, b.n_nan), f"step {t} tensor {k} worker {p}"
            assert_array_close(wd[off:off + length].cpu().numpy(), w_o[off:off + length], f"step {t} w tensor {k}")
            off += length
    A.a2sgd_lazy_materialize(plan, s, ws)
    off = 0
    for k, length in enumerate(seg):
        for p in range(P):
            assert_array_close(s[p][off:off + length].cpu().numpy(), e_o[p][off:off + length], f"materialised e[{p}] tensor {k}")
        off += length


SIGN_CASES = [  # (n, lengths, offsets or None)
    (sum(LAZY_LAYOUTS[9]), LAZY_LAYOUTS[9], None),
    (sum(LAZY_LAYOUTS[11]), LAZY_LAYOUTS[11], None),
    (sum(LAYOUTS[7]), LAYOUTS[7], None),
    (sum(LAYOUTS[2]), LAYOUTS[2], None),
    PADDED[3], PADDED[4], PADDED[6],
    (8195, [2048, 2046], [2048, 6149]),
]


@pytest.mark.parametrize("case", SIGN_CASES, ids=[f"signs{i}" for i in range(len(SIGN_CASES))])
def test_stored_sign_words_on_tensor_plans(A, case):
    """pos(v) of Eq. 2 as the lazy state of a plan with tensors stores it: every bit of the sign words after each of
    two lazy reductions against the per-tensor oracle's masks; padding, float4 groups past the end and the last n % 4
    elements have no bit."""
    n, lengths, offsets = case
    P = 3
    rng = np.random.default_rng(n)
    offs = offsets if offsets is not None else list(np.concatenate([[0], np.cumsum(lengths)[:-1]]))
    member = np.zeros(n, bool)
    for o, l in zip(offs, lengths):
        member[o:o + l] = True
    e_o = [(rng.standard_normal(n) * 0.5).astype(f32) for _ in range(P)]
    w_o = (rng.standard_normal(n) * 0.02).astype(f32)
    for x in e_o + [w_o]:
        x[~member] = np.nan
    plan = A.a2sgd_plan(n, P, 0, 0, seg_lengths=lengths, seg_offsets=offsets)
    ws = A.alloc_workspace(plan)
    ws.fill_(-1)  # stale ones everywhere: whatever is 0 afterwards was written
    A.a2sgd_workspace_init(plan, ws)
    s, wd = [dev(x) for x in e_o], dev(w_o)
    A.a2sgd_lazy_reset(plan, ws)
    covered = (n >> 2) << 2
    for t in range(2):
        g = [rng.standard_normal(n).astype(f32) for _ in range(P)]
        for x in g:
            x[~member] = np.nan
        gd = [dev(x) for x in g]
        res, e_o, w_o = O.step_segmented(g, e_o, w_o, 0.1, 0, lengths, offsets)
        A.a2sgd_lazy_local_averages(plan, gd, s, ws)
        torch.cuda.synchronize()
        bits = stored_sign_bits(A, plan, ws, n, P)
        for p in range(P):
            want = np.zeros(max(n, bits.shape[1]), np.uint8)
            for k, (o, l) in enumerate(zip(offs, lengths)):
                want[o:o + l] = res[k].mask[p]
            want[covered:] = 0
            assert np.array_equal(bits[p], want[:bits.shape[1]]), f"step {t} worker {p}: stored signs differ"
        A.a2sgd_global_average(plan, ws)
        A.a2sgd_lazy_apply(plan, s, wd, 0.1, ws)
        w_got = wd.cpu().numpy()
        for o, l in zip(offs, lengths):
            assert_array_close(w_got[o:o + l], w_o[o:o + l], f"step {t} w tensor at {o}")


def test_config2_full_size_replicas_and_lazy_state_per_tensor(A):
    """ResNet-50 shape at full size (161 tensors, 8 workers, inputs generated on the device): one per-replica step and
    one lazy step with per-tensor means, every element against the oracle."""
    wl = workloads.config2()
    n, P = wl.n, wl.num_workers
    seg = [numel for _, numel in wl.tensors]
    plan = A.a2sgd_plan(n, P, 0, 0, seg_lengths=seg)
    ws = A.alloc_workspace(plan)
    g = [wl.gradient(p, 0, device="cuda") for p in range(P)]
    gh = [x.cpu().numpy() for x in g]
    eh = [wl.synthetic_error(p).numpy() for p in range(P)]
    wh = wl.weights().numpy()
    # replicas: all start from the same weights
    ed, wr = [dev(x) for x in eh], [dev(wh) for _ in range(P)]
    A.a2sgd_step_replicas(plan, g, ed, wr, wl.eta, ws)
    e_ref, w_ref = O.step_replicas_segmented(gh, eh, [wh] * P, wl.eta, 0, seg)
    offs = np.concatenate([[0], np.cumsum(seg)])
    for p in range(P):
        e_got, w_got = ed[p].cpu().numpy(), wr[p].cpu().numpy()
        for k in range(len(seg)):
            lo, hi = int(offs[k]), int(offs[k + 1])
            assert_array_close(e_got[lo:hi], e_ref[p][lo:hi], f"replica e[{p}] tensor {k}")
            assert_array_close(w_got[lo:hi], w_ref[p][lo:hi], f"replica w[{p}] tensor {k}")
    del wr
    # lazy state: one step from true errors, then materialise
    s, wd = [dev(x) for x in eh], dev(wh)
    A.a2sgd_lazy_reset(plan, ws)
    A.a2sgd_lazy_step(plan, g, s, wd, wl.eta, ws)
    A.a2sgd_lazy_materialize(plan, s, ws)
    _, e_ref, w_ref = O.step_segmented(gh, eh, wh, wl.eta, 0, seg)
    w_got = wd.cpu().numpy()
    for k in range(len(seg)):
        lo, hi = int(offs[k]), int(offs[k + 1])
        assert_array_close(w_got[lo:hi], w_ref[lo:hi], f"lazy w tensor {k}")
    for p in range(P):
        e_got = s[p].cpu().numpy()
        for k in range(len(seg)):
            lo, hi = int(offs[k]), int(offs[k + 1])
            assert_array_close(e_got[lo:hi], e_ref[p][lo:hi], f"lazy e[{p}] tensor {k}")


# ---- the single-launch step on plans with tensors -------------------------------------------------------------------

@pytest.mark.parametrize("model,P", [("fnn3", 4), ("fnn3", 16), ("resnet20", 4), ("resnet20", 8), ("vgg16_cifar", 1)])
def test_single_launch_step_on_the_papers_own_models(A, model, P):
    """Table 1's models as per-layer tensors, small enough to stay in the caches: a2sgd_step is one kernel launch
    with per-tensor means.  Three steps on carried state in both modes, every tensor's statistics and every element
    of e and w against the per-tensor oracle; then the same plan's three calls give the same result."""
    wl = workloads.table1(model, num_workers=P)
    n = wl.n
    seg = [numel for _, numel in wl.tensors]
    offs = np.concatenate([[0], np.cumsum(seg)])
    for mode in (0, 1):
        plan = A.a2sgd_plan(n, P, mode, 0, seg_lengths=seg)
        # one launch up to about 4 M elements; the 14.7 M-parameter VGG-16 runs the three passes, which are faster there
        assert (A.a2sgd_plan_single_launch_cell(plan) >= 0) == (model != "vgg16_cifar")
        ws = A.alloc_workspace(plan)
        e_o = [wl.synthetic_error(p).numpy() for p in range(P)]
        w_o = wl.weights().numpy()
        ed, wd = [dev(x) for x in e_o], dev(w_o)
        for t in range(3):
            g = [wl.gradient(p, t).numpy() for p in range(P)]
            gd = [dev(x) for x in g]
            if t == 2:  # last step through the three calls, from the same state: the same kernels' tables, other route
                e3, w3 = [x.clone() for x in ed], wd.clone()
                A.a2sgd_local_averages(plan, gd, e3, ws)
                A.a2sgd_global_average(plan, ws)
                A.a2sgd_apply_and_update_error(plan, gd, e3, w3, wl.eta, ws)
            A.a2sgd_step(plan, gd, ed, wd, wl.eta, ws)
            stats, gmu = A.a2sgd_read_segment_stats(plan, ws)
            res, e_o, w_o = O.step_segmented(g, e_o, w_o, wl.eta, mode, seg)
            for k, r in enumerate(res):
                for p in range(P):
                    a, b = stats[p][k], r.workers[p]
                    assert (a.n_pos, a.n_neg, a.n_zero, a.n_nan) == (b.n_pos, b.n_neg, b.n_zero, b.n_nan), f"step {t} tensor {k} worker {p}"
                    close(a.mu_pos, b.mu_pos, f"step {t} tensor {k} worker {p} mu_pos")
                    close(a.mu_neg, b.mu_neg, f"step {t} tensor {k} worker {p} mu_neg")
                close(gmu[k][0], r.gmu_pos, f"step {t} tensor {k} gmu_pos")
                close(gmu[k][1], r.gmu_neg, f"step {t} tensor {k} gmu_neg")
            w_got = wd.cpu().numpy()
            for k in range(len(seg)):
                lo, hi = int(offs[k]), int(offs[k + 1])
                assert_array_close(w_got[lo:hi], w_o[lo:hi], f"step {t} w tensor {k}")
                for p in range(P):
                    assert_array_close(ed[p][lo:hi].cpu().numpy(), e_o[p][lo:hi], f"step {t} e[{p}] tensor {k}")
        for k in range(len(seg)):
            lo, hi = int(offs[k]), int(offs[k + 1])
            assert_array_close(w3[lo:hi].cpu().numpy(), w_o[lo:hi], f"three calls: w tensor {k}")


def test_single_launch_step_on_tensors_is_deterministic_and_graph_capturable(A):
    """Same inputs twice: bit-identical outputs.  Captured in a HIP graph and replayed with eager work between the
    replays: every replay equals the eager step from the same state."""
    wl = workloads.table1("resnet20", num_workers=4)
    n, P = wl.n, wl.num_workers
    seg = [numel for _, numel in wl.tensors]
    plan = A.a2sgd_plan(n, P, 0, 0, seg_lengths=seg)
    ws = A.alloc_workspace(plan)
    g = [wl.gradient(p, 0, device="cuda") for p in range(P)]
    e0 = [wl.synthetic_error(p, device="cuda") for p in range(P)]
    w0 = wl.weights(device="cuda")
    runs = []
    for _ in range(2):
        e, w = [x.clone() for x in e0], w0.clone()
        A.a2sgd_step(plan, g, e, w, wl.eta, ws)
        runs.append((e, w))
    torch.cuda.synchronize()
    assert torch.equal(runs[0][1], runs[1][1]) and all(torch.equal(a, b) for a, b in zip(runs[0][0], runs[1][0]))
    ws_ref = A.alloc_workspace(plan)
    e_ref, w_ref = [x.clone() for x in e0], w0.clone()
    expected = []
    for _ in range(3):
        A.a2sgd_step(plan, g, e_ref, w_ref, wl.eta, ws_ref)
        expected.append(([x.clone() for x in e_ref], w_ref.clone()))
    e, w = [x.clone() for x in e0], w0.clone()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        A.a2sgd_step(plan, g, e, w, wl.eta, ws)
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        busy = (w0 * 2.0).sum().item()  # unrelated eager work and a host wait between replays
        assert busy == busy
        assert torch.equal(w, expected[k][1]), f"replay {k}: w differs from the eager step"
        assert all(torch.equal(a, b) for a, b in zip(e, expected[k][0])), f"replay {k}: e differs from the eager step"


@pytest.mark.parametrize("calls,P", [("lazy", 3), ("lazy", 8), ("three", 8)])
def test_tensor_plan_steps_captured_in_a_hip_graph(A, calls, P):
    """The lazy step on a plan with tensors (one-shot reduction, fold, second level, global pass, sign-reading apply
    pass) and the eager step whose apply pass is two kernels only enqueue kernels: captured once and replayed three
    times with eager work between the replays, they leave exactly what three eager calls leave."""
    seg = [1_000_003, 5, 777_777, 64, 1_300_001, 131_072, 2, 291_079]
    n = sum(seg)
    rng = np.random.default_rng(P)
    scale = torch.from_numpy(scales_for(seg, 3)).cuda()
    g = [torch.from_numpy(rng.standard_normal(n).astype(f32)).cuda() * scale for _ in range(P)]
    e0 = [torch.from_numpy((rng.standard_normal(n) * 0.5).astype(f32)).cuda() * scale for _ in range(P)]
    w0 = torch.from_numpy((rng.standard_normal(n) * 0.02).astype(f32)).cuda()
    plan = A.a2sgd_plan(n, P, 0, 0, seg_lengths=seg)

    def one_step(e, w, ws):
        if calls == "lazy":
            A.a2sgd_lazy_step(plan, g, e, w, 0.1, ws)
        else:
            A.a2sgd_local_averages(plan, g, e, ws)
            A.a2sgd_global_average(plan, ws)
            A.a2sgd_apply_and_update_error(plan, g, e, w, 0.1, ws)

    ws_ref = A.alloc_workspace(plan)
    e_ref, w_ref = [x.clone() for x in e0], w0.clone()
    if calls == "lazy":
        A.a2sgd_lazy_reset(plan, ws_ref)
    expected = []
    for _ in range(3):
        one_step(e_ref, w_ref, ws_ref)
        expected.append(([x.clone() for x in e_ref], w_ref.clone()))
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
        assert busy == busy
        assert torch.equal(w, expected[k][1]), f"replay {k}: w differs from the eager step"
        assert all(torch.equal(a, b) for a, b in zip(e, expected[k][0])), f"replay {k}: state differs from the eager step"


def random_layout(rng, target_n, padded):
    """Tensor lengths (and offsets, if padded) with boundaries of every kind: tiny tensors, lengths around the sizes the
    kernels work in (4, 256, 1024, 2048, 4096, 65536 elements), and a few large ones."""
    lengths = []
    while sum(lengths) < target_n:
        kind = rng.random()
        if kind < 0.25:
            lengths.append(int(rng.integers(1, 10)))
        elif kind < 0.55:
            lengths.append(int(rng.integers(10, 3000)))
        elif kind < 0.8:
            unit = int(rng.choice([4, 256, 1024, 2048, 4096, 65_536]))
            lengths.append(max(1, unit * int(rng.integers(1, 4)) + int(rng.choice([-3, -1, 0, 0, 1, 3]))))
        else:
            lengths.append(int(rng.integers(3000, max(3001, target_n // 3))))
    if not padded:
        return sum(lengths), lengths, None
    offsets, pos = [], int(rng.integers(0, 6))
    for length in lengths:
        offsets.append(pos)
        gap = rng.random()
        pos += length + (0 if gap < 0.6 else int(rng.integers(1, 8)) if gap < 0.8 else
                         int(rng.integers(255, 258)) if gap < 0.9 else int(rng.integers(1000, 3000)))
    return pos + int(rng.integers(0, 10)), lengths, offsets


def run_random_case(A, rng, case, n, lengths, offsets, P, mode, pooled, path):
    print(f"case {case}: n={n} S={len(lengths)} padded={offsets is not None} P={P} mode={mode} pooled={pooled} path={path}",
          flush=True)
    if path == "step":
        offs = offsets if offsets is not None else [int(x) for x in np.concatenate([[0], np.cumsum(lengths)[:-1]])]
        run_padded_case(A, 1000 + case, n, P, mode, lengths, offs, pooled, with_e=bool(mode == 0 or rng.integers(0, 2)))
    elif path == "lazy":
        run_lazy_case(A, 1000 + case, n, P, mode, lengths, offsets, pooled, steps=2)
    else:
        run_replica_case(A, 1000 + case, n, P, mode, lengths, offsets, pooled)


def test_random_tensor_layouts_against_the_oracle(A):
    """Seeded random draws of the tensor layout (with and without padding), P, mode, pooled means and the path taken
    (a2sgd_step, the lazy state, one weight vector per worker): the combinations nobody thought of."""
    rng = np.random.default_rng(20261127)
    for case in range(36):
        padded = bool(rng.integers(0, 2))
        n, lengths, offsets = random_layout(rng, int(rng.choice([60, 3000, 40_000, 300_000])), padded)
        P = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16]))
        run_random_case(A, rng, case, n, lengths, offsets, P, int(rng.integers(0, 2)), bool(rng.integers(0, 2)),
                        str(rng.choice(["step", "lazy", "replicas"])))


@pytest.mark.parametrize("P", [8, 9, 16, 33])
def test_random_tensor_layouts_at_streaming_sizes(A, P):
    """The same draws at sizes above the cache limit, where the streaming instantiations run (non-temporal loads,
    write-through stores, the two-kernel apply pass, one worker per workgroup in the replica pass)."""
    rng = np.random.default_rng(977 + P)
    need = (192 << 20) // (4 * (2 * P + 1)) + 1
    for k, path in enumerate(["step", "lazy", "replicas"]):
        padded = bool((P + k) % 2)
        n, lengths, offsets = random_layout(rng, need + int(rng.integers(1, 5000)), padded)
        assert (2 * P + 1) * 4 * n > 192 << 20
        run_random_case(A, rng, 100 * P + k, n, lengths, offsets, P, int(k == 1 and P == 9), bool(P == 16 and k != 2), path)
