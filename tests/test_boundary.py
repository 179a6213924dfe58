"""CPU-only checks of the C ABI: the library loads, exports everything include/a2sgd.h declares, and rejects bad
arguments before launching anything (so these run with no GPU present)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "a2sgd.h")


@pytest.fixture(scope="module")
def A():
    import paper_2006_07405_amd as A
    return A


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(a2sgd_[a-z_]+)\s*\(", src)))


def test_header_functions_are_exported(A):
    names = declared_functions()
    assert {"a2sgd_plan", "a2sgd_local_averages", "a2sgd_global_average", "a2sgd_apply_and_update_error",
            "a2sgd_step", "a2sgd_read_stats", "a2sgd_export_mask", "a2sgd_dense_step", "a2sgd_workspace_bytes",
            "a2sgd_plan_destroy", "a2sgd_status_string", "a2sgd_plan_blocks_per_worker"} <= set(names)
    lib = C.CDLL(A.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in a2sgd.h but not exported"


def test_binding_has_the_same_names(A):
    for name in declared_functions():
        if name == "a2sgd_plan_destroy" or name == "a2sgd_status_string":
            continue  # owned by Plan.__del__ / A2sgdError
        assert hasattr(A, name), f"binding lacks {name}"


def test_struct_layouts_match_header(A):
    from paper_2006_07405_amd import binding as B
    assert C.sizeof(B.a2sgd_worker_stats_t) == 40
    assert C.sizeof(B.a2sgd_config_t) == 48
    assert C.sizeof(B.a2sgd_global_stats_t) == 8
    assert C.sizeof(B.a2sgd_device_info_t) == 32
    assert A.raw.a2sgd_device_info(None) == A.A2SGD_ERR_INVALID_ARG


@pytest.mark.parametrize("n,P,mode,bpw", [(0, 4, 0, 0), (10, 0, 0, 0), (10, 65, 0, 0), (10, 4, 2, 0), (10, 4, -1, 0),
                                          ((1 << 38) + 1, 4, 0, 0), (10, 4, 0, 65537)])
def test_plan_rejects_bad_config(A, n, P, mode, bpw):
    with pytest.raises(A.A2sgdError) as ei:
        A.a2sgd_plan(n, P, mode, bpw)
    assert ei.value.status == A.A2SGD_ERR_INVALID_ARG


def test_plan_null_pointers(A):
    from paper_2006_07405_amd import binding as B
    cfg = B.a2sgd_config_t(10, 2, 0, 0, 0, None)
    h = C.c_void_p()
    assert A.raw.a2sgd_plan(None, C.byref(h)) == A.A2SGD_ERR_INVALID_ARG
    assert A.raw.a2sgd_plan(C.byref(cfg), None) == A.A2SGD_ERR_INVALID_ARG
    cfg.num_segments = 3  # segments announced, no lengths given
    assert A.raw.a2sgd_plan(C.byref(cfg), C.byref(h)) == A.A2SGD_ERR_INVALID_ARG
    assert A.raw.a2sgd_workspace_bytes(None) == 0
    assert A.raw.a2sgd_plan_destroy(None) == A.A2SGD_OK


def test_plan_geometry(A):
    p = A.a2sgd_plan(1_500_000_000, 4)
    assert A.a2sgd_plan_blocks_per_worker(p) == 128  # 256 CUs x 2 resident workgroups / 4 workers
    # header, the 128 records per worker of the reduction pass, then (256-byte aligned) one record per 2048
    # elements and worker for the lazy state's reduction pass and one per 4096 of those, then (aligned again) one
    # sign bit per element and worker, rounded up to whole 2048-element blocks
    blocks = -(-(1_500_000_000 // 4) // 512)
    records = 4096 + 5 * 8 * 4 * 128 + 5 * 8 * 4 * (blocks + -(-blocks // 4096))
    assert A.a2sgd_workspace_bytes(p) == -(-records // 256) * 256 + 4 * blocks * 2048 // 8
    p = A.a2sgd_plan(5, 3)
    assert A.a2sgd_plan_blocks_per_worker(p) == 1
    p = A.a2sgd_plan(1 << 38, 64)  # the largest plan: host arithmetic only, sizes stay in 64 bits
    assert A.a2sgd_plan_blocks_per_worker(p) == 8
    assert A.a2sgd_workspace_bytes(p) > 64 * (1 << 38) // 8
    p = A.a2sgd_plan(1000, 2, blocks_per_worker=7)
    assert A.a2sgd_plan_blocks_per_worker(p) == 7


def test_segmented_plan_validation_and_workspace(A):
    for bad in ([5, 4], [5, 6], [10, 0], [0, 10], [3, 3, 3]):
        with pytest.raises(A.A2sgdError) as ei:
            A.a2sgd_plan(10, 2, 0, 0, seg_lengths=bad)
        assert ei.value.status == A.A2SGD_ERR_INVALID_ARG
    whole = A.a2sgd_plan(1_000_000, 4)
    seg = A.a2sgd_plan(1_000_000, 4, 0, 0, seg_lengths=[1, 70_000, 3, 929_996])
    # the tables of the per-tensor plan come after the header and the whole-model partial records
    assert A.a2sgd_workspace_bytes(seg) > 4096 + 5 * 8 * 4 * A.a2sgd_plan_blocks_per_worker(whole)
    one = A.a2sgd_plan(1_000_000, 4, 0, 0, seg_lengths=[1_000_000])  # one tensor: the same means, the tensor path
    assert one.num_segments == 1
    # retained-error mode keeps one sign bit per element and worker for the lazy state and the two-kernel apply pass,
    # in rows of 2048 elements, at the very end of the workspace; literal mode has no use for them
    for n, P, lengths in ((1_000_000, 4, [1, 70_000, 3, 929_996]), (2049, 3, [2049]), (3, 1, [1, 2]), (8192, 9, [4096, 4096])):
        ret = A.a2sgd_plan(n, P, 0, 0, seg_lengths=lengths)
        lit = A.a2sgd_plan(n, P, 1, 0, seg_lengths=lengths)
        rows = max(1, -(-(n >> 2) // 512))
        assert A.a2sgd_workspace_bytes(ret) - A.a2sgd_workspace_bytes(lit) == 256 * P * rows
    # with offsets: ascending, not overlapping, inside [0, n); sizes need not add up to n
    ok = A.a2sgd_plan(100, 2, 0, 0, seg_lengths=[10, 20, 5], seg_offsets=[3, 13, 90])
    assert ok.num_segments == 3
    for lengths, offsets in (([10, 20], [5, 14]), ([10, 20], [20, 0]), ([10, 20], [0, 81]), ([10], [100]), ([0], [5])):
        with pytest.raises(A.A2sgdError) as ei:
            A.a2sgd_plan(100, 2, 0, 0, seg_lengths=lengths, seg_offsets=offsets)
        assert ei.value.status == A.A2SGD_ERR_INVALID_ARG
    # pooled means and offsets belong to plans with tensors
    from paper_2006_07405_amd import binding as B
    h = C.c_void_p()
    for cfg in (B.a2sgd_config_t(10, 2, 0, 0, 0, None, None, 1, 0),
                B.a2sgd_config_t(10, 2, 0, 0, 0, None, (C.c_uint64 * 1)(0), 0, 0),
                B.a2sgd_config_t(10, 2, 0, 0, 1, (C.c_uint64 * 1)(10), None, 2, 0),
                B.a2sgd_config_t(10, 2, 0, 0, 1, (C.c_uint64 * 1)(10), None, 0, -2)):
        assert A.raw.a2sgd_plan(C.byref(cfg), C.byref(h)) == A.A2SGD_ERR_INVALID_ARG
    pooled = A.a2sgd_plan(100, 2, 0, 0, seg_lengths=[10, 20], seg_offsets=[4, 50], pooled_means=True)
    assert A.raw.a2sgd_read_stats(pooled.handle, None, None, None, None) == A.A2SGD_ERR_INVALID_ARG  # NULL workspace
    R = A.raw
    assert R.a2sgd_read_stats(seg.handle, 0x30000, None, None, None) == A.A2SGD_ERR_INVALID_ARG
    assert R.a2sgd_read_segment_stats(whole.handle, 0x30000, None, None, None) == A.A2SGD_ERR_INVALID_ARG
    assert R.a2sgd_workspace_init(whole.handle, 0x30000, None) == A.A2SGD_OK  # nothing to upload


def test_grid_barrier_cells_are_owned_by_live_plans(A):
    """A plan whose model fits the caches owns one of the 64 grid-barrier cells from a2sgd_plan to
    a2sgd_plan_destroy: live plans never share a cell, a plan made while all are taken runs the three passes, and
    destroying a plan frees its cell for the next one."""
    import gc
    gc.collect()  # plans of earlier tests give their cells back when they are collected
    plans, cells = [], []
    for _ in range(70):
        p = A.a2sgd_plan(5000, 2)
        c = A.a2sgd_plan_single_launch_cell(p)
        if c < 0:
            spare = p
            break
        plans.append(p)
        cells.append(c)
    else:
        raise AssertionError("more than 64 plans got a cell")
    assert 1 <= len(cells) <= 64 and len(set(cells)) == len(cells) and all(0 <= c < 64 for c in cells)
    assert A.a2sgd_plan_single_launch_cell(spare) == -1
    # the workspace does not depend on whether the plan got a cell
    assert A.a2sgd_workspace_bytes(spare) == A.a2sgd_workspace_bytes(plans[0])
    # models too large for the caches never take one
    assert A.a2sgd_plan_single_launch_cell(A.a2sgd_plan(1 << 28, 4)) == -1
    victim = plans.pop(len(plans) // 2)
    freed = A.a2sgd_plan_single_launch_cell(victim)
    assert A.raw.a2sgd_plan_destroy(victim.handle) == A.A2SGD_OK
    victim.handle = None
    again = A.a2sgd_plan(5000, 2)
    assert A.a2sgd_plan_single_launch_cell(again) == freed
    assert A.a2sgd_plan_single_launch_cell(A.a2sgd_plan(5000, 2)) == -1  # all taken once more
    assert A.raw.a2sgd_plan_single_launch_cell(None) == -1
    del plans, again, spare
    gc.collect()
    # plans with tensors take one too, unless their means are pooled
    assert A.a2sgd_plan_single_launch_cell(A.a2sgd_plan(5000, 2, seg_lengths=[5000], pooled_means=True)) == -1
    assert A.a2sgd_plan_single_launch_cell(A.a2sgd_plan(5000, 2, seg_lengths=[3000, 2000])) >= 0
    assert A.a2sgd_plan_single_launch_cell(A.a2sgd_plan(5000, 2)) >= 0


def test_workspace_check_and_new_status_codes(A):
    plan = A.a2sgd_plan(1000, 2)
    need = A.a2sgd_workspace_bytes(plan)
    R, h = A.raw, plan.handle
    assert R.a2sgd_workspace_check(h, 0x30000, need) == A.A2SGD_OK
    assert R.a2sgd_workspace_check(h, 0x30000, need + 1) == A.A2SGD_OK
    assert R.a2sgd_workspace_check(h, 0x30000, need - 1) == A.A2SGD_ERR_WORKSPACE_TOO_SMALL
    assert R.a2sgd_workspace_check(h, 0x30000, 0) == A.A2SGD_ERR_WORKSPACE_TOO_SMALL
    assert R.a2sgd_workspace_check(h, None, need) == A.A2SGD_ERR_INVALID_ARG
    assert R.a2sgd_workspace_check(None, 0x30000, need) == A.A2SGD_ERR_INVALID_ARG
    assert R.a2sgd_workspace_check(h, 0x30008, need) == A.A2SGD_ERR_ALIGNMENT
    assert A.A2SGD_ERR_WORKSPACE_TOO_SMALL == 5 and A.A2SGD_ERR_WORKSPACE_STATE == 6
    assert b"workspace" in R.a2sgd_status_string(5) and b"a2sgd_workspace_init" in R.a2sgd_status_string(6)
    assert R.a2sgd_status_string(99) == b"unknown status"


def test_plan_for_a_device(A):
    """The device index is part of the plan; -1 means no check.  (What a mismatch does is a GPU test.)"""
    assert A.a2sgd_plan(1000, 2, device=0).handle and A.a2sgd_plan(1000, 2, device=3).handle
    with pytest.raises(A.A2sgdError) as ei:
        A.a2sgd_plan(1000, 2, device=-2)
    assert ei.value.status == A.A2SGD_ERR_INVALID_ARG


def _tab(vals):
    return (C.c_void_p * len(vals))(*vals)


def test_step_calls_validate_before_launch(A):
    """Hand-made pointer values: nothing is dereferenced on the host, and every call must fail in validation."""
    plan = A.a2sgd_plan(1000, 2)
    good = _tab([0x10000, 0x20000])
    misaligned = _tab([0x10000, 0x20004])
    with_null = _tab([0x10000, 0])
    ws, w = 0x30000, 0x40000
    R, h = A.raw, plan.handle
    INV, ALN = A.A2SGD_ERR_INVALID_ARG, A.A2SGD_ERR_ALIGNMENT
    assert R.a2sgd_local_averages(None, good, good, ws, None) == INV
    assert R.a2sgd_local_averages(h, None, good, ws, None) == INV
    assert R.a2sgd_local_averages(h, good, None, ws, None) == INV  # retained-error mode needs e
    assert R.a2sgd_local_averages(h, with_null, good, ws, None) == INV
    assert R.a2sgd_local_averages(h, good, misaligned, ws, None) == ALN
    assert R.a2sgd_local_averages(h, good, good, None, None) == INV
    assert R.a2sgd_local_averages(h, good, good, ws + 8, None) == ALN
    assert R.a2sgd_global_average(None, ws, None) == INV
    assert R.a2sgd_global_average(h, None, None) == INV
    assert R.a2sgd_apply_and_update_error(h, good, good, None, 0.1, ws, None) == INV
    assert R.a2sgd_apply_and_update_error(h, good, good, w + 4, 0.1, ws, None) == ALN
    assert R.a2sgd_apply_and_update_error(h, misaligned, good, w, 0.1, ws, None) == ALN
    assert R.a2sgd_step(h, good, with_null, w, 0.1, ws, None) == INV
    assert R.a2sgd_step(h, good, good, w, 0.1, ws + 4, None) == ALN
    assert R.a2sgd_export_mask(h, good, good, None, None) == INV
    assert R.a2sgd_export_mask(h, good, misaligned, ws, None) == ALN
    assert R.a2sgd_dense_step(h, None, w, 0.1, None) == INV
    assert R.a2sgd_dense_step(h, good, w + 2, 0.1, None) == ALN
    assert R.a2sgd_read_stats(h, None, None, None, None) == INV
    assert R.a2sgd_export_local_means(h, ws, None, None) == INV
    assert R.a2sgd_export_local_means(h, ws, 0x50002, None) == ALN
    assert R.a2sgd_import_global_means(h, None, 0x50000, None) == INV
    assert R.a2sgd_import_global_means(h, ws + 8, 0x50000, None) == ALN
    # aliasing: a written buffer may not overlap anything else of the call; read-only ones may coincide
    other = _tab([0x50000, 0x60000])
    same_g = _tab([0x10000, 0x10000])
    assert R.a2sgd_step(h, good, good, w, 0.1, ws, None) == INV                    # e^p is g^p
    assert R.a2sgd_step(h, good, _tab([0x50000, 0x50000 + 3984]), w, 0.1, ws, None) == INV  # e^0 and e^1 overlap by 16 B
    assert R.a2sgd_step(h, good, other, 0x50000 + 2000, 0.1, ws, None) == INV      # w inside e^0
    assert R.a2sgd_apply_and_update_error(h, good, other, w, 0.1, 0x60000 + 1600, None) == INV  # workspace inside e^1
    assert R.a2sgd_local_averages(h, good, other, 0x10000 + 3200, None) == INV     # workspace inside g^0
    assert R.a2sgd_dense_step(h, good, 0x20000 + 160, 0.1, None) == INV            # w inside g^1
    assert R.a2sgd_lazy_step(h, same_g, other, 0x50000 + 800, 0.1, ws, None) == INV
    assert R.a2sgd_step_replicas(h, same_g, other, _tab([0x70000, 0x70000]), 0.1, ws, None) == INV  # w^0 is w^1
    assert R.a2sgd_status_string(ALN) == b"device pointer not 16-byte aligned"


def test_step_static_validates_before_it_touches_the_device(A):
    """The entry point for callers that cannot allocate rejects bad arguments, plans with tensors and plans whose
    records do not fit its built-in array, all before the first HIP call."""
    R = A.raw
    INV, ALN = A.A2SGD_ERR_INVALID_ARG, A.A2SGD_ERR_ALIGNMENT
    plan = A.a2sgd_plan(1000, 2)
    good, other = _tab([0x10000, 0x20000]), _tab([0x50000, 0x60000])
    w = 0x40000
    assert R.a2sgd_step_static(None, good, other, w, 0.1, None) == INV
    assert R.a2sgd_step_static(plan.handle, good, None, w, 0.1, None) == INV
    assert R.a2sgd_step_static(plan.handle, good, other, None, 0.1, None) == INV
    assert R.a2sgd_step_static(plan.handle, good, other, w + 8, 0.1, None) == ALN
    assert R.a2sgd_step_static(plan.handle, good, good, w, 0.1, None) == INV  # e^p is g^p
    tensors = A.a2sgd_plan(1000, 2, seg_lengths=[400, 600])
    assert R.a2sgd_step_static(tensors.handle, good, other, w, 0.1, None) == INV
    # 4096 + 40 * P * B bytes must fit the array
    limit = (A.A2SGD_STATIC_SCRATCH_BYTES - 4096) // (40 * 2)
    big = A.a2sgd_plan(1000, 2, blocks_per_worker=limit + 1)
    assert R.a2sgd_step_static(big.handle, good, other, w, 0.1, None) == A.A2SGD_ERR_SCRATCH_LIMIT
    assert A.A2SGD_ERR_SCRATCH_LIMIT == 7 and b"built-in" in R.a2sgd_status_string(7)
    # every plan that lets the library choose the grid fits
    for n, P in ((1 << 38, 64), (1_500_000_000, 4), (5, 1), (138_357_544, 16)):
        assert 4096 + 40 * P * A.a2sgd_plan_blocks_per_worker(A.a2sgd_plan(n, P)) <= A.A2SGD_STATIC_SCRATCH_BYTES


def test_binding_checks_shapes_without_touching_the_gpu(A):
    import torch
    plan = A.a2sgd_plan(100, 2)
    cpu = [torch.zeros(100), torch.zeros(100)]
    with pytest.raises(TypeError):
        A.a2sgd_local_averages(plan, cpu, cpu, torch.zeros(1000))
    with pytest.raises(ValueError):
        A.a2sgd_local_averages(plan, cpu[:1], cpu, torch.zeros(1000))


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2006_07405_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2006_07405_amd" not in text and "a2sgd.h" not in text


def test_bench_refuses_more_than_one_gpu():
    """One GPU is all this build uses: the benchmark says so and exits before it touches torch or the device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=60)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout == ""


def test_streaming_kernel_library_loads_and_validates():
    """The benchmark's plain streaming kernels (bandwidth ceilings) are a library of their own: it loads, prices its
    launches, and turns bad arguments down before any launch."""
    path = os.path.join(ROOT, "paper_2006_07405_amd", "libhbm_streams.so")
    assert os.path.exists(path), "run build() first"
    L = C.CDLL(path)
    L.hbm_stream_bytes.restype = C.c_uint64
    L.hbm_stream_bytes.argtypes = [C.c_int, C.c_int, C.c_int, C.c_uint64]
    L.hbm_stream_run.argtypes = [C.c_int, C.POINTER(C.c_void_p), C.c_int, C.c_int, C.c_uint64, C.c_void_p]
    n = 1 << 20
    assert [L.hbm_stream_bytes(k, 9, 5, n) for k in (0, 1, 2, 3, 4, 5)] == [4 * n, 8 * n, 12 * n, 56 * n, 4 * n, 0]
    tab = (C.c_void_p * 9)(*[0x10000 * (k + 1) for k in range(9)])
    assert L.hbm_stream_run(1, None, 2, 1, n, None) == 1       # no table
    assert L.hbm_stream_run(7, tab, 2, 1, n, None) == 1        # unknown kind
    assert L.hbm_stream_run(1, tab, 2, 1, n + 1, None) == 1    # whole float4 groups only
    assert L.hbm_stream_run(3, tab, 8, 4, n, None) == 1        # the mix is 2P + 1 read, P + 1 written
    assert L.hbm_stream_run(3, tab, 9, 4, n, None) == 1
    bad = (C.c_void_p * 2)(0x10000, 0x20004)
    assert L.hbm_stream_run(1, bad, 2, 1, n, None) == 2        # alignment


def test_header_is_plain_c(tmp_path):
    """include/a2sgd.h compiles as C99 with no extensions and no other headers than the two standard ones."""
    import subprocess
    src = tmp_path / "client.c"
    src.write_text('#include "a2sgd.h"\n'
                   "int main(void)\n{\n    a2sgd_config_t cfg;\n    a2sgd_worker_stats_t st;\n"
                   "    cfg.n = 1;\n    st.n_pos = 0;\n"
                   "    return (int)(cfg.n + st.n_pos) - 1 + (int)sizeof(a2sgd_device_info_t) - 32;\n}\n")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                           "-I", os.path.join(ROOT, "include"), str(src)])
