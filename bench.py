#!/usr/bin/env python3
"""Benchmark of the A2SGD step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic gradients: a2sgd_local_averages ->
a2sgd_global_average -> a2sgd_apply_and_update_error (Algorithm 1 lines 3-7), with g, e and w already resident
in HBM.  The same g is reused every step; e and w evolve, which does not change the traffic.

Prints ONE JSON line: params/s (model parameters updated per second) of the headline workload (config 5 unless
--config says otherwise), the roofline of the dominant kernel (the fused apply pass) from HIP events recorded around
it on the launch stream in every timed step, the same figures for the other four workloads (`other_configs`),
bandwidth ceilings measured in this run with plain streaming kernels (`hbm_reference`), and the CPU oracle timed on
this machine's host cores (`cpu_baseline`: one thread, a bounded sample; `cpu_baseline_threads`: one whole streamed step
on the host's cores).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--no-cpu-baseline] [--no-other-configs]
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak

# HBM bytes per launch of the apply kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this program, each
# scaled by the same counter's reading of a plain copy of known size.  This run reads no counter: the figure is
# carried over from the named profile, and the JSON line says so in roofline.traffic_source.
MEASURED_TRAFFIC = {"config5": (8.40001e10, "profiles/a2sgd_step_config5_hbm_counters.txt (rocprofv3 --pmc, an earlier "
                                            "run of this command; not measured in this run)")}


def time_steps(A, torch, plan, g, e, w, eta, ws, steps, warmup, single_call=False, hip_graph=False):
    """W untimed steps, then K timed ones between two synchronisations.  Returns wall ms per step and, for the
    three-call form, the per-kernel averages and the median step from HIP events on the launch stream."""
    def step(ev=None):
        if single_call:
            A.a2sgd_step(plan, g, e, w, eta, ws)
            return
        if ev is not None:
            ev[0].record()
        A.a2sgd_local_averages(plan, g, e, ws)
        if ev is not None:
            ev[1].record()
        A.a2sgd_global_average(plan, ws)
        if ev is not None:
            ev[2].record()
        A.a2sgd_apply_and_update_error(plan, g, e, w, eta, ws)
        if ev is not None:
            ev[3].record()

    for _ in range(warmup):
        step()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    torch.cuda.synchronize()
    if hip_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        t0 = time.perf_counter()
        for k in range(steps):
            step(events[k])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    res = {"ms_per_step": (t1 - t0) * 1e3 / steps, "ms_median": None, "ms_reduce": None, "ms_global": None,
           "ms_apply": None}
    if not (single_call or hip_graph):
        res["ms_median"] = sorted(ev[0].elapsed_time(ev[3]) for ev in events)[steps // 2]
        res["ms_reduce"] = sum(ev[0].elapsed_time(ev[1]) for ev in events) / steps
        res["ms_global"] = sum(ev[1].elapsed_time(ev[2]) for ev in events) / steps
        res["ms_apply"] = sum(ev[2].elapsed_time(ev[3]) for ev in events) / steps
    return res


def alloc_and_fill(torch, wl):
    """The big buffers are allocated before anything else touches the device heap, then filled in place."""
    n, P = wl.n, wl.num_workers
    g = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(P)]
    e = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(P)]  # every workload starts from e = 0
    w = torch.empty(n, dtype=torch.float32, device="cuda")
    for p in range(P):
        wl.gradient(p, 0, out=g[p])
    wl.weights(out=w)
    return g, e, w


def other_config(A, torch, workloads, k, steps, warmup):
    """The same measurement on one of the other workloads, reduced to a few figures."""
    wl = workloads.FULL[k]()
    n, P = wl.n, wl.num_workers
    g, e, w = alloc_and_fill(torch, wl)
    plan = A.a2sgd_plan(n, P, A.A2SGD_MODE_RETAINED_ERROR)
    ws = A.alloc_workspace(plan)
    t = time_steps(A, torch, plan, g, e, w, wl.eta, ws, steps, warmup)
    bytes_step, bytes_apply = 20 * n * P + 8 * n, 12 * n * P + 8 * n
    out = {"workload": f"config{k}:{wl.name}", "n": n, "num_workers": P, "steps": steps,
           "ms_per_step": t["ms_per_step"], "params_per_s": n / (t["ms_per_step"] * 1e-3),
           "kernels_ms": {"local_averages": t["ms_reduce"], "global_average": t["ms_global"],
                          "apply_and_update_error": t["ms_apply"]},
           "step_hbm_gbps": bytes_step / (t["ms_per_step"] * 1e-3) / 1e9,
           "step_frac_of_peak": bytes_step / (t["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
           "apply_frac_of_peak": bytes_apply / (t["ms_apply"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
           "cache_resident": A.a2sgd_plan_single_launch_cell(plan) >= 0}
    # a2sgd_step: the same passes in one call with no events recorded between them (what a caller who wants no
    # per-pass times pays; at the smaller sizes the events cost several percent)
    t1 = time_steps(A, torch, plan, g, e, w, wl.eta, ws, steps, warmup, single_call=True)
    if out["cache_resident"]:
        # g + e + w fit the last-level cache: the fractions above are not HBM fractions, and a2sgd_step is one launch
        out["ms_per_step_single_launch"] = t1["ms_per_step"]
    else:
        out["ms_per_step_one_call"] = t1["ms_per_step"]
    del g, e, w, ws
    torch.cuda.empty_cache()
    return out


def hbm_ceilings(torch, g, e, w):
    """Plain streaming kernels (csrc/hbm_streams.hip) on the headline workload's own buffers, after everything else
    has been measured (they overwrite e and w): GB/s of a read stream, a write stream, a copy, an add of two streams
    and the apply pass's mix of 2P + 1 read and P + 1 write streams.  None for a figure that cannot be measured here.
    `apply_pass_ms_at_plain_rates`: the time the apply pass's bytes would take if its reads went at the plain read
    stream's rate and its writes at the plain write stream's, one after the other."""
    path = os.path.join(ROOT, "paper_2006_07405_amd", "libhbm_streams.so")
    if not os.path.exists(path):
        return {"error": "libhbm_streams.so is not built"}
    L = ctypes.CDLL(path)
    L.hbm_stream_run.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_void_p), ctypes.c_int, ctypes.c_int,
                                 ctypes.c_uint64, ctypes.c_void_p]
    L.hbm_stream_bytes.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_uint64]
    L.hbm_stream_bytes.restype = ctypes.c_uint64
    P, n = len(g), w.numel() & ~3
    stream = torch.cuda.current_stream().cuda_stream
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def run(kind, bufs, reads, writes, reps=5):
        tab = (ctypes.c_void_p * len(bufs))(*[b.data_ptr() for b in bufs])
        if L.hbm_stream_run(kind, tab, reads, writes, n, stream) != 0:
            return None
        ev0.record()
        for _ in range(reps):
            L.hbm_stream_run(kind, tab, reads, writes, n, stream)
        ev1.record()
        torch.cuda.synchronize()
        return L.hbm_stream_bytes(kind, reads, writes, n) / (ev0.elapsed_time(ev1) / reps * 1e-3) / 1e9

    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    out = {"read_gbps": run(0, [g[0], sink], 1, 0), "copy_gbps": run(1, [g[0], e[0]], 2, 1)}
    out["add_gbps"] = run(2, [e[0], g[0], g[1 % P]], 3, 1)
    out["fill_gbps"] = run(4, [e[0]], 0, 1)
    if out["read_gbps"] and out["fill_gbps"]:
        out["apply_pass_ms_at_plain_rates"] = ((8 * P + 4) * n / out["read_gbps"] + (4 * P + 4) * n / out["fill_gbps"]) / 1e6
    mix = f"mix_{2 * P + 1}r_{P + 1}w_gbps"
    out[mix] = run(3, list(e) + [w] + list(g), 2 * P + 1, P + 1) if P in (1, 2, 4, 8, 16) else None
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--blocks-per-worker", type=int, default=0)
    ap.add_argument("--n", type=int, default=0, help="override n (config 1 only: one flat tensor)")
    ap.add_argument("--workers", type=int, default=0, help="override P (config 1 only)")
    ap.add_argument("--table1", choices=["fnn3", "resnet20", "vgg16_cifar"], default=None,
                    help="instead of a benchmark configuration: one of the paper's own small models (Table 1) as "
                         "per-layer tensors; combine with --per-tensor and --single-call, --workers sets P (default 4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short runs of the other four workloads (they are part of the default run only)")
    ap.add_argument("--per-tensor", action="store_true",
                    help="one pair of means per worker and tensor of the workload's layout instead of per worker")
    ap.add_argument("--pooled", action="store_true",
                    help="with --per-tensor: the plan knows the tensors but every worker has one pair of means over all "
                         "of them together (the whole-model method on the tensor path)")
    ap.add_argument("--single-call", action="store_true",
                    help="time a2sgd_step (one call per step; a single cooperative launch when the model fits the "
                         "caches) instead of the three calls with events between them")
    ap.add_argument("--replicas", action="store_true",
                    help="also time the step with one weight vector per worker (outside the timed region)")
    ap.add_argument("--hip-graph", action="store_true",
                    help="capture one step in a HIP graph and time its replays (no events inside the step)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain copy of n floats (for scaling rocprofv3 HBM counters)")
    ap.add_argument("--cpu-sample", type=int, default=1 << 28, help="parameters in the single-thread CPU-baseline sample")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the P workers are simulated as P buffer pairs on it. "
              "--gpus must be 1.", file=sys.stderr)
        return 2

    import torch
    import paper_2006_07405_amd as A
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = workloads.FULL[args.config]()
    if args.table1:
        wl = workloads.table1(args.table1, num_workers=args.workers or 4)
    elif args.n or args.workers:
        assert args.config == 1, "--n and --workers apply to the flat workload of config 1"
        wl = workloads.config1(n=args.n or wl.n, num_workers=args.workers or wl.num_workers)
    n, P = wl.n, wl.num_workers
    g, e, w = alloc_and_fill(torch, wl)
    seg = [numel for _, numel in wl.tensors] if args.per_tensor else None
    plan = A.a2sgd_plan(n, P, A.A2SGD_MODE_RETAINED_ERROR, args.blocks_per_worker, seg_lengths=seg,
                        pooled_means=bool(seg) and args.pooled)
    ws = A.alloc_workspace(plan)

    if args.calibration_copy:
        # a plain device-to-device copy of known size (4n bytes read, 4n written), for scaling HBM counters
        scratch = torch.empty_like(w)
        scratch.copy_(w)
        torch.cuda.synchronize()
        del scratch

    t = time_steps(A, torch, plan, g, e, w, wl.eta, ws, args.steps, args.warmup, args.single_call, args.hip_graph)
    ms_per_step = t["ms_per_step"]
    no_events = args.single_call or args.hip_graph  # then the roofline entry is the whole step
    bytes_reduce = 8 * n * P
    bytes_apply = 12 * n * P + 8 * n
    bytes_step = bytes_reduce + bytes_apply
    ms_reduce, ms_global, ms_apply = t["ms_reduce"], t["ms_global"], t["ms_apply"]
    if no_events:
        ms_apply = ms_per_step
        bytes_apply = bytes_step
    achieved = bytes_apply / (ms_apply * 1e-3) / 1e9
    if plan.num_segments:
        seg_stats, seg_gmu = A.a2sgd_read_segment_stats(plan, ws)
        stats, gmu = [row[0] for row in seg_stats], seg_gmu[0]
    else:
        stats, gmu = A.a2sgd_read_stats(plan, ws)
    traffic, traffic_source = (None, None) if (no_events or plan.num_segments or args.n or args.workers or args.table1) else \
        MEASURED_TRAFFIC.get(f"config{args.config}", (None, None))

    out = {
        "metric": "a2sgd_step_params_per_s",
        "value": n / (ms_per_step * 1e-3),
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": wl.name if args.table1 else f"config{args.config}:{wl.name}", "n": n, "num_workers": P, "seed": wl.seed,
                   "recipe": wl.recipe, "mode": "retained_error", "eta": wl.eta, "per_tensor_means": plan.num_segments, "pooled_means": bool(seg) and args.pooled,
                   "blocks_per_worker": A.a2sgd_plan_blocks_per_worker(plan),
                   "launch": ("one_call" if args.single_call else "three_calls") + ("+hip_graph_replay" if args.hip_graph else "")},
        "ms_per_step_median_events": t["ms_median"],
        "worker_params_per_s": n * P / (ms_per_step * 1e-3),
        "step_hbm_gbps": bytes_step / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_peak": bytes_step / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "kernels_ms": {"local_averages": ms_reduce, "global_average": ms_global, "apply_and_update_error": ms_apply},
        "local_averages_gbps": None if ms_reduce is None else bytes_reduce / (ms_reduce * 1e-3) / 1e9,
        "roofline": {"kernel": "whole step" if no_events else "k_apply (a2sgd_apply_and_update_error)",
                     "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "algorithmic_bytes_per_launch": bytes_apply,
                     "traffic": traffic, "traffic_source": traffic_source},
        "result_check": {"gmu_pos": gmu[0], "gmu_neg": gmu[1], "n_pos_worker0": stats[0].n_pos},
    }

    # Outside the timed region: the dense data-parallel step (Eq. 1; Algorithm 1 lines 9-10) on the same buffers,
    # the "no compression" reference (reads every g and w once, writes w once).
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    A.a2sgd_dense_step(plan, g, w, wl.eta)
    ev0.record()
    for _ in range(5):
        A.a2sgd_dense_step(plan, g, w, wl.eta)
    ev1.record()
    torch.cuda.synchronize()
    ms_dense = ev0.elapsed_time(ev1) / 5
    out["dense_step"] = {"ms": ms_dense, "gbps": (4 * n * P + 8 * n) / (ms_dense * 1e-3) / 1e9,
                         "params_per_s": n / (ms_dense * 1e-3)}

    if args.replicas:
        # Algorithm 1 line 7 as each worker runs it: 8nP bytes for the reduction, 20nP for the apply pass
        wr = [w.clone() for _ in range(P)]
        A.a2sgd_step_replicas(plan, g, e, wr, wl.eta, ws)
        ev0.record()
        for _ in range(5):
            A.a2sgd_step_replicas(plan, g, e, wr, wl.eta, ws)
        ev1.record()
        torch.cuda.synchronize()
        ms_rep = ev0.elapsed_time(ev1) / 5
        out["replica_step"] = {"ms": ms_rep, "gbps": 28 * n * P / (ms_rep * 1e-3) / 1e9,
                               "params_per_s": n / (ms_rep * 1e-3)}
        del wr

    if True:
        # The same step on the lazy error state: the buffers keep v, the error is formed on the next read, and in
        # this mode the apply pass reads one sign bit per element-worker that the reduction pass left (12nP + 8n
        # bytes plus nP/8 written and read), with whole-model and with per-tensor means.  A different contract for
        # what e holds.
        lazy_bytes = 12.25 * n * P + 8 * n
        A.a2sgd_lazy_reset(plan, ws)
        for _ in range(2):
            A.a2sgd_lazy_step(plan, g, e, w, wl.eta, ws)
        ev0.record()
        for _ in range(5):
            A.a2sgd_lazy_step(plan, g, e, w, wl.eta, ws)
        ev1.record()
        torch.cuda.synchronize()
        ms_lazy = ev0.elapsed_time(ev1) / 5
        ev0.record()
        A.a2sgd_lazy_materialize(plan, e, ws)
        ev1.record()
        torch.cuda.synchronize()
        out["lazy_step"] = {"ms": ms_lazy, "gbps": lazy_bytes / (ms_lazy * 1e-3) / 1e9,
                            "params_per_s": n / (ms_lazy * 1e-3), "materialize_ms": ev0.elapsed_time(ev1)}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, g, w, min(args.cpu_sample, n))
        out["cpu_baseline_threads"] = cpu_baseline_threads(torch, wl, g, w)

    # Bandwidth references measured in this run, on this workload's buffers, last of all: a torch copy of n floats
    # and the plain streaming kernels, which overwrite e and w.
    scratch = torch.empty_like(w)
    scratch.copy_(w)
    ev0.record()
    for _ in range(5):
        scratch.copy_(w)
    ev1.record()
    torch.cuda.synchronize()
    del scratch
    out["hbm_reference"] = {"published_peak_gbps": HBM_PEAK_GBPS, "used_for_frac": "published_peak_gbps",
                            "torch_copy_gbps": 8 * n / (ev0.elapsed_time(ev1) / 5 * 1e-3) / 1e9,
                            "plain_streaming_kernels": hbm_ceilings(torch, g, e, w),
                            "device_reports": A.a2sgd_device_info()}
    copy_gbps = out["hbm_reference"]["plain_streaming_kernels"].get("copy_gbps")
    if copy_gbps:
        out["step_frac_of_plain_copy"] = out["step_hbm_gbps"] / copy_gbps

    default_run = args.config == 5 and not (args.n or args.workers or args.per_tensor or args.single_call or args.hip_graph
                                            or args.table1)
    if default_run and not args.no_other_configs:
        del g, e, w, ws
        torch.cuda.empty_cache()
        out["other_configs"] = [other_config(A, torch, workloads, k, 50, args.warmup) for k in (1, 2, 3, 4)]
    print(json.dumps(out))
    return 0


def cpu_baseline_threads(torch, wl, g, w, chunk=1 << 21, group=16):
    """One whole step of the oracle over ALL n parameters of all P workers, streamed: the gradients and weights come
    from the GPU in groups of `group` chunks (copies not timed), and the oracle's own calls run on a pool of host
    threads (the C calls release the interpreter lock): pass A feeds one accumulator per worker in index order (one
    thread per worker), pass B runs one chunk per task.  The arithmetic and its order per worker are the oracle's
    own.  e = 0, the workload's first step."""
    import numpy as np
    from concurrent.futures import ThreadPoolExecutor
    from oracle import a2sgd_oracle as O
    n, P = wl.n, wl.num_workers
    threads = max(1, min(16, len(os.sched_getaffinity(0))))
    O.lib()
    span = chunk * group
    stage_g = [torch.empty(span, dtype=torch.float32, pin_memory=True) for _ in range(P)]
    stage_w = torch.empty(span, dtype=torch.float32, pin_memory=True)
    zeros = np.zeros(chunk, dtype=np.float32)
    accs = [O.LocalAccumulator() for _ in range(P)]
    seconds = 0.0
    with ThreadPoolExecutor(threads) as pool:
        def fetch(lo, hi, with_w):
            for p in range(P):
                stage_g[p][:hi - lo].copy_(g[p][lo:hi])
            if with_w:
                stage_w[:hi - lo].copy_(w[lo:hi])
            torch.cuda.synchronize()
            return [x[:hi - lo].numpy() for x in stage_g], stage_w[:hi - lo].numpy()

        for lo in range(0, n, span):
            hi = min(n, lo + span)
            gh, _ = fetch(lo, hi, False)

            def pass_a(p):
                for a in range(0, hi - lo, chunk):
                    b = min(hi - lo, a + chunk)
                    accs[p].feed(gh[p][a:b], zeros[:b - a])

            t0 = time.perf_counter()
            list(pool.map(pass_a, range(P)))
            seconds += time.perf_counter() - t0
        workers = [a.stats() for a in accs]
        gp, gn = O.global_means(workers)
        for lo in range(0, n, span):
            hi = min(n, lo + span)
            gh, wh = fetch(lo, hi, True)

            def pass_b(a):
                b = min(hi - lo, a + chunk)
                O.apply_chunk([x[a:b] for x in gh], [zeros[:b - a]] * P, wh[a:b], workers, gp, gn, wl.eta,
                              O.RETAINED_ERROR)

            t0 = time.perf_counter()
            list(pool.map(pass_b, range(0, hi - lo, chunk)))
            seconds += time.perf_counter() - t0
    return {"value": n / seconds, "unit": "params/s", "cores": threads, "kind": "oracle", "seconds": seconds,
            "sample": f"all {n} parameters of all {P} workers, one whole streamed step (both passes), e = 0; pass A on "
                      f"min(P, cores) = {min(P, threads)} threads (one worker each), pass B on {threads} threads (one "
                      f"chunk of {chunk} each); device-to-host copies not timed"}


def cpu_baseline(wl, g, w, m):
    """The oracle as it stands, single-threaded, on the first m parameters of every worker: one whole step (both
    passes).  Only the compute is timed; the device-to-host copies are not."""
    import numpy as np
    from oracle import a2sgd_oracle as O
    P = wl.num_workers
    gh = [x[:m].cpu().numpy() for x in g]
    eh = [np.zeros(m, dtype=np.float32) for _ in range(P)]
    wh = w[:m].cpu().numpy()
    O.lib()
    t0 = time.perf_counter()
    O.step(gh, eh, wh, wl.eta, O.RETAINED_ERROR)
    dt = time.perf_counter() - t0
    return {"value": m / dt, "unit": "params/s", "cores": 1, "kind": "oracle", "seconds": dt,
            "sample": f"first {m} of {wl.n} parameters of all {P} workers, one whole step (both passes), e = 0"}


if __name__ == "__main__":
    sys.exit(main())
