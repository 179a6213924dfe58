"""Shared by the GPU parity tests: run one step through the C ABI (via the binding) and compare with the oracle.

Tolerances (stated here once, used everywhere):
  - counts (n_pos, n_neg, n_zero, n_nan) and mask bits: equal;
  - local and global means: |gpu - ref| <= 1e-5 * |ref|;
  - e and w: |gpu_i - ref_i| <= 1e-5 * max(|ref_i|, rms(ref)).  A purely per-element relative bound is
    ill-posed for e, because v - mu cancels to about 0 wherever v is close to mu.
A wrong sign-group decision moves e by mu_pos + mu_neg, orders of magnitude above this bound, so the check
on e also verifies the mask the fused kernel used, element by element.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import a2sgd_oracle as O

RTOL = 1e-5


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def gpu_step(A, g, e, w, eta, mode=0, blocks_per_worker=0, split_calls=True, want_mask=False):
    """g, e: lists of numpy fp32 arrays (e may be None); w: numpy fp32.  Returns (stats, gmu, e_new, w_new, mask)."""
    n, P = int(w.shape[0]), len(g)
    plan = A.a2sgd_plan(n, P, mode, blocks_per_worker)
    ws = A.alloc_workspace(plan)
    gd = [dev(x) for x in g]
    ed = [dev(x) for x in e] if e is not None else None
    wd = dev(w)
    mask = None
    if want_mask:
        words = (n + 63) // 64
        md = torch.full((P * words,), -1, dtype=torch.int64, device="cuda")
        A.a2sgd_export_mask(plan, gd, ed, md)
        bits = np.unpackbits(md.cpu().numpy().view(np.uint8), bitorder="little").reshape(P, words * 64)
        assert not bits[:, n:].any(), "mask bits beyond n must be 0"
        mask = [bits[p, :n] for p in range(P)]
    if split_calls:
        A.a2sgd_local_averages(plan, gd, ed, ws)
        A.a2sgd_global_average(plan, ws)
        A.a2sgd_apply_and_update_error(plan, gd, ed, wd, eta, ws)
    else:
        A.a2sgd_step(plan, gd, ed, wd, eta, ws)
    stats, gmu = A.a2sgd_read_stats(plan, ws)
    torch.cuda.synchronize()
    for p in range(P):  # g is read-only
        assert np.array_equal(gd[p].cpu().numpy().view(np.uint32), np.ascontiguousarray(g[p]).view(np.uint32))
    e_new = [x.cpu().numpy() for x in ed] if ed is not None else None
    return stats, gmu, e_new, wd.cpu().numpy(), mask


def close(got, ref, what):
    assert abs(got - ref) <= RTOL * abs(ref), f"{what}: gpu {got!r} vs oracle {ref!r}"


def assert_array_close(got: np.ndarray, ref: np.ndarray, what: str):
    nan_g, nan_r = np.isnan(got), np.isnan(ref)
    assert np.array_equal(nan_g, nan_r), f"{what}: NaN positions differ"
    ok = ~nan_r
    if not ok.any():
        return
    r = ref[ok].astype(np.float64)
    d = np.abs(got[ok].astype(np.float64) - r)
    rms = float(np.sqrt(np.mean(r * r)))
    bound = RTOL * np.maximum(np.abs(r), rms)
    bad = d > bound
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {r.size} elements out of tolerance; worst abs err "
                           f"{float(d.max()):.3e} at rms {rms:.3e}")


def assert_chunk_close(got: np.ndarray, ref: np.ndarray, what: str):
    """assert_array_close for one chunk of a long vector (the rms that scales the bound is the chunk's own), with a
    short cut: a chunk that equals the reference bit for bit needs no arithmetic."""
    if np.array_equal(got.view(np.uint32), ref.view(np.uint32)):
        return
    assert_array_close(got, ref, what)


def compare_stats(stats, gmu, ref: "O.StepResult"):
    for p, (s, r) in enumerate(zip(stats, ref.workers)):
        assert (s.n_pos, s.n_neg, s.n_zero, s.n_nan) == (r.n_pos, r.n_neg, r.n_zero, r.n_nan), \
            f"worker {p} counts: gpu {(s.n_pos, s.n_neg, s.n_zero, s.n_nan)} oracle {(r.n_pos, r.n_neg, r.n_zero, r.n_nan)}"
        close(s.mu_pos, r.mu_pos, f"worker {p} mu_pos")
        close(s.mu_neg, r.mu_neg, f"worker {p} mu_neg")
    close(gmu[0], ref.gmu_pos, "gmu_pos")
    close(gmu[1], ref.gmu_neg, "gmu_neg")


def check_against_oracle(A, g, e, w, eta, mode=0, **kw):
    """Whole-vector parity of one step.  Returns (gpu outputs, oracle result) for further checks."""
    want_mask = kw.pop("want_mask", True)
    stats, gmu, e_new, w_new, mask = gpu_step(A, g, e, w, eta, mode, want_mask=want_mask, **kw)
    ref = O.step(g, e, w, eta, mode)
    compare_stats(stats, gmu, ref)
    if e_new is not None:
        for p in range(len(g)):
            assert_array_close(e_new[p], ref.e_new[p], f"e[{p}]")
    assert_array_close(w_new, ref.w_new, "w")
    if mask is not None:
        for p in range(len(g)):
            assert np.array_equal(mask[p], ref.mask[p]), f"mask[{p}] differs from pos(v)"
    return (stats, gmu, e_new, w_new, mask), ref


def stored_sign_bits(A, plan, ws, n, P):
    """Decodes the sign words that a2sgd_lazy_local_averages leaves at the end of the workspace in retained-error
    mode: uint16 sign[b][h][p][tid], block b covering 2048 elements, thread tid owning the float4 groups
    b*512 + (4h + u)*64 + tid, u = 0..3, whose component c is bit 15 - (4u + c).  Returns bits[P][blocks*2048] in
    element order."""
    nvec = n >> 2
    blocks = max(1, -(-nvec // 512))
    off = A.a2sgd_workspace_bytes(plan) - 256 * P * blocks
    words = ws.view(torch.uint8)[off:off + 256 * P * blocks].cpu().numpy().view(np.uint16).reshape(blocks, 2, P, 64)
    bits = np.zeros((P, blocks, 2, 4, 64, 4), np.uint8)  # [p][b][h][u][tid][c]: element b*2048 + h*1024 + u*256 + tid*4 + c
    for u in range(4):
        for c in range(4):
            bits[:, :, :, u, :, c] = ((words >> (15 - (4 * u + c))) & 1).transpose(2, 0, 1, 3)
    return bits.reshape(P, blocks * 2048)
