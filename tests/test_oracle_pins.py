"""CPU-only pins of the oracle: each test fixes the oracle to something other than itself.

  - a hand-worked example (tests/golden/worked_example.txt, derived from Sec. 3.1 / Eq. 2 / Algorithm 1);
  - exact rational brute force of the definitions on tiny dyadic inputs;
  - identities that follow from the definitions (reconstruction, zero-sum of errors per group, counts);
  - special cases that reduce to a textbook or library routine (P = 1 literal mode is plain SGD; Theorem 1's
    form is the dense average plus a two-valued vector; math.fsum gives the exactly rounded means);
  - symmetries (power-of-two scaling, permutation, sign flip) and closed forms for the input distributions.

The battery at the bottom re-runs the pins against builds of the C source with one planted mistake each and
requires every mutant to be caught.
"""
import math
import os
import subprocess
import tempfile
from fractions import Fraction

import numpy as np
import pytest

from oracle import a2sgd_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example.txt")
f32 = np.float32


def arr(x):
    return np.asarray(x, dtype=np.float32)


def load_golden():
    d = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        k, v = line.split("=")
        d[k.strip()] = [float(t) for t in v.split()]
    return d


# ---------------------------------------------------------------------------------------------------------
# P2: the hand-worked example
# ---------------------------------------------------------------------------------------------------------
def check_worked_example():
    G = load_golden()
    w = np.zeros(6, dtype=f32)
    e = None
    for s in ("step1", "step2"):
        g = [arr(G[f"{s}.gA"]), arr(G[f"{s}.gB"])]
        r = O.step(g, e, w, 0.5, O.RETAINED_ERROR)
        for name, st in zip("AB", r.workers):
            assert st.n_pos == G[f"{s}.{name}.n_pos"][0]
            assert st.n_neg == G[f"{s}.{name}.n_neg"][0]
            assert st.n_zero == G[f"{s}.{name}.n_zero"][0]
            assert st.n_nan == 0
            assert st.mu_pos == G[f"{s}.{name}.mu_pos"][0]
            assert st.mu_neg == G[f"{s}.{name}.mu_neg"][0]
        assert r.gmu_pos == G[f"{s}.gmu_pos"][0] and r.gmu_neg == G[f"{s}.gmu_neg"][0]
        assert np.array_equal(r.e_new[0], arr(G[f"{s}.eA"])) and np.array_equal(r.e_new[1], arr(G[f"{s}.eB"]))
        assert np.array_equal(r.mask[0], np.array(G[f"{s}.maskA"], dtype=np.uint8))
        assert np.array_equal(r.mask[1], np.array(G[f"{s}.maskB"], dtype=np.uint8))
        assert np.array_equal(r.w_new, arr(G[f"{s}.w"]))
        # U is recovered from the weights: w_new = w - eta*U
        assert np.array_equal((w.astype(np.float64) - r.w_new) / 0.5, np.array(G[f"{s}.U"]))
        e, w = r.e_new, r.w_new
    g = [arr(G["step1.gA"]), arr(G["step1.gB"])]
    r = O.step(g, None, np.zeros(6, dtype=f32), 0.5, O.ALG1_LITERAL)
    assert np.array_equal(r.w_new, arr(G["step1.literal.w"]))
    assert np.array_equal(-r.w_new.astype(np.float64) / 0.5, np.array(G["step1.literal.U"]))
    # with zero old error, passing e = zeros and e = None must agree
    r0 = O.step(g, [np.zeros(6, dtype=f32)] * 2, np.zeros(6, dtype=f32), 0.5, O.ALG1_LITERAL)
    assert np.array_equal(r0.w_new, r.w_new)


def test_worked_example():
    check_worked_example()


# ---------------------------------------------------------------------------------------------------------
# P1: exact rational brute force of the definitions on tiny dyadic inputs
# ---------------------------------------------------------------------------------------------------------
def rf32(x: Fraction) -> Fraction:
    """Round an exact rational to fp32 (through the correctly rounded double; the two roundings differ from
    one only when the double lands exactly on an fp32 midpoint, which the fixed seed below does not hit)."""
    return Fraction(float(np.float32(float(x))))


def brute_force(g, e, w, eta, mode):
    """Sec. 3.1 definitions and Algorithm 1 lines 3-7 in exact rationals, in set notation rather than running
    sums.  The only roundings are the ones the definition has: the fold g + e (exact here, inputs are short
    dyadics), the two fp32 numbers each worker transmits, the two fp32 global means, and the fp32 results."""
    P, n = len(g), len(g[0])
    F = Fraction
    v = [[F(float(g[p][i])) + F(float(e[p][i])) for i in range(n)] for p in range(P)]
    mu_pos, mu_neg = [], []
    for p in range(P):
        pos = [x for x in v[p] if x >= 0]
        neg = [-x for x in v[p] if x < 0]
        mu_pos.append(rf32(sum(pos, F(0)) / len(pos)) if pos else F(0))
        mu_neg.append(rf32(sum(neg, F(0)) / len(neg)) if neg else F(0))
    gp, gn = rf32(sum(mu_pos, F(0)) / P), rf32(sum(mu_neg, F(0)) / P)
    enc = [[mu_pos[p] if x >= 0 else -mu_neg[p] for x in v[p]] for p in range(P)]
    err = [[v[p][i] - enc[p][i] for i in range(n)] for p in range(P)]
    glob = [[gp if x >= 0 else -gn for x in v[p]] for p in range(P)]
    if mode == O.ALG1_LITERAL:
        upd = [[err[p][i] + glob[p][i] for i in range(n)] for p in range(P)]
    else:
        upd = glob
    w_new = [F(float(w[i])) - F(float(eta)) * sum((upd[p][i] for p in range(P)), F(0)) / P for i in range(n)]
    return mu_pos, mu_neg, gp, gn, [[rf32(x) for x in row] for row in err], [rf32(x) for x in w_new]


def check_brute_force(trials=60, seed=1234):
    rng = np.random.default_rng(seed)
    for t in range(trials):
        P = int(rng.integers(1, 4))
        n = int(rng.integers(1, 17))
        g = [arr(rng.integers(-32, 33, n) / 8.0) for _ in range(P)]  # multiples of 1/8 in [-4, 4]
        e = [arr(rng.integers(-16, 17, n) / 8.0) for _ in range(P)]
        w = arr(rng.integers(-64, 65, n) / 16.0)
        eta = float(2.0 ** -int(rng.integers(0, 4)))
        for mode in (O.RETAINED_ERROR, O.ALG1_LITERAL):
            r = O.step(g, e, w, eta, mode)
            mu_pos, mu_neg, gp, gn, err, w_new = brute_force(g, e, w, eta, mode)
            for p in range(P):
                assert r.workers[p].mu_pos == float(mu_pos[p]) and r.workers[p].mu_neg == float(mu_neg[p])
                assert r.workers[p].n_pos == sum(1 for i in range(n) if float(g[p][i]) + float(e[p][i]) >= 0)
                assert r.workers[p].n_pos + r.workers[p].n_neg == n
                assert [float(x) for x in err[p]] == [float(x) for x in r.e_new[p]]
            assert r.gmu_pos == float(gp) and r.gmu_neg == float(gn)
            assert [float(x) for x in w_new] == [float(x) for x in r.w_new]


def test_brute_force_exact_rationals():
    check_brute_force()


def test_per_tensor_variant_worked_example_and_brute_force():
    """The per-tensor variant is Sec. 3.1 / Algorithm 1 lines 3-7 restricted to each tensor.  Pinned by a case
    worked by hand (the step-1 gradients of the worked example cut into two tensors of three elements) and by the
    exact-rational brute force on every tensor of random splits."""
    gA, gB = arr([1, -2, 3, 0, -4, 2]), arr([-1, -3, 2, -2, 4, 0])
    zero = arr([0] * 6)
    per_seg, e_new, w_new = O.step_segmented([gA, gB], [zero, zero], zero, 0.5, O.RETAINED_ERROR, [3, 3])
    # tensor 0: A = [1,-2,3] and B = [-1,-3,2] both have mu+ = 2, mu- = 2
    # tensor 1: A = [0,-4,2] has mu+ = 1, mu- = 4; B = [-2,4,0] has mu+ = 2, mu- = 2; global 1.5 and 3
    assert [(s.mu_pos, s.mu_neg) for s in per_seg[0].workers] == [(2.0, 2.0), (2.0, 2.0)]
    assert [(s.mu_pos, s.mu_neg) for s in per_seg[1].workers] == [(1.0, 4.0), (2.0, 2.0)]
    assert (per_seg[0].gmu_pos, per_seg[0].gmu_neg) == (2.0, 2.0)
    assert (per_seg[1].gmu_pos, per_seg[1].gmu_neg) == (1.5, 3.0)
    assert e_new[0].tolist() == [-1, 0, 1, -1, 0, 1]
    assert e_new[1].tolist() == [1, -1, 0, 0, 2, -2]
    assert w_new.tolist() == [0, 1, -1, 0.375, 0.375, -0.75]

    rng = np.random.default_rng(77)
    for _ in range(25):
        P, S = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        seg = [int(x) for x in rng.integers(1, 7, S)]
        n = sum(seg)
        g = [arr(rng.integers(-32, 33, n) / 8.0) for _ in range(P)]
        e = [arr(rng.integers(-16, 17, n) / 8.0) for _ in range(P)]
        w = arr(rng.integers(-64, 65, n) / 16.0)
        for mode in (O.RETAINED_ERROR, O.ALG1_LITERAL):
            per_seg, e_new, w_new = O.step_segmented(g, e, w, 0.25, mode, seg)
            off = 0
            for k, length in enumerate(seg):
                sl = slice(off, off + length)
                mu_pos, mu_neg, gp, gn, err, wn = brute_force([x[sl] for x in g], [x[sl] for x in e], w[sl], 0.25, mode)
                assert [s.mu_pos for s in per_seg[k].workers] == [float(x) for x in mu_pos]
                assert [s.mu_neg for s in per_seg[k].workers] == [float(x) for x in mu_neg]
                assert (per_seg[k].gmu_pos, per_seg[k].gmu_neg) == (float(gp), float(gn))
                for p in range(P):
                    assert e_new[p][sl].tolist() == [float(x) for x in err[p]]
                assert w_new[sl].tolist() == [float(x) for x in wn]
                off += length


def test_tensors_with_padding_and_pooled_means():
    """Buffers that hold tensors with padding between them: per tensor, each tensor is the brute force on its own
    slice; pooled, all tensors laid end to end are one brute-force vector; padding comes back bit for bit, whatever it
    holds (here NaN, which would poison any sum it entered)."""
    rng = np.random.default_rng(78)
    for _ in range(25):
        P, S = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        lengths = [int(x) for x in rng.integers(1, 6, S)]
        gaps = [int(x) for x in rng.integers(0, 4, S + 1)]
        offsets, pos = [], gaps[0]
        for k in range(S):
            offsets.append(pos)
            pos += lengths[k] + gaps[k + 1]
        n = pos if pos > 0 else 1
        member = np.zeros(n, bool)
        for o, l in zip(offsets, lengths):
            member[o:o + l] = True
        g = [arr(rng.integers(-32, 33, n) / 8.0) for _ in range(P)]
        e = [arr(rng.integers(-16, 17, n) / 8.0) for _ in range(P)]
        w = arr(rng.integers(-64, 65, n) / 16.0)
        for x in g + e + [w]:
            x[~member] = np.nan
        for mode in (O.RETAINED_ERROR, O.ALG1_LITERAL):
            for pooled in (False, True):
                res, e_new, w_new = O.step_segmented(g, e, w, 0.25, mode, lengths, offsets, pooled)
                for p in range(P):
                    assert np.isnan(e_new[p][~member]).all() and not np.isnan(e_new[p][member]).any()
                assert np.isnan(w_new[~member]).all() and not np.isnan(w_new[member]).any()
                if pooled:
                    cat = lambda x: np.concatenate([x[o:o + l] for o, l in zip(offsets, lengths)])
                    mu_pos, mu_neg, gp, gn, err, wn = brute_force([cat(x) for x in g], [cat(x) for x in e], cat(w), 0.25, mode)
                    assert len(res) == 1 and [s.mu_pos for s in res[0].workers] == [float(x) for x in mu_pos]
                    assert [s.n_nan for s in res[0].workers] == [0] * P
                    assert (res[0].gmu_pos, res[0].gmu_neg) == (float(gp), float(gn))
                    for p in range(P):
                        assert cat(e_new[p]).tolist() == [float(x) for x in err[p]]
                    assert cat(w_new).tolist() == [float(x) for x in wn]
                else:
                    for k, (o, l) in enumerate(zip(offsets, lengths)):
                        sl = slice(o, o + l)
                        mu_pos, mu_neg, gp, gn, err, wn = brute_force([x[sl] for x in g], [x[sl] for x in e], w[sl], 0.25, mode)
                        assert [s.mu_neg for s in res[k].workers] == [float(x) for x in mu_neg]
                        assert (res[k].gmu_pos, res[k].gmu_neg) == (float(gp), float(gn))
                        for p in range(P):
                            assert e_new[p][sl].tolist() == [float(x) for x in err[p]]
                        assert w_new[sl].tolist() == [float(x) for x in wn]


def test_per_tensor_replicas():
    """One weight vector per worker on buffers that consist of tensors.  Pinned by the hand-worked per-tensor case
    (each worker's rebuilt update is +gmu_pos or -gmu_neg of the element's tensor) and, on random dyadic cases with
    padding, per tensor and pooled, by two identities: the errors are those of the shared-weight form, and the mean
    of the replicas, all started from the same w, is the shared form's new w (Eq. 1 with rebuilt gradients)."""
    gA, gB = arr([1, -2, 3, 0, -4, 2]), arr([-1, -3, 2, -2, 4, 0])
    zero = arr([0] * 6)
    e_new, w_new = O.step_replicas_segmented([gA, gB], [zero, zero], [zero, zero], 0.5, O.RETAINED_ERROR, [3, 3])
    # tensor 0: global means (2, 2); tensor 1: (1.5, 3); w^p = -0.5 * (+gmu_pos or -gmu_neg by the sign of g^p)
    assert w_new[0].tolist() == [-1, 1, -1, -0.75, 1.5, -0.75]
    assert w_new[1].tolist() == [1, 1, -1, 1.5, -0.75, -0.75]
    assert e_new[0].tolist() == [-1, 0, 1, -1, 0, 1] and e_new[1].tolist() == [1, -1, 0, 0, 2, -2]
    rng = np.random.default_rng(79)
    for _ in range(25):
        P, S = int(rng.choice([1, 2, 4])), int(rng.integers(1, 5))
        lengths = [int(x) for x in rng.integers(1, 6, S)]
        gaps = [int(x) for x in rng.integers(0, 4, S + 1)]
        offsets, pos = [], gaps[0]
        for k in range(S):
            offsets.append(pos)
            pos += lengths[k] + gaps[k + 1]
        n = max(pos, 1)
        member = np.zeros(n, bool)
        for o, l in zip(offsets, lengths):
            member[o:o + l] = True
        g = [arr(rng.integers(-32, 33, n) / 8.0) for _ in range(P)]
        e = [arr(rng.integers(-16, 17, n) / 8.0) for _ in range(P)]
        w = arr(rng.integers(-64, 65, n) / 16.0)
        for x in g + e + [w]:
            x[~member] = np.nan
        for mode in (O.RETAINED_ERROR, O.ALG1_LITERAL):
            for pooled in (False, True):
                _, e_ref, w_ref = O.step_segmented(g, e, w, 0.25, mode, lengths, offsets, pooled)
                e_new, w_new = O.step_replicas_segmented(g, e, [w.copy() for _ in range(P)], 0.25, mode, lengths,
                                                         offsets, pooled)
                for p in range(P):
                    assert np.array_equal(e_new[p], e_ref[p], equal_nan=True)
                    assert np.isnan(w_new[p][~member]).all() and not np.isnan(w_new[p][member]).any()
                # each replica and the shared w are rounded to fp32 once: the identity holds to a few ulp
                mean = np.mean(np.stack(w_new).astype(np.float64), axis=0)
                assert np.allclose(mean[member], w_ref[member].astype(np.float64), rtol=4e-7, atol=1e-7)


# ---------------------------------------------------------------------------------------------------------
# exactly rounded means: math.fsum is an exact sum, so fl32(fsum/n) is the definition's value
# ---------------------------------------------------------------------------------------------------------
def check_means_against_fsum():
    rng = np.random.default_rng(7)
    n = 200_003
    g = (rng.standard_normal(n) * 1e-3).astype(f32)
    e = (rng.standard_normal(n) * 3e-4).astype(f32)
    g[::97] = 0.0
    e[::97] = 0.0
    v = g + e  # numpy fp32 add: the same single rounding
    acc = O.LocalAccumulator()
    for lo in range(0, n, 33_333):  # ragged chunking must not matter
        acc.feed(g[lo:lo + 33_333], e[lo:lo + 33_333])
    st = acc.stats()
    pos = v[v >= 0].astype(np.float64)
    neg = -v[v < 0].astype(np.float64)
    assert st.n_pos == pos.size and st.n_neg == neg.size and st.n_zero == int((v == 0).sum()) and st.n_nan == 0
    assert st.mu_pos == f32(math.fsum(pos) / pos.size)
    assert st.mu_neg == f32(math.fsum(neg) / neg.size)


def test_means_against_fsum():
    check_means_against_fsum()


# ---------------------------------------------------------------------------------------------------------
# identities and invariants
# ---------------------------------------------------------------------------------------------------------
def random_case(rng, n, P, scale=1e-3, zeros=True):
    g = [(rng.standard_normal(n) * scale).astype(f32) for _ in range(P)]
    e = [(rng.standard_normal(n) * scale * 0.5).astype(f32) for _ in range(P)]
    if zeros:
        for p in range(P):
            idx = rng.integers(0, n, max(1, n // 50))
            g[p][idx] = 0.0
            e[p][idx] = 0.0
    w = (rng.standard_normal(n) * 0.02).astype(f32)
    return g, e, w


def check_reconstruction_and_zero_sum():
    """enc_local(v) + e_new == g + e_old elementwise (Algorithm 1 line 4), and the new errors of each sign
    group sum to zero because the group's mean was subtracted."""
    rng = np.random.default_rng(11)
    n, P = 50_021, 3
    g, e, w = random_case(rng, n, P)
    r = O.step(g, e, w, 0.1)
    for p in range(P):
        v = (g[p] + e[p]).astype(np.float64)
        st = r.workers[p]
        enc = np.where(r.mask[p] == 1, st.mu_pos, -st.mu_neg)
        assert np.array_equal(r.mask[p] == 1, v >= 0)
        # one fp32 rounding of (v - mu): half an ulp of the result, bounded by ulp of max(|v|, mu)
        ulp = np.spacing(np.maximum(np.abs(v), max(st.mu_pos, st.mu_neg)).astype(f32)).astype(np.float64)
        assert np.all(np.abs(enc + r.e_new[p].astype(np.float64) - v) <= ulp)
        en = r.e_new[p].astype(np.float64)
        tol = n * 1e-3 * 2.0 ** -23
        assert abs(math.fsum(en[v >= 0])) <= tol and abs(math.fsum(en[v < 0])) <= tol
        assert st.n_pos + st.n_neg + st.n_nan == n


def test_reconstruction_and_zero_sum():
    check_reconstruction_and_zero_sum()


def check_nan_handling():
    """NaN is in neither group: counted apart, leaves both means untouched, poisons only its own index."""
    rng = np.random.default_rng(5)
    n, P = 1000, 2
    g, e, w = random_case(rng, n, P)
    clean = O.step(g, e, w, 0.1)
    g2 = [x.copy() for x in g]
    bad = [3, 500, 999]
    # replace by NaN, but first move those entries' values out of the sums of the clean run for comparison:
    g3 = [x.copy() for x in g]
    e3 = [x.copy() for x in e]
    for i in bad:
        g2[0][i] = np.nan
    r = O.step(g2, e, w, 0.1)
    assert r.workers[0].n_nan == 3 and r.workers[1].n_nan == 0
    assert r.workers[0].n_pos + r.workers[0].n_neg + 3 == n
    # means of worker 0 equal those of the vector with the three entries deleted
    keep = np.ones(n, bool)
    keep[bad] = False
    rd = O.step([g3[0][keep], g3[1][keep]], [e3[0][keep], e3[1][keep]], w[keep], 0.1)
    assert rd.workers[0].mu_pos == r.workers[0].mu_pos and rd.workers[0].mu_neg == r.workers[0].mu_neg
    assert np.all(np.isnan(r.w_new[bad])) and np.all(np.isnan(r.e_new[0][bad]))
    assert not np.any(np.isnan(r.w_new[keep])) and not np.any(np.isnan(r.e_new[1]))
    assert np.array_equal(r.e_new[1], clean.e_new[1])


def test_nan_handling():
    check_nan_handling()


def check_p1_literal_is_plain_sgd():
    """P = 1, Algorithm-1-literal: the global means equal the local ones, the net gain is zero, and the step
    is w - eta*g (Theorem 1's update with grad-mu = 0), i.e. a plain axpy computed here with numpy."""
    rng = np.random.default_rng(21)
    n = 40_000
    g, _, w = random_case(rng, n, 1)
    r = O.step(g, None, w, 0.05, O.ALG1_LITERAL)
    assert r.gmu_pos == r.workers[0].mu_pos and r.gmu_neg == r.workers[0].mu_neg
    # the oracle evaluates (v - mu) + mu in double: exact up to double rounding, then one fp32 rounding
    ref = (w.astype(np.float64) - np.float64(f32(0.05)) * g[0].astype(np.float64))
    assert np.max(np.abs(r.w_new.astype(np.float64) - ref)) <= np.max(np.spacing(np.abs(r.w_new))) * 0.5000001


def test_p1_literal_is_plain_sgd():
    check_p1_literal_is_plain_sgd()


def check_p1_retained_is_local_encoding():
    rng = np.random.default_rng(22)
    n = 10_000
    g, e, w = random_case(rng, n, 1)
    r = O.step(g, e, w, 0.25)
    v = g[0] + e[0]
    st = r.workers[0]
    enc = np.where(v >= 0, np.float64(st.mu_pos), -np.float64(st.mu_neg))
    ref = (w.astype(np.float64) - 0.25 * enc).astype(f32)
    assert np.array_equal(r.w_new, ref)


def test_p1_retained_is_local_encoding():
    check_p1_retained_is_local_encoding()


def check_theorem1_form():
    """Algorithm-1-literal, any P: update = dense average of g + average net gain, where the net gain of a
    worker is (global-mean vector) - enc(g) (Sec. 3.2, the definitions before Assumption 3; Theorem 1)."""
    rng = np.random.default_rng(23)
    n, P = 20_000, 4
    g, _, w = random_case(rng, n, P)
    eta = 0.1
    r = O.step(g, None, w, eta, O.ALG1_LITERAL)
    dense = O.dense_step(g, w, eta).astype(np.float64)
    gain = np.zeros(n)
    for p in range(P):
        st = r.workers[p]
        pos = g[p] >= 0
        gbar = np.where(pos, np.float64(r.gmu_pos), -np.float64(r.gmu_neg))
        enc = np.where(pos, np.float64(st.mu_pos), -np.float64(st.mu_neg))
        gain += (gbar - enc) / P
        assert len(np.unique(gbar - enc)) <= 2
    ref = dense - np.float64(f32(eta)) * gain
    assert np.allclose(r.w_new, ref, rtol=0, atol=1e-8)
    # and the dense step itself against numpy
    ref_dense = w.astype(np.float64) - np.float64(f32(eta)) * np.mean(np.stack(g).astype(np.float64), axis=0)
    assert np.allclose(dense, ref_dense, rtol=0, atol=4e-9)  # half an fp32 ulp of |w| < 0.125


def test_theorem1_form():
    check_theorem1_form()


def check_same_sign_and_two_valued():
    z = np.zeros(4, dtype=f32)
    r = O.step([arr([1, 2, 3, 0])], None, z, 1.0)
    st = r.workers[0]
    assert (st.n_pos, st.n_neg, st.mu_pos, st.mu_neg) == (4, 0, 1.5, 0.0)
    assert np.array_equal(r.e_new[0], arr([-0.5, 0.5, 1.5, -1.5])) and np.array_equal(r.w_new, arr([-1.5] * 4))
    r = O.step([arr([-1, -2, -3, -2])], None, z, 1.0)
    st = r.workers[0]
    assert (st.n_pos, st.n_neg, st.mu_pos, st.mu_neg) == (0, 4, 0.0, 2.0)
    assert np.array_equal(r.e_new[0], arr([1, 0, -1, 0])) and np.array_equal(r.w_new, arr([2.0] * 4))
    # an empty group on one worker enters the global average as 0 with weight 1/P
    r = O.step([arr([1, 2, 3, 0]), arr([-1, -2, -3, -2])], None, z, 1.0)
    assert (r.gmu_pos, r.gmu_neg) == (0.75, 1.0)
    assert np.array_equal(r.w_new, arr([-(0.75 - 1.0) / 2] * 4))
    # a vector with one value per sign is encoded without loss
    v = arr([0.375, -1.25, 0.375, 0.375, -1.25])
    r = O.step([v], None, np.zeros(5, dtype=f32), 1.0)
    assert r.workers[0].mu_pos == 0.375 and r.workers[0].mu_neg == 1.25
    assert np.array_equal(r.e_new[0], np.zeros(5, dtype=f32)) and np.array_equal(r.w_new, -v)
    # -0.0 is in the ">= 0" group
    r = O.step([arr([-0.0, 4.0, -2.0])], None, np.zeros(3, dtype=f32), 1.0)
    st = r.workers[0]
    assert (st.n_pos, st.n_neg, st.n_zero, st.mu_pos, st.mu_neg) == (2, 1, 1, 2.0, 2.0)
    assert list(r.mask[0]) == [1, 1, 0]


def test_same_sign_and_two_valued():
    check_same_sign_and_two_valued()


def check_identical_workers():
    rng = np.random.default_rng(31)
    g, e, w = random_case(rng, 5000, 1)
    r1 = O.step(g, e, w, 0.1)
    for mode in (O.RETAINED_ERROR, O.ALG1_LITERAL):
        r1 = O.step(g, e, w, 0.1, mode)
        r3 = O.step(g * 3, e * 3, w, 0.1, mode)
        assert (r3.gmu_pos, r3.gmu_neg) == (r1.workers[0].mu_pos, r1.workers[0].mu_neg)
        assert np.allclose(r3.w_new, r1.w_new, rtol=0, atol=1e-9)
        assert all(np.array_equal(x, r1.e_new[0]) for x in r3.e_new)


def test_identical_workers():
    check_identical_workers()


def check_power_of_two_scaling():
    """g, e scaled by 2^k and eta by 2^-k: means and errors scale by 2^k bit for bit; counts, masks and the
    new weights do not change at all."""
    rng = np.random.default_rng(41)
    g, e, w = random_case(rng, 30_011, 3)
    for mode in (O.RETAINED_ERROR, O.ALG1_LITERAL):
        a = O.step(g, e, w, 0.125, mode)
        k = 5
        b = O.step([x * f32(2.0 ** k) for x in g], [x * f32(2.0 ** k) for x in e], w, 0.125 * 2.0 ** -k, mode)
        for p in range(3):
            assert b.workers[p].mu_pos == a.workers[p].mu_pos * 2 ** k
            assert b.workers[p].mu_neg == a.workers[p].mu_neg * 2 ** k
            assert (b.workers[p].n_pos, b.workers[p].n_neg, b.workers[p].n_zero) == \
                   (a.workers[p].n_pos, a.workers[p].n_neg, a.workers[p].n_zero)
            assert np.array_equal(b.e_new[p], a.e_new[p] * f32(2.0 ** k)) and np.array_equal(b.mask[p], a.mask[p])
        assert np.array_equal(a.w_new, b.w_new)


def test_power_of_two_scaling():
    check_power_of_two_scaling()


def check_permutation_and_sign_flip():
    rng = np.random.default_rng(43)
    n, P = 20_000, 2
    g, e, w = random_case(rng, n, P, zeros=False)
    a = O.step(g, e, w, 0.1)
    perm = rng.permutation(n)
    b = O.step([x[perm] for x in g], [x[perm] for x in e], w[perm], 0.1)
    for p in range(P):
        assert (a.workers[p].n_pos, a.workers[p].n_neg) == (b.workers[p].n_pos, b.workers[p].n_neg)
        # long-double sums in another order: same fp32 mean except in a near-tie of vanishing probability
        assert a.workers[p].mu_pos == b.workers[p].mu_pos and a.workers[p].mu_neg == b.workers[p].mu_neg
        assert np.array_equal(a.e_new[p][perm], b.e_new[p])
    assert np.array_equal(a.w_new[perm], b.w_new)
    # sign flip, no zeros present: the two groups trade places
    c = O.step([-x for x in g], [-x for x in e], w, 0.1)
    for p in range(P):
        assert (c.workers[p].n_pos, c.workers[p].n_neg) == (a.workers[p].n_neg, a.workers[p].n_pos)
        assert (c.workers[p].mu_pos, c.workers[p].mu_neg) == (a.workers[p].mu_neg, a.workers[p].mu_pos)
        assert np.array_equal(c.e_new[p], -a.e_new[p])
    assert np.allclose(c.w_new.astype(np.float64) - w, -(a.w_new.astype(np.float64) - w), rtol=0, atol=8e-9)
    # with zeros present the symmetry breaks: zeros stay in the ">= 0" group on both sides
    gz = [x.copy() for x in g]
    ez = [x.copy() for x in e]
    gz[0][:100] = 0
    ez[0][:100] = 0
    d = O.step(gz, ez, w, 0.1)
    f = O.step([-x for x in gz], [-x for x in ez], w, 0.1)
    assert f.workers[0].n_pos == d.workers[0].n_neg + 100 and f.workers[0].n_neg == d.workers[0].n_pos - 100


def test_permutation_and_sign_flip():
    check_permutation_and_sign_flip()


def check_closed_forms():
    """Half-normal, Laplace and Student-t(3) absolute means; the zero-inflated positive mean."""
    import workloads
    n = 400_000
    wl = workloads.config1(n=n)
    g = wl.gradient(0).numpy()
    st = O.step([g], None, np.zeros(n, f32), 0.1).workers[0]
    z, sigma = 0.01, 1e-3
    hn = sigma * math.sqrt(2 / math.pi)
    assert abs(st.mu_neg / hn - 1) < 5 / math.sqrt(n / 2)
    assert abs(st.mu_pos / ((1 - z) / (1 + z) * hn) - 1) < 8 / math.sqrt(n / 2)
    assert abs(st.n_pos / n - (1 + z) / 2) < 4 / math.sqrt(n)
    # Laplace(0, b): E|v| = b
    rng = np.random.default_rng(3)
    b = 3e-4
    v = rng.laplace(0, b, n).astype(f32)
    st = O.step([v], None, np.zeros(n, f32), 0.1).workers[0]
    assert abs(st.mu_pos / b - 1) < 8 / math.sqrt(n / 2) and abs(st.mu_neg / b - 1) < 8 / math.sqrt(n / 2)
    # Student-t(3) * s: E|v| = 2*sqrt(3)/pi * s (heavy tail: loose)
    s = 1e-4
    v = (rng.standard_t(3, n) * s).astype(f32)
    st = O.step([v], None, np.zeros(n, f32), 0.1).workers[0]
    assert abs(st.mu_pos / (2 * math.sqrt(3) / math.pi * s) - 1) < 0.03
    assert abs(st.mu_neg / (2 * math.sqrt(3) / math.pi * s) - 1) < 0.03


def test_closed_forms():
    check_closed_forms()


def test_fold_is_one_fp32_add():
    """The sign of fl32(g + e) decides the group; cases where double and single rounding part ways."""
    g = arr([1.0, -1.0, 1e-30, 16777216.0])
    e = arr([-1.0, 1.0, -1e-30, 1.0])
    r = O.step([g], [e], np.zeros(4, f32), 1.0)
    assert r.workers[0].n_pos == 4 and r.workers[0].n_zero == 3
    # 2^24 + 1 rounds to 2^24 in fp32 (ties to even): the mean sees 16777216, not 16777217
    assert r.workers[0].mu_pos == f32(16777216.0 / 4)


def test_chunk_split_invariance():
    rng = np.random.default_rng(77)
    g, e, w = random_case(rng, 10_007, 3)
    a = O.step(g, e, w, 0.1, chunk=1 << 22)
    b = O.step(g, e, w, 0.1, chunk=1001)
    assert a.workers == b.workers and (a.gmu_pos, a.gmu_neg) == (b.gmu_pos, b.gmu_neg)
    assert np.array_equal(a.w_new, b.w_new) and all(np.array_equal(x, y) for x, y in zip(a.e_new, b.e_new))


# ---------------------------------------------------------------------------------------------------------
# per-replica weights (Algorithm 1 line 7 as printed) and the final synchronisation on replicas
# ---------------------------------------------------------------------------------------------------------
def check_replicas():
    rng = np.random.default_rng(91)
    n, P = 30_011, 4
    g, e, w = random_case(rng, n, P)
    wr = [(w + (rng.standard_normal(n) * 1e-3).astype(f32)) for _ in range(P)]
    for mode in (O.RETAINED_ERROR, O.ALG1_LITERAL):
        shared = O.step(g, e, np.mean(np.stack(wr).astype(np.float64), axis=0).astype(f32), 0.1, mode)
        workers, gmu, e_new, w_new = O.step_replicas(g, e, wr, 0.1, mode)
        assert workers == shared.workers and gmu == (shared.gmu_pos, shared.gmu_neg)
        assert all(np.array_equal(a, b) for a, b in zip(e_new, shared.e_new))
        # the mean of the replicas moves like the shared weight vector (no update depends on w)
        mean_new = np.mean(np.stack(w_new).astype(np.float64), axis=0)
        mean_old = np.mean(np.stack(wr).astype(np.float64), axis=0)
        assert np.allclose(mean_new - mean_old, shared.w_new.astype(np.float64) - mean_old.astype(f32), rtol=0, atol=2e-8)
        # each replica separately: retained mode moves it by one of two values
        for p in range(P):
            step_p = (wr[p].astype(np.float64) - w_new[p]) / np.float64(f32(0.1))
            if mode == O.RETAINED_ERROR:
                want = np.where(shared.mask[p] == 1, np.float64(gmu[0]), -np.float64(gmu[1]))
                assert np.allclose(step_p, want, rtol=0, atol=1e-7)
    # P = 1: the replica path is the shared path
    r1 = O.step([g[0]], [e[0]], wr[0], 0.1)
    _, _, e1, w1 = O.step_replicas([g[0]], [e[0]], [wr[0]], 0.1)
    assert np.array_equal(w1[0], r1.w_new) and np.array_equal(e1[0], r1.e_new[0])
    # final synchronisation: every replica takes the dense averaged gradient; drift is unchanged by it
    d0 = O.replica_drift(wr)
    ws = O.dense_step_replicas(g, wr, 0.1)
    for p in range(P):
        ref = wr[p].astype(np.float64) - np.float64(f32(0.1)) * np.mean(np.stack(g).astype(np.float64), axis=0)
        assert np.allclose(ws[p], ref, rtol=0, atol=4e-9)
    d1 = O.replica_drift(ws)
    assert np.allclose(d0[0], d1[0], rtol=0, atol=1e-8) and np.allclose(d0[1], d1[1], rtol=1e-5)
    # drift against numpy
    W = np.stack(wr).astype(np.float64)
    dev = W - W.mean(axis=0)
    assert np.allclose(d0[0], np.abs(dev).max(axis=1), rtol=1e-12) and np.allclose(d0[1], np.sqrt((dev ** 2).mean(axis=1)), rtol=1e-10)
    same = O.replica_drift([wr[0]] * 3)
    assert same[0] == [0.0] * 3 and same[1] == [0.0] * 3


def test_replicas():
    check_replicas()


# ---------------------------------------------------------------------------------------------------------
# mutation battery: every planted mistake must trip at least one pin
# ---------------------------------------------------------------------------------------------------------
PINS = [check_worked_example, check_brute_force, check_means_against_fsum, check_reconstruction_and_zero_sum,
        check_nan_handling, check_p1_literal_is_plain_sgd, check_p1_retained_is_local_encoding,
        check_theorem1_form, check_same_sign_and_two_valued, check_identical_workers,
        check_power_of_two_scaling, check_permutation_and_sign_flip, check_closed_forms, check_replicas]

MUTANTS = [
    ("zero_in_negative_group", "if (v >= 0.0f) {\n            acc->n_pos", "if (v > 0.0f) {\n            acc->n_pos"),
    ("neg_sum_sign", "acc->s_neg += -(long double)v;", "acc->s_neg += (long double)v;"),
    ("mean_divides_by_wrong_count", "(float)(acc->s_neg / (long double)acc->n_neg)",
     "(float)(acc->s_neg / (long double)acc->n_pos)"),
    ("global_mean_not_divided", "*gmu_pos = (float)(sp / (double)P);", "*gmu_pos = (float)(sp);"),
    ("global_means_swapped", "sn += (double)mu_neg[p];", "sn += (double)mu_pos[p];"),
    ("error_sign_neg_group", "err = (double)v + (double)mu_neg[p]; /* v - enc", "err = (double)v - (double)mu_neg[p]; /* v - enc"),
    ("error_uses_global_mean", "err = (double)v - (double)mu_pos[p]; /* v - enc", "err = (double)v - (double)gmu_pos; /* v - enc"),
    ("update_sign_neg_group", "glob = -(double)gmu_neg;\n            } else { /* NaN", "glob = (double)gmu_neg;\n            } else { /* NaN"),
    ("replica_error_sign_neg_group", "err = (double)v + (double)mu_neg[p];\n", "err = (double)v - (double)mu_neg[p];\n"),
    ("replica_update_sign_neg_group", "glob = -(double)gmu_neg;\n            } else {\n", "glob = (double)gmu_neg;\n            } else {\n"),
    ("update_not_averaged", "double U = usum / (double)P;", "double U = usum;"),
    ("weight_update_sign", "(double)w[i] - (double)eta * U", "(double)w[i] + (double)eta * U"),
    ("literal_drops_error", "usum += (mode == A2SGD_ORACLE_ALG1_LITERAL) ? err + glob : glob;", "usum += glob;"),
    ("retained_adds_error", "usum += (mode == A2SGD_ORACLE_ALG1_LITERAL) ? err + glob : glob;", "usum += err + glob;"),
    ("fold_drops_error", "float v = g[i] + e[i];", "float v = g[i];"),
    ("mask_strict", "mask[p][i] = (uint8_t)(v >= 0.0f);", "mask[p][i] = (uint8_t)(v > 0.0f);"),
    ("apply_strict_compare", "if (v >= 0.0f) {\n                err = (double)v - (double)mu_pos[p]; /* v",
     "if (v > 0.0f) {\n                err = (double)v - (double)mu_pos[p]; /* v"),
    ("dense_not_averaged", "w_new[i] = (float)((double)w[i] - (double)eta * (s / (double)P));",
     "w_new[i] = (float)((double)w[i] - (double)eta * (s));"),
    ("replica_update_sign", "w_new[p][i] = (float)((double)w[p][i] - (double)eta * u);",
     "w_new[p][i] = (float)((double)w[p][i] + (double)eta * u);"),
    ("replica_literal_drops_error", "double u = (mode == A2SGD_ORACLE_ALG1_LITERAL) ? err + glob : glob;",
     "double u = glob;"),
    ("replica_dense_not_averaged", "w_new[p][i] = (float)((double)w[p][i] - (double)eta * (s / (double)P));",
     "w_new[p][i] = (float)((double)w[p][i] - (double)eta * s);"),
    ("drift_mean_not_divided", "double mean = s / (double)P;", "double mean = s;"),
]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_planted_mistake(name, old, new):
    src = open(O._SRC).read()
    assert src.count(old) == 1, f"mutation anchor for {name} not found exactly once"
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "mutant.c")
        so = os.path.join(d, "mutant.so")
        open(c, "w").write(src.replace(old, new))
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared", "-o", so, c, "-lm"])
        caught = []
        with O.use_library(so):
            for pin in PINS:
                try:
                    pin()
                except AssertionError:
                    caught.append(pin.__name__)
        assert caught, f"no pin noticed the planted mistake {name!r}"
