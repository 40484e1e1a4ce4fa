"""Pins for the CPU oracle: what the paper and the mathematics fix, never the oracle itself.

Each test names the passage it rests on.  A dropped term, a wrong sign, a transposed operand or
an off-by-one in the oracle fails at least one of them (test_planted_mistakes_are_caught shows
this for a handful of plausible slips, planted in a copy of the oracle's source on the CPU).
"""
import ctypes
import itertools
import os
import subprocess
import sys

import numpy as np
import pytest
from scipy.optimize import minimize_scalar

sys.path.insert(0, os.path.dirname(__file__))
import bruteforce as bf                                   # noqa: E402
from oracle import duhl_oracle as orc                     # noqa: E402
from paper_1708_05357_amd import synth                    # noqa: E402

LASSO, SVM = orc.LASSO, orc.SVM


# ----------------------------------------------------------------------------- instances
def tiny_lasso(seed, d=8, n=6, c=0.3):
    rng = np.random.default_rng(seed)
    cols = rng.standard_normal((n, d)).astype(np.float32)
    b = rng.standard_normal(d).astype(np.float32)
    A = cols.T.astype(np.float64)
    lam = c * np.abs(A.T @ b).max() / d
    return cols, b, A, lam


def tiny_svm(seed, n=8, d=6):
    rng = np.random.default_rng(seed)
    cols = rng.standard_normal((n, d)).astype(np.float32)
    y = np.where(rng.standard_normal(n) >= 0, 1.0, -1.0).astype(np.float32)
    lam = 0.5 / n * (1 + seed % 3)
    return cols, y, cols.T.astype(np.float64), lam


def hadamard16():
    H = np.array([[1.0]])
    for _ in range(4):
        H = np.block([[H, H], [H, -H]])
    return (H / 4.0).astype(np.float32)        # 16 x 16, exactly orthonormal in fp32


def mid_lasso(seed=3, d=60, n=40):
    p = synth.lasso_dense(d, n, 0.2, 0.1, seed=seed)
    return p["cols"].numpy(), p["target"].numpy(), p["lam"]


def run_passes(o, passes, seed=0):
    rng = np.random.default_rng(seed)
    for _ in range(passes):
        o.cd_pass(rng.permutation(o.n).astype(np.int32))


# ----------------------------------------------------------------------------- Lasso gaps
def test_lasso_gap_sum_equals_primal_minus_dual():
    """Section 2, eq. (2) with f*(w) = w^T b + (d/2)||w||^2 and the Lipschitzed g_i* (App. E):
    gap = (1/d)[||v||^2 + b^T v + Lambda ||alpha||_1 + B sum [|c_i| - Lambda]_+] -- a form
    that never multiplies alpha_i with c_i column by column."""
    cols, b, lam = mid_lasso()
    o = orc.Oracle(LASSO, b, lam, cols=cols)
    A = cols.T.astype(np.float64)
    d = A.shape[0]
    for passes in (0, 1, 3):
        run_passes(o, passes)
        total = o.gaps()
        v = A @ o.alpha - b
        Bnd = float(b.astype(np.float64) @ b) / (2 * lam * d)
        c = A.T @ v
        ref = (v @ v + b @ v + lam * d * np.abs(o.alpha).sum()
               + Bnd * np.maximum(np.abs(c) - lam * d, 0).sum()) / d
        assert total == pytest.approx(ref, rel=1e-11, abs=1e-14)
        assert total == pytest.approx(o.z.sum(), rel=1e-12)
        assert o.z.min() >= -1e-13 * max(1.0, o.z.max())          # Section 2: gap non-negative


def test_lasso_gap_zero_at_zero_when_lambda_large():
    """Lambda >= ||A^T b||_inf makes alpha = 0 optimal, so every coordinate gap at 0 vanishes."""
    cols, b, _ = mid_lasso()
    A = cols.T.astype(np.float64)
    lam = 1.0000001 * np.abs(A.T @ b).max() / A.shape[0]
    o = orc.Oracle(LASSO, b, lam, cols=cols)
    assert o.gaps() == 0.0 and np.all(o.z == 0.0)
    lam2 = 0.5 * lam
    o2 = orc.Oracle(LASSO, b, lam2, cols=cols)
    assert o2.gaps() > 0.0


def test_lasso_orthonormal_closed_form():
    """Orthonormal columns: the minimiser is the soft-thresholding of A^T b at Lambda; there all
    coordinate gaps are 0 (App. E formula) and a single CD pass from 0 lands on it (App. D)."""
    H = hadamard16()
    cols = np.ascontiguousarray(H[:10])
    rng = np.random.default_rng(5)
    b = rng.standard_normal(16).astype(np.float32)
    atb = cols.astype(np.float64) @ b
    Lam = 0.4 * np.abs(atb).max()
    lam = Lam / 16
    star = np.sign(atb) * np.maximum(np.abs(atb) - Lam, 0)
    assert 0 < np.count_nonzero(star) < 10
    o = orc.Oracle(LASSO, b, lam, cols=cols)
    assert o.gaps() > 1e-3
    o.set_state(star)
    assert abs(o.gaps()) < 1e-14 and np.abs(o.z).max() < 1e-14
    o2 = orc.Oracle(LASSO, b, lam, cols=cols)
    o2.cd_pass(np.arange(10, dtype=np.int32)[::-1].copy())
    np.testing.assert_allclose(o2.alpha, star, atol=1e-14)
    np.testing.assert_allclose(o2.v, cols.T.astype(np.float64) @ star - b, atol=1e-14)


@pytest.mark.parametrize("seed", range(4))
def test_lasso_gap_bounds_suboptimality_and_cd_reaches_bruteforce_optimum(seed):
    """App. A (gap >= O(alpha) - O(alpha*)) and Alg. 3: on 8 x 6 instances the optimum is found
    by enumerating all 3^6 sign patterns; the oracle's CD limit must coincide with it."""
    cols, b, A, lam = tiny_lasso(seed)
    ostar, astar = bf.lasso_optimum(A, b.astype(np.float64), lam)
    o = orc.Oracle(LASSO, b, lam, cols=cols)
    prev = o.objective()
    assert prev == pytest.approx(bf.lasso_objective(A, b, o.alpha, lam), rel=1e-13)
    for it in range(400):
        gap = o.gaps()
        obj = o.objective()
        assert gap >= obj - ostar - 1e-12
        assert obj <= prev + 1e-15                                 # exact steps never go up
        prev = obj
        o.cd_pass(np.roll(np.arange(6, dtype=np.int32), it))
    assert o.objective() == pytest.approx(ostar, rel=1e-9, abs=1e-12)
    assert o.objective() == pytest.approx(bf.lasso_objective(A, b, o.alpha, lam), rel=1e-12)
    np.testing.assert_allclose(o.alpha, astar, atol=1e-7)
    assert o.gaps() < 1e-9
    assert np.abs(o.alpha).sum() <= o.B                            # App. E: iterates stay in the box


def test_lasso_with_zero_lambda_is_least_squares():
    """Lambda = 0 turns the Lasso step into the plain exact line search of least squares, whose
    limit is numpy's lstsq solution."""
    rng = np.random.default_rng(11)
    cols = rng.standard_normal((5, 12)).astype(np.float32)
    b = rng.standard_normal(12).astype(np.float32)
    o = orc.Oracle(LASSO, b, 0.0, cols=cols)
    for _ in range(600):
        o.cd_pass(np.arange(5, dtype=np.int32))
    ref, *_ = np.linalg.lstsq(cols.T.astype(np.float64), b.astype(np.float64), rcond=None)
    np.testing.assert_allclose(o.alpha, ref, atol=1e-10)


# ----------------------------------------------------------------------------- SVM gaps
@pytest.mark.parametrize("seed", range(3))
def test_svm_gap_is_primal_plus_dual_and_equals_one_at_zero(seed):
    """App. E: with w = A alpha/(lambda n) the gap is P(w) + O(alpha) (Section 2, eq. (2)); at
    alpha = 0 every z_i is exactly 1/n and the total gap is 1."""
    cols, y, A, lam = tiny_svm(seed, n=30, d=7)
    n = 30
    o = orc.Oracle(SVM, y, lam, cols=cols)
    assert o.gaps() == pytest.approx(1.0, rel=1e-14)
    np.testing.assert_array_equal(o.z, np.full(n, 1.0 / n))
    for passes in (1, 2, 5):
        run_passes(o, passes, seed)
        total = o.gaps()
        w = A @ o.alpha / (lam * n)
        ref = bf.svm_primal_objective(A, y, w, lam) + bf.svm_dual_objective(A, y, o.alpha, lam)
        assert total == pytest.approx(ref, rel=1e-11, abs=1e-14)
        assert o.objective() == pytest.approx(bf.svm_dual_objective(A, y, o.alpha, lam), rel=1e-12)
        assert o.z.min() >= -1e-15
        assert np.all(y * o.alpha >= 0) and np.all(y * o.alpha <= 1)


@pytest.mark.parametrize("seed", range(4))
def test_svm_cd_reaches_bruteforce_optimum(seed):
    """App. C(c)/D: 8-sample duals solved exactly by enumerating the 3^8 active sets."""
    cols, y, A, lam = tiny_svm(seed)
    ostar, _ = bf.svm_dual_optimum(A, y.astype(np.float64), lam)
    o = orc.Oracle(SVM, y, lam, cols=cols)
    prev = o.objective()
    for it in range(3000):
        if it % 100 == 0:
            assert o.gaps() >= o.objective() - ostar - 1e-12
        o.cd_pass(np.roll(np.arange(8, dtype=np.int32), it))
        assert o.objective() <= prev + 1e-15
        prev = o.objective()
    assert o.objective() == pytest.approx(ostar, rel=1e-9, abs=1e-12)


# ----------------------------------------------------------------------------- single steps
@pytest.mark.parametrize("model", [LASSO, SVM])
def test_each_step_is_the_one_dimensional_argmin(model):
    """Alg. 3, the update of the chosen coordinate: the step minimises O over that coordinate alone.  Checked with scipy's
    scalar minimiser on an objective evaluated from A and alpha directly."""
    if model == LASSO:
        cols, tgt, A, lam = tiny_lasso(7, d=9, n=5)
        fobj = lambda a: bf.lasso_objective(A, tgt, a, lam)
    else:
        cols, tgt, A, lam = tiny_svm(7, n=7, d=4)
        fobj = lambda a: bf.svm_dual_objective(A, tgt, a, lam)
    o = orc.Oracle(model, tgt, lam, cols=cols)
    rng = np.random.default_rng(0)
    for step in range(40):
        j = int(rng.integers(o.n))
        base = o.alpha.copy()

        def line(t):
            a = base.copy()
            a[j] = t
            return fobj(a)
        if model == LASSO:
            res = minimize_scalar(line, bracket=(-3, 3), tol=1e-13)
        else:
            lo, hi = (0.0, 1.0) if tgt[j] > 0 else (-1.0, 0.0)
            res = minimize_scalar(line, bounds=(lo, hi), method="bounded",
                                  options={"xatol": 1e-13})
        o.cd_pass(np.array([j], dtype=np.int32))
        assert fobj(o.alpha) <= res.fun + 1e-12
        assert abs(o.alpha[j] - res.x) < 2e-5
        shift = tgt if model == LASSO else 0.0
        np.testing.assert_allclose(o.v, A @ o.alpha - shift, atol=1e-13)   # App. D: v stays A alpha (- b)


def test_zero_column_steps():
    """A column of zeros: the one-dimensional problems reduce to lam|t| (min at 0) and -y t/n
    on the box (min at y)."""
    cols, b, A, lam = tiny_lasso(1)
    cols = cols.copy()
    cols[2] = 0
    o = orc.Oracle(LASSO, b, lam, cols=cols)
    o.alpha[2] = 0.7
    o.cd_pass(np.array([2], dtype=np.int32))
    assert o.alpha[2] == 0.0
    cols, y, A, lam = tiny_svm(1)
    cols = cols.copy()
    cols[3] = 0
    o = orc.Oracle(SVM, y, lam, cols=cols)
    o.cd_pass(np.array([3], dtype=np.int32))
    assert o.alpha[3] == y[3]


# ----------------------------------------------------------------------------- selection
@pytest.mark.parametrize("seed", range(5))
def test_selection_is_the_argmax_over_all_subsets(seed):
    """eq. (11)/(13): P maximises the sum of z over all subsets of size m (brute force, n <= 12);
    eq. (7): rho of that P lies in [1, n/m]."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(5, 13))
    z = rng.random(n) ** 3
    for m in range(1, n + 1):
        P = orc.select_topm(z, m)
        assert P.size == m and np.all(np.diff(P) > 0)
        assert z[P].sum() == pytest.approx(bf.best_subset_sum(z, m), rel=1e-14)
        r = orc.rho(z, P)
        assert 1 - 1e-12 <= r <= n / m + 1e-12
        assert r == pytest.approx((z[P].mean()) / z.mean(), rel=1e-13)


def test_selection_ties_and_limits():
    z = np.full(9, 1.0 / 9)                     # the SVM at alpha = 0: all gaps equal
    np.testing.assert_array_equal(orc.select_topm(z, 4), [0, 1, 2, 3])
    z = np.array([0.5, 2.0, 0.5, 0.5, 3.0, 0.5])
    np.testing.assert_array_equal(orc.select_topm(z, 4), [0, 1, 2, 4])
    np.testing.assert_array_equal(orc.select_topm(z, 6), np.arange(6))
    np.testing.assert_array_equal(orc.select_topm(z, 60), np.arange(6))
    np.testing.assert_array_equal(orc.select_topm(z, 1), [4])


def test_rho_reaches_n_over_m_when_support_fits():
    """Section 5.1: on a sparse problem whose support fits in the block, rho -> n/m."""
    p = synth.lasso_dense(200, 100, 0.05, 0.2, seed=2)
    o = orc.Oracle(LASSO, p["target"].numpy(), p["lam"], cols=p["cols"].numpy())
    m = 25
    rng = np.random.default_rng(0)
    for _ in range(30):
        P, _ = o.round(m, passes=5, rng=rng)
    o.gaps()
    P = o.select(m)
    assert orc.rho(o.z, P) == pytest.approx(100 / m, rel=1e-6)


# ----------------------------------------------------------------------------- whole scheme
@pytest.mark.parametrize("seed", range(3))
def test_block_rounds_converge_to_the_full_optimum(seed):
    """Alg. 1 with rule (11) and m < n: the block scheme must reach the optimum of the whole
    problem (brute force), and m = n with one pass is plain CD (Remark after Thm 2)."""
    cols, b, A, lam = tiny_lasso(seed)
    ostar, astar = bf.lasso_optimum(A, b.astype(np.float64), lam)
    o = orc.Oracle(LASSO, b, lam, cols=cols)
    for _ in range(300):
        P, total = o.round(3, passes=2)
        assert P.size == 3
    assert o.objective() == pytest.approx(ostar, rel=1e-9, abs=1e-12)
    o_full = orc.Oracle(LASSO, b, lam, cols=cols)
    o_plain = orc.Oracle(LASSO, b, lam, cols=cols)
    for _ in range(5):
        o_full.round(6, passes=1)
        o_plain.cd_pass(np.arange(6, dtype=np.int32))
    np.testing.assert_array_equal(o_full.alpha, o_plain.alpha)

    cols, y, A, lam = tiny_svm(seed)
    ostar, _ = bf.svm_dual_optimum(A, y.astype(np.float64), lam)
    o = orc.Oracle(SVM, y, lam, cols=cols)
    for _ in range(1500):
        o.round(4, passes=2)
    assert o.objective() == pytest.approx(ostar, rel=1e-9, abs=1e-12)


# ----------------------------------------------------------------------------- Algorithm 2
def test_rho_hand_computed():
    """eq. (7) on numbers small enough to do in the head: z = (4, 2, 1, 1), P = {0, 1}: the mean over
    P is 3, the mean over all is 2, so rho = 3/2; P = {2, 3} gives 1/2; P = everything gives 1; and
    a single coordinate that holds the whole gap gives n/m = 4."""
    z = np.array([4.0, 2.0, 1.0, 1.0])
    assert orc.rho(z, np.array([0, 1], dtype=np.int32)) == 1.5
    assert orc.rho(z, np.array([2, 3], dtype=np.int32)) == 0.5
    assert orc.rho(z, np.arange(4, dtype=np.int32)) == 1.0
    assert orc.rho(np.array([0.0, 0.0, 7.0, 0.0]), np.array([2], dtype=np.int32)) == 4.0
    # a slip in either normalisation (1/m or 1/n) changes these: (6)/(8) = 0.75, (6/2)/8 = 0.375, ...
    assert orc.rho(z, np.array([0], dtype=np.int32)) == 2.0


def _delayed_by_hand(o, m, refresh, passes):
    """Algorithm 2's round written out with nothing but the oracle's pinned steps and a SECOND oracle
    object that is put at alpha^(t) to evaluate unit A's samples there."""
    P = orc.select_topm(o.z, m)
    at_t = orc.Oracle(o.model, o.target, o.lam, cols=o._keep[0], eta=o.eta)
    at_t.set_state(o.alpha.copy(), o.v.copy())
    for _ in range(passes):
        o.cd_pass(P)
    at_t.gaps(refresh)
    o.z[refresh] = at_t.z[refresh]
    return P


@pytest.mark.parametrize("seed", range(3))
def test_delayed_round_evaluates_samples_at_the_start_of_the_round(seed):
    """Alg. 2: unit A's samples are gap_j(alpha^(t)) -- the iterate BEFORE unit B's update of the same
    round -- they enter the gap memory after the selection, and every other entry keeps its value."""
    p = synth.lasso_dense(60, 40, 0.2, 0.1, seed=seed)
    cols, b = p["cols"].numpy(), p["target"].numpy()
    o = orc.Oracle(LASSO, b, p["lam"], cols=cols)
    ref = orc.Oracle(LASSO, b, p["lam"], cols=cols)
    o.gaps()
    ref.gaps()
    rng = np.random.default_rng(seed)
    differs = False
    for t in range(12):
        refresh = np.sort(rng.choice(40, 7, replace=False)).astype(np.int32)
        z_before = o.z.copy()
        P = o.round_delayed(8, refresh, passes=2)
        P_ref = _delayed_by_hand(ref, 8, refresh, 2)
        np.testing.assert_array_equal(P, P_ref)
        np.testing.assert_array_equal(P, orc.select_topm(z_before, 8))       # selection saw the OLD memory
        np.testing.assert_array_equal(o.alpha, ref.alpha)
        np.testing.assert_array_equal(o.z, ref.z)
        rest = np.ones(40, dtype=bool)
        rest[refresh] = False
        np.testing.assert_array_equal(o.z[rest], z_before[rest])               # stale entries stay
        # and the refreshed ones are NOT the gaps at the new iterate (unless B did not move)
        now = orc.Oracle(LASSO, b, p["lam"], cols=cols)
        now.set_state(o.alpha.copy(), o.v.copy())
        now.gaps(refresh)
        differs = differs or np.abs(now.z[refresh] - o.z[refresh]).max() > 0
        # the running v still is A alpha - b
        np.testing.assert_allclose(o.v, cols.astype(np.float64).T @ o.alpha - b, atol=1e-12)
    assert differs            # (many Lasso gaps are exactly 0 at both iterates, but not all of them)


def test_delayed_round_special_cases_reduce_to_algorithm_1():
    """m = n: the working set is everything whatever the memory says, so the iterates are those of
    plain coordinate descent (round() with m = n).  Refreshing every coordinate BEFORE the selection
    (fresh_idx = all) is Alg. 1 with rule (11) itself.  Refreshing every coordinate as unit A does
    (after the selection) is rule (11) one round late: round t+1 selects by the gaps at alpha^(t)."""
    p = synth.lasso_dense(60, 40, 0.2, 0.1, seed=5)
    cols, b = p["cols"].numpy(), p["target"].numpy()
    everything = np.arange(40, dtype=np.int32)
    a = orc.Oracle(LASSO, b, p["lam"], cols=cols)
    c = orc.Oracle(LASSO, b, p["lam"], cols=cols)
    for _ in range(6):
        a.round_delayed(40, everything[:5], passes=1)
        c.round(40, passes=1)
        np.testing.assert_array_equal(a.alpha, c.alpha)
    a = orc.Oracle(LASSO, b, p["lam"], cols=cols)
    c = orc.Oracle(LASSO, b, p["lam"], cols=cols)
    for _ in range(8):
        Pa = a.round_delayed(9, None, passes=2, fresh_idx=everything)
        Pc, _ = c.round(9, passes=2)
        np.testing.assert_array_equal(Pa, Pc)
        np.testing.assert_array_equal(a.alpha, c.alpha)
    a = orc.Oracle(LASSO, b, p["lam"], cols=cols)
    a.gaps()
    for _ in range(8):
        shadow = orc.Oracle(LASSO, b, p["lam"], cols=cols)
        shadow.set_state(a.alpha.copy(), a.v.copy())
        shadow.gaps()                                        # the gaps at alpha^(t)
        a.round_delayed(9, everything, passes=2)
        np.testing.assert_array_equal(a.z, shadow.z)          # what round t+1 will select by


@pytest.mark.parametrize("seed", range(3))
def test_delayed_rounds_converge_to_the_full_optimum(seed):
    """Alg. 2 with a gap memory refreshed a few coordinates per round still reaches the optimum of the
    whole problem (brute force over sign patterns / active sets), Lasso and SVM."""
    cols, b, A, lam = tiny_lasso(seed)
    ostar, _ = bf.lasso_optimum(A, b.astype(np.float64), lam)
    o = orc.Oracle(LASSO, b, lam, cols=cols)
    o.gaps()
    for t in range(400):
        o.round_delayed(3, np.array([(2 * t) % 6, (2 * t + 1) % 6], dtype=np.int32), passes=2)
    assert o.objective() == pytest.approx(ostar, rel=1e-9, abs=1e-12)
    cols, y, A, lam = tiny_svm(seed)
    ostar, _ = bf.svm_dual_optimum(A, y.astype(np.float64), lam)
    o = orc.Oracle(SVM, y, lam, cols=cols)
    o.gaps()
    for t in range(2500):
        o.round_delayed(4, np.array([(3 * t + k) % 8 for k in range(3)], dtype=np.int32), passes=2)
    assert o.objective() == pytest.approx(ostar, rel=1e-9, abs=1e-12)


# ----------------------------------------------------------------------------- storage forms
@pytest.mark.parametrize("model", [LASSO, SVM])
def test_sparse_and_dense_storage_agree(model):
    """The CSR branch against the dense branch on the same matrix (index or transpose slips)."""
    rng = np.random.default_rng(4)
    n, d = 23, 17
    dense = (rng.standard_normal((n, d)) * (rng.random((n, d)) < 0.3)).astype(np.float32)
    dense[5] = 0
    rowptr = np.zeros(n + 1, dtype=np.int64)
    colidx, val = [], []
    for i in range(n):
        nz = np.flatnonzero(dense[i])
        colidx += list(nz)
        val += list(dense[i, nz])
        rowptr[i + 1] = len(colidx)
    csr = (rowptr, np.array(colidx, dtype=np.int32), np.array(val, dtype=np.float32))
    if model == LASSO:
        tgt = rng.standard_normal(d).astype(np.float32)
        lam = 0.1 * np.abs(dense.astype(np.float64) @ tgt).max() / d
    else:
        tgt = np.where(rng.standard_normal(n) >= 0, 1.0, -1.0).astype(np.float32)
        lam = 1.0 / n
    a = orc.Oracle(model, tgt, lam, cols=dense)
    s = orc.Oracle(model, tgt, lam, csr=csr, d=d)
    np.testing.assert_allclose(a.q, s.q, rtol=1e-14)
    for it in range(4):
        order = rng.permutation(n).astype(np.int32)
        a.cd_pass(order)
        s.cd_pass(order)
        np.testing.assert_allclose(a.alpha, s.alpha, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(a.v, s.v, rtol=1e-12, atol=1e-14)
        idx = rng.permutation(n)[:9].astype(np.int32)
        assert a.gaps(idx) == pytest.approx(s.gaps(idx), rel=1e-12)
        np.testing.assert_allclose(a.z, s.z, rtol=1e-11, atol=1e-15)
        assert a.objective() == pytest.approx(s.objective(), rel=1e-13)


def test_strided_dense_columns():
    """Columns with a leading dimension larger than d give the same results."""
    cols, b, lam = mid_lasso(d=30, n=20)
    wide = np.full((20, 37), np.nan, dtype=np.float32)
    wide[:, :30] = cols
    a = orc.Oracle(LASSO, b, lam, cols=cols)
    s = orc.Oracle(LASSO, b, lam, cols=wide[:, :30])
    run_passes(a, 2)
    run_passes(s, 2)
    np.testing.assert_array_equal(a.alpha, s.alpha)
    assert a.gaps() == s.gaps()


# ----------------------------------------------------------------------------- planted mistakes
MUTATIONS = [
    ("B * over", "B * 0.5 * over"),                               # scaled conjugate term
    ("Lam * fabs(alpha[i])) / d", "Lam * alpha[i]) / d"),         # |alpha| -> alpha
    ("alpha[i] * c + B", "-alpha[i] * c + B"),                    # sign of the coupling term
    ("double hinge = 1.0 - (double)y[i] * s;", "double hinge = 1.0 - s;"),
    ("- (double)y[i] * alpha[i]) / n", "+ (double)y[i] * alpha[i]) / n"),
    ("double tau = Lam / qj;", "double tau = Lam;"),              # threshold not divided by q_j
    ("(alpha[j] * qj - col_dot(M, j, v)) / qj", "(alpha[j] * qj + col_dot(M, j, v)) / qj"),
    ("(yj - col_dot(M, j, v) / lam_n) / (qj / lam_n)", "(yj - col_dot(M, j, v)) / (qj / lam_n)"),
    ("if (a->z > b->z) return -1;\n    if (a->z < b->z) return 1;",
     "if (a->z > b->z) return 1;\n    if (a->z < b->z) return -1;"),
    ("return sq / (2.0 * lambda * (double)M->d);", "return sq / (2.0 * (double)M->d);"),
]


@pytest.mark.parametrize("which", range(len(MUTATIONS)))
def test_planted_mistakes_are_caught(which, tmp_path, monkeypatch):
    """Plant one slip in a copy of the oracle's C source and check that the pins above notice."""
    src = open(os.path.join(os.path.dirname(orc.__file__), "duhl_oracle.c")).read()
    old, new = MUTATIONS[which]
    assert src.count(old) == 1, old
    mutated = tmp_path / "mut.c"
    mutated.write_text(src.replace(old, new))
    lib = tmp_path / "libmut.so"
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-shared", "-fPIC", "-o", str(lib),
                           str(mutated), "-lm"])
    good = orc._lib
    monkeypatch.setattr(orc, "_lib", None)
    monkeypatch.setattr(orc, "build", lambda force=False: str(lib))
    pins = [test_lasso_gap_sum_equals_primal_minus_dual,
            test_lasso_orthonormal_closed_form,
            lambda: test_lasso_gap_bounds_suboptimality_and_cd_reaches_bruteforce_optimum(0),
            lambda: test_svm_gap_is_primal_plus_dual_and_equals_one_at_zero(0),
            lambda: test_svm_cd_reaches_bruteforce_optimum(0),
            lambda: test_selection_is_the_argmax_over_all_subsets(0)]
    caught = False
    for pin in pins:
        try:
            pin()
        except AssertionError:
            caught = True
            break
    monkeypatch.setattr(orc, "_lib", good)
    assert caught, f"mutation {old!r} -> {new!r} slipped through"


# ----------------------------------------------------------------------------- elastic net / ridge
ENET = orc.ENET


@pytest.mark.parametrize("eta", [1.0, 0.5, 0.1])
def test_enet_gap_is_primal_minus_dual_and_cd_reaches_the_optimum(eta):
    """App. D (elastic-net step), App. E (ridge gap = the eta = 1 case): the gap equals eq. (2)
    written from the conjugates; the CD limit is the enumerated KKT solution; for eta = 1 that is
    the ridge normal-equations solution; every step is the 1-D argmin."""
    cols, b, A, lam = tiny_lasso(3, d=9, n=6, c=0.2)
    b64 = b.astype(np.float64)
    o = orc.Oracle(ENET, b, lam, cols=cols, eta=eta)
    ostar, astar = bf.enet_optimum(A, b64, lam, eta)
    if eta == 1.0:
        ridge = np.linalg.solve(A.T @ A / 9 + lam * np.eye(6), A.T @ b64 / 9)
        np.testing.assert_allclose(astar, ridge, atol=1e-12)
    rng = np.random.default_rng(0)
    prev = o.objective()
    for it in range(300):
        total = o.gaps()
        assert total == pytest.approx(bf.enet_gap(A, b64, o.alpha, lam, eta), rel=1e-10, abs=1e-15)
        assert o.z.min() >= -1e-15
        assert total >= o.objective() - ostar - 1e-12
        if it < 30:
            j = int(rng.integers(6))
            base = o.alpha.copy()

            def line(t):
                a = base.copy()
                a[j] = t
                return bf.enet_objective(A, b64, a, lam, eta)
            res = minimize_scalar(line, bracket=(-3, 3), tol=1e-13)
            o.cd_pass(np.array([j], dtype=np.int32))
            assert line(o.alpha[j]) <= res.fun + 1e-12
            np.testing.assert_allclose(o.v, A @ o.alpha - b64, atol=1e-13)
        else:
            o.cd_pass(rng.permutation(6).astype(np.int32))
        obj = o.objective()
        assert obj == pytest.approx(bf.enet_objective(A, b64, o.alpha, lam, eta), rel=1e-12)
        assert obj <= prev + 1e-15
        prev = obj
    assert o.objective() == pytest.approx(ostar, rel=1e-10)
    np.testing.assert_allclose(o.alpha, astar, atol=1e-8)
    assert o.gaps() < 1e-12


def test_enet_tends_to_lasso_for_small_eta():
    """eta -> 0 recovers the Lasso step (App. D with eta = 0)."""
    cols, b, A, lam = tiny_lasso(2)
    e = orc.Oracle(ENET, b, lam, cols=cols, eta=1e-12)
    l = orc.Oracle(LASSO, b, lam, cols=cols)
    for _ in range(50):
        e.cd_pass(np.arange(6, dtype=np.int32))
        l.cd_pass(np.arange(6, dtype=np.int32))
    np.testing.assert_allclose(e.alpha, l.alpha, atol=1e-9)


# ---------------------------------------------------------------------------------- hand-worked fixtures
def _golden():
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")) as f:
        return json.load(f)


@pytest.mark.parametrize("name", ["lasso_identity_2x2", "svm_two_points_1d", "ridge_one_column"])
def test_oracle_reproduces_the_hand_worked_examples(name):
    """Tiny instances worked by hand from App. C, D and E (tests/golden/hand_worked.json holds the
    derivations): objective, gaps, one pass in index order, all exact in floating point."""
    case = _golden()[name]
    model = {"lasso": orc.LASSO, "svm_t": orc.SVM, "ridge": orc.ENET}[name[:5]]
    cols = np.array(case["cols"], dtype=np.float32)
    o = orc.Oracle(model, np.array(case["target"], dtype=np.float32), case["lambda"], cols=cols,
                   eta=case.get("eta", 1.0))
    if "B" in case:
        assert o.B == case["B"]
    assert o.objective() == case["objective_at_zero"]
    assert o.gaps() == sum(case["gaps_at_zero"])
    np.testing.assert_array_equal(o.z, case["gaps_at_zero"])
    o.cd_pass(np.arange(cols.shape[0], dtype=np.int32))
    np.testing.assert_array_equal(o.alpha, case["alpha_after_pass_0_1"])
    np.testing.assert_array_equal(o.v, case["v_after_pass"])
    assert o.objective() == case["objective_after_pass"]
    o.gaps()
    np.testing.assert_array_equal(o.z, case["gaps_after_pass"])
