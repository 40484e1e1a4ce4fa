"""The inequality that the guard of the concurrent passes rests on, checked with the oracle (CPU only).

A concurrent pass moves the iterate from (alpha, v) to (alpha + D, v + Dv).  The objectives of
Appendix C are a quadratic in v plus a sum of convex terms g_j(alpha_j), so for 0 <= theta <= 1

    O(alpha + theta D)  <=  O(alpha) + theta * lin + theta^2 * curv,
    lin = 2 q <v, Dv> + sum_j [g_j(alpha_j + D_j) - g_j(alpha_j)],   curv = q ||Dv||^2,

q = 1/(2d) (Lasso, elastic net) or 1/(2 lambda n^2) (SVM dual): the quadratic part exactly, every
g_j by its chord.  The right-hand side is smallest at theta* = -lin / (2 curv); at theta = 1 it is
the true change of the objective, so the pass raised the objective exactly when theta* < 1/2.
The device code forms lin and curv from its own sums; here the same quantities are formed from the
oracle's objective and state, for steps that really collide (every coordinate stepped against the
same stale v), and the claims are checked against the oracle's objective along the line.
"""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
from oracle import duhl_oracle as orc                     # noqa: E402
from paper_1708_05357_amd import synth                    # noqa: E402


def _problem(model, seed):
    if model == "svm":
        p = synth.svm_dense(60, 24, seed=seed)
        cols = np.repeat(p["cols"].numpy(), 3, axis=0)               # every sample three times: steps collide
        y = np.repeat(p["target"].numpy(), 3)
        return orc.Oracle(orc.SVM, y, 1.0 / cols.shape[0], cols=np.ascontiguousarray(cols)), cols.shape[0]
    p = synth.lasso_clustered(40, 90, 9, 0.2, seed=seed)             # 9 groups of 10 near-duplicates
    cols = np.ascontiguousarray(p["cols"].numpy())
    if model == "enet":
        return orc.Oracle(orc.ENET, p["target"].numpy(), p["lam"], cols=cols, eta=0.5), cols.shape[0]
    return orc.Oracle(orc.LASSO, p["target"].numpy(), p["lam"], cols=cols), cols.shape[0]


def _jacobi_step(o, coords):
    """Every coordinate of `coords` solved exactly against the same v: the new alpha (v not moved)."""
    a0, v0 = o.alpha.copy(), o.v.copy()
    new = a0.copy()
    for j in coords:
        o.set_state(a0, v0)
        o.cd_pass(np.array([j], dtype=np.int32))
        new[j] = o.alpha[j]
    o.set_state(a0, v0)
    return new


def _objective_at(o, alpha):
    keep = (o.alpha.copy(), o.v.copy())
    o.set_state(alpha)                                    # v from its definition
    val = o.objective()
    o.set_state(*keep)
    return val


@pytest.mark.parametrize("model", ["lasso", "enet", "svm"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_line_bound_and_its_minimiser(model, seed):
    o, n = _problem(model, seed)
    rng = np.random.default_rng(seed)
    o.cd_pass(rng.permutation(n)[: n // 3].astype(np.int32))         # some non-trivial iterate
    a0, v0, O0 = o.alpha.copy(), o.v.copy(), o.objective()
    coords = rng.permutation(n)[: n // 2]
    a1 = _jacobi_step(o, coords)
    o.set_state(a1)
    v1 = o.v.copy()
    o.set_state(a0, v0)
    dv = v1 - v0
    q = 0.5 / o.d if model != "svm" else 0.5 / (o.lam * o.n * o.n)
    # sum of the terms in alpha alone: O minus the quadratic part, at both ends
    g0 = O0 - q * (v0 @ v0)
    g1 = _objective_at(o, a1) - q * (v1 @ v1)
    lin, curv = 2.0 * q * (v0 @ dv) + (g1 - g0), q * (dv @ dv)
    assert curv > 0.0
    # each coordinate step descends on its own, so the line starts downhill
    assert lin < 0.0
    for theta in np.linspace(0.0, 1.0, 21):
        got = _objective_at(o, a0 + theta * (a1 - a0))
        assert got <= O0 + theta * lin + theta * theta * curv + 1e-12 * abs(O0)
    # at theta = 1 the bound is the change of the objective itself
    O1 = _objective_at(o, a1)
    assert abs((O1 - O0) - (lin + curv)) <= 1e-12 * max(abs(O0), abs(O1))
    theta_star = -lin / (2.0 * curv)
    assert (O1 > O0) == (theta_star < 0.5)
    # scaled back to min(1, theta*), the pass never raises the objective
    t = min(1.0, theta_star)
    assert _objective_at(o, a0 + t * (a1 - a0)) <= O0 + 1e-12 * abs(O0)


def test_colliding_steps_overshoot_and_sequential_ones_do_not():
    """Ten near-duplicates of each column stepped at once overshoot about tenfold (theta* near 1/10,
    objective up); the same coordinates one after the other give theta* >= 1/2 and descend."""
    o, n = _problem("lasso", 5)
    a0, v0, O0 = o.alpha.copy(), o.v.copy(), o.objective()
    q = 0.5 / o.d
    g0 = O0 - q * (v0 @ v0)

    def theta_of(a1):
        o.set_state(a1)
        v1, O1 = o.v.copy(), o.objective()
        o.set_state(a0, v0)
        dv = v1 - v0
        lin = 2.0 * q * (v0 @ dv) + (O1 - q * (v1 @ v1) - g0)
        return -lin / (2.0 * q * (dv @ dv)), O1

    th_jacobi, O_jacobi = theta_of(_jacobi_step(o, np.arange(n)))
    assert th_jacobi < 0.3 and O_jacobi > O0
    o.cd_pass(np.arange(n, dtype=np.int32))
    a_seq = o.alpha.copy()
    th_seq, O_seq = theta_of(a_seq)
    assert th_seq >= 0.5 and O_seq < O0
