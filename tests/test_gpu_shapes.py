"""Seeded sweeps over problem shapes: the sizes at which the library switches kernels (threads per
coordinate, register/LDS split of the private v, compute units per worker, ranges and slices of
the sparse copy), their neighbours, and sizes drawn at random in between.  Each shape is checked
against the oracle the same way as the hand-picked cases of test_gpu_parity.py: gap vectors
(App. E) at the state a few concurrent passes leave, the invariant v = A alpha (- b) that those
passes must keep (App. D), and sequential steps on a few coordinates."""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import gpu_common
    return gpu_common


DENSE_EDGES = [1, 3, 4, 5, 63, 64, 65, 255, 256, 257, 2047, 2048, 2049, 4095, 4096, 4097, 13311, 13312, 13313,
               53247, 53248, 53249, 106495, 106496, 106497, 212992, 212993]


@pytest.mark.parametrize("seed", [1, 2])
def test_dense_shapes(G, seed):
    from paper_1708_05357_amd import duhl, synth
    rng = np.random.default_rng(seed)
    for it in range(30):
        d = int(rng.choice(DENSE_EDGES)) if rng.random() < 0.7 else int(rng.integers(1, 120000))
        n = int(rng.choice([1, 2, 7, 64, 65, 130, int(rng.integers(1, 300))]))
        if d * n > 3e7:
            n = max(1, int(3e7 // d))
        model = str(rng.choice(["lasso", "svm", "enet"]))
        if model == "svm":
            prob = synth.svm_dense(n, d, seed=int(rng.integers(1 << 30)))
        else:
            prob = synth.lasso_dense(d, n, 0.2, 0.1, seed=int(rng.integers(1 << 30)))
            if model == "enet":
                prob["model"], prob["eta"] = "enet", float(rng.choice([1.0, 0.5]))
        ld = None                                        # ld = d, or padded to whole 16-byte chunks and beyond
        if rng.random() < 0.6:
            ld = (d + 3) // 4 * 4 + 4 * int(rng.integers(0, 3))
        what = f"{model} d={d} n={n} ld={ld}"
        p = G.Pair(prob, ld=ld)
        m = max(1, n // 2)
        for rnd in range(3):
            p.g.gap(want_sum=False)
            p.g.select(m, want_stats=False)
            p.g.commit_swap()
            p.g.cd_epoch(duhl.CD_ASYNC, seed=rnd)
        a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
        p.o.set_state(a.astype(np.float64))              # v from its definition
        scale = max(np.abs(p.o.v).max(), 1e-30,
                    np.abs(G.to_np(prob["target"])).max() if model != "svm" else 1.0)
        assert np.abs(v - p.o.v).max() <= 2e-5 * scale, what
        p.o.set_state(a.astype(np.float64), v.astype(np.float64))
        p.o.gaps()
        p.g.gap(want_sum=False)
        z, zo = p.g.get(duhl.Z), np.maximum(p.o.z, 0.0)
        G.assert_gaps_close(z, zo, floor=G.gap_floor(p), label=f"dense shapes {model}")
        members = set(p.g.get(duhl.P).tolist())
        order = np.array([j for j in rng.permutation(n)[:5] if j in members], dtype=np.int32)
        if order.size:
            p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(order))
            p.o.cd_pass(order)
            a2, v2 = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
            assert np.abs(a2 - p.o.alpha).max() <= 1e-5 * max(np.abs(p.o.alpha).max(), 1e-30) + 1e-7, what
            assert np.abs(v2 - p.o.v).max() <= 1e-5 * scale, what
        p.close()


@pytest.mark.parametrize("seed", [1, 2])
def test_sparse_shapes(G, monkeypatch, seed):
    """The sliced copy at row counts around a slice (64) and a sorting window (1,024), column
    counts around a range of v (34,560), and row lengths from one entry to several hundred;
    full pass and index list (the threshold is lowered so that lists take the copy too)."""
    from paper_1708_05357_amd import duhl, synth
    monkeypatch.setenv("DUHL_CSR_BLOCKED_LIST_MIN", "1")
    rng = np.random.default_rng(seed)
    for it in range(40):
        n = int(rng.choice([1, 2, 63, 64, 65, 1000, 1023, 1024, 1025, 3000, int(rng.integers(1, 6000))]))
        d = int(rng.choice([1, 3, 4, 5, 100, 34559, 34560, 34561, 69121, 100000, int(rng.integers(1, 250000))]))
        density = min(1.0, float(rng.choice([1, 3, 8, 33, 100, 400])) / d)
        if n * density * d > 3e6:
            density = 3e6 / (n * d)
        prob = synth.svm_csr(n, d, density, seed=int(rng.integers(1 << 30)))
        what = f"n={n} d={d} density={density:.3g}"
        p = G.Pair(prob)
        y = prob["target"].numpy()
        alpha = (y * rng.random(n) * (rng.random(n) < 0.5)).astype(np.float32)   # feasible: y alpha in [0, 1]
        v = rng.standard_normal(d).astype(np.float32)                            # any v: only the formula is tested
        p.g.set(duhl.ALPHA, alpha)
        p.g.set(duhl.V, v)
        p.o.set_state(alpha.astype(np.float64), v.astype(np.float64))
        p.o.gaps()
        zo = np.maximum(p.o.z, 0.0)                      # the library clamps at 0 (Section 2)
        rowptr, colidx, val = prob["rowptr"].numpy(), prob["colidx"].numpy(), prob["val"].numpy()
        rows = np.repeat(np.arange(n), np.diff(rowptr))
        S = np.bincount(rows, weights=np.abs(val.astype(np.float64) * v[colidx]), minlength=n)
        floor = 8 * 2.0 ** -24 / n * (1 + (1 + np.abs(alpha)) * S / (prob["lam"] * n))
        tol = 1e-4 * np.abs(zo) + floor
        total = p.g.gap()
        z = p.g.get(duhl.Z).astype(np.float64)
        assert (np.abs(z - zo) <= tol).all(), what
        assert abs(total - zo.sum()) <= 1e-4 * zo.sum() + n * floor.max(), what
        listed = rng.permutation(n)[:max(1, n // 2)].astype(np.int32)
        p.g.set(duhl.Z, np.full(n, -1.0, dtype=np.float32))
        p.g.gap(G.dev_i32(listed), want_sum=False)
        z2 = p.g.get(duhl.Z).astype(np.float64)
        rest = np.ones(n, dtype=bool)
        rest[listed] = False
        assert (np.abs(z2[listed] - zo[listed]) <= tol[listed]).all(), what
        assert (z2[rest] == -1.0).all(), what
        p.close()
