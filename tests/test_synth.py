"""The seeded input generators: shapes, normalisation and the structure each recipe promises (CPU only).
They hold none of the method's arithmetic; both the oracle's tests and the GPU tests draw from them."""
import numpy as np
import pytest
import torch

from paper_1708_05357_amd import synth


def test_dense_lasso_recipe():
    p = synth.lasso_dense(200, 80, 0.1, 0.1, seed=3)
    A = p["cols"].numpy().astype(np.float64)                # row i = column a_i
    assert A.shape == (80, 200)
    np.testing.assert_allclose(np.linalg.norm(A, axis=1), 1.0, rtol=1e-6)
    assert np.count_nonzero(p["alpha_star"].numpy()) == 8
    # Lambda = lambda * d = c * ||A^T b||_inf
    b = p["target"].numpy().astype(np.float64)
    assert p["lam"] * 200 == pytest.approx(0.1 * np.abs(A @ b).max(), rel=1e-5)
    # the same seed gives the same bits, another seed another matrix
    q = synth.lasso_dense(200, 80, 0.1, 0.1, seed=3)
    assert torch.equal(p["cols"], q["cols"]) and torch.equal(p["target"], q["target"])
    assert not torch.equal(p["cols"], synth.lasso_dense(200, 80, 0.1, 0.1, seed=4)["cols"])


def test_clustered_columns_are_alike_within_a_group_only():
    """Column j = centre of group j mod clusters + spread * noise, unit norm: cosine about
    1 / (1 + spread^2) within a group, about 0 between groups -- from the all-at-once generator and
    from the block-wise one that the 100 GB workload uses."""
    for p in (synth.lasso_clustered(4000, 120, 12, 0.3, seed=1),
              synth.lasso_dense(4000, 120, 0.05, 0.1, seed=1, clusters=12, spread=0.3, block_cols=50)):
        A = p["cols"].numpy().astype(np.float64)
        np.testing.assert_allclose(np.linalg.norm(A, axis=1), 1.0, rtol=1e-6)
        G = A @ A.T
        group = np.arange(120) % 12
        same = (group[:, None] == group[None, :]) & ~np.eye(120, dtype=bool)
        assert abs(G[same].mean() - 1.0 / 1.09) < 0.01
        assert np.abs(G[~same & ~np.eye(120, dtype=bool)]).mean() < 0.03


def test_sparse_svm_recipe():
    p = synth.svm_csr(500, 300, 0.05, seed=2)
    rowptr, colidx, val = p["rowptr"].numpy(), p["colidx"].numpy(), p["val"].numpy().astype(np.float64)
    assert rowptr[0] == 0 and rowptr[-1] == val.size and np.all(np.diff(rowptr) >= 1)
    for i in (0, 17, 499):
        seg = slice(rowptr[i], rowptr[i + 1])
        assert np.all(np.diff(colidx[seg]) > 0) and colidx[seg].min() >= 0 and colidx[seg].max() < 300
        assert np.linalg.norm(val[seg]) == pytest.approx(1.0, rel=1e-5)
    y = p["target"].numpy()
    assert set(np.unique(y)) <= {-1.0, 1.0}
    assert p["lam"] == 1.0 / 500


def test_every_named_workload_has_a_recipe():
    for name, cfg in synth.CONFIGS.items():
        assert cfg["kind"] in ("lasso_dense", "lasso_clustered", "svm_dense", "svm_csr"), name
        assert 0 < cfg["m"] <= cfg["n"]
    small = synth.make("cfg1", seed=0)
    assert small["cols"].shape == (500, 1000) and small["m"] == 125
    tiny = synth.make("cfg2clustered", seed=0, scale=0.01)
    assert tiny["cols"].shape == (500, 10000) and tiny["m"] == 50
