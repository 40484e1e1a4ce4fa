"""Seeded synthetic inputs shaped like the workloads of the paper's experiments.

The paper trains on two fully dense single-precision datasets (Section 5.1 and 5.3) that are
not available here; these generators stand in for them.  This module only draws data: it holds
none of the method's arithmetic (no gaps, no updates, no selection) and is the one piece that
both the HIP path's tests and the CPU oracle's tests are allowed to share.

Everything is written with torch ops so the same recipe runs on the CPU (small cases for the
oracle) and on the GPU (the large benchmark cases, generated block by block in HBM).

Dense problems are returned "by columns": a float32 tensor ``cols`` of shape (n, d) whose row i
is the column a_i of the paper's d x n matrix A, i.e. A stored column-major.
"""
import math

import torch


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _segments(out, j0, j1):
    """The rows [j0, j1) of a matrix stored as one (n, d) tensor or as a list of (rows_k, d) pieces
    (all of the same height but the last): (tensor slice, first row, end row) per piece touched."""
    if isinstance(out, torch.Tensor):
        yield out[j0:j1], j0, j1
        return
    per = out[0].shape[0]
    while j0 < j1:
        k, a = divmod(j0, per)
        b = min(out[k].shape[0], a + (j1 - j0))
        yield out[k][a:b], j0, j0 + (b - a)
        j0 += b - a


def lasso_dense(d, n, support_frac, c_lambda, seed=0, device="cpu", out=None, block_cols=None,
                noise=0.01, clusters=0, spread=0.0):
    """Dense Lasso instance.

    Entries of A ~ N(0,1), every column scaled to unit L2 norm; alpha* has floor(support_frac*n)
    non-zeros at uniformly random positions with N(0,1) values; b = A alpha* + N(0, noise^2).
    The regulariser is set through Lambda = lambda*d = c_lambda * ||A^T b||_inf, so that the
    returned ``lam`` is the lambda of the paper's objective ||A alpha - b||^2/(2d) + lambda||alpha||_1.

    clusters > 0: the columns come in that many groups of near-duplicates instead -- column j is the
    centre of group j mod clusters (N(0,1) entries) plus ``spread`` times N(0,1) noise, scaled to
    unit norm (see lasso_clustered, the all-at-once version for small instances).

    ``out`` (optional) is a preallocated float32 (n, d) tensor to fill -- on the device, or in
    pinned host memory for the out-of-budget case --, or a list of such tensors that hold the
    columns in order, piece by piece; blocks are generated on ``device`` and copied.
    """
    dev = torch.device(device)
    g = _gen(seed, dev)
    if out is None:
        out = torch.empty((n, d), dtype=torch.float32, device=dev)
    if isinstance(out, torch.Tensor):
        assert out.shape == (n, d) and out.dtype == torch.float32
    else:
        assert sum(t.shape[0] for t in out) == n and all(t.shape[1] == d and t.dtype == torch.float32 for t in out)
        assert all(t.shape[0] == out[0].shape[0] for t in out[:-1]) and out[-1].shape[0] <= out[0].shape[0]
    if block_cols is None:
        block_cols = max(1, min(n, (256 << 20) // (4 * d)))
    k = int(math.floor(support_frac * n))
    perm = torch.randperm(n, generator=g, device=dev)
    support = perm[:k].sort().values
    alpha_star = torch.zeros(n, dtype=torch.float32, device=dev)
    alpha_star[support] = torch.randn(k, generator=g, device=dev, dtype=torch.float32)
    b = torch.zeros(d, dtype=torch.float32, device=dev)
    centres = torch.randn((clusters, d), generator=g, dtype=torch.float32, device=dev) if clusters > 0 else None
    for j0 in range(0, n, block_cols):
        j1 = min(n, j0 + block_cols)
        x = torch.randn((j1 - j0, d), generator=g, device=dev, dtype=torch.float32)
        if centres is not None:
            x *= spread
            x += centres[torch.arange(j0, j1, device=dev) % clusters]
        x /= x.norm(dim=1, keepdim=True)
        b += x.t() @ alpha_star[j0:j1]
        for piece, a, e in _segments(out, j0, j1):
            piece.copy_(x[a - j0:e - j0])
    b += noise * torch.randn(d, generator=g, device=dev, dtype=torch.float32)
    atb_inf = 0.0
    for j0 in range(0, n, block_cols):
        j1 = min(n, j0 + block_cols)
        for piece, a, e in _segments(out, j0, j1):
            x = piece.to(dev, non_blocking=False)
            atb_inf = max(atb_inf, float((x @ b).abs().max()))
    lam = c_lambda * atb_inf / d
    return {"model": "lasso", "d": d, "n": n, "cols": out, "target": b, "lam": lam,
            "alpha_star": alpha_star}


def lasso_clustered(d, n, clusters, spread, support_frac=0.05, c_lambda=0.1, seed=0, noise=0.01, device="cpu"):
    """Dense Lasso instance whose columns come in `clusters` groups of near-duplicates: column j is
    the centre of group j mod clusters plus `spread` times N(0,1) noise, scaled to unit norm (cosine
    within a group about 1/(1+spread^2), between groups about 0).  Features of real datasets are
    often this alike; a working set chosen by gap then gathers whole groups.  alpha*, b and lambda
    as in lasso_dense."""
    dev = torch.device(device)
    g = _gen(seed, dev)
    centres = torch.randn((clusters, d), generator=g, dtype=torch.float32, device=dev)
    cols = torch.randn((n, d), generator=g, dtype=torch.float32, device=dev)
    cols *= spread
    cols += centres[torch.arange(n, device=dev) % clusters]
    cols /= cols.norm(dim=1, keepdim=True)
    k = int(math.floor(support_frac * n))
    alpha_star = torch.zeros(n, dtype=torch.float32, device=dev)
    alpha_star[torch.randperm(n, generator=g, device=dev)[:k]] = torch.randn(k, generator=g, dtype=torch.float32, device=dev)
    b = cols.t() @ alpha_star + noise * torch.randn(d, generator=g, dtype=torch.float32, device=dev)
    lam = c_lambda * float((cols @ b).abs().max()) / d
    return {"model": "lasso", "d": d, "n": n, "cols": cols.contiguous(), "target": b, "lam": lam,
            "alpha_star": alpha_star}


def orthonormal_lasso(d, n, seed=0):
    """Lasso instance whose columns are exactly orthonormal (n <= d); used for closed forms."""
    g = _gen(seed, "cpu")
    x = torch.randn((d, n), generator=g, dtype=torch.float64)
    qmat, _ = torch.linalg.qr(x)
    cols = qmat.t().contiguous().to(torch.float32)
    b = torch.randn(d, generator=g, dtype=torch.float32)
    return {"model": "lasso", "d": d, "n": n, "cols": cols, "target": b}


def _labels(margin, flip_frac, g, dev):
    n = margin.numel()
    y = torch.where(margin >= 0, 1.0, -1.0).to(torch.float32)      # sign(0) := +1
    nflip = int(math.floor(flip_frac * n))
    flip = torch.randperm(n, generator=g, device=dev)[:nflip]
    y[flip] = -y[flip]
    return y


def svm_dense(n, d, flip_frac=0.05, seed=0, device="cpu"):
    """Dense SVM instance: n samples (= columns of A, = coordinates) with d features each.

    Features ~ U(0,1) - 0.5, every sample scaled to unit L2 norm; labels sign(X w*) with
    w* ~ N(0,I) and a fraction flipped; lambda = 1/n.  ``cols[i]`` is sample i."""
    dev = torch.device(device)
    g = _gen(seed, dev)
    x = torch.rand((n, d), generator=g, device=dev, dtype=torch.float32)
    x -= 0.5
    x /= x.norm(dim=1, keepdim=True)
    w = torch.randn(d, generator=g, device=dev, dtype=torch.float32)
    y = _labels(x @ w, flip_frac, g, dev)
    return {"model": "svm", "d": d, "n": n, "cols": x, "target": y, "lam": 1.0 / n}


def svm_csr(n, d, density, flip_frac=0.05, seed=0, device="cpu"):
    """Sparse SVM instance as CSR over samples (row i = sample i = column a_i of the paper's A).

    Row lengths ~ Binomial(d, density) (at least 1), distinct sorted uniformly random feature
    indices, values U(0,1), rows scaled to unit L2 norm; labels sign(X w*) with w* ~ N(0,I) and a
    fraction flipped; lambda = 1/n."""
    dev = torch.device(device)
    g = _gen(seed, dev)
    counts = torch.binomial(torch.full((n,), float(d), device=dev),
                            torch.full((n,), float(density), device=dev), generator=g)
    counts = counts.clamp_(min=1).to(torch.int64)
    rows = torch.repeat_interleave(torch.arange(n, device=dev), counts)
    colsd = torch.randint(0, d, (rows.numel(),), generator=g, device=dev)
    key = torch.unique(rows * d + colsd)            # sorted, duplicates inside a row removed
    del rows, colsd
    rows = torch.div(key, d, rounding_mode="floor")
    colidx = (key - rows * d).to(torch.int32)
    del key
    counts = torch.bincount(rows, minlength=n)
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    rowptr[1:] = torch.cumsum(counts, 0)
    val = torch.rand(rows.numel(), generator=g, device=dev, dtype=torch.float32)
    val = val.clamp_(min=1e-3)
    sq = torch.zeros(n, dtype=torch.float32, device=dev).index_add_(0, rows, val * val)
    val /= sq.sqrt()[rows]
    w = torch.randn(d, generator=g, device=dev, dtype=torch.float32)
    margin = torch.zeros(n, dtype=torch.float32, device=dev).index_add_(
        0, rows, val * w[colidx.long()])
    y = _labels(margin, flip_frac, g, dev)
    return {"model": "svm", "d": d, "n": n, "rowptr": rowptr, "colidx": colidx, "val": val,
            "target": y, "lam": 1.0 / n}


# The five workloads of the benchmark plan, by name -> (generator, kwargs, m, rounds).
CONFIGS = {
    "cfg1": dict(kind="lasso_dense", d=1000, n=500, support_frac=0.10, c_lambda=0.1, m=125,
                 rounds=20),
    "cfg2": dict(kind="lasso_dense", d=10_000, n=50_000, support_frac=0.02, c_lambda=0.05,
                 m=5_000, rounds=50),
    "cfg3": dict(kind="svm_csr", n=1_000_000, d=100_000, density=1e-3, m=200_000, rounds=50),
    "cfg4": dict(kind="lasso_dense", d=100_000, n=200_000, support_frac=0.01, c_lambda=0.05,
                 m=20_000, rounds=20, host_resident=True),
    "cfg5": dict(kind="lasso_dense", d=50_000, n=500_000, support_frac=0.005, c_lambda=0.05,
                 m=50_000, rounds=20),
    # the 2 GB workload with correlated features, as real feature matrices have them (Section 5.3 uses
    # image features): 1,250 groups of 40 near-duplicate columns (cosine about 0.9 within a group)
    "cfg2clustered": dict(kind="lasso_clustered", d=10_000, n=50_000, clusters=1_250, spread=0.3,
                          support_frac=0.02, c_lambda=0.05, m=5_000, rounds=50),
    # the 100 GB workload with columns in 12,500 groups of 40 near-duplicates (on demand only:
    # `bench.py --workload cfg5clustered`)
    "cfg5clustered": dict(kind="lasso_dense", d=50_000, n=500_000, support_frac=0.005, c_lambda=0.05,
                          clusters=12_500, spread=0.3, m=50_000, rounds=20),
    # the shape of the paper's large-scale SVM experiment (Section 5.3: 40,000 samples with 200,704
    # dense single-precision features, 30 GB, a quarter of them on the accelerator)
    "fig5svm": dict(kind="svm_dense", n=40_000, d=200_704, m=10_000, rounds=20),
    # the shape of the paper's convergence experiments (Section 5.1: a dense dataset of 400,000
    # samples and 2,000 features, a quarter of the coordinates on the accelerator, Lasso support ~12 %)
    "sec51lasso": dict(kind="lasso_dense", d=400_000, n=2_000, support_frac=0.12, c_lambda=0.1,
                       m=500, rounds=20),
    # the same dataset shape for the SVM dual, where the coordinates are the samples
    "sec51svm": dict(kind="svm_dense", n=400_000, d=2_000, m=100_000, rounds=20),
}


def make(name, seed=0, device="cpu", scale=1.0, out=None):
    """Instantiate one of CONFIGS; ``scale`` < 1 shrinks n (and m) at fixed d for tests."""
    cfg = dict(CONFIGS[name])
    kind = cfg.pop("kind")
    m, rounds = cfg.pop("m"), cfg.pop("rounds")
    cfg.pop("host_resident", None)
    if scale != 1.0:
        cfg["n"] = max(8, int(cfg["n"] * scale))
        m = max(1, int(m * scale))
    if kind == "lasso_dense":
        p = lasso_dense(seed=seed, device=device, out=out, **cfg)
    elif kind == "lasso_clustered":
        p = lasso_clustered(seed=seed, device=device, **cfg)
    elif kind == "svm_dense":
        p = svm_dense(seed=seed, device=device, **cfg)
    else:
        p = svm_csr(seed=seed, device=device, **cfg)
    p["m"], p["rounds"], p["name"] = m, rounds, name
    return p
