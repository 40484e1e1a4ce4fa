"""Parity of the HIP path with the CPU oracle, element by element, through the C ABI.

Tolerances (the benchmark spec): gap vectors 1e-4 relative in fp32 (normwise, and entrywise on the
entries that matter), selection bit-exact on the same fp32 z, sequential CD iterates 1e-5
relative, asynchronous CD final objective 1e-5 relative.
"""
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(__file__))

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import gpu_common
    return gpu_common


def lasso_problem(d, n, frac=0.1, c=0.1, seed=0):
    from paper_1708_05357_amd import synth
    return synth.lasso_dense(d, n, frac, c, seed=seed)


# ------------------------------------------------------------------------------------ gaps
@pytest.mark.parametrize("d,n,ld", [(1000, 500, None), (1003, 37, None), (64, 9, None), (1, 5, None),
                                    (257, 130, 300), (4100, 67, 4104), (10, 3, 13),
                                    (60000, 1400, None), (60002, 1500, 60004)])
def test_dense_lasso_gaps_match_oracle(G, d, n, ld):
    """App. E (Lasso): z from the first pass of set_data, from a full pass at a later state, and
    from an index-list refresh; sizes cover whole tiles, ragged tails, unaligned leading
    dimensions (scalar path) and fewer columns than one wavefront group.  The last two have
    columns long enough (three parts of v) for the pass that keeps v on chip, one of them with
    d % 4 != 0."""
    from paper_1708_05357_amd import duhl
    p = G.Pair(lasso_problem(d, n, 0.2, 0.1, seed=d + n), ld=ld)
    np.testing.assert_allclose(p.g.get(duhl.SQNORM), p.o.q, rtol=2e-6)
    total_or = p.o.gaps()
    G.assert_gaps_close(p.g.get(duhl.Z), p.o.z, label=f"dense lasso {d}x{n} at alpha=0")   # the bare rule
    rng = np.random.default_rng(1)
    m = max(1, n // 2)
    for rnd in range(3):
        p.g.select(m)
        p.g.commit_swap()
        order = rng.permutation(p.g.get(duhl.P)).astype(np.int32)
        p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(order))
        p.sync_oracle_to_gpu_state()
        total_gpu = p.g.gap()
        total_or = p.o.gaps()
        floor = G.gap_floor(p)
        G.assert_gaps_close(p.g.get(duhl.Z), p.o.z, floor=floor, label=f"dense lasso {d}x{n} round {rnd + 1}")
        assert total_gpu == pytest.approx(total_or, rel=1e-4, abs=float(floor.sum()))
    # stale entries stay, listed entries are refreshed
    zero = np.zeros(n, dtype=np.float32)
    p.g.set(duhl.Z, zero)
    idx = rng.permutation(n)[: max(1, n // 3)].astype(np.int32)
    part = p.g.gap(G.dev_i32(idx))
    z = p.g.get(duhl.Z)
    mask = np.zeros(n, dtype=bool)
    mask[idx] = True
    assert np.all(z[~mask] == 0)
    G.assert_gaps_close(z[idx], p.o.z[idx], floor=floor[idx], label=f"dense lasso {d}x{n} index list")
    assert part == pytest.approx(float(p.o.z[mask].sum()), rel=1e-4, abs=float(floor[idx].sum()))
    p.close()


def test_svm_gaps_match_oracle_dense_and_csr(G):
    """App. E (SVM): all gaps equal 1/n at alpha = 0; parity after some passes, both storages."""
    from paper_1708_05357_amd import duhl, synth
    for prob in (synth.svm_dense(300, 41, seed=3), synth.svm_csr(1500, 400, 0.02, seed=4),
                 synth.svm_dense(1400, 60000, seed=5)):          # long columns: v on chip, three parts
        p = G.Pair(prob)
        n = prob["n"]
        np.testing.assert_allclose(p.g.get(duhl.Z), np.full(n, 1.0 / n), rtol=1e-6)
        np.testing.assert_allclose(p.g.get(duhl.SQNORM), p.o.q, rtol=2e-6)
        assert p.g.gap() == pytest.approx(1.0, rel=1e-6)
        rng = np.random.default_rng(0)
        for rnd in range(3):
            p.g.select(n // 2)
            p.g.commit_swap()
            order = rng.permutation(p.g.get(duhl.P)).astype(np.int32)
            p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(order))
            p.sync_oracle_to_gpu_state()
            total = p.g.gap()
            assert total == pytest.approx(p.o.gaps(), rel=1e-4)
            G.assert_gaps_close(p.g.get(duhl.Z), p.o.z, floor=G.gap_floor(p, partials=128 if "cols" in prob else 1),
                                label=f"svm {'dense' if 'cols' in prob else 'csr'} n={n} round {rnd + 1}")
        p.close()


@pytest.mark.parametrize("n,d,density", [
    (3000, 400, 0.02),        # one range, ~8 non-zeros per row: two quad-rows per slice
    (2000, 50000, 0.002),     # two ranges, ~50 per row and range
    (1500, 80000, 0.004),     # three ranges, ~107 per row and range
    (1200, 3000, 0.1),        # one range, ~300 per row: slices longer than a wavefront's share
    (700, 2000, 0.3),         # ~600 per row; a last window of 700 rows, the rest of it empty
    (900, 36865, 0.001),      # d % 4 != 0; fewer rows than one sorting window
    (65, 3, 0.7),             # two slices, the second with one row; columns shorter than a quad
    (1, 5, 1.0),              # a single row
])
def test_sparse_full_gap_pass_from_the_blocked_copy(G, n, d, density):
    """The full gap pass over CSR data runs from the library's range-blocked, sliced copy of the
    matrix; at every density it must give the oracle's gaps (App. E), and the same values as the
    plain CSR kernel that serves short index lists."""
    from paper_1708_05357_amd import duhl, synth
    prob = synth.svm_csr(n, d, density, seed=11)
    p = G.Pair(prob)
    rng = np.random.default_rng(1)
    for rnd in range(2):
        p.g.select(max(1, n // 3))
        p.g.commit_swap()
        p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(rng.permutation(p.g.get(duhl.P)).astype(np.int32)))
    p.sync_oracle_to_gpu_state()
    total = p.g.gap()                                        # blocked copy
    z_blocked = p.g.get(duhl.Z)
    assert total == pytest.approx(p.o.gaps(), rel=1e-4)
    floor = G.gap_floor(p, partials=1)
    G.assert_gaps_close(z_blocked, p.o.z, floor=floor, label=f"svm csr blocked {n}x{d}")
    assert total == pytest.approx(float(z_blocked.astype(np.float64).sum()), rel=1e-9)
    p.g.set(duhl.Z, np.full(n, -1.0, dtype=np.float32))
    p.g.gap(G.dev_i32(np.arange(n)), want_sum=False)         # index list: plain CSR kernel
    z_plain = p.g.get(duhl.Z)
    G.assert_gaps_close(z_plain, p.o.z, floor=floor, label=f"svm csr plain {n}x{d}")
    assert np.all(np.abs(z_blocked.astype(np.float64) - z_plain) <= 1e-4 * z_plain + 2 * floor)
    p.close()


@pytest.mark.parametrize("n,d,density", [
    (3000, 400, 0.02),        # ~8 non-zeros per row
    (2000, 50000, 0.002),     # two ranges, ~50 per row and range
    (1200, 3000, 0.1),        # ~300 per row
    (700, 2000, 0.3),         # ~600 per row
])
def test_sparse_index_lists_from_the_blocked_copy(G, monkeypatch, n, d, density):
    """Long index lists over CSR data are evaluated from the range-blocked copy too -- the dot
    products of all rows, then the gap formula for the listed ones (the threshold is lowered here
    so that short lists take that path): listed coordinates get the
    oracle's gaps (App. E), coordinates not listed keep their old entry, entries that name no
    coordinate are skipped, and the sum is that of the listed gaps."""
    from paper_1708_05357_amd import duhl, synth
    monkeypatch.setenv("DUHL_CSR_BLOCKED_LIST_MIN", "1")
    prob = synth.svm_csr(n, d, density, seed=12)
    p = G.Pair(prob)
    rng = np.random.default_rng(2)
    p.g.select(n // 3)
    p.g.commit_swap()
    p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(rng.permutation(p.g.get(duhl.P)).astype(np.int32)))
    p.sync_oracle_to_gpu_state()
    p.o.gaps()
    for count in (1, 37, n // 2, n - 1):
        listed = rng.permutation(n)[:count].astype(np.int32)
        with_bad = listed.copy()
        if count >= 37:
            with_bad[5], with_bad[count - 1] = -3, n           # skipped; their rows drop out
            listed = np.delete(listed, [5, count - 1])
        p.g.set(duhl.Z, np.full(n, -1.0, dtype=np.float32))
        total = p.g.gap(G.dev_i32(with_bad))
        z = p.g.get(duhl.Z)
        rest = np.ones(n, dtype=bool)
        rest[listed] = False
        assert (z[rest] == -1.0).all()
        G.assert_gaps_close(z[listed], p.o.z[listed], floor=G.gap_floor(p, idx=listed, partials=1),
                            label=f"svm csr blocked list {n}x{d}")
        assert total == pytest.approx(float(z[listed].astype(np.float64).sum()), rel=1e-9)
    p.close()


def uneven_csr(n, d, short, long_rows, long_len, seed):
    """SVM instance whose rows have `short` non-zeros except `long_rows` of them, which have
    `long_len`; unit rows, labels from a random separator."""
    rng = np.random.default_rng(seed)
    counts = np.full(n, short, dtype=np.int64)
    counts[rng.choice(n, size=long_rows, replace=False)] = long_len
    rowptr = np.zeros(n + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(counts)
    colidx = np.concatenate([np.sort(rng.choice(d, size=k, replace=False)) for k in counts]).astype(np.int32)
    val = rng.uniform(0.1, 1.0, size=colidx.size).astype(np.float32)
    rows = np.repeat(np.arange(n), counts)
    val /= np.sqrt(np.bincount(rows, weights=val.astype(np.float64) ** 2, minlength=n))[rows].astype(np.float32)
    w = rng.standard_normal(d)
    y = np.where(np.bincount(rows, weights=val * w[colidx], minlength=n) >= 0, 1.0, -1.0).astype(np.float32)
    t = torch.from_numpy
    return {"model": "svm", "d": d, "n": n, "rowptr": t(rowptr), "colidx": t(colidx), "val": t(val),
            "target": t(y), "lam": 1.0 / n}


@pytest.mark.parametrize("n,d,short,long_rows,long_len", [
    (3000, 5000, 5, 5, 3000),       # a few rows 600 times longer: slices would be padding, plain pass
    (5000, 40000, 8, 700, 400),     # a seventh of the rows 50 times longer: sorted into slices of their own
    (1100, 70000, 3, 64, 20000),    # three ranges, one slice's worth of very long rows
])
def test_sparse_rows_of_uneven_length(G, n, d, short, long_rows, long_len):
    """The sliced copy of a sparse matrix pads every 64 rows to the longest of them (after
    sorting 1,024 at a time); with rows of very different length it is either still compact or
    not built at all, and the gaps (App. E) are the oracle's either way."""
    from paper_1708_05357_amd import duhl
    prob = uneven_csr(n, d, short, long_rows, long_len, seed=21)
    p = G.Pair(prob)
    rng = np.random.default_rng(3)
    assert p.g.gap() == pytest.approx(1.0, rel=1e-6)         # every z_i = 1/n at alpha = 0
    p.g.select(n // 4)
    p.g.commit_swap()
    p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(rng.permutation(p.g.get(duhl.P)).astype(np.int32)))
    p.sync_oracle_to_gpu_state()
    total = p.g.gap()
    assert total == pytest.approx(p.o.gaps(), rel=1e-4)
    G.assert_gaps_close(p.g.get(duhl.Z), p.o.z, floor=G.gap_floor(p, partials=1), label=f"svm csr uneven rows {n}x{d}")
    p.close()


def sparse_regression(n, d, density, model, eta, seed):
    """Lasso / elastic-net instance with sparse columns, as CSR over coordinates: unit columns with
    ~density*d non-zeros, b = A alpha* + noise for a sparse alpha*, lambda d = 0.1 ||A^T b||_inf."""
    from paper_1708_05357_amd import synth
    base = synth.svm_csr(n, d, density, seed=seed)           # the sparsity pattern and unit rows
    rng = np.random.default_rng(seed)
    rowptr, colidx = base["rowptr"].numpy(), base["colidx"].numpy()
    val = (base["val"].numpy() * rng.choice([-1.0, 1.0], size=colidx.size)).astype(np.float32)
    rows = np.repeat(np.arange(n), np.diff(rowptr))
    alpha = np.where(rng.random(n) < 0.1, rng.standard_normal(n), 0.0)
    b = np.bincount(colidx, weights=val * alpha[rows], minlength=d) + 0.01 * rng.standard_normal(d)
    b = b.astype(np.float32)
    corr = np.abs(np.bincount(rows, weights=val.astype(np.float64) * b[colidx], minlength=n)).max()
    t = torch.from_numpy
    return {"model": model, "eta": eta, "d": d, "n": n, "rowptr": t(rowptr), "colidx": t(colidx),
            "val": t(val), "target": t(b), "lam": 0.1 * corr / d}


@pytest.mark.parametrize("model,eta", [("lasso", 1.0), ("enet", 0.4)])
def test_sparse_lasso_and_elastic_net(G, model, eta):
    """The regression models on CSR data (rows = coordinates = sparse columns of A): gaps of the
    full pass and of a list (App. E, eq. (4)), sequential iterates (App. D), and the objective the
    concurrent scheme reaches, against the oracle."""
    from paper_1708_05357_amd import duhl
    n, d, m = 2500, 40000, 500
    prob = sparse_regression(n, d, 0.002, model, eta, seed=17)
    p = G.Pair(prob)
    np.testing.assert_allclose(p.g.get(duhl.SQNORM), p.o.q, rtol=2e-6)
    assert p.g.gap() == pytest.approx(p.o.gaps(), rel=1e-4)
    G.assert_gaps_close(p.g.get(duhl.Z), p.o.z, label=f"sparse {model} at alpha=0")           # the bare rule
    rng = np.random.default_rng(5)
    for rnd in range(4):
        p.g.gap(want_sum=False)
        p.g.select(m, want_stats=False)
        p.g.commit_swap()
        order = rng.permutation(p.g.get(duhl.P)).astype(np.int32)
        p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(order))
        p.o.cd_pass(order)
        a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
        assert np.abs(a - p.o.alpha).max() <= 1e-5 * np.abs(p.o.alpha).max()
        assert np.abs(v - p.o.v).max() <= 1e-5 * np.abs(p.o.v).max()
        p.sync_oracle_to_gpu_state()
        total_gpu, total_or = p.g.gap(), p.o.gaps()
        floor = G.gap_floor(p, partials=1)
        assert total_gpu == pytest.approx(total_or, rel=1e-4, abs=float(floor.sum()))
        G.assert_gaps_close(p.g.get(duhl.Z), p.o.z, floor=floor, label=f"sparse {model} round {rnd + 1}")
        listed = rng.permutation(n)[:n // 5].astype(np.int32)
        p.g.set(duhl.Z, np.zeros(n, dtype=np.float32))
        p.g.gap(G.dev_i32(listed), want_sum=False)
        G.assert_gaps_close(p.g.get(duhl.Z)[listed], p.o.z[listed], floor=floor[listed],
                            label=f"sparse {model} list round {rnd + 1}")
    # concurrent scheme: rounds until both have converged, then the objectives agree
    for rnd in range(150):
        p.g.gap(want_sum=False)
        p.g.select(m, want_stats=False)
        p.g.commit_swap()
        p.g.cd_epoch(duhl.CD_ASYNC, seed=rnd)
    rng2 = np.random.default_rng(0)
    for rnd in range(150):
        p.o.round(m, passes=1, rng=rng2)
    og, oo = p.g.objective(), p.o.objective()
    assert abs(og - oo) <= 1e-5 * abs(oo), (og, oo)
    p.close()


@pytest.mark.parametrize("eta", [1.0, 0.3])
def test_elastic_net_gaps_steps_and_objective_match_oracle(G, eta):
    """App. D elastic-net step and the gap of eq. (4) (ridge gap of App. E for eta = 1): gap vectors,
    sequential iterates and the concurrent schemes' objective, on ragged shapes."""
    from paper_1708_05357_amd import duhl
    prob = lasso_problem(1503, 260, 0.1, 0.02, seed=41)
    prob["model"], prob["eta"] = "enet", eta
    p = G.Pair(prob)
    m = 80
    rng = np.random.default_rng(4)
    assert p.g.gap() == pytest.approx(p.o.gaps(), rel=1e-4)
    G.assert_gaps_close(p.g.get(duhl.Z), p.o.z, label=f"enet eta={eta} at alpha=0")                # the bare rule
    for rnd in range(6):
        p.g.gap(want_sum=False)
        p.g.select(m, want_stats=False)
        p.g.commit_swap()
        order = rng.permutation(p.g.get(duhl.P)).astype(np.int32)
        p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(order))
        p.o.cd_pass(order)
        a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
        assert np.abs(a - p.o.alpha).max() <= 1e-5 * np.abs(p.o.alpha).max()
        assert np.abs(v - p.o.v).max() <= 1e-5 * np.abs(p.o.v).max()
        p.sync_oracle_to_gpu_state()
        total = p.g.gap()
        total_or = p.o.gaps()
        floor = G.gap_floor(p)
        assert total == pytest.approx(total_or, rel=1e-4, abs=float(floor.sum()))
        G.assert_gaps_close(p.g.get(duhl.Z), p.o.z, floor=floor, label=f"enet eta={eta} round {rnd + 1}")
        assert p.g.objective() == pytest.approx(p.o.objective(), rel=1e-6)
        p.o.set_state(a.astype(np.float64))            # back to the oracle's own v
    for mode in (duhl.CD_ASYNC, duhl.CD_ATOMIC):
        p.g.set(duhl.ALPHA, np.zeros(prob["n"], dtype=np.float32))
        p.g.recompute_v()
        p.o.set_state(np.zeros(prob["n"]))
        converge_async(G, p, m, 150, 2, 1e-9, mode)
        converge_oracle(p, m, 150, 2, 1e-11)
        assert abs(p.g.objective() - p.o.objective()) <= 1e-5 * abs(p.o.objective())
    p.close()


# ------------------------------------------------------------------------------------ selection
@pytest.mark.parametrize("n", [7, 500, 2048, 2049, 70001])
def test_selection_is_bit_exact_on_the_same_z(G, n):
    """eq. (13): same fp32 z into both selectors -> identical sets (ascending), incl. heavy ties,
    m = 1, m = n, the threshold (the m-th largest entry) and rho of eq. (7)."""
    from oracle import duhl_oracle as orc
    from paper_1708_05357_amd import duhl
    p = G.Pair(lasso_problem(16, n, 0.1, 0.1, seed=n))
    rng = np.random.default_rng(n)
    cases = {
        "random": rng.random(n).astype(np.float32) ** 4,
        "many zeros": np.where(rng.random(n) < 0.9, 0.0, rng.random(n)).astype(np.float32),
        "all equal": np.full(n, 1.0 / n, dtype=np.float32),
        "few levels": rng.integers(0, 4, n).astype(np.float32),
        "tiny spread": (1.0 + rng.integers(0, 3, n) * 2.0 ** -23).astype(np.float32),
    }
    for name, z in cases.items():
        p.g.set(duhl.Z, z)
        for m in sorted({1, 2, max(1, n // 10), max(1, n // 2), n - 1 if n > 1 else 1, n}):
            out = torch.full((m,), -7, dtype=torch.int32, device="cuda:0")
            nsw, rho = p.g.select(m, out)
            want = orc.select_topm(z.astype(np.float64), m)
            np.testing.assert_array_equal(out.cpu().numpy(), want, err_msg=f"{name} m={m}")
            assert p.g.selection_threshold() == np.sort(z)[n - m], (name, m)   # the m-th largest, exactly
            if z.sum() > 0:
                assert rho == pytest.approx(orc.rho(z.astype(np.float64), want), rel=1e-12), (name, m)
            else:
                assert rho == 1.0               # all gaps zero: the ratio of eq. (7) is 0/0
            p.g.commit_swap()
            np.testing.assert_array_equal(p.g.get(duhl.P), want)
    p.close()


def test_selection_counts_new_columns(G):
    from paper_1708_05357_amd import duhl
    n = 3000
    p = G.Pair(lasso_problem(8, n, 0.1, 0.1, seed=1))
    z = np.zeros(n, dtype=np.float32)
    z[:100] = 1.0
    p.g.set(duhl.Z, z)
    assert p.g.select(100)[0] == 100
    p.g.commit_swap()
    z[:] = 0
    z[50:150] = 1.0
    p.g.set(duhl.Z, z)
    assert p.g.select(100)[0] == 50
    p.close()


# ------------------------------------------------------------------------------------ sequential CD
def run_rounds_sequential(G, p, m, rounds, seed=0, check_selection=True):
    """The loop of Alg. 1 with rule (11) on both sides: fresh gaps, top-m, one pass in a random
    order that is passed to both as data.  The oracle follows the GPU's working set after it has
    been checked against its own choice outside the tie band."""
    from paper_1708_05357_amd import duhl
    rng = np.random.default_rng(seed)
    worst_a = worst_v = 0.0
    for rnd in range(rounds):
        p.g.gap(want_sum=False)
        p.g.select(m, want_stats=False)
        p.g.commit_swap()
        P = p.g.get(duhl.P)
        if check_selection:
            p.o.gaps()
            Po = p.o.select(m)
            if not np.array_equal(P, Po):
                thr = np.sort(p.o.z)[-m]
                # tie band: the 1e-4 relative agreement of the gaps plus their fp32 rounding floor
                band = 1e-4 * p.o.z.max() + (G.lasso_gap_floor(p) if p.model == duhl.LASSO else 1e-7 / p.o.n)
                diff = np.setxor1d(P, Po)
                assert np.all(np.abs(p.o.z[diff] - thr) <= band), (rnd, diff, p.o.z[diff], thr)
        order = rng.permutation(P).astype(np.int32)
        p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(order))
        p.o.cd_pass(order)
        a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
        ea = np.abs(a - p.o.alpha).max() / max(np.abs(p.o.alpha).max(), 1e-30)
        ev = np.abs(v - p.o.v).max() / max(np.abs(p.o.v).max(), 1e-30)
        worst_a, worst_v = max(worst_a, ea), max(worst_v, ev)
        assert ea <= 1e-5 and ev <= 1e-5, (rnd, ea, ev)
    return worst_a, worst_v


def test_sequential_cd_iterates_match_oracle_cfg1(G):
    """Tiny dense Lasso of the benchmark plan: 1000 x 500, m = 125, 20 rounds of one pass."""
    from paper_1708_05357_amd import duhl, synth
    prob = synth.make("cfg1")
    p = G.Pair(prob)
    wa, wv = run_rounds_sequential(G, p, prob["m"], prob["rounds"])
    print("cfg1 worst relative deviation alpha %.2e v %.2e" % (wa, wv))
    assert np.count_nonzero(p.g.get(duhl.ALPHA)) > 10          # the regulariser leaves a support
    assert p.g.objective() == pytest.approx(p.o.objective(), rel=1e-6)
    p.close()


@pytest.mark.parametrize("kind", ["lasso_ragged", "lasso_padded", "svm_dense", "svm_csr"])
def test_sequential_cd_iterates_match_oracle_other_shapes(G, kind):
    from paper_1708_05357_amd import synth
    if kind == "lasso_ragged":
        p = G.Pair(lasso_problem(4099, 300, 0.1, 0.1, seed=5))
        m = 90
    elif kind == "lasso_padded":
        p = G.Pair(lasso_problem(515, 200, 0.1, 0.1, seed=6), ld=519)
        m = 77
    elif kind == "svm_dense":
        p = G.Pair(synth.svm_dense(600, 50, seed=7))
        m = 150
    else:
        p = G.Pair(synth.svm_csr(2000, 300, 0.03, seed=8))
        m = 500
    run_rounds_sequential(G, p, m, 8, seed=3)
    assert p.g.objective() == pytest.approx(p.o.objective(), rel=1e-6)
    p.close()


def test_sequential_default_order_is_ascending(G):
    from paper_1708_05357_amd import duhl
    p = G.Pair(lasso_problem(200, 60, 0.2, 0.1, seed=9))
    p.g.select(20)
    p.g.commit_swap()
    P = p.g.get(duhl.P)
    p.g.cd_epoch(duhl.CD_SEQUENTIAL)
    p.o.cd_pass(P)
    np.testing.assert_allclose(p.g.get(duhl.ALPHA), p.o.alpha, rtol=1e-5, atol=1e-7)
    p.close()


# ------------------------------------------------------------------------------------ asynchronous CD
def converge_async(G, p, m, max_rounds, passes, target_rel_gap, mode=None):
    from paper_1708_05357_amd import duhl
    mode = duhl.CD_ASYNC if mode is None else mode
    o0 = p.g.objective()
    for rnd in range(max_rounds):
        gap = p.g.gap()
        if gap <= target_rel_gap * abs(o0):
            break
        p.g.select(m, want_stats=False)
        p.g.commit_swap()
        for k in range(passes):
            p.g.cd_epoch(mode, seed=rnd * 131 + k)
    return rnd


def converge_oracle(p, m, max_rounds, passes, target_rel_gap):
    o0 = p.o.objective()
    rng = np.random.default_rng(0)
    for rnd in range(max_rounds):
        if p.o.gaps() <= target_rel_gap * abs(o0):
            break
        P = p.o.select(m)
        for k in range(passes):
            p.o.cd_pass(P[rng.permutation(P.size)])
    return rnd


@pytest.mark.parametrize("scheme", ["async", "atomic"])
@pytest.mark.parametrize("kind", ["cfg1", "lasso_mid", "lasso_ragged", "lasso_long", "lasso_longer",
                                  "lasso_longest", "lasso_extended", "lasso_eight_units", "lasso_unaligned",
                                  "lasso_long_unaligned", "svm_dense", "svm_csr", "svm_csr_long_rows"])
def test_async_cd_reaches_the_oracle_objective(G, kind, scheme):
    """The asynchronous scheme is compared on what is unique: the objective at convergence
    (1e-5 relative), and on the invariant v = A alpha (- b) that the atomic adds must keep."""
    from paper_1708_05357_amd import duhl, synth
    if kind == "cfg1":
        prob = synth.make("cfg1")
        m = prob["m"]
    elif kind == "lasso_mid":
        prob = lasso_problem(5000, 3000, 0.03, 0.05, seed=11)
        m = 300
    elif kind == "lasso_ragged":
        prob = lasso_problem(14003, 700, 0.05, 0.05, seed=14)       # 1024-thread workers, tail rows
        m = 200
    elif kind == "lasso_long":
        prob = lasso_problem(50002, 300, 0.05, 0.05, seed=15)       # private v in registers + LDS
        m = 120
    elif kind == "lasso_longer":
        prob = lasso_problem(75001, 260, 0.05, 0.05, seed=16)       # column re-read on update
        m = 100
    elif kind == "lasso_longest":
        prob = lasso_problem(100003, 220, 0.05, 0.05, seed=17)      # largest register/LDS split
        m = 90
    elif kind == "lasso_extended":
        prob = lasso_problem(150002, 160, 0.05, 0.05, seed=18)      # part of the private v in device memory
        m = 70
    elif kind == "lasso_eight_units":
        prob = lasso_problem(300004, 96, 0.05, 0.05, seed=20)       # eight compute units per worker
        m = 40
    elif kind == "lasso_unaligned":
        prob = lasso_problem(50002, 300, 0.05, 0.05, seed=15)       # leading dimension = d: scalar kernels
        m = 120
    elif kind == "lasso_long_unaligned":
        prob = lasso_problem(90001, 200, 0.05, 0.05, seed=19)       # two units per worker, dword loads
        m = 90
    elif kind == "svm_dense":
        prob = synth.svm_dense(2000, 300, seed=12)
        m = 500
    elif kind == "svm_csr_long_rows":
        prob = synth.svm_csr(3000, 6000, 0.06, seed=21)             # ~360 non-zeros per row: a wavefront per row
        m = 600
    else:
        prob = synth.svm_csr(20000, 2000, 0.01, seed=13)
        m = 4000
    # columns padded to a multiple of four floats take the 16-byte kernels (with a ragged tail when
    # d itself is not a multiple of four); "lasso_unaligned" keeps ld = d and the scalar ones
    ld = None
    if "cols" in prob and "unaligned" not in kind and prob["d"] % 4 != 0:
        ld = (prob["d"] + 3) // 4 * 4
    p = G.Pair(prob, ld=ld)
    tol = 1e-7 if prob["model"] == "lasso" else 1e-6
    mode = duhl.CD_ASYNC if scheme == "async" else duhl.CD_ATOMIC
    r_gpu = converge_async(G, p, m, 400, 3, tol, mode)
    r_or = converge_oracle(p, m, 400, 3, tol)
    og, oo = p.g.objective(), p.o.objective()
    print(f"{kind}: rounds gpu {r_gpu} oracle {r_or} objective gpu {og:.9e} oracle {oo:.9e}")
    assert abs(og - oo) <= 1e-5 * abs(oo)
    # the shared vector still is what its definition says (App. D), up to fp32 accumulation
    a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
    p.o.set_state(a.astype(np.float64))
    scale = max(np.abs(p.o.v).max(), np.abs(G.to_np(prob["target"])).max() if prob["model"] == "lasso" else 1.0)
    assert np.abs(v - p.o.v).max() <= 2e-4 * scale
    p.g.recompute_v()
    np.testing.assert_allclose(p.g.get(duhl.V), p.o.v, rtol=0, atol=G.v_accumulation_floor(p, a))
    p.close()


# ------------------------------------------------------------------------------------ host residency
def test_resident_columns_counts_device_slots(G):
    """Host residency: the slots in use are the working set after the first commit, and never
    more than the budget; device residency: every column."""
    from paper_1708_05357_amd import duhl
    prob = lasso_problem(600, 90, 0.1, 0.05, seed=61)
    p = G.Pair(prob)
    assert p.g.resident_columns() == 90
    p.close()
    p = G.Pair(prob, budget=40, host_resident=True)
    assert p.g.resident_columns() == 0
    p.g.select(20)
    p.g.commit_swap()
    assert p.g.resident_columns() == 20
    for rnd in range(3):
        p.g.cd_epoch(duhl.CD_ASYNC, seed=rnd)
        p.g.gap(want_sum=False)
        p.g.select(20)
        p.g.commit_swap()
        assert 20 <= p.g.resident_columns() <= 40
    p.close()


def test_host_resident_swap_matches_oracle(G):
    """Alg. 2 with the matrix in pinned host memory and fewer device slots than columns: the
    copies run on the side stream while the previous set is being worked on; iterates must still
    match the oracle, and the slots must hold the selected columns."""
    from paper_1708_05357_amd import duhl
    run_host_resident(G, lasso_problem(1028, 400, 0.1, 0.1, seed=21), 60)


def test_host_resident_swap_long_columns(G):
    """The same with the column length of the out-of-budget workload (d = 100,000): slots with a
    padded leading dimension, the longest register/LDS split of the workers."""
    run_host_resident(G, lasso_problem(100000, 160, 0.1, 0.1, seed=22), 30, rounds=4)


def test_host_resident_matrix_in_pieces(G):
    """The host matrix handed over as separately pinned pieces (a short last one; padded leading
    dimension): same iterates, slots and gaps as from one allocation."""
    prob = lasso_problem(1028, 400, 0.1, 0.1, seed=23)
    run_host_resident(G, prob, 60, rounds=6, chunk_cols=130, ld=1040)
    run_host_resident(G, prob, 60, rounds=3, chunk_cols=1)        # a piece per column
    run_host_resident(G, prob, 60, rounds=3, chunk_cols=400)      # one piece through the table


@pytest.mark.parametrize("d,n,m,ld,stage_mb", [(1028, 400, 60, None, None), (1027, 400, 60, 1031, None),
                                                (100000, 160, 30, None, None), (5000, 900, 200, None, 1),
                                                (300, 6000, 600, None, 1)])
def test_pageable_host_matrix_through_staging_buffers(G, monkeypatch, d, n, m, ld, stage_mb):
    """The host matrix in ordinary memory that the device cannot read (Assumption 1 of Sec. 3 on a
    machine that cannot pin everything): the first pass, index-list gap passes and the column swap of
    Alg. 2 go through the library's pinned staging buffers, a background thread doing the swap.  Same
    iterates, slots and gaps as with pinned memory; ragged and padded columns; staging buffers of
    1 MB, so that a pass takes many batches and the buffers are reused.  The last case has enough
    columns (more than 2,048) for the first pass to leave those with the largest gaps in the device
    slots: the first working set then finds part of its columns there, and every later read of
    them -- gaps of the residents, the passes -- must see the right data."""
    if stage_mb is not None:
        monkeypatch.setenv("DUHL_STAGE_MB", str(stage_mb))
    run_host_resident(G, lasso_problem(d, n, 0.1, 0.1, seed=24), m, rounds=4, ld=ld, pageable=True)


def test_first_pass_keeping_can_be_switched_off(G, monkeypatch):
    """DUHL_KEEP_FIRST_PASS=0: the first pass over a staged matrix leaves the slots empty and the first
    working set crosses the link whole; the rounds are the same."""
    monkeypatch.setenv("DUHL_STAGE_MB", "1")
    monkeypatch.setenv("DUHL_KEEP_FIRST_PASS", "0")
    from paper_1708_05357_amd import duhl
    prob = lasso_problem(300, 6000, 0.1, 0.1, seed=24)
    p = G.Pair(prob, budget=1200, host_resident=True, pageable=True)
    assert p.g.resident_columns() == 0
    nsw, rho = p.g.select(600)
    assert nsw == 600
    p.g.commit_swap()
    p.close()


def run_host_resident(G, prob, m, rounds=10, chunk_cols=None, ld=None, pageable=False):
    from paper_1708_05357_amd import duhl
    for budget in (2 * m, m + 7):                  # overlapping copies / in-place replacement
        p = G.Pair(prob, budget=budget, host_resident=True, chunk_cols=chunk_cols, ld=ld, pageable=pageable)
        np.testing.assert_allclose(p.g.get(duhl.SQNORM), p.o.q, rtol=2e-6)
        p.o.gaps()
        G.assert_gaps_close(p.g.get(duhl.Z), p.o.z)
        rng = np.random.default_rng(2)
        all_idx = G.dev_i32(np.arange(prob["n"]))
        kept = p.g.resident_columns()              # (pageable memory: what the first pass left in the slots)
        assert 0 <= kept <= budget and (kept == 0 or (pageable and prob["n"] > 2048))
        nsw, rho = p.g.select(m)
        assert m - kept <= nsw <= m
        if pageable and prob["n"] > 2048:
            assert kept > 0 and nsw < m
        p.g.commit_swap()
        for rnd in range(rounds):
            P = p.g.get(duhl.P)
            order = rng.permutation(P).astype(np.int32)
            if budget >= 2 * m:
                # time-delayed scheme: choose the next set from the gaps before this pass,
                # copy while the pass runs, then switch
                p.g.gap(all_idx, want_sum=False)
                nsw, rho = p.g.select(m)
                p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(order))
                p.g.commit_swap()
            else:
                p.g.cd_epoch(duhl.CD_SEQUENTIAL, G.dev_i32(order))
                p.g.gap(all_idx, want_sum=False)
                nsw, rho = p.g.select(m)
                with pytest.raises(duhl.DuhlError):
                    p.g.cd_epoch(duhl.CD_SEQUENTIAL)       # slots are being overwritten
                p.g.commit_swap()
            p.o.cd_pass(order)
            a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
            assert np.abs(a - p.o.alpha).max() <= 1e-5 * np.abs(p.o.alpha).max()
            assert np.abs(v - p.o.v).max() <= 1e-5 * np.abs(p.o.v).max()
            Pn = p.g.get(duhl.P)
            fresh = np.setdiff1d(Pn, P).size       # spare slots may still hold some of them
            assert fresh - (budget - m) <= nsw <= fresh
            assert 1.0 - 1e-9 <= rho <= prob["n"] / m + 1e-9
        # gaps of the resident columns (idx = NULL) equal the oracle's at the same state
        p.sync_oracle_to_gpu_state()
        p.o.gaps()
        p.g.set(duhl.Z, np.full(prob["n"], -1.0, dtype=np.float32))
        p.g.gap(want_sum=False)
        z = p.g.get(duhl.Z)
        Pn = p.g.get(duhl.P)
        assert np.all(z[Pn] >= 0)
        G.assert_gaps_close(z[Pn], p.o.z[Pn], floor=G.gap_floor(p, idx=Pn), label="host-resident lasso, residents")
        assert np.count_nonzero(z >= 0) <= budget
        # the concurrent schemes read the working set from the slots too: the objective must not
        # rise and v must stay A alpha - b (App. D)
        for mode in (duhl.CD_ASYNC, duhl.CD_ATOMIC):
            before = p.g.objective()
            p.g.cd_epoch(mode, seed=5)
            assert p.g.objective() <= before * (1 + 1e-6) + 1e-12
            a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
            p.o.set_state(a.astype(np.float64))
            assert np.abs(v - p.o.v).max() <= 1e-4 * max(np.abs(p.o.v).max(), np.abs(G.to_np(prob["target"])).max())
        p.close()


# ------------------------------------------------------------------------------------ API behaviour
def test_error_paths(G):
    from paper_1708_05357_amd import duhl
    dev = "cuda:0"
    g = duhl.Duhl(duhl.LASSO, 8, 6, 3)
    with pytest.raises(duhl.DuhlError) as e:
        g.gap()
    assert e.value.status == duhl.ESTATE
    cols = torch.randn(6, 8, device=dev)
    b = torch.randn(8, device=dev)
    for lam in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(duhl.DuhlError) as e:
            g.set_data_dense(cols, b, lam)
        assert e.value.status == duhl.EINVAL
    with pytest.raises(duhl.DuhlError) as e:
        g.set_data_dense(cols, torch.full((8,), float("nan"), device=dev), 0.1)
    assert e.value.status == duhl.EINVAL
    for bad in (float("nan"), float("inf")):                      # a non-finite entry of the matrix
        spoiled = cols.clone()
        spoiled[4, 3] = bad
        with pytest.raises(duhl.DuhlError) as e:
            g.set_data_dense(spoiled, b, 0.1)
        assert e.value.status == duhl.EINVAL
        with pytest.raises(duhl.DuhlError) as e:
            g.gap()
        assert e.value.status == duhl.ESTATE
    g.set_data_dense(cols, b, 0.1)
    with pytest.raises(duhl.DuhlError) as e:
        g.cd_epoch()
    assert e.value.status == duhl.ESTATE
    with pytest.raises(duhl.DuhlError) as e:
        g.select(4)
    assert e.value.status == duhl.EBUDGET
    with pytest.raises(duhl.DuhlError) as e:
        g.select(0)
    assert e.value.status == duhl.EINVAL
    with pytest.raises(duhl.DuhlError) as e:
        g.commit_swap()
    assert e.value.status == duhl.ESTATE
    with pytest.raises(duhl.DuhlError) as e:
        g.selection_threshold()
    assert e.value.status == duhl.ESTATE
    g.select(3)
    g.commit_swap()
    g.cd_epoch()
    # a host matrix in pieces: the counts must fit n, and every piece must be readable by the device
    import ctypes as C
    pieces = [torch.randn(4, 8).pin_memory(), torch.randn(2, 8).pin_memory()]
    ptrs = (C.c_void_p * 2)(*[t.data_ptr() for t in pieces])
    bp = C.c_void_p(b.data_ptr())
    for n_chunks, per in ((3, 3), (2, 2), (1, 4), (2, 0), (0, 6)):
        assert g.lib.duhl_set_data_dense_chunks(g._h, ptrs, n_chunks, per, 8, bp, 0.1) == duhl.EINVAL
    assert g.lib.duhl_set_data_dense_chunks(g._h, None, 2, 4, 8, bp, 0.1) == duhl.EINVAL
    assert g.lib.duhl_set_data_dense_chunks(g._h, ptrs, 2, 4, 7, bp, 0.1) == duhl.EINVAL       # ld < d
    null_piece = (C.c_void_p * 2)(pieces[0].data_ptr(), None)
    assert g.lib.duhl_set_data_dense_chunks(g._h, null_piece, 2, 4, 8, bp, 0.1) == duhl.EINVAL
    pageable = torch.randn(2, 8)
    not_pinned = (C.c_void_p * 2)(pieces[0].data_ptr(), pageable.data_ptr())
    assert g.lib.duhl_set_data_dense_chunks(g._h, not_pinned, 2, 4, 8, bp, 0.1) == duhl.EINVAL
    with pytest.raises(duhl.DuhlError) as e:
        g.gap()                                                  # the failed call left no data behind
    assert e.value.status == duhl.ESTATE
    g.set_data_dense_chunks(pieces, b, 0.1)
    assert g.gap() >= 0.0
    g.close()
    with pytest.raises(duhl.DuhlError) as e:
        duhl.Duhl(duhl.LASSO, 8, 6, 3).set_eta(0.5)              # eta belongs to the elastic net
    assert e.value.status == duhl.EINVAL
    en = duhl.Duhl(duhl.ELASTIC_NET, 8, 6, 3)
    for bad in (0.0, -0.1, 1.5, float("nan")):
        with pytest.raises(duhl.DuhlError) as e:
            en.set_eta(bad)
        assert e.value.status == duhl.EINVAL
    en.set_eta(0.25)
    en.close()
    s = duhl.Duhl(duhl.SVM, 8, 6, 6)
    with pytest.raises(duhl.DuhlError) as e:
        s.set_data_dense(cols, torch.tensor([1, -1, 1, 0.5, 1, -1.0], device=dev), 0.1)
    assert e.value.status == duhl.EINVAL
    rowptr = torch.tensor([0, 2, 2, 3, 3, 3, 4], dtype=torch.int64, device=dev)
    val = torch.ones(4, device=dev)
    y = torch.tensor([1, -1, 1, 1, 1, -1.0], device=dev)
    for bad in ([1, 0, 2, 3], [0, 8, 2, 3], [0, 0, 2, 3]):
        with pytest.raises(duhl.DuhlError) as e:
            s.set_data_csr(rowptr, torch.tensor(bad, dtype=torch.int32, device=dev), val, y, 0.1)
        assert e.value.status == duhl.EINVAL
    bad_ptr = torch.tensor([0, 2, 1, 3, 3, 3, 4], dtype=torch.int64, device=dev)
    with pytest.raises(duhl.DuhlError) as e:
        s.set_data_csr(bad_ptr, torch.tensor([0, 1, 2, 3], dtype=torch.int32, device=dev), val, y, 0.1)
    assert e.value.status == duhl.EINVAL
    # a rowptr that is locally fine but points outside the nnz = rowptr[n] entries of colidx / val must
    # be refused before any row is walked: negative, far above nnz (increasing from there), decreasing
    good_idx = torch.tensor([0, 1, 2, 3], dtype=torch.int32, device=dev)
    for ptr in ([0, -2, 2, 3, 3, 3, 4], [0, 10 ** 12, 10 ** 12 + 5, 10 ** 12 + 6, 10 ** 12 + 6, 10 ** 12 + 7, 4],
                [0, 2, 5, 5, 5, 5, 4], [0, 4, 3, 2, 1, 0, 4], [1, 2, 2, 3, 3, 3, 4]):
        with pytest.raises(duhl.DuhlError) as e:
            s.set_data_csr(torch.tensor(ptr, dtype=torch.int64, device=dev), good_idx, val, y, 0.1)
        assert e.value.status == duhl.EINVAL, ptr
        with pytest.raises(duhl.DuhlError) as e:
            s.gap()                                              # the failed call left no data behind
        assert e.value.status == duhl.ESTATE
    s.set_data_csr(rowptr, good_idx, val, y, 0.1)
    assert s.gap() == pytest.approx(1.0)
    s.close()


def test_list_entries_outside_the_problem_are_skipped(G):
    """Index lists come from the caller: entries that name no coordinate must neither be read
    through nor change anything, in every kernel that takes a list."""
    from paper_1708_05357_amd import duhl
    from paper_1708_05357_amd import synth
    prob = lasso_problem(300, 40, 0.2, 0.1, seed=31)
    csr = synth.svm_csr(60, 30, 0.2, seed=32)
    for pr in (prob, csr):
        p = G.Pair(pr)
        n = pr["n"]
        m = 12
        p.g.select(m)
        p.g.commit_swap()
        P = p.g.get(duhl.P)
        good = P[:6].astype(np.int32)
        mixed = np.array([good[0], -1, good[1], n, good[2], 2 ** 31 - 1, good[3], -2 ** 31, good[4], good[5]],
                         dtype=np.int32)
        for mode in (duhl.CD_SEQUENTIAL, duhl.CD_ASYNC, duhl.CD_ATOMIC):
            p.g.set(duhl.ALPHA, np.zeros(n, dtype=np.float32))
            p.g.recompute_v()
            p.g.cd_epoch(mode, G.dev_i32(good), max_inflight=1)
            want_a, want_v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
            p.g.set(duhl.ALPHA, np.zeros(n, dtype=np.float32))
            p.g.recompute_v()
            p.g.cd_epoch(mode, G.dev_i32(mixed), max_inflight=1)
            np.testing.assert_allclose(p.g.get(duhl.ALPHA), want_a, rtol=1e-6, atol=1e-9)
            np.testing.assert_allclose(p.g.get(duhl.V), want_v, rtol=1e-5, atol=1e-7)
        p.g.set(duhl.Z, np.full(n, -1.0, dtype=np.float32))
        p.g.gap(G.dev_i32(mixed), want_sum=False)
        z = p.g.get(duhl.Z)
        assert np.all(z[good] >= 0)
        assert np.count_nonzero(z >= 0) == good.size
        p.close()


def test_long_column_gap_pass_skips_bad_entries_and_matches_the_other_kernel(G, monkeypatch):
    """The gap pass that keeps v on chip (columns of more than 51,200 entries, long lists): entries
    of the list that name no coordinate write nothing, a list shorter than one workgroup's share
    falls back to the other kernel, and both kernels give the same gaps to fp32 rounding."""
    from paper_1708_05357_amd import duhl
    prob = lasso_problem(52000, 1500, 0.1, 0.1, seed=33)
    n = prob["n"]
    p = G.Pair(prob)
    p.g.select(300)
    p.g.commit_swap()
    p.g.cd_epoch(duhl.CD_SEQUENTIAL)
    p.sync_oracle_to_gpu_state()
    p.o.gaps()
    floor = G.gap_floor(p)
    rng = np.random.default_rng(5)
    good = rng.permutation(n)[:1400].astype(np.int32)
    mixed = good.copy()
    mixed[::7] = np.array([-1, n, 2 ** 31 - 1, -2 ** 31], dtype=np.int64)[np.arange(mixed[::7].size) % 4].astype(np.int32)
    kept = np.setdiff1d(np.arange(1400), np.arange(0, 1400, 7))
    p.g.set(duhl.Z, np.full(n, -1.0, dtype=np.float32))
    part = p.g.gap(G.dev_i32(mixed))
    z = p.g.get(duhl.Z)
    written = np.flatnonzero(z >= 0)
    assert np.array_equal(np.sort(written), np.sort(good[kept]))
    G.assert_gaps_close(z[good[kept]], p.o.z[good[kept]], floor=floor[good[kept]], label="long columns, list with bad entries")
    assert part == pytest.approx(float(p.o.z[good[kept]].sum()), rel=1e-4, abs=float(floor.sum()))
    z_lds = p.g.get(duhl.Z).copy()
    short = good[:100]                                      # 100 x 3 parts: fewer than 16 workgroups' worth
    p.g.set(duhl.Z, np.full(n, -1.0, dtype=np.float32))
    p.g.gap(G.dev_i32(short), want_sum=False)
    z_short = p.g.get(duhl.Z)
    both = np.intersect1d(short, good[kept])
    assert np.count_nonzero(z_short >= 0) == 100
    assert np.abs(z_short[both] - z_lds[both]).max() <= 2.0 * floor[both].max() + 1e-6 * np.abs(z_lds[both]).max()
    p.close()


def test_zero_columns_and_empty_rows(G):
    """Degenerate coordinates: a zero column (Lasso -> alpha_j = 0) and an empty CSR row
    (SVM -> alpha_j = y_j), both schemes."""
    from paper_1708_05357_amd import duhl, synth
    prob = lasso_problem(300, 40, 0.2, 0.1, seed=31)
    prob["cols"][7] = 0
    p = G.Pair(prob)
    a0 = np.zeros(40, dtype=np.float32)
    a0[7] = 0.3
    for mode in (duhl.CD_SEQUENTIAL, duhl.CD_ASYNC, duhl.CD_ATOMIC):
        p.g.set(duhl.ALPHA, a0)
        p.g.set(duhl.Z, np.arange(40, 0, -1).astype(np.float32))
        p.g.select(40)
        p.g.commit_swap()
        p.g.cd_epoch(mode, max_inflight=1)
        assert p.g.get(duhl.ALPHA)[7] == 0.0
    p.close()
    sp = synth.svm_csr(64, 50, 0.1, seed=2)
    rp = sp["rowptr"].clone()
    cut = int(rp[6] - rp[5])
    keep = torch.ones(sp["val"].numel(), dtype=torch.bool)
    keep[int(rp[5]):int(rp[6])] = False
    sp["val"], sp["colidx"] = sp["val"][keep], sp["colidx"][keep]
    rp[6:] -= cut
    sp["rowptr"] = rp
    p = G.Pair(sp)
    for mode in (duhl.CD_ASYNC, duhl.CD_ATOMIC, duhl.CD_SEQUENTIAL):
        p.g.set(duhl.ALPHA, np.zeros(64, dtype=np.float32))
        p.g.recompute_v()
        p.g.select(64)
        p.g.commit_swap()
        p.g.cd_epoch(mode, max_inflight=1)
        assert p.g.get(duhl.ALPHA)[5] == G.to_np(sp["target"])[5]
    o = p.o
    o.cd_pass(np.arange(64, dtype=np.int32))
    np.testing.assert_allclose(p.g.get(duhl.ALPHA), o.alpha, rtol=1e-5, atol=1e-6)
    p.close()


def test_degenerate_problems(G):
    """What the method does at its corners: a zero target (everything is optimal at alpha = 0), a
    regulariser at or above ||A^T b||_inf / d (alpha = 0 is optimal, every gap 0: App. E), a single
    coordinate, m = 1 and m = n, an empty visiting order, an empty refresh list."""
    from paper_1708_05357_amd import duhl, synth
    from oracle import duhl_oracle as orc
    base = lasso_problem(260, 33, 0.2, 0.1, seed=51)
    # b = 0: v = 0, B = 0, all gaps 0, selection falls back on the index order, rho = 1, nothing moves
    prob = dict(base)
    prob["target"] = torch.zeros_like(base["target"])
    p = G.Pair(prob)
    assert p.g.gap() == 0.0 and p.g.objective() == 0.0
    out = torch.empty(5, dtype=torch.int32, device="cuda:0")
    nsw, rho = p.g.select(5, out)
    np.testing.assert_array_equal(out.cpu().numpy(), np.arange(5))        # ties: smaller index first
    assert rho == 1.0
    p.g.commit_swap()
    for mode in (duhl.CD_SEQUENTIAL, duhl.CD_ASYNC, duhl.CD_ATOMIC):
        p.g.cd_epoch(mode)
    assert not p.g.get(duhl.ALPHA).any() and not p.g.get(duhl.V).any()
    p.close()
    # lambda d >= ||A^T b||_inf: alpha = 0 is the optimum, every gap is exactly 0 on both sides
    A = G.to_np(base["cols"]).astype(np.float64)
    b = G.to_np(base["target"]).astype(np.float64)
    prob = dict(base)
    prob["lam"] = float(np.abs(A @ b).max() * 1.001 / base["d"])
    p = G.Pair(prob)
    assert p.g.gap() == 0.0 and p.o.gaps() == 0.0
    p.g.select(base["n"])
    p.g.commit_swap()
    p.g.cd_epoch(duhl.CD_ASYNC)
    assert not p.g.get(duhl.ALPHA).any()
    assert p.g.objective() == pytest.approx(p.o.objective(), rel=1e-6)
    p.close()
    # one coordinate; m = 1 out of many; m = n; empty lists
    one = lasso_problem(64, 1, 1.0, 0.1, seed=52)
    p = G.Pair(one)
    p.g.select(1)
    p.g.commit_swap()
    p.g.cd_epoch(duhl.CD_SEQUENTIAL)
    p.o.cd_pass(np.zeros(1, dtype=np.int32))
    np.testing.assert_allclose(p.g.get(duhl.ALPHA), p.o.alpha, rtol=1e-5)
    p.close()
    p = G.Pair(base)
    z32 = p.g.get(duhl.Z)
    out = torch.empty(1, dtype=torch.int32, device="cuda:0")
    p.g.select(1, out)
    assert out.item() == int(np.flatnonzero(z32 == z32.max())[0])
    p.g.commit_swap()
    alln = torch.empty(base["n"], dtype=torch.int32, device="cuda:0")
    nsw, rho = p.g.select(base["n"], alln)
    np.testing.assert_array_equal(alln.cpu().numpy(), np.arange(base["n"]))
    assert rho == pytest.approx(1.0)
    p.g.commit_swap()
    before = (p.g.get(duhl.ALPHA), p.g.get(duhl.V), p.g.get(duhl.Z))
    empty = torch.empty(0, dtype=torch.int32, device="cuda:0")
    for mode in (duhl.CD_SEQUENTIAL, duhl.CD_ASYNC, duhl.CD_ATOMIC):
        p.g.cd_epoch(mode, empty)
    assert p.g.gap(empty) == 0.0                                          # nothing refreshed: sum of nothing
    for x, y in zip(before, (p.g.get(duhl.ALPHA), p.g.get(duhl.V), p.g.get(duhl.Z))):
        np.testing.assert_array_equal(x, y)
    p.close()


# ------------------------------------------------------------------------------------ reference selection rules
def test_block_and_random_selection_rules(G):
    """The sequential-block and random reference schemes (Sections 5.1, 5.2): exact block contents
    with wrap-around, random subsets that are valid, seed-dependent and roughly uniform, rho of
    eq. (7) evaluated on z for the chosen set; and the paper's qualitative claim that gap selection
    converges faster than random selection."""
    from oracle import duhl_oracle as orc
    from paper_1708_05357_amd import duhl
    n, m = 5003, 700
    p = G.Pair(lasso_problem(64, n, 0.05, 0.1, seed=51))
    z = p.g.get(duhl.Z)
    out = torch.empty(m, dtype=torch.int32, device="cuda:0")
    nblocks = -(-n // m)
    for arg in (0, 1, nblocks - 1, nblocks, 3 * nblocks + 2):
        nsw, rho = p.g.select(m, out, rule=duhl.SELECT_BLOCK, arg=arg)
        start = (arg % nblocks) * m % n
        want = np.sort((start + np.arange(m)) % n).astype(np.int32)
        np.testing.assert_array_equal(out.cpu().numpy(), want)
        assert rho == pytest.approx(orc.rho(z.astype(np.float64), want), rel=1e-10)
    counts = np.zeros(n)
    seen = []
    for seed in range(60):
        nsw, rho = p.g.select(m, out, rule=duhl.SELECT_RANDOM, arg=seed)
        P = out.cpu().numpy()
        assert P.size == m and np.all(np.diff(P) > 0) and P[0] >= 0 and P[-1] < n
        assert rho == pytest.approx(orc.rho(z.astype(np.float64), P), rel=1e-10)
        counts[P] += 1
        seen.append(P.copy())
    assert not np.array_equal(seen[0], seen[1])
    expect = 60 * m / n
    assert abs(counts.mean() - expect) < 1e-9 and counts.std() < 2.0 * np.sqrt(expect)
    assert np.abs(counts.reshape(-1)[: n // 2].mean() - counts[n // 2:].mean()) < 0.5   # no positional bias
    p.close()

    prob = lasso_problem(1000, 500, 0.1, 0.1, seed=0)
    finals = {}
    for rule in (duhl.SELECT_GAP, duhl.SELECT_RANDOM, duhl.SELECT_BLOCK):
        q = G.Pair(prob)
        for rnd in range(12):
            q.g.gap(want_sum=False)
            q.g.select(125, want_stats=False, rule=rule, arg=rnd)
            q.g.commit_swap()
            q.g.cd_epoch(duhl.CD_ASYNC, seed=rnd)
        finals[rule] = q.g.gap()
        q.close()
    assert finals[duhl.SELECT_GAP] < 0.1 * finals[duhl.SELECT_RANDOM]
    assert finals[duhl.SELECT_GAP] < 0.1 * finals[duhl.SELECT_BLOCK]


# ------------------------------------------------------------------------------------ unit A's gap sampler
@pytest.mark.parametrize("chunk_cols", [None, 170])
def test_host_gap_sampler_matches_oracle(G, chunk_cols):
    """Alg. 2, unit A's loop: host threads refresh z_j := gap_j(alpha^(t)) from the host matrix while
    the GPU runs the pass on the current block.  The refreshed entries must equal the oracle's gaps
    at the snapshot alpha^(t) (not at the state after the pass); other entries stay untouched."""
    from paper_1708_05357_amd import duhl
    prob = lasso_problem(2051, 600, 0.1, 0.1, seed=61)
    m = 90
    p = G.Pair(prob, budget=2 * m, host_resident=True, chunk_cols=chunk_cols)   # one allocation, or pieces
    rng = np.random.default_rng(7)
    p.g.select(m)
    p.g.commit_swap()
    for rnd in range(4):
        p.g.cd_epoch(duhl.CD_ASYNC, seed=rnd)                 # some state alpha^(t)
        p.sync_oracle_to_gpu_state()
        p.o.gaps()
        snapshot = p.o.z.copy()
        floor = G.gap_floor(p, partials=8)                    # the host threads keep eight running sums
        marker = np.full(prob["n"], -3.0, dtype=np.float32)
        p.g.set(duhl.Z, marker)
        idx = rng.permutation(prob["n"])[:250].astype(np.int32)
        p.g.host_sample_begin(idx, nthreads=4)
        with pytest.raises(duhl.DuhlError) as e:
            p.g.host_sample_begin(idx, nthreads=4)            # one round at a time
        assert e.value.status == duhl.ESTATE
        p.g.cd_epoch(duhl.CD_ASYNC, seed=100 + rnd)           # B works meanwhile and moves alpha, v
        done = p.g.host_sample_end(wait_all=True)
        assert done == idx.size
        z = p.g.get(duhl.Z)
        mask = np.zeros(prob["n"], dtype=bool)
        mask[idx] = True
        assert np.all(z[~mask] == -3.0)
        G.assert_gaps_close(z[idx], snapshot[idx], floor=floor[idx], label="host sampler")
    # stopping early refreshes a prefix-like subset only, and only with valid values
    p.sync_oracle_to_gpu_state()
    p.o.gaps()
    p.g.set(duhl.Z, np.full(prob["n"], -3.0, dtype=np.float32))
    idx = rng.permutation(prob["n"]).astype(np.int32)
    p.g.host_sample_begin(idx, nthreads=2)
    done = p.g.host_sample_end(wait_all=False)
    z = p.g.get(duhl.Z)
    touched = z != -3.0
    assert 0 <= done <= idx.size and touched.sum() == done
    floor = G.gap_floor(p, partials=8)
    if done:
        G.assert_gaps_close(z[touched], p.o.z[touched], floor=floor[touched], label="host sampler, stopped early")
    with pytest.raises(duhl.DuhlError) as e:
        p.g.host_sample_end()
    assert e.value.status == duhl.ESTATE
    # a pool of another size, built in the middle of the context's life, does one round's work once
    for threads in (3, 5):
        p.g.set(duhl.Z, np.full(prob["n"], -3.0, dtype=np.float32))
        p.g.host_sample_begin(idx, nthreads=threads)
        assert p.g.host_sample_end(wait_all=True) == idx.size
        G.assert_gaps_close(p.g.get(duhl.Z), p.o.z, floor=floor, label="host sampler, other pool sizes")
    p.close()
    q = G.Pair(lasso_problem(64, 40, 0.1, 0.1, seed=1))           # device residency: not applicable
    with pytest.raises(duhl.DuhlError) as e:
        q.g.host_sample_begin(np.arange(5, dtype=np.int32))
    assert e.value.status == duhl.EINVAL
    q.close()


def test_stream_read_probe(G):
    """The measurement aid reads what it is given and rejects what it cannot read."""
    from paper_1708_05357_amd import duhl
    g = duhl.Duhl(duhl.LASSO, 64, 8, 8)
    x = torch.ones(1 << 22, dtype=torch.float32, device="cuda:0")
    ms = g.probe_stream_read(x, reps=2)
    assert 0.0 < ms < 50.0
    with pytest.raises(duhl.DuhlError):
        g.probe_stream_read(x[1:], reps=1)               # not 16-byte aligned
    with pytest.raises(duhl.DuhlError):
        g.probe_stream_read(x, reps=0)
    g.close()


def test_first_gap_call_reuses_the_pass_of_set_data_and_nothing_later(G):
    """set_data's own pass leaves every gap at alpha = 0 in z; a full duhl_gap before anything has moved
    returns their sum without a second pass (z untouched: a poisoned entry written behind the
    library's back through a device pointer is the only way to tell, and handing such a pointer out
    switches the shortcut off).  After a pass, a duhl_set or duhl_recompute_v the gaps are computed."""
    from paper_1708_05357_amd import duhl
    prob = lasso_problem(500, 300, 0.2, 0.1, seed=12)
    p = G.Pair(prob)
    total0 = p.o.gaps()
    assert p.g.gap() == pytest.approx(total0, rel=1e-4)
    G.assert_gaps_close(p.g.get(duhl.Z), p.o.z)
    z_dev = p.g.device_view(duhl.Z)                       # from here on every call computes
    z_dev[7] = -5.0
    assert p.g.gap() == pytest.approx(total0, rel=1e-4)
    assert p.g.get(duhl.Z)[7] >= 0.0
    p.close()
    for change in ("pass", "set", "recompute"):
        p = G.Pair(prob)
        if change == "pass":
            p.g.select(60)
            p.g.commit_swap()
            p.g.cd_epoch(duhl.CD_SEQUENTIAL)
        elif change == "set":
            a = np.zeros(prob["n"], dtype=np.float32)
            a[3] = 0.25
            p.g.set(duhl.ALPHA, a)
            p.g.recompute_v()
        else:
            p.g.recompute_v()
        p.sync_oracle_to_gpu_state()
        total = p.g.gap()
        assert total == pytest.approx(p.o.gaps(), rel=1e-4, abs=1e-7)
        G.assert_gaps_close(p.g.get(duhl.Z), p.o.z, floor=G.gap_floor(p))
        p.close()


def test_scatter_add_probe_leaves_v_alone(G):
    """The second measurement aid: atomic adds of +0 to random elements of v.  v keeps its bits, the
    rate is a positive number, and the call needs data and sane arguments."""
    from paper_1708_05357_amd import duhl
    g = duhl.Duhl(duhl.LASSO, 1000, 64, 16)
    with pytest.raises(duhl.DuhlError) as e:
        g.probe_scatter_add(1000)
    assert e.value.status == duhl.ESTATE
    prob = lasso_problem(1000, 64, 0.2, 0.1, seed=3)
    g.set_data_dense(prob["cols"].cuda(), prob["target"].cuda(), prob["lam"])
    g.gap(want_sum=False)
    g.select(16, want_stats=False)
    g.commit_swap()
    g.cd_epoch(duhl.CD_SEQUENTIAL)
    before = g.get(duhl.V).copy()
    rate = g.probe_scatter_add(2_000_000, reps=2)
    assert 1e8 < rate < 1e13
    assert np.array_equal(before.view(np.uint32), g.get(duhl.V).view(np.uint32))
    for ops, reps in ((0, 1), (1000, 0)):
        with pytest.raises(duhl.DuhlError) as e:
            g.probe_scatter_add(ops, reps=reps)
        assert e.value.status == duhl.EINVAL
    g.close()


def test_guard_books_need_data_and_start_empty(G):
    from paper_1708_05357_amd import duhl
    g = duhl.Duhl(duhl.LASSO, 100, 40, 10)
    with pytest.raises(duhl.DuhlError) as e:
        g.cd_stats()
    assert e.value.status == duhl.ESTATE
    prob = lasso_problem(100, 40, 0.2, 0.1, seed=3)
    g.set_data_dense(prob["cols"].cuda(), prob["target"].cuda(), prob["lam"])
    assert g.cd_stats() == (0, 0, 0, 1.0)               # no working set, no pass yet
    g.gap(want_sum=False)
    g.select(10, want_stats=False)
    g.commit_swap()
    g.cd_epoch(duhl.CD_ASYNC, seed=1)
    damped, bound, kept, theta = g.cd_stats()
    assert damped in (0, 1) and 1 <= bound <= 10 and kept in (0, 10) and 0.0 <= theta <= 1.0
    g.set_data_dense(prob["cols"].cuda(), prob["target"].cuda(), prob["lam"])     # the books start afresh
    assert g.cd_stats()[0] == 0 and g.cd_stats()[2] == 0
    g.close()


def test_partner_wait_of_multi_unit_workers_is_bounded(G, monkeypatch):
    """Workers that span several compute units wait for each other's partial dot products.  With
    the wait cut to a single poll (forced from the host; every kernel still ends normally) some
    workgroup gives up, all of them leave their loops, and the next call that returns a scalar
    reports it; setting the data again clears the condition."""
    from paper_1708_05357_amd import duhl
    prob = lasso_problem(120000, 300, 0.05, 0.05, seed=71)           # two compute units per worker
    monkeypatch.setenv("DUHL_CD_SPIN_LIMIT", "0")
    g = duhl.Duhl(duhl.LASSO, prob["d"], prob["n"], prob["n"])
    monkeypatch.delenv("DUHL_CD_SPIN_LIMIT")
    cols, b = prob["cols"].cuda(), prob["target"].cuda()
    g.set_data_dense(cols, b, prob["lam"])
    g.select(256, want_stats=False)
    g.commit_swap()
    for k in range(3):
        g.cd_epoch(duhl.CD_ASYNC, seed=k)
    with pytest.raises(duhl.DuhlError) as e:
        g.objective()
    assert e.value.status == duhl.EHIP and "timed out" in str(e.value)
    g.close()
    # the same problem with the normal limit: no error, and the pass decreases the objective
    g = duhl.Duhl(duhl.LASSO, prob["d"], prob["n"], prob["n"])
    g.set_data_dense(cols, b, prob["lam"])
    before = g.objective()
    g.select(256, want_stats=False)
    g.commit_swap()
    g.cd_epoch(duhl.CD_ASYNC, seed=0)
    assert g.objective() < before
    g.close()


def test_selection_barrier_wait_is_bounded_and_the_context_recovers(G):
    """The selection kernel's workgroups meet at barriers.  With the wait cut to a single poll
    (forced from the host; every kernel still ends normally) the first workgroup to arrive gives up,
    the rest follow, and the call that reads a scalar reports it.  Setting the data again on the SAME
    context makes it usable: the next selection is the oracle's and the objective is read."""
    from oracle import duhl_oracle as orc
    from paper_1708_05357_amd import duhl
    prob = lasso_problem(96, 20000, 0.05, 0.1, seed=73)              # ten workgroups in the selection
    cols, b = prob["cols"].cuda(), prob["target"].cuda()
    g = duhl.Duhl(duhl.LASSO, prob["d"], prob["n"], 4000)
    g.set_data_dense(cols, b, prob["lam"])
    g.select(4000)                                                   # fine with the normal limit
    g.commit_swap()
    g.set_wait_limit(0)
    with pytest.raises(duhl.DuhlError) as e:
        g.select(4000)                                               # reads rho: reports the time-out
    assert e.value.status == duhl.EHIP and "timed out" in str(e.value)
    with pytest.raises(duhl.DuhlError) as e:
        g.objective()                                                # and so does every later scalar
    assert e.value.status == duhl.EHIP
    g.set_wait_limit(1 << 22)
    for attempt in range(2):                                         # recovery, twice over
        g.set_data_dense(cols, b, prob["lam"])
        out = torch.empty(4000, dtype=torch.int32, device="cuda:0")
        nsw, rho = g.select(4000, out)
        want = orc.select_topm(g.get(duhl.Z).astype(np.float64), 4000)
        np.testing.assert_array_equal(out.cpu().numpy(), want)
        g.commit_swap()
        before = g.objective()
        g.cd_epoch(duhl.CD_SEQUENTIAL, out[:64].contiguous())
        assert g.objective() < before
    with pytest.raises(duhl.DuhlError) as e:
        g.set_wait_limit(-1)
    assert e.value.status == duhl.EINVAL
    g.close()


@pytest.mark.parametrize("name", ["lasso_identity_2x2", "svm_two_points_1d", "ridge_one_column"])
def test_hand_worked_examples_on_the_gpu(G, name):
    """The instances worked by hand from App. C, D and E (tests/golden/hand_worked.json): the HIP
    path must give those numbers, which are exact in single precision, in every scheme."""
    import json
    from paper_1708_05357_amd import duhl
    with open(os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")) as f:
        case = json.load(f)[name]
    model = {"lasso": duhl.LASSO, "svm_t": duhl.SVM, "ridge": duhl.ELASTIC_NET}[name[:5]]
    cols = torch.tensor(case["cols"], dtype=torch.float32, device="cuda:0")
    target = torch.tensor(case["target"], dtype=torch.float32, device="cuda:0")
    n, d = cols.shape
    for mode in (duhl.CD_SEQUENTIAL, duhl.CD_ASYNC, duhl.CD_ATOMIC):
        g = duhl.Duhl(model, d, n, n)
        if model == duhl.ELASTIC_NET:
            g.set_eta(case["eta"])
        g.set_data_dense(cols, target, case["lambda"])
        assert g.objective() == pytest.approx(case["objective_at_zero"], abs=1e-7)
        np.testing.assert_allclose(g.get(duhl.Z), case["gaps_at_zero"], rtol=1e-6, atol=1e-7)
        assert g.gap() == pytest.approx(sum(case["gaps_at_zero"]), rel=1e-6)
        g.select(n, want_stats=False)
        g.commit_swap()
        g.cd_epoch(mode, G.dev_i32(np.arange(n)), max_inflight=1)       # index order, one at a time
        np.testing.assert_allclose(g.get(duhl.ALPHA), case["alpha_after_pass_0_1"], rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(g.get(duhl.V), case["v_after_pass"], rtol=1e-6, atol=1e-7)
        assert g.objective() == pytest.approx(case["objective_after_pass"], abs=1e-7)
        g.gap(want_sum=False)
        np.testing.assert_allclose(g.get(duhl.Z), case["gaps_after_pass"], atol=1e-7)
        g.close()


def test_context_reused_for_other_data(G):
    """duhl_set_data_* may be called again on a context, with another matrix, storage or residency:
    everything the previous data left behind (slots, the sparse copy, worker buffers, selection
    state) must be rebuilt or reset, so the rounds that follow equal those of a fresh context."""
    from paper_1708_05357_amd import duhl, synth
    dev = "cuda:0"
    n, d, m = 900, 2600, 200
    dense = [synth.svm_dense(n, d, seed=s) for s in (71, 72)]
    sparse = synth.svm_csr(n, d, 0.02, seed=73)

    def rounds(g, reproducible):
        out = []
        for rnd in range(4):
            g.gap(want_sum=False)
            g.select(m, want_stats=False)
            g.commit_swap()
            g.cd_epoch(duhl.CD_ASYNC if reproducible else duhl.CD_SEQUENTIAL, seed=rnd)
        out.append(g.get(duhl.ALPHA))
        out.append(g.get(duhl.V))
        out.append(np.float32(g.gap()))
        out.append(g.get(duhl.P))
        return out

    def load(g, kind, prob, keep):
        y = prob["target"].to(dev)
        if kind == "device":
            cols = prob["cols"].to(dev)
            keep += [cols, y]
            g.set_data_dense(cols, y, prob["lam"])
        elif kind == "host":
            cols = prob["cols"].pin_memory()
            keep += [cols, y]
            g.set_data_dense(cols, y, prob["lam"], duhl.RESIDENT_HOST)
        elif kind == "pieces":
            pieces = [prob["cols"][a:a + 350].clone().pin_memory() for a in range(0, n, 350)]
            keep += pieces + [y]
            g.set_data_dense_chunks(pieces, y, prob["lam"])
        else:
            arrs = [prob[k].to(dev) for k in ("rowptr", "colidx", "val")]
            keep += arrs + [y]
            g.set_data_csr(*arrs, y, prob["lam"])

    plan = [("device", dense[0]), ("csr", sparse), ("host", dense[1]), ("pieces", dense[0]),
            ("csr", sparse), ("device", dense[1])]
    keep = []
    reused = duhl.Duhl(duhl.SVM, d, n, 2 * m)
    for kind, prob in plan:
        # dense workers are reproducible for a seed; sparse concurrent passes are not, so the
        # sparse data are compared on sequential passes
        reproducible = kind != "csr"
        load(reused, kind, prob, keep)
        got = rounds(reused, reproducible)
        fresh = duhl.Duhl(duhl.SVM, d, n, 2 * m)
        load(fresh, kind, prob, keep)
        want = rounds(fresh, reproducible)
        fresh.close()
        for a, b in zip(got, want):
            assert np.array_equal(a, b), kind
    reused.close()


def test_plain_c_client_matches_oracle(G):
    """The library driven by a client written in C (HIP runtime C interface, default stream, no
    torch objects): rounds of Algorithm 1 with sequential passes give the oracle's iterates (1e-5),
    gaps (1e-4) and working set."""
    import ctypes as C
    from oracle import duhl_oracle as orc
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    path = os.path.join(root, "tests", "c_client", "libduhl_c_client.so")
    assert os.path.exists(path), "build it with __graft_entry__.build()"
    lib = C.CDLL(path)
    d, n, ld, m, rounds = 1003, 260, 1004, 60, 5
    prob = lasso_problem(d, n, 0.1, 0.1, seed=81)
    A = np.full((n, ld), np.nan, dtype=np.float32)             # padding must never be read
    A[:, :d] = prob["cols"].numpy()
    b = prob["target"].numpy().astype(np.float32)
    alpha, v, z = np.empty(n, np.float32), np.empty(d, np.float32), np.empty(n, np.float32)
    P = np.empty(m, np.int32)
    obj, gap = C.c_double(0.0), C.c_double(0.0)
    fp, ip = C.POINTER(C.c_float), C.POINTER(C.c_int32)
    lib.duhl_c_client_rounds.argtypes = [fp, fp, C.c_int64, C.c_int64, C.c_int64, C.c_double, C.c_int64, C.c_int,
                                         fp, fp, fp, ip, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    rc = lib.duhl_c_client_rounds(A.ctypes.data_as(fp), b.ctypes.data_as(fp), d, n, ld, prob["lam"], m, rounds,
                                  alpha.ctypes.data_as(fp), v.ctypes.data_as(fp), z.ctypes.data_as(fp),
                                  P.ctypes.data_as(ip), C.byref(obj), C.byref(gap))
    assert rc == 0, rc
    o = orc.Oracle(orc.LASSO, b, prob["lam"], cols=np.ascontiguousarray(A[:, :d]))
    for _ in range(rounds):
        o.gaps()
        Po = o.select(m)
        o.cd_pass(np.sort(Po).astype(np.int32))
    assert np.array_equal(np.sort(P), np.sort(Po))
    assert np.abs(alpha - o.alpha).max() <= 1e-5 * np.abs(o.alpha).max()
    assert np.abs(v - o.v).max() <= 1e-5 * np.abs(o.v).max()
    assert obj.value == pytest.approx(o.objective(), rel=1e-5)
    o.set_state(alpha.astype(np.float64), v.astype(np.float64))      # the gaps at the client's own iterate
    total = o.gaps()

    class _P:
        pass
    pp = _P()
    pp.o = o
    pp.prob = {"model": "lasso", "cols": np.ascontiguousarray(A[:, :d]), "d": d, "n": n}
    floor = G.gap_floor(pp)
    G.assert_gaps_close(z, o.z, floor=floor, label="plain C client")
    assert gap.value == pytest.approx(total, rel=1e-4, abs=float(floor.sum()))
