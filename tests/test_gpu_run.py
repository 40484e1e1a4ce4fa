"""The native round loop (duhl_run) against the oracle's own loop of Algorithm 1, and its
stopping rule, sampling windows and host-thread sampler against what they must satisfy."""
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


def _lasso(d, n, frac=0.1, c=0.1, seed=0):
    from paper_1708_05357_amd import synth
    return synth.lasso_dense(d, n, frac, c, seed=seed)


@pytest.mark.parametrize("kind,passes", [("lasso", 1), ("lasso", 3), ("svm_csr", 2)])
def test_sequential_rounds_match_the_oracle_loop(G, kind, passes):
    """Alg. 1 with eq. (11): every round refreshes all gaps, takes the top m and runs `passes`
    sequential passes in ascending order -- the oracle's round() does the same, so the iterates
    agree to the sequential tolerance after every number of rounds."""
    from paper_1708_05357_amd import duhl, synth
    prob = _lasso(700, 300, seed=41) if kind == "lasso" else synth.svm_csr(900, 200, 0.05, seed=42)
    m = 40
    for rounds in (1, 4, 9):
        p = G.Pair(prob)
        st = p.g.run(m, rounds, passes=passes, mode=duhl.CD_SEQUENTIAL)
        assert st["rounds"] == rounds and st["passes"] == rounds * passes and st["converged"] == 0
        for _ in range(rounds):
            p.o.round(m, passes=passes)
        a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
        assert np.abs(a - p.o.alpha).max() <= 1e-5 * max(np.abs(p.o.alpha).max(), 1e-30)
        assert np.abs(v - p.o.v).max() <= 1e-5 * np.abs(p.o.v).max()
        # the sum read back at the last check is the total gap before the last round
        assert st["gap_memory_sum"] > 0
        p.close()


def test_stops_on_the_gap_and_reports_it(G):
    from paper_1708_05357_amd import duhl
    prob = _lasso(2000, 1500, 0.05, 0.1, seed=43)
    p = G.Pair(prob)
    m = 300
    g0 = p.g.gap()
    tol = 1e-4 * g0
    st = p.g.run(m, 500, passes=2, mode=duhl.CD_ASYNC, gap_tol=tol, seed=7)
    assert st["converged"] == 1 and 0 < st["rounds"] < 500
    assert st["gap_memory_sum"] <= tol
    assert p.g.working_set_size() == m                      # nothing left pending
    # the state was not touched after the check: a fresh pass gives the same sum
    assert p.g.gap() == pytest.approx(st["gap_memory_sum"], rel=1e-6)
    # and the oracle agrees that this point is that close to optimal
    p.sync_oracle_to_gpu_state()
    assert p.o.gaps() == pytest.approx(st["gap_memory_sum"], rel=1e-3, abs=1e-4 * tol)
    rng = np.random.default_rng(0)
    for _ in range(150):
        p.o.round(m, passes=2, rng=rng)
    assert abs(p.g.objective() - p.o.objective()) <= max(1e-5 * abs(p.o.objective()), 2 * tol)
    # check_every: fewer read-backs, the loop may overshoot by at most check_every - 1 rounds
    p2 = G.Pair(prob)
    st2 = p2.g.run(m, 500, passes=2, mode=duhl.CD_ASYNC, gap_tol=tol, seed=7, check_every=4)
    assert st2["converged"] == 1 and st["rounds"] <= st2["rounds"] <= st["rounds"] + 3
    assert st2["rounds"] % 4 == 0
    p.close()
    p2.close()


def test_stale_gap_memory_windows_on_device_data(G):
    """Section 4.1 on a device-resident matrix: per round only the working set and a window of
    the sample list are refreshed.  After the run, entries are either fresh (equal to the oracle at
    the final state, for the last working set) or stale; the problem still converges."""
    from paper_1708_05357_amd import duhl
    prob = _lasso(1500, 1200, 0.05, 0.1, seed=44)
    p = G.Pair(prob)
    n, m = prob["n"], 200
    perm = torch.randperm(n, generator=torch.Generator().manual_seed(3)).to(torch.int32).cuda()
    st = p.g.run(m, 120, passes=2, mode=duhl.CD_ASYNC, sample=perm, sample_per_round=n // 7, seed=1)
    assert st["rounds"] == 120
    full = p.g.gap()
    assert full <= 1e-3 * G.to_np(prob["target"]).var()     # far below O(0) = ||b||^2/(2d)
    rng = np.random.default_rng(0)
    for _ in range(150):
        p.o.round(m, passes=2, rng=rng)
    assert abs(p.g.objective() - p.o.objective()) <= 1e-5 * abs(p.o.objective())
    # stopping on the estimate alone is refused until the windows have covered the list once;
    # with `confirm` the loop only ends on the true total gap
    p3 = G.Pair(prob)
    tol = 1e-4 * p3.g.gap()
    st = p3.g.run(m, 3000, passes=2, mode=duhl.CD_ASYNC, sample=perm, sample_per_round=n // 7, gap_tol=tol,
                  confirm=True, seed=1)
    assert st["converged"] == 1 and st["confirmations"] >= 1 and st["rounds"] >= 7
    assert st["gap_memory_sum"] <= tol
    assert p3.g.gap() == pytest.approx(st["gap_memory_sum"], rel=1e-6)
    p3.sync_oracle_to_gpu_state()
    assert p3.o.gaps() == pytest.approx(st["gap_memory_sum"], rel=1e-3, abs=1e-4 * tol)
    p3.close()
    # windows wrap: a list that is not a multiple of the window, and bad arguments
    p.g.run(m, 5, sample=perm[:1000].contiguous(), sample_per_round=300)
    for bad in (dict(sample=perm, sample_per_round=0), dict(sample=perm, sample_per_round=n + 1),
                dict(passes=-1), dict(check_every=-1)):
        with pytest.raises(duhl.DuhlError) as e:
            p.g.run(m, 2, **bad)
        assert e.value.status == duhl.EINVAL
    with pytest.raises(duhl.DuhlError) as e:
        p.g.run(n + 1, 2)
    assert e.value.status == duhl.EINVAL
    p.g.select(m)
    with pytest.raises(duhl.DuhlError) as e:
        p.g.run(m, 2)                                       # a selection is pending
    assert e.value.status == duhl.ESTATE
    p.close()


@pytest.mark.parametrize("threads,pageable", [(0, False), (3, False), (0, True), (3, True)])
def test_host_resident_rounds_converge_to_the_oracle(G, threads, pageable):
    """Alg. 2 with the matrix in pinned host memory: residents refreshed from their slots, a
    window of the others over the link (threads = 0) or by host threads while the passes run."""
    from paper_1708_05357_amd import duhl
    prob = _lasso(1200, 900, 0.05, 0.1, seed=45)
    n, m = prob["n"], 120
    p = G.Pair(prob, budget=2 * m, host_resident=True, pageable=pageable)
    perm = torch.randperm(n, generator=torch.Generator().manual_seed(5)).to(torch.int32).cuda()
    before = p.g.objective()
    st = p.g.run(m, 200, passes=2, mode=duhl.CD_ASYNC, sample=perm, sample_per_round=n // 5,
                 host_threads=threads, seed=2)
    assert st["rounds"] == 200 and st["columns_swapped"] >= m
    if threads:
        assert st["host_sampled"] > 0
    assert p.g.objective() < before
    a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
    p.o.set_state(a.astype(np.float64))                     # v = A alpha - b must still hold
    assert np.abs(v - p.o.v).max() <= 1e-4 * np.abs(G.to_np(prob["target"])).max()
    o2 = G.Pair(prob)
    rng = np.random.default_rng(0)
    for _ in range(200):
        o2.o.round(m, passes=2, rng=rng)
    assert abs(p.g.objective() - o2.o.objective()) <= 1e-5 * abs(o2.o.objective())
    o2.close()
    p.close()
    # the stopping rule with confirmation: ends on the true total gap, evaluated over the link
    p = G.Pair(prob, budget=2 * m, host_resident=True, pageable=pageable)
    all_idx = G.dev_i32(np.arange(n))
    tol = 1e-4 * p.g.gap(all_idx)
    st = p.g.run(m, 3000, passes=2, mode=duhl.CD_ASYNC, sample=perm, sample_per_round=n // 5,
                 host_threads=threads, gap_tol=tol, confirm=True, seed=2)
    assert st["converged"] == 1 and st["confirmations"] >= 1
    assert p.g.gap(all_idx) == pytest.approx(st["gap_memory_sum"], rel=1e-6)
    assert st["gap_memory_sum"] <= tol
    p.close()


@pytest.mark.parametrize("threads", [0, 2])
def test_host_resident_svm_and_elastic_net_rounds(G, threads):
    """The other two models through the host-resident path (slots, copies, unit A's sampler reads
    the labels / the elastic-net constants): rounds converge to the oracle's objective."""
    from paper_1708_05357_amd import duhl, synth
    sv = synth.svm_dense(700, 260, seed=61)
    en = dict(synth.lasso_dense(900, 500, 0.05, 0.1, seed=62))
    en["model"], en["eta"] = "enet", 0.4
    for prob, m, rounds in ((sv, 150, 250), (en, 80, 150)):
        n = prob["n"]
        # with host threads the matrix comes in pinned pieces of 97 columns, otherwise in one
        p = G.Pair(prob, budget=2 * m, host_resident=True, chunk_cols=97 if threads else None)
        perm = torch.randperm(n, generator=torch.Generator().manual_seed(7)).to(torch.int32).cuda()
        st = p.g.run(m, rounds, passes=2, mode=duhl.CD_ASYNC, sample=perm, sample_per_round=max(1, n // 4),
                     host_threads=threads, seed=3)
        assert st["rounds"] == rounds
        if threads:
            assert st["host_sampled"] > 0
        ref = G.Pair(prob)
        rng = np.random.default_rng(0)
        for _ in range(rounds):
            ref.o.round(m, passes=2, rng=rng)
        og, oo = p.g.objective(), ref.o.objective()
        assert abs(og - oo) <= (1e-5 if prob["model"] != "svm" else 1e-4) * abs(oo), (prob["model"], og, oo)
        # the gap memory of the resident columns equals the oracle's gaps at the GPU's state
        p.sync_oracle_to_gpu_state()
        p.o.gaps()
        p.g.set(duhl.Z, np.full(n, -1.0, dtype=np.float32))
        p.g.gap(want_sum=False)
        z = p.g.get(duhl.Z)
        res = np.flatnonzero(z >= 0)
        assert res.size >= m
        np.testing.assert_allclose(z[res], p.o.z[res], rtol=1e-4, atol=1e-4 * p.o.z.max() + 1e-9)
        ref.close()
        p.close()


@pytest.mark.parametrize("clusters,spread", [(50, 0.3), (10, 0.3)])
def test_guard_of_concurrent_passes_on_near_duplicate_columns(G, clusters, spread):
    """Columns in groups of near-duplicates, and a selection by gap that gathers whole groups: more
    alike than the library's bound on concurrent steps assumes from the mean correlation, so the
    concurrent passes overshoot.  duhl_run's guard (adapt_inflight) notices the objective rising --
    exact steps never raise it (App. D) --, returns to the last good iterate and halves the bound
    until the passes descend again; the run then reaches the oracle's objective."""
    from paper_1708_05357_amd import duhl, synth
    prob = synth.lasso_clustered(3000, 2000, clusters, spread, seed=1)
    m = 200
    p = G.Pair(prob)
    start = p.g.objective()
    st = p.g.run(m, 150, passes=1, mode=duhl.CD_ASYNC, seed=3, adapt_inflight=True)
    assert st["rounds"] == 150
    # (either guard may be the one that acts: the pass's own, or the loop's on checked rounds)
    assert st["inflight_halvings"] + p.g.cd_stats()[0] >= 1
    og = p.g.objective()
    assert np.isfinite(og) and og < start
    a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
    p.o.set_state(a.astype(np.float64))                     # v = A alpha - b still holds (App. D)
    assert np.abs(v - p.o.v).max() <= 1e-4 * np.abs(G.to_np(prob["target"])).max()
    ref = G.Pair(prob)
    rng = np.random.default_rng(0)
    for _ in range(150):
        ref.o.round(m, passes=1, rng=rng)
    oo = ref.o.objective()
    print(f"clusters {clusters}: halvings {st['inflight_halvings']} in flight at the end {st['inflight_last']} "
          f"objective gpu {og:.9e} oracle {oo:.9e}")
    assert abs(og - oo) <= 1e-5 * abs(oo)
    ref.close()
    p.close()


@pytest.mark.parametrize("model,rep", [("lasso", 40), ("svm", 40), ("svm", 8)])
def test_guard_on_exact_duplicates(G, model, rep):
    """Every column `rep` times over (duplicated samples are common in real data; for the Lasso the
    minimiser is then not unique, the objective is): duplicates have equal gaps, are selected
    together and collide when solved at once.  With the guard the rounds reach the oracle's
    objective (1e-5)."""
    from paper_1708_05357_amd import duhl, synth
    base_n = 2000 // rep
    prob = dict(synth.lasso_dense(3000, base_n, 0.1, 0.1, seed=4) if model == "lasso"
                else synth.svm_dense(base_n, 3000, seed=4))
    prob["cols"] = prob["cols"].repeat_interleave(rep, dim=0).contiguous()
    prob["n"] = base_n * rep
    if model == "svm":
        prob["target"] = prob["target"].repeat_interleave(rep)
        prob["lam"] = 1.0 / prob["n"]
    m = prob["n"] // 5
    p = G.Pair(prob)
    st = p.g.run(m, 120, passes=1, mode=duhl.CD_ASYNC, seed=3, adapt_inflight=True)
    rng = np.random.default_rng(0)
    for _ in range(120):
        p.o.round(m, passes=1, rng=rng)
    og, oo = p.g.objective(), p.o.objective()
    print(f"{model} x{rep}: halvings {st['inflight_halvings']} objective gpu {og:.9e} oracle {oo:.9e}")
    assert abs(og - oo) <= 1e-5 * abs(oo)
    p.close()


def _duplicated_sparse_rows(rep):
    from paper_1708_05357_amd import synth
    base = synth.svm_csr(400, 3000, 0.02, seed=9)
    rowptr, colidx, val = (base[k].numpy() for k in ("rowptr", "colidx", "val"))
    lens = np.repeat(np.diff(rowptr), rep)
    new_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    pieces_c, pieces_v = [], []
    for i in range(400):
        for _ in range(rep):
            pieces_c.append(colidx[rowptr[i]:rowptr[i + 1]])
            pieces_v.append(val[rowptr[i]:rowptr[i + 1]])
    n = 400 * rep
    return {"model": "svm", "n": n, "d": 3000, "rowptr": torch.from_numpy(new_ptr),
            "colidx": torch.from_numpy(np.concatenate(pieces_c).astype(np.int32)),
            "val": torch.from_numpy(np.concatenate(pieces_v).astype(np.float32)),
            "target": base["target"].repeat_interleave(rep), "lam": 1.0 / n}


def test_default_pass_reaches_the_gap_on_clustered_columns_as_fast_as_sequential_steps(G):
    """Groups of 40 near-duplicate columns, which a selection by gap gathers into the working set: the
    rounds of the six named calls with max_inflight = 0 must not only descend but arrive -- total
    duality gap 1e-3 (eq. (2), from a fresh full pass) in no more rounds than 1.5 times what the
    oracle's sequential steps (Algorithm 1) need from the same start."""
    from paper_1708_05357_amd import duhl, synth
    prob = synth.lasso_clustered(2000, 10000, 250, 0.3, support_frac=0.02, c_lambda=0.05, seed=3)
    m, limit = 1000, 900
    p = G.Pair(prob)
    rng = np.random.default_rng(0)
    rounds_or = None
    for r in range(limit):
        if p.o.gaps() <= 1e-3:
            rounds_or = r
            break
        P = p.o.select(m)
        p.o.cd_pass(rng.permutation(P))
    assert rounds_or is not None
    rounds_gpu = None
    for r in range(limit):
        if p.g.gap() <= 1e-3:
            rounds_gpu = r
            break
        p.g.select(m, want_stats=False)
        p.g.commit_swap()
        p.g.cd_epoch(duhl.CD_ASYNC, seed=r)
    damped, inflight, kept, theta = p.g.cd_stats()
    print(f"rounds to total gap 1e-3: oracle {rounds_or}, gpu {rounds_gpu}; passes damped {damped}, bound now {inflight}")
    assert rounds_gpu is not None and rounds_gpu <= 1.5 * rounds_or + 10
    p.close()


@pytest.mark.parametrize("case", ["clustered", "lasso_x40", "svm_x40", "sparse_x16", "short_columns",
                                  "lasso_x40_d20000", "lasso_x40_d100000"])
def test_plain_cd_epoch_never_raises_the_objective(G, case):
    """The six named calls alone, on data that the library's bound on concurrent steps gets wrong:
    groups of near-duplicate columns, exact duplicates (dense and sparse), and a working set forty
    times larger than the columns are long.  Every DUHL_CD_ASYNC pass is guarded on the device (exact
    steps never raise the objective, App. D; a pass whose steps overshot is scaled back along its own
    direction and the bound halved), so with max_inflight = 0 the objective never rises from pass to
    pass, nothing turns into NaN, v stays A alpha - b, and the rounds reach the oracle's objective to 1e-5."""
    from paper_1708_05357_amd import duhl, synth
    rounds = 150
    if case == "clustered":
        prob, m = synth.lasso_clustered(3000, 2000, 50, 0.3, seed=1), 200
    elif case in ("lasso_x40", "svm_x40"):
        rep = 40
        prob = dict(synth.lasso_dense(3000, 50, 0.1, 0.1, seed=4) if case == "lasso_x40"
                    else synth.svm_dense(50, 3000, seed=4))
        prob["cols"] = prob["cols"].repeat_interleave(rep, dim=0).contiguous()
        prob["n"] = 50 * rep
        if case == "svm_x40":
            prob["target"] = prob["target"].repeat_interleave(rep)
            prob["lam"] = 1.0 / prob["n"]
        m = prob["n"] // 5
    elif case in ("lasso_x40_d20000", "lasso_x40_d100000"):
        # the same with columns long enough for the workers of 1,024 threads, and for those that span
        # two compute units
        rep, base = 40, (30 if case == "lasso_x40_d20000" else 16)
        prob = dict(synth.lasso_dense(20000 if case == "lasso_x40_d20000" else 100000, base, 0.2, 0.1, seed=4))
        prob["cols"] = prob["cols"].repeat_interleave(rep, dim=0).contiguous()
        prob["n"] = base * rep
        m, rounds = prob["n"] // 5, 100
    elif case == "sparse_x16":
        prob = _duplicated_sparse_rows(16)
        m = prob["n"] // 5
    else:
        prob, m, rounds = synth.lasso_dense(96, 8000, 0.01, 0.1, seed=6), 2000, 200
    p = G.Pair(prob)
    last = p.g.objective()
    for rnd in range(rounds):
        p.g.gap(want_sum=False)
        p.g.select(m, want_stats=False)
        p.g.commit_swap()
        p.g.cd_epoch(duhl.CD_ASYNC, seed=rnd)               # max_inflight = 0: the library's own bound
        now = p.g.objective()
        assert np.isfinite(now) and now <= last + 1e-6 * abs(last) + 1e-30, (rnd, last, now)
        last = now
    undone, inflight, kept, theta = p.g.cd_stats()
    # the host read the guard's books before every pass here, so no pass ran throttled: every step
    # counts but those of passes that had to be undone altogether (a damped pass keeps its steps)
    assert (rounds - undone) * m <= kept <= rounds * m
    assert 0.0 <= theta <= 1.0
    a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
    if prob["model"] == "svm":                              # a damped pass is a convex combination: the box holds
        ya = a * G.to_np(prob["target"])
        assert ya.min() >= -1e-6 and ya.max() <= 1.0 + 1e-6
    keep = p.o.alpha.copy()
    p.o.set_state(a.astype(np.float64))                     # v = A alpha (- b) still holds (App. D)
    scale = max(np.abs(p.o.v).max(), np.abs(G.to_np(prob["target"])).max() if prob["model"] != "svm" else 0.0, 1e-30)
    assert np.abs(v - p.o.v).max() <= 1e-4 * scale
    p.o.set_state(keep)
    rng = np.random.default_rng(0)
    for _ in range(rounds):
        p.o.round(m, passes=1, rng=rng)
    oo = p.o.objective()
    print(f"{case}: passes damped {undone}, bound now {inflight}, objective gpu {last:.9e} oracle {oo:.9e}")
    assert undone >= 1
    assert abs(last - oo) <= 1e-5 * abs(oo)
    p.close()


def test_guard_on_duplicated_sparse_rows(G):
    """The same for CSR data, whose concurrent passes add to v with atomics: every sample 16 times
    over.  The guard brings the rounds to the oracle's objective."""
    from paper_1708_05357_amd import duhl, synth
    rep = 16
    base = synth.svm_csr(400, 3000, 0.02, seed=9)
    rowptr, colidx, val = (base[k].numpy() for k in ("rowptr", "colidx", "val"))
    lens = np.repeat(np.diff(rowptr), rep)
    new_ptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    pieces_c, pieces_v = [], []
    for i in range(400):
        for _ in range(rep):
            pieces_c.append(colidx[rowptr[i]:rowptr[i + 1]])
            pieces_v.append(val[rowptr[i]:rowptr[i + 1]])
    n = 400 * rep
    prob = {"model": "svm", "n": n, "d": 3000, "rowptr": torch.from_numpy(new_ptr),
            "colidx": torch.from_numpy(np.concatenate(pieces_c).astype(np.int32)),
            "val": torch.from_numpy(np.concatenate(pieces_v).astype(np.float32)),
            "target": base["target"].repeat_interleave(rep), "lam": 1.0 / n}
    m = n // 5
    p = G.Pair(prob)
    st = p.g.run(m, 150, passes=1, mode=duhl.CD_ASYNC, seed=3, adapt_inflight=True)
    rng = np.random.default_rng(0)
    for _ in range(150):
        p.o.round(m, passes=1, rng=rng)
    og, oo = p.g.objective(), p.o.objective()
    print(f"sparse x{rep}: halvings {st['inflight_halvings']} in flight {st['inflight_last']} gpu {og:.9e} oracle {oo:.9e}")
    assert abs(og - oo) <= 1e-5 * abs(oo)
    a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
    p.o.set_state(a.astype(np.float64))
    assert np.abs(v - p.o.v).max() <= 1e-4 * max(np.abs(p.o.v).max(), 1e-30)
    p.close()


def _windows(length, per_round, rounds, wrap):
    """The windows duhl_run takes from a sample list of `length` entries: `per_round` consecutive
    positions from a cursor that advances round by round; `wrap`: a window runs on from the start of
    the list (GPU-evaluated windows), otherwise it is cut at the end of the list (host threads)."""
    cursor, out = 0, []
    for _ in range(rounds):
        if wrap:
            pos = [(cursor + k) % length for k in range(per_round)]
        else:
            pos = list(range(cursor, min(length, cursor + per_round)))
        out.append(np.array(pos, dtype=np.int64))
        cursor = (cursor + len(pos)) % length
    return out


def _check_gap_memory(G, p, z_gpu, refreshed, states, label, partials=128):
    """The gap memory after some rounds, entry by entry: entry i was last evaluated in round
    refreshed[i], i.e. at the iterate the GPU had after that many rounds (states[t] = its alpha, v),
    and must equal the oracle's gap at that very iterate to the 1e-4 bar."""
    n = z_gpu.size
    z_want, floor = np.zeros(n), np.zeros(n)
    for t in np.unique(refreshed):
        idx = np.flatnonzero(refreshed == t).astype(np.int32)
        p.o.set_state(states[t][0].astype(np.float64), states[t][1].astype(np.float64))
        p.o.gaps(idx)
        z_want[idx] = p.o.z[idx]
        floor[idx] = G.gap_floor(p, idx=idx, partials=partials)
    G.assert_gaps_close(z_gpu, z_want, floor=floor, label=label)


def _same_working_set_outside_the_tie_band(G, p, P_gpu, P_or, z_sel):
    """The two selections may differ only in coordinates whose gap-memory entry lies within the
    tie band around the m-th largest entry: the 1e-4 agreement of the gaps plus their fp32 resolution
    (an entry that is 1e-13 in double precision is an exact 0 in single, and ranks with the zeros)."""
    if np.array_equal(P_gpu, P_or):
        return
    diff = np.setxor1d(P_gpu, P_or).astype(np.int32)
    thr = np.sort(z_sel)[-P_or.size]
    band = 1e-4 * z_sel.max() + G.gap_floor(p, idx=diff).max()
    assert np.all(np.abs(z_sel[diff] - thr) <= band), (diff, z_sel[diff], thr, band)


@pytest.mark.parametrize("kind", ["lasso", "svm"])
def test_stale_memory_rounds_match_the_oracle_round_by_round(G, kind):
    """Sec. 4.1 / eq. (13) on a device-resident matrix, the GPU evaluating the windows: per round the
    gap memory is refreshed for the last working set and one window of the sample list at the current
    iterate, the m largest entries of the (otherwise stale) memory are taken, and `passes` sequential
    passes run over them in ascending order.  The oracle does the same rounds with the same windows:
    iterates 1e-5 and identical working sets after every number of rounds up to 9; and every entry
    of the gap memory equals the oracle's gap at the iterate of the round that last refreshed it."""
    from paper_1708_05357_amd import duhl, synth
    prob = _lasso(700, 300, seed=46) if kind == "lasso" else synth.svm_dense(400, 96, seed=47)
    n, m, per_round, passes = prob["n"], 40, 57, 2
    perm = np.random.default_rng(8).permutation(n).astype(np.int32)[: n - 11]       # 11 coordinates never sampled
    wins = _windows(perm.size, per_round, 9, wrap=True)
    states, refreshed = {}, np.zeros(n, dtype=np.int64)
    p = G.Pair(prob)
    states[0] = (p.g.get(duhl.ALPHA), p.g.get(duhl.V))
    p.o.gaps()                                                # set_data's first pass: every gap at alpha = 0
    P_prev = None
    for rounds in range(1, 10):
        q = G.Pair(prob)
        st = q.g.run(m, rounds, passes=passes, mode=duhl.CD_SEQUENTIAL, sample=G.dev_i32(perm),
                     sample_per_round=per_round)
        assert st["rounds"] == rounds
        # the oracle's round number rounds-1: what is refreshed at alpha^(t) before the selection
        t = rounds - 1
        fresh = np.arange(n) if P_prev is None else np.union1d(P_prev, perm[wins[t]])
        refreshed[fresh] = t
        p.o.gaps(fresh.astype(np.int32))
        # the GPU's working set of this round must be the oracle's outside the tie band; the oracle
        # then goes on with the GPU's choice, so that later rounds compare like with like
        P_prev = q.g.get(duhl.P)
        _same_working_set_outside_the_tie_band(G, p, P_prev, p.o.select(m), p.o.z)
        p.o.round_delayed(m, None, passes=passes, P=P_prev)
        a, v = q.g.get(duhl.ALPHA), q.g.get(duhl.V)
        states[rounds] = (a, v)
        assert np.abs(a - p.o.alpha).max() <= 1e-5 * max(np.abs(p.o.alpha).max(), 1e-30), rounds
        assert np.abs(v - p.o.v).max() <= 1e-5 * np.abs(p.o.v).max(), rounds
        if rounds in (1, 4, 9):
            keep = (p.o.alpha.copy(), p.o.v.copy(), p.o.z.copy())
            _check_gap_memory(G, p, q.g.get(duhl.Z), refreshed, states, f"stale memory ({kind}), {rounds} rounds")
            p.o.set_state(keep[0], keep[1])
            p.o.z[:] = keep[2]
        q.close()
    p.close()


def test_state_dumped_and_restored_continues_the_same_run(G):
    """Checkpoint and resume with the getters and setters: alpha and z are dumped after three rounds,
    a new context gets the data, alpha, v rebuilt from alpha (duhl_recompute_v) and z, and three more
    rounds there give the iterates of six uninterrupted rounds (sequential steps, 1e-5: v rebuilt
    from alpha differs from the running v by rounding only)."""
    from paper_1708_05357_amd import duhl
    prob = _lasso(700, 500, 0.1, 0.1, seed=70)
    m = 80

    def rounds(g, k):
        for _ in range(k):
            g.gap(want_sum=False)
            g.select(m, want_stats=False)
            g.commit_swap()
            g.cd_epoch(duhl.CD_SEQUENTIAL)

    p = G.Pair(prob)
    rounds(p.g, 6)
    want_a, want_v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
    p.close()
    q = G.Pair(prob)
    rounds(q.g, 3)
    dump_a, dump_z = q.g.get(duhl.ALPHA), q.g.get(duhl.Z)
    q.close()
    r = G.Pair(prob)
    r.g.set(duhl.ALPHA, dump_a)
    r.g.recompute_v()
    r.g.set(duhl.Z, dump_z)
    rounds(r.g, 3)
    a, v = r.g.get(duhl.ALPHA), r.g.get(duhl.V)
    assert np.abs(a - want_a).max() <= 1e-5 * np.abs(want_a).max()
    assert np.abs(v - want_v).max() <= 1e-5 * np.abs(want_v).max()
    r.close()


def test_native_loop_chooses_its_passes_per_round(G):
    """passes = 0 in the options: one pass in the first round, then a number between 1 and 8 from the
    measured cost of a refresh and of a pass; the loop converges to the same optimum (objective of
    the oracle's rounds to 1e-5) and accounts for its passes."""
    from paper_1708_05357_amd import duhl
    prob = _lasso(3000, 4000, 0.05, 0.1, seed=61)
    m = 400
    p = G.Pair(prob)
    st = p.g.run(m, 200, passes=0, mode=duhl.CD_ASYNC, gap_tol=1e-6, seed=3)
    assert st["converged"] == 1
    ppr = st["passes_per_round"]
    assert 1 <= ppr <= 8
    assert st["passes"] == 1 + (st["rounds"] - 1) * ppr
    print(f"passes per round chosen: {ppr}; {st['rounds']} rounds, {st['passes']} passes")
    rng = np.random.default_rng(0)
    for _ in range(200):
        p.o.round(m, passes=1, rng=rng)
    assert abs(p.g.objective() - p.o.objective()) <= 1e-5 * abs(p.o.objective())
    with pytest.raises(duhl.DuhlError):
        p.g.run(m, 1, passes=-1)
    p.close()


@pytest.mark.parametrize("pageable", [False, True])
def test_extra_passes_while_the_copies_are_in_flight(G, pageable):
    """theta sized to the copy (Sec. 5.2) in the native loop: with max_extra_passes the rounds run
    further passes on the current set for as long as the next set's columns are still arriving, and
    none once they are there.  How many depends on timing; what must hold: between passes and
    passes + max_extra_passes per round, none without host residency, v = A alpha - b, and the
    objective no higher than without them after the same rounds on the same sets (sequential exact
    steps never raise it, App. D)."""
    from paper_1708_05357_amd import duhl
    prob = _lasso(60000, 300, 0.1, 0.1, seed=50)
    m, rounds = 40, 5
    p = G.Pair(prob, budget=2 * m, host_resident=True, pageable=pageable)
    o0 = p.g.objective()
    st = p.g.run(m, rounds, passes=1, mode=duhl.CD_SEQUENTIAL, max_extra_passes=12)
    assert st["rounds"] == rounds and rounds <= st["passes"] <= rounds * 13
    print(f"passes run in {rounds} rounds: {st['passes']}")
    a, v = p.g.get(duhl.ALPHA), p.g.get(duhl.V)
    p.o.set_state(a.astype(np.float64))
    assert np.abs(v - p.o.v).max() <= 1e-5 * max(np.abs(p.o.v).max(), 1e-30)
    assert p.g.objective() < o0
    with pytest.raises(duhl.DuhlError):
        p.g.run(m, 1, max_extra_passes=-1)
    p.close()
    q = G.Pair(prob)                                        # the matrix on the device: nothing to wait for
    st = q.g.run(m, rounds, passes=2, mode=duhl.CD_SEQUENTIAL, max_extra_passes=12)
    assert st["passes"] == 2 * rounds
    q.close()


@pytest.mark.parametrize("chunk_cols", [None, 128, "pageable"])
def test_delayed_rounds_with_unit_a_threads_match_the_oracle_round_by_round(G, chunk_cols):
    """Alg. 2 as printed, on a matrix in host memory: unit B (the GPU) selects by eq. (13) and runs its
    passes while unit A's host threads evaluate z_j = gap_j(alpha^(t)) for the round's window; those
    values enter the gap memory after the round.  With host_wait_all the threads finish every window,
    so the rounds are reproducible and the oracle's round_delayed() -- same windows, samples taken at
    alpha^(t), residents refreshed before the selection -- must give the same iterates (1e-5) and
    working sets after every number of rounds up to 9, and every entry of the gap memory must be the
    oracle's gap at the iterate of the round that last refreshed it.  The device holds exactly m
    columns, so the columns in its slots at the start of a round are the previous working set."""
    from paper_1708_05357_amd import duhl
    prob = _lasso(900, 380, 0.1, 0.1, seed=48)
    n, m, per_round, passes = prob["n"], 50, 64, 2
    perm = np.random.default_rng(9).permutation(n).astype(np.int32)
    wins = _windows(perm.size, per_round, 9, wrap=False)
    states, refreshed = {}, np.zeros(n, dtype=np.int64)
    by_host = np.zeros(n, dtype=bool)
    p = G.Pair(prob)
    states[0] = (p.g.get(duhl.ALPHA), p.g.get(duhl.V))
    p.o.gaps()
    P_prev = None
    for rounds in range(1, 10):
        pageable = chunk_cols == "pageable"                    # ordinary host memory, staged by the library
        q = G.Pair(prob, budget=m, host_resident=True, chunk_cols=None if pageable else chunk_cols, pageable=pageable)
        st = q.g.run(m, rounds, passes=passes, mode=duhl.CD_SEQUENTIAL, sample=G.dev_i32(perm),
                     sample_per_round=per_round, host_threads=3, host_wait_all=True)
        assert st["rounds"] == rounds
        assert st["host_sampled"] == sum(w.size for w in wins[:rounds])
        t = rounds - 1
        if P_prev is not None:
            refreshed[P_prev] = t
            by_host[P_prev] = False
        refreshed[perm[wins[t]]] = t                          # unit A's samples: also at alpha^(t)
        by_host[perm[wins[t]]] = True
        if P_prev is not None:
            p.o.gaps(P_prev)                                   # residents, before the selection
        P_prev = q.g.get(duhl.P)                              # (the oracle follows the GPU among ties)
        _same_working_set_outside_the_tie_band(G, p, P_prev, p.o.select(m), p.o.z)
        p.o.round_delayed(m, perm[wins[t]], passes=passes, P=P_prev)
        a, v = q.g.get(duhl.ALPHA), q.g.get(duhl.V)
        states[rounds] = (a, v)
        assert np.abs(a - p.o.alpha).max() <= 1e-5 * max(np.abs(p.o.alpha).max(), 1e-30), rounds
        assert np.abs(v - p.o.v).max() <= 1e-5 * np.abs(p.o.v).max(), rounds
        if rounds in (1, 4, 9):
            keep = (p.o.alpha.copy(), p.o.v.copy(), p.o.z.copy())
            _check_gap_memory(G, p, q.g.get(duhl.Z), refreshed, states,
                              f"delayed rounds with host threads, {rounds} rounds", partials=8)
            p.o.set_state(keep[0], keep[1])
            p.o.z[:] = keep[2]
        q.close()
    p.close()
