"""duhl_gap_dense_static -- the gap pass for callers that cannot allocate -- against duhl_gap.

Both run the same kernels; the static variant keeps the per-workgroup partial sums in a static
device array instead of the context's buffer.  Checked through the C ABI on two calls in a row, the
second on a smaller input, so that whatever the first call left in the shared array would show."""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_1708_05357_amd import duhl, synth

pytestmark = pytest.mark.gpu


def _lasso_bound(prob):
    b = prob["target"].numpy().astype(np.float64)
    return float(b @ b) / (2.0 * prob["lam"] * prob["d"])          # App. E: ||b||^2 / (2 lambda d)


def _advance(g, m, rounds):
    """A few rounds so that alpha and v are no longer the starting point."""
    for r in range(rounds):
        g.gap(want_sum=False)
        g.select(m, want_stats=False)
        g.commit_swap()
        g.cd_epoch(duhl.CD_ASYNC, seed=r)


def _check(z_static, sum_static, z_ref, sum_ref, touched):
    zs = z_static.cpu().numpy()
    zmax = float(z_ref.max())
    # the bar of the gap vectors (1e-4 relative); the two paths share their kernels, so in fact equal
    assert np.abs(zs[touched] - z_ref[touched]).max() <= 1e-4 * zmax
    assert np.array_equal(zs[touched], z_ref[touched])
    untouched = np.ones(zs.size, dtype=bool)
    untouched[touched] = False
    assert np.all(zs[untouched] == -1.0)
    assert abs(float(sum_static.cpu()[0]) - sum_ref) <= 1e-12 * max(abs(sum_ref), 1e-300)


@pytest.mark.parametrize("model", ["lasso", "svm", "enet"])
def test_static_gap_pass_equals_duhl_gap_on_two_calls_in_a_row(model):
    dev = torch.device("cuda", 0)
    if model == "lasso":
        prob = synth.lasso_dense(1037, 3000, 0.05, 0.1, seed=5)
        mid, bound, eta = duhl.LASSO, _lasso_bound(prob), 1.0
    elif model == "enet":
        prob = synth.lasso_dense(1037, 3000, 0.05, 0.1, seed=6)
        mid, bound, eta = duhl.ELASTIC_NET, 0.0, 0.4
    else:
        prob = synth.svm_dense(2500, 515, seed=7)
        mid, bound, eta = duhl.SVM, 0.0, 1.0
    d, n = prob["d"], prob["n"]
    cols = prob["cols"].to(dev).contiguous()
    target = prob["target"].to(dev).contiguous()
    g = duhl.Duhl(mid, d, n, n // 4)
    if mid == duhl.ELASTIC_NET:
        g.set_eta(eta)
    g.set_data_dense(cols, target, prob["lam"])
    _advance(g, n // 4, 3)
    alpha, v = g.device_view(duhl.ALPHA), g.device_view(duhl.V)

    # first call: every coordinate
    sum_ref = g.gap()
    z_ref = g.get(duhl.Z)
    z1 = torch.full((n,), -1.0, dtype=torch.float32, device=dev)
    s1 = torch.full((1,), -7.0, dtype=torch.float64, device=dev)
    duhl.gap_dense_static(mid, cols, v, alpha, z1, prob["lam"], target=target, eta=eta, bound=bound, gap_sum=s1)
    torch.cuda.synchronize()
    _check(z1, s1, z_ref, sum_ref, np.arange(n))

    # second call, smaller: a list of 701 coordinates in no particular order
    rng = np.random.default_rng(11)
    pick = rng.permutation(n)[:701].astype(np.int32)
    idx = torch.as_tensor(pick, device=dev)
    sum_ref2 = g.gap(idx)
    z_ref2 = g.get(duhl.Z)
    z2 = torch.full((n,), -1.0, dtype=torch.float32, device=dev)
    s2 = torch.full((1,), -7.0, dtype=torch.float64, device=dev)
    duhl.gap_dense_static(mid, cols, v, alpha, z2, prob["lam"], target=target, eta=eta, bound=bound, idx=idx,
                          gap_sum=s2)
    torch.cuda.synchronize()
    _check(z2, s2, z_ref2, sum_ref2, pick)

    # third: an empty list writes nothing and sums to zero
    empty = torch.zeros(1, dtype=torch.int32, device=dev)[:0]
    z3 = torch.full((n,), -1.0, dtype=torch.float32, device=dev)
    s3 = torch.full((1,), -7.0, dtype=torch.float64, device=dev)
    lib = duhl.load()
    st = lib.duhl_gap_dense_static(mid, d, n, C.c_void_p(cols.data_ptr()), cols.stride(0), C.c_void_p(v.data_ptr()),
                                   C.c_void_p(alpha.data_ptr()), C.c_void_p(target.data_ptr()), prob["lam"], eta,
                                   bound, C.c_void_p(torch.zeros(1, dtype=torch.int32, device=dev).data_ptr()), 0,
                                   C.c_void_p(z3.data_ptr()), C.c_void_p(s3.data_ptr()), 0,
                                   C.c_void_p(torch.cuda.current_stream().cuda_stream), None, 0)
    assert st == duhl.OK
    torch.cuda.synchronize()
    assert float(s3.cpu()[0]) == 0.0 and bool((z3 == -1.0).all())
    del empty
    g.close()


def test_static_gap_pass_smaller_problem_after_a_larger_one():
    """Second call on a matrix with fewer and shorter columns than the first."""
    dev = torch.device("cuda", 0)
    for (d, n, seed) in [(4100, 6000, 1), (260, 900, 2)]:
        prob = synth.lasso_dense(d, n, 0.05, 0.1, seed=seed)
        cols = prob["cols"].to(dev).contiguous()
        target = prob["target"].to(dev).contiguous()
        g = duhl.Duhl(duhl.LASSO, d, n, n // 5)
        g.set_data_dense(cols, target, prob["lam"])
        _advance(g, n // 5, 2)
        sum_ref = g.gap()
        z_ref = g.get(duhl.Z)
        z = torch.full((n,), -1.0, dtype=torch.float32, device=dev)
        s = torch.full((1,), -7.0, dtype=torch.float64, device=dev)
        duhl.gap_dense_static(duhl.LASSO, cols, g.device_view(duhl.V), g.device_view(duhl.ALPHA), z, prob["lam"],
                              bound=_lasso_bound(prob), gap_sum=s)
        torch.cuda.synchronize()
        _check(z, s, z_ref, sum_ref, np.arange(n))
        g.close()


def test_static_gap_pass_refuses_what_its_array_cannot_hold():
    """Sizes beyond the static array are refused on the host, before anything is launched."""
    dev = torch.device("cuda", 0)
    small = torch.zeros(64, dtype=torch.float32, device=dev)
    lib = duhl.load()
    err = C.create_string_buffer(256)
    p = C.c_void_p(small.data_ptr())
    n_big = 32 * 65536 + 1                                   # one workgroup more than the array has entries
    st = lib.duhl_gap_dense_static(duhl.LASSO, 16, n_big, p, 16, p, p, None, 0.1, 1.0, 1.0, None, 0, p, None, 0,
                                   None, err, len(err))
    assert st == duhl.EINVAL and b"static scratch array" in err.value
    st = lib.duhl_gap_dense_static(duhl.LASSO, 16, 10, p, 8, p, p, None, 0.1, 1.0, 1.0, None, 0, p, None, 0, None,
                                   err, len(err))
    assert st == duhl.EINVAL and b"ld" in err.value
    st = lib.duhl_gap_dense_static(duhl.SVM, 16, 4, p, 16, p, p, None, 0.1, 1.0, 0.0, None, 0, p, None, 0, None,
                                   err, len(err))
    assert st == duhl.EINVAL
