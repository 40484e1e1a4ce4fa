"""Helpers of the GPU parity tests: build the HIP context and the oracle on the same inputs."""
import numpy as np
import torch

from oracle import duhl_oracle as orc
from paper_1708_05357_amd import duhl, synth


def to_np(t):
    return t if isinstance(t, np.ndarray) else t.detach().cpu().numpy()


class Pair:
    """The same seeded problem in the HIP library (self.g) and in the CPU oracle (self.o)."""

    def __init__(self, prob, budget=None, host_resident=False, ld=None, chunk_cols=None, pageable=False):
        self.prob = prob
        model = {"lasso": duhl.LASSO, "svm": duhl.SVM, "enet": duhl.ELASTIC_NET}[prob["model"]]
        self.model = model
        eta = float(prob.get("eta", 1.0))
        d, n = prob["d"], prob["n"]
        dev = torch.device("cuda", 0)
        self.target = prob["target"].to(dev).contiguous()
        self.g = duhl.Duhl(model, d, n, budget if budget is not None else n)
        if model == duhl.ELASTIC_NET:
            self.g.set_eta(eta)
        if "cols" in prob:
            ld_eff = ld if ld is not None else d
            if chunk_cols is not None:
                # the host matrix in separately pinned pieces of chunk_cols columns (the last one shorter)
                assert host_resident
                self.pieces = []
                for first in range(0, n, chunk_cols):
                    rows = min(chunk_cols, n - first)
                    piece = torch.full((rows, ld_eff), float("nan"), dtype=torch.float32).pin_memory()
                    piece[:, :d].copy_(prob["cols"][first:first + rows])
                    self.pieces.append(piece[:, :d])
                self.g.set_data_dense_chunks(self.pieces, self.target, prob["lam"])
            else:
                if host_resident and pageable:                      # ordinary host memory, staged by the library
                    store = torch.empty((n, ld_eff), dtype=torch.float32)
                elif host_resident:
                    store = torch.empty((n, ld_eff), dtype=torch.float32, pin_memory=True)
                else:
                    store = torch.empty((n, ld_eff), dtype=torch.float32, device=dev)
                if ld_eff > d:
                    store.fill_(float("nan"))                      # padding must never be read
                store[:, :d].copy_(prob["cols"])
                self.cols = store[:, :d]
                self.g.set_data_dense(self.cols, self.target, prob["lam"],
                                      (duhl.RESIDENT_HOST_PAGEABLE if pageable else duhl.RESIDENT_HOST)
                                      if host_resident else duhl.RESIDENT_DEVICE)
            self.o = orc.Oracle(model, to_np(prob["target"]), prob["lam"],
                                cols=np.ascontiguousarray(to_np(prob["cols"])), eta=eta)
        else:
            self.rowptr = prob["rowptr"].to(dev)
            self.colidx = prob["colidx"].to(dev)
            self.val = prob["val"].to(dev)
            self.g.set_data_csr(self.rowptr, self.colidx, self.val, self.target, prob["lam"])
            self.o = orc.Oracle(model, to_np(prob["target"]), prob["lam"],
                                csr=(to_np(prob["rowptr"]), to_np(prob["colidx"]), to_np(prob["val"])),
                                d=d, eta=eta)

    def sync_oracle_to_gpu_state(self):
        """Put the GPU's (alpha, v) into the oracle so both evaluate at the same point."""
        self.o.set_state(self.g.get(duhl.ALPHA).astype(np.float64), self.g.get(duhl.V).astype(np.float64))

    def close(self):
        self.g.close()


# ---- tolerance of the gap vectors -------------------------------------------------------------------
# The bar is 1e-4 relative.  The kernels compute in single precision, so an entry whose terms cancel
# (near the optimum alpha_i c_i = -Lambda |alpha_i|) cannot be better than the rounding of those
# terms.  That resolution is modelled PER ENTRY from the entry's own terms (gap_floor below) and is
# only granted to an entry where it exceeds the 1e-4 bar; everywhere else the bare bar applies.
EPS = 2.0 ** -24          # unit roundoff of fp32
DOT_SIGMAS = 8.0          # multiples of the modelled standard deviation of a dot product's rounding error
FORM_ULPS = 4.0           # roundings of a term of the gap formula, in units of EPS times the term

MARGINS = {}              # label -> worst observed err / floor (written out at the end of the session)


def dot_rounding(sumsq_prod, length, partials):
    """Modelled standard deviation of the rounding error of an fp32 dot product whose `length`
    terms a_k v_k (sumsq_prod = sum_k (a_k v_k)^2) are accumulated with fused multiply-adds into
    `partials` running sums which are then added pairwise: every rounding is independent,
    uniform within half an ulp of the running sum, and the running sum of random-sign terms grows
    like a random walk.  The variance is EPS^2 * sumsq_prod * (length/(6 partials) + log2(partials)/3 + 1/3)."""
    partials = max(1.0, min(float(partials), float(length)))
    return EPS * np.sqrt(sumsq_prod) * np.sqrt(length / (6.0 * partials) + np.log2(partials) / 3.0 + 1.0 / 3.0)


def column_stats(pair, idx=None):
    """c_i = a_i^T v in double and sum_k (a_ik v_k)^2, at the oracle's v, for all or the listed columns."""
    prob, v = pair.prob, pair.o.v
    if "cols" in prob:
        cols = to_np(prob["cols"])
        if idx is not None:
            cols = cols[idx]
        cols = cols.astype(np.float64)
        return cols @ v, (cols * cols) @ (v * v), float(prob["d"])
    import scipy.sparse as sp
    rowptr, colidx, val = (to_np(prob[k]) for k in ("rowptr", "colidx", "val"))
    X = sp.csr_matrix((val.astype(np.float64), colidx, rowptr), shape=(prob["n"], prob["d"]))
    if idx is not None:
        X = X[idx]
    length = float(np.diff(X.indptr).max()) if X.shape[0] else 1.0
    return X @ v, X.multiply(X) @ (v * v), length


def gap_floor(pair, idx=None, partials=128):
    """Per-entry resolution of the fp32 gap at the oracle's current (alpha, v): DOT_SIGMAS modelled
    standard deviations of the dot product's rounding error, carried through the formula's derivative
    with respect to c_i, plus FORM_ULPS roundings of each term of the formula (App. E / eq. (4)).
    `partials`: running sums of the kernel's dot product (dense gap kernel: 64 lanes x 2; one per lane
    and a tree of 16 for sparse rows; 8 for the host sampler)."""
    o = pair.o
    c, sumsq, length = column_stats(pair, idx)
    signed = o.alpha if idx is None else o.alpha[idx]
    alpha = np.abs(signed)
    dot = DOT_SIGMAS * dot_rounding(sumsq, length, partials)
    if pair.prob["model"] == "svm":
        y = o.target.astype(np.float64) if idx is None else o.target[idx].astype(np.float64)
        lam_n = o.lam * o.n
        s = c / lam_n
        active = (1.0 - y * s) > -dot / lam_n                 # the hinge term is, or may round to, non-zero
        hinge = np.maximum(1.0 - y * s, 0.0)
        form = FORM_ULPS * EPS * (alpha * np.abs(s) * 2 + hinge + active * (1.0 + np.abs(s)) + alpha)
        return (dot / lam_n * (alpha + active) + form) / o.n
    Lam = o.lam * o.d
    if pair.prob["model"] == "lasso":
        active = np.abs(c) > Lam - dot                         # [|c| - Lambda]_+ is, or may round to, non-zero
        over = np.maximum(np.abs(c) - Lam, 0.0)
        form = FORM_ULPS * EPS * (alpha * np.abs(c) + Lam * alpha + o.B * over + active * o.B * Lam)
        return (dot * (alpha + active * o.B) + form) / o.d
    eta = o.eta
    l1, l2 = Lam * (1.0 - eta), Lam * eta
    active = np.abs(c) > l1 - dot
    over = np.maximum(np.abs(c) - l1, 0.0)
    form = FORM_ULPS * EPS * (alpha * np.abs(c) + l2 * alpha * alpha + l1 * alpha + over * over / l2
                              + active * over * l1 / l2)
    # dz/dc = alpha_i + sign(c_i) [|c_i| - l1]_+ / l2, which vanishes at the optimum of an active
    # coordinate: the dot product's error then enters through the second-order term only
    slope = np.abs(signed + np.sign(c) * over / l2)
    return (dot * slope + active * dot * dot / (2.0 * l2) + form) / o.d


def assert_gaps_close(z_gpu, z_or, tol=1e-4, floor=None, label=None):
    """The 1e-4 bar on a gap vector: normwise, |z_i - zhat_i| <= tol * max zhat for every entry, and
    entrywise, <= tol * zhat_i on the entries that matter (zhat_i >= 1e-3 of the largest).  `floor`
    (per entry, or one number) is the fp32 resolution of the entry; it is added to a bound only where
    it exceeds that bound, i.e. where single precision cannot do better -- never in the first
    rounds, where the bare rule must hold.  Records the worst err/floor under `label`."""
    z_or = np.maximum(np.asarray(z_or, dtype=np.float64), 0.0)      # the device clamps at 0
    zmax = float(np.max(z_or)) if z_or.size else 0.0
    err = np.abs(np.asarray(z_gpu, dtype=np.float64) - z_or)
    fl = np.zeros_like(err) if floor is None else np.broadcast_to(np.asarray(floor, dtype=np.float64), err.shape)
    bound = tol * zmax + np.where(fl > tol * zmax, fl, 0.0)
    bad = err > bound
    assert not bad.any(), ("normwise", int(bad.sum()), float(err[bad].max()), zmax, float(fl[bad].max()))
    big = z_or >= 1e-3 * zmax
    if zmax > 0 and big.any():
        bound_e = tol * z_or[big] + np.where(fl[big] > tol * z_or[big], fl[big], 0.0)
        bad = err[big] > bound_e
        assert not bad.any(), ("entrywise", int(bad.sum()), float((err[big] / z_or[big])[bad].max()))
    if label is not None and floor is not None and (fl > 0).any():
        pos = fl > 0
        worst = float((err[pos] / fl[pos]).max())
        needed = int((fl > tol * zmax).sum())
        prev = MARGINS.get(label, (0.0, 0, 0))
        MARGINS[label] = (max(prev[0], worst), max(prev[1], needed), prev[2] + 1)
        print(f"[gap tolerance] {label}: worst err/floor {worst:.3f}, entries that needed the floor {needed}/{err.size}, "
              f"max err/zmax {err.max() / max(zmax, 1e-300):.2e}")


def lasso_gap_floor(pair):
    """Largest per-entry resolution of the Lasso gap (for bands around selection thresholds)."""
    return float(gap_floor(pair).max())


def enet_gap_floor(pair):
    return float(gap_floor(pair).max())


def dev_i32(a):
    return torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32), device="cuda:0")


def v_accumulation_floor(pair, alpha):
    """Rounding floor of v = A alpha (- b) (App. D) accumulated in fp32 in any order.  Each of the
    N = nnz(alpha) additions rounds a partial sum that is at most S_i = sum_j |a_ij alpha_j| (+ |b_i|)
    in size, by at most u = 2^-24 of it; N such errors add up like a random walk, sqrt(N) u S_i
    (worst case N u S_i).  A fixed 8 u S_i covers short sums."""
    prob = pair.prob
    a = np.abs(np.asarray(alpha, dtype=np.float64))
    if "cols" in prob:
        mag = np.abs(to_np(prob["cols"]).astype(np.float64)).T @ a
    else:
        rowptr, colidx, val = (to_np(prob[k]) for k in ("rowptr", "colidx", "val"))
        rows = np.repeat(np.arange(prob["n"]), np.diff(rowptr))
        mag = np.bincount(colidx, weights=np.abs(val.astype(np.float64)) * a[rows], minlength=prob["d"])
    if prob["model"] != "svm":
        mag = mag + np.abs(to_np(prob["target"]).astype(np.float64))
    return (8.0 + np.sqrt(np.count_nonzero(a))) * 2.0 ** -24 * float(mag.max())
