"""Helpers of the GPU parity tests: build the HIP context and the oracle on the same inputs."""
import numpy as np
import torch

from oracle import duhl_oracle as orc
from paper_1708_05357_amd import duhl, synth


def to_np(t):
    return t.detach().cpu().numpy()


class Pair:
    """The same seeded problem in the HIP library (self.g) and in the CPU oracle (self.o)."""

    def __init__(self, prob, budget=None, host_resident=False, ld=None, chunk_cols=None):
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
                if host_resident:
                    store = torch.empty((n, ld_eff), dtype=torch.float32, pin_memory=True)
                else:
                    store = torch.empty((n, ld_eff), dtype=torch.float32, device=dev)
                if ld_eff > d:
                    store.fill_(float("nan"))                      # padding must never be read
                store[:, :d].copy_(prob["cols"])
                self.cols = store[:, :d]
                self.g.set_data_dense(self.cols, self.target, prob["lam"],
                                      duhl.RESIDENT_HOST if host_resident else duhl.RESIDENT_DEVICE)
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


def assert_gaps_close(z_gpu, z_or, tol=1e-4, floor=0.0):
    """Normwise 1e-4 relative on the whole vector, entrywise 1e-4 relative on the entries that
    matter (>= 1e-3 of the largest).  `floor` is the absolute rounding floor of the formula."""
    zmax = float(np.max(z_or))
    err = np.abs(z_gpu.astype(np.float64) - z_or)
    assert err.max() <= tol * zmax + floor, (err.max(), zmax, floor)
    big = z_or >= 1e-3 * zmax
    if zmax > 0 and big.any():
        rel = err[big] / z_or[big]
        assert rel.max() <= tol + floor / max(zmax * 1e-3, 1e-300), rel.max()


def lasso_gap_floor(pair):
    """Rounding floor of the fp32 Lasso gap: the terms alpha_i c_i and Lambda |alpha_i| cancel
    near the optimum, leaving an absolute error of a few ulps of Lambda |alpha_i| / d, plus the
    error of the fp32 dot product scaled by |alpha_i| + B."""
    o = pair.o
    Lam = o.lam * o.d
    eps = 2.0 ** -24
    dot_err = 8 * eps * np.sqrt(o.d) * np.linalg.norm(o.v) * np.sqrt(o.q.max())
    return float((4 * eps * Lam * np.abs(o.alpha).max() + dot_err * (np.abs(o.alpha).max() + o.B)) / o.d)


def enet_gap_floor(pair):
    """Rounding floor of the fp32 elastic-net gap: the three terms cancel to ~0 at the optimum, each
    carrying a few ulps of its own size, plus the fp32 dot error times |alpha_i| + |c_i|/(Lambda eta)."""
    o = pair.o
    Lam = o.lam * o.d
    eps = 2.0 ** -24
    amax = np.abs(o.alpha).max()
    dot_err = 8 * eps * np.sqrt(o.d) * np.linalg.norm(o.v) * np.sqrt(o.q.max())
    cmax = np.linalg.norm(o.v) * np.sqrt(o.q.max())
    terms = amax * cmax + Lam * (o.eta * amax * amax + amax) + cmax * cmax / (Lam * o.eta)
    return float((8 * eps * terms + dot_err * (amax + cmax / (Lam * o.eta))) / o.d)


def svm_gap_floor_csr(rowptr, colidx, val, v, alpha, lam):
    """Rounding floor of the fp32 SVM gap on sparse data.  The dot product a_i^T v is summed in
    fp32 (per lane and range one after the other, then the ranges): its error is a small multiple
    of eps * S_i, S_i = sum_k |x_ik v_k|, which enters z_i through s_i = a_i^T v / (lambda n)
    multiplied by (1 + |alpha_i|) / n; the formula itself adds a few eps / n."""
    n = rowptr.size - 1
    rows = np.repeat(np.arange(n), np.diff(rowptr))
    S = np.bincount(rows, weights=np.abs(val.astype(np.float64) * np.asarray(v, dtype=np.float64)[colidx]),
                    minlength=n)
    eps = 2.0 ** -24
    return float(4 * eps / n * (1.0 + (1.0 + np.abs(alpha).max()) * S.max() / (lam * n)))


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
