"""Python face of the DuHL reference oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Thin ctypes wrapper around ``duhl_oracle.c`` (compiled with gcc, host only) plus the
outer round loop of Algorithms 1/2 written on top of its steps.  Everything is
sequential and in double precision on the single-precision data.  It shares nothing
with the HIP library and must not be imported by it; only tests, the smoke check and
the benchmark's CPU-baseline leg use it.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "duhl_oracle.c")
_LIB = os.path.join(_HERE, "libduhl_oracle.so")

LASSO, SVM, ENET = 0, 1, 2


def build(force=False):
    """Compile the C oracle with the host compiler."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Matrix(C.Structure):
    _fields_ = [("d", C.c_int64), ("n", C.c_int64), ("dense", C.c_void_p), ("ld", C.c_int64),
                ("rowptr", C.c_void_p), ("colidx", C.c_void_p), ("val", C.c_void_p)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        dbl = C.c_double
        p = C.c_void_p
        lib.or_lasso_objective.restype = dbl
        lib.or_lasso_objective.argtypes = [p, p, p, dbl]
        lib.or_svm_objective.restype = dbl
        lib.or_svm_objective.argtypes = [p, p, p, p, dbl]
        lib.or_lasso_bound.restype = dbl
        lib.or_lasso_bound.argtypes = [p, p, dbl]
        lib.or_lasso_gaps.restype = dbl
        lib.or_lasso_gaps.argtypes = [p, p, p, dbl, dbl, p, C.c_int64, p]
        lib.or_svm_gaps.restype = dbl
        lib.or_svm_gaps.argtypes = [p, p, p, p, dbl, p, C.c_int64, p]
        lib.or_select_topm.restype = C.c_int
        lib.or_select_topm.argtypes = [C.c_int64, p, C.c_int64, p]
        lib.or_rho.restype = dbl
        lib.or_rho.argtypes = [C.c_int64, p, p, C.c_int64]
        lib.or_col_sqnorms.restype = None
        lib.or_col_sqnorms.argtypes = [p, p]
        lib.or_matvec.restype = None
        lib.or_matvec.argtypes = [p, p, p, p]
        lib.or_lasso_cd_pass.restype = None
        lib.or_lasso_cd_pass.argtypes = [p, p, dbl, p, C.c_int64, p, p]
        lib.or_svm_cd_pass.restype = None
        lib.or_svm_cd_pass.argtypes = [p, p, p, dbl, p, C.c_int64, p, p]
        lib.or_enet_objective.restype = dbl
        lib.or_enet_objective.argtypes = [p, p, p, dbl, dbl]
        lib.or_enet_gaps.restype = dbl
        lib.or_enet_gaps.argtypes = [p, p, p, dbl, dbl, p, C.c_int64, p]
        lib.or_enet_cd_pass.restype = None
        lib.or_enet_cd_pass.argtypes = [p, p, dbl, dbl, p, C.c_int64, p, p]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def select_topm(z, m):
    """Indices of the m largest entries of z (ties to the smaller index), ascending."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    m = min(int(m), z.size)
    P = np.empty(m, dtype=np.int32)
    if _load().or_select_topm(z.size, _ptr(z), m, _ptr(P)) != 0:
        raise MemoryError
    return P


def rho(z, P):
    z = np.ascontiguousarray(z, dtype=np.float64)
    P = np.ascontiguousarray(P, dtype=np.int32)
    return _load().or_rho(z.size, _ptr(z), _ptr(P), P.size)


class Oracle:
    """State (alpha, v, z) of one problem and the steps of the scheme acting on it.

    dense problems: ``cols`` is a float32 array of shape (n, d) whose row i is column a_i
    (i.e. the column-major d x n matrix); sparse problems: ``csr=(rowptr, colidx, val)`` of A^T
    with ``d`` given.  ``target`` is b (length d) for the Lasso and y (length n, +-1) for the SVM.
    """

    def __init__(self, model, target, lam, cols=None, csr=None, d=None, eta=1.0):
        self.lib = _load()
        self.model = model
        self.lam = float(lam)
        self.eta = float(eta)          # elastic-net mix (ENET only): 1 = ridge
        self.target = np.ascontiguousarray(target, dtype=np.float32)
        M = _Matrix()
        if cols is not None:
            assert cols.dtype == np.float32 and cols.ndim == 2 and cols.strides[1] == 4
            self._keep = (cols,)
            M.n, M.d = cols.shape
            M.dense, M.ld = cols.ctypes.data, cols.strides[0] // 4
        else:
            rowptr = np.ascontiguousarray(csr[0], dtype=np.int64)
            colidx = np.ascontiguousarray(csr[1], dtype=np.int32)
            val = np.ascontiguousarray(csr[2], dtype=np.float32)
            self._keep = (rowptr, colidx, val)
            M.n, M.d = rowptr.size - 1, int(d)
            M.dense, M.ld = None, 0
            M.rowptr, M.colidx, M.val = rowptr.ctypes.data, colidx.ctypes.data, val.ctypes.data
        self.M = M
        self._Mp = C.cast(C.pointer(M), C.c_void_p)
        self.n, self.d = int(M.n), int(M.d)
        assert self.target.size == (self.n if model == SVM else self.d)
        self.q = np.empty(self.n, dtype=np.float64)
        self.lib.or_col_sqnorms(self._Mp, _ptr(self.q))
        self.alpha = np.zeros(self.n, dtype=np.float64)
        self.z = np.zeros(self.n, dtype=np.float64)
        self.v = np.empty(self.d, dtype=np.float64)
        self.recompute_v()
        self.B = (self.lib.or_lasso_bound(self._Mp, _ptr(self.target), self.lam)
                  if model == LASSO else 0.0)

    # -- state ---------------------------------------------------------------------------
    def recompute_v(self):
        """v := A alpha - b (Lasso) or A alpha (SVM), from its definition."""
        shift = None if self.model == SVM else self.target
        self.lib.or_matvec(self._Mp, _ptr(self.alpha), _ptr(shift), _ptr(self.v))
        return self.v

    def set_state(self, alpha, v=None):
        self.alpha[:] = alpha
        if v is None:
            self.recompute_v()
        else:
            self.v[:] = v

    # -- steps ---------------------------------------------------------------------------
    def objective(self):
        if self.model == LASSO:
            return self.lib.or_lasso_objective(self._Mp, _ptr(self.v), _ptr(self.alpha), self.lam)
        if self.model == ENET:
            return self.lib.or_enet_objective(self._Mp, _ptr(self.v), _ptr(self.alpha), self.lam, self.eta)
        return self.lib.or_svm_objective(self._Mp, _ptr(self.v), _ptr(self.alpha),
                                         _ptr(self.target), self.lam)

    def gaps(self, idx=None):
        """Refresh z for idx (None: all coordinates); returns the sum of the refreshed entries."""
        if idx is not None:
            idx = np.ascontiguousarray(idx, dtype=np.int32)
        count = self.n if idx is None else idx.size
        if self.model == LASSO:
            return self.lib.or_lasso_gaps(self._Mp, _ptr(self.v), _ptr(self.alpha), self.lam,
                                          self.B, _ptr(idx), count, _ptr(self.z))
        if self.model == ENET:
            return self.lib.or_enet_gaps(self._Mp, _ptr(self.v), _ptr(self.alpha), self.lam, self.eta,
                                         _ptr(idx), count, _ptr(self.z))
        return self.lib.or_svm_gaps(self._Mp, _ptr(self.v), _ptr(self.alpha), _ptr(self.target),
                                    self.lam, _ptr(idx), count, _ptr(self.z))

    def select(self, m):
        return select_topm(self.z, m)

    def cd_pass(self, order):
        order = np.ascontiguousarray(order, dtype=np.int32)
        if self.model == LASSO:
            self.lib.or_lasso_cd_pass(self._Mp, _ptr(self.q), self.lam, _ptr(order), order.size,
                                      _ptr(self.alpha), _ptr(self.v))
        elif self.model == ENET:
            self.lib.or_enet_cd_pass(self._Mp, _ptr(self.q), self.lam, self.eta, _ptr(order),
                                     order.size, _ptr(self.alpha), _ptr(self.v))
        else:
            self.lib.or_svm_cd_pass(self._Mp, _ptr(self.q), _ptr(self.target), self.lam,
                                    _ptr(order), order.size, _ptr(self.alpha), _ptr(self.v))

    # -- outer loop (Algorithm 1 with the selection rule of eq. (11)) ----------------------
    def round(self, m, passes=1, rng=None, order_fn=None):
        """One round: fresh gaps for all coordinates, top-m selection, `passes` passes over P.

        The visiting order of each pass is a permutation of P: from `order_fn(P, pass_no)` when
        given, from `rng` when given, else P as it stands (ascending).  Returns (P, total gap
        before the round)."""
        total = self.gaps()
        P = self.select(m)
        for k in range(passes):
            if order_fn is not None:
                order = order_fn(P, k)
            elif rng is not None:
                order = P[rng.permutation(P.size)]
            else:
                order = P
            self.cd_pass(order)
        return P, total

    # -- outer loop with a gap memory that may be stale (Algorithm 2; Section 4.1, eq. (13)) -----
    def round_delayed(self, m, refresh_idx, passes=1, rng=None, order_fn=None, fresh_idx=None, P=None):
        """One round t of Algorithm 2 on the gap memory self.z, whose entries may stem from earlier
        iterates (Section 4.1).

        1. (optional, not part of the printed algorithm) entries `fresh_idx` are evaluated at the
           round's starting point alpha^(t) BEFORE the selection -- what a unit that holds columns in
           its own memory can do for them at no cost to the other;
        2. P := the m largest entries of the gap memory as it stands (eq. (13));
        3. unit B: `passes` passes of exact coordinate steps over P (visiting order as in round());
        4. unit A, meanwhile: z_j := gap_j(alpha^(t)) for the sampled coordinates `refresh_idx` --
           at the round's STARTING point, whatever B has done since; they are seen by the selection
           of round t+1;
        5. alpha^(t+1) := alpha^(t) + B's update.
        `P` (optional) replaces step 2 by a given working set: eq. (13) has several maximisers when
        entries of the memory tie, and a caller that checks another implementation's choice among
        them passes that choice on.  Returns P."""
        if fresh_idx is not None and len(fresh_idx):
            self.gaps(fresh_idx)
        P = self.select(m) if P is None else np.ascontiguousarray(P, dtype=np.int32)
        alpha_t, v_t = self.alpha.copy(), self.v.copy()
        for k in range(passes):
            if order_fn is not None:
                order = order_fn(P, k)
            elif rng is not None:
                order = P[rng.permutation(P.size)]
            else:
                order = P
            self.cd_pass(order)
        if refresh_idx is not None and len(refresh_idx):
            alpha_next, v_next = self.alpha.copy(), self.v.copy()
            self.alpha[:], self.v[:] = alpha_t, v_t
            self.gaps(refresh_idx)
            self.alpha[:], self.v[:] = alpha_next, v_next
        return P

