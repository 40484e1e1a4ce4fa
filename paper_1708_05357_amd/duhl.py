"""ctypes binding of libduhl.so -- argument marshalling only; every step runs in the HIP kernels.

The names mirror the C ABI of ``include/duhl.h``.  torch is used for device memory and streams:
tensors are passed as raw device pointers, the compute stream is torch's current stream at
construction time (so ``torch.cuda.Event`` timing brackets the library's kernels) and the copy
stream is a second torch stream of default priority.
"""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libduhl.so")

LASSO, SVM, ELASTIC_NET = 0, 1, 2
RESIDENT_DEVICE, RESIDENT_HOST, RESIDENT_HOST_PAGEABLE = 0, 1, 2
ALPHA, V, Z, P, SQNORM = 0, 1, 2, 3, 4
CD_SEQUENTIAL, CD_ASYNC, CD_ATOMIC = 0, 1, 2
SELECT_GAP, SELECT_RANDOM, SELECT_BLOCK = 0, 1, 2
OK, EINVAL, ENOMEM, EHIP, ESTATE, EBUDGET = 0, -1, -2, -3, -4, -5

EXPORTS = ["duhl_create", "duhl_set_eta", "duhl_set_wait_limit", "duhl_set_data_dense", "duhl_set_data_dense_chunks", "duhl_set_data_csr", "duhl_gap", "duhl_select",
           "duhl_gap_dense_static",
           "duhl_select_rule_apply", "duhl_host_sample_begin", "duhl_host_sample_end",
           "duhl_commit_swap", "duhl_cd_epoch", "duhl_cd_stats", "duhl_run", "duhl_objective", "duhl_recompute_v", "duhl_get",
           "duhl_set", "duhl_device_ptr", "duhl_probe_stream_read", "duhl_probe_scatter_add", "duhl_selection_threshold",
           "duhl_resident_columns", "duhl_swap_stats",
           "duhl_working_set_size", "duhl_last_error",
           "duhl_destroy"]

_lib = None


class RunOpts(C.Structure):
    _fields_ = [("m", C.c_int64), ("passes", C.c_int), ("mode", C.c_int), ("max_inflight", C.c_int),
                ("rule", C.c_int), ("seed", C.c_uint64), ("max_rounds", C.c_int64), ("gap_tol", C.c_double),
                ("check_every", C.c_int), ("sample_dev", C.c_void_p), ("sample_host", C.c_void_p),
                ("sample_len", C.c_int64), ("sample_per_round", C.c_int64), ("host_threads", C.c_int),
                ("confirm", C.c_int), ("adapt_inflight", C.c_int), ("host_wait_all", C.c_int),
                ("max_extra_passes", C.c_int)]


class RunStats(C.Structure):
    _fields_ = [("rounds", C.c_int64), ("passes", C.c_int64), ("converged", C.c_int), ("confirmations", C.c_int),
                ("gap_memory_sum", C.c_double), ("rho", C.c_double), ("columns_swapped", C.c_int64),
                ("host_sampled", C.c_int64), ("seconds", C.c_double), ("inflight_halvings", C.c_int),
                ("inflight_last", C.c_int), ("passes_per_round", C.c_int)]


class DuhlError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"duhl status {status}: {text}")
        self.status = status


def load():
    """Load the HIP library; fails loudly when it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1708_05357_amd.build`")
    lib = C.CDLL(LIB_PATH)
    p, i64, i32, dbl = C.c_void_p, C.c_int64, C.c_int, C.c_double
    lib.duhl_create.argtypes = [C.POINTER(p), i32, i64, i64, i64, i32, p, p]
    lib.duhl_set_eta.argtypes = [p, dbl]
    lib.duhl_set_wait_limit.argtypes = [p, i64]
    lib.duhl_set_data_dense.argtypes = [p, p, i64, i32, p, dbl]
    lib.duhl_set_data_dense_chunks.argtypes = [p, p, i64, i64, i64, p, dbl]
    lib.duhl_set_data_csr.argtypes = [p, p, p, p, i32, p, dbl]
    lib.duhl_gap.argtypes = [p, p, i64, C.POINTER(dbl)]
    lib.duhl_select.argtypes = [p, i64, p, C.POINTER(i64), C.POINTER(dbl)]
    lib.duhl_select_rule_apply.argtypes = [p, i32, C.c_uint64, i64, p, C.POINTER(i64), C.POINTER(dbl)]
    lib.duhl_host_sample_begin.argtypes = [p, p, i64, i32]
    lib.duhl_host_sample_end.argtypes = [p, i32, C.POINTER(i64)]
    lib.duhl_commit_swap.argtypes = [p]
    lib.duhl_cd_epoch.argtypes = [p, i32, p, i64, C.c_uint64, i32]
    lib.duhl_cd_stats.argtypes = [p, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64), C.POINTER(C.c_double)]
    lib.duhl_objective.argtypes = [p, C.POINTER(dbl)]
    lib.duhl_recompute_v.argtypes = [p]
    lib.duhl_get.argtypes = [p, i32, p, i64]
    lib.duhl_set.argtypes = [p, i32, p, i64]
    lib.duhl_device_ptr.argtypes = [p, i32, C.POINTER(p)]
    lib.duhl_selection_threshold.argtypes = [p, C.POINTER(C.c_float)]
    lib.duhl_resident_columns.argtypes = [p, C.POINTER(i64)]
    lib.duhl_swap_stats.argtypes = [p, C.POINTER(i64), C.POINTER(dbl)]
    lib.duhl_working_set_size.argtypes = [p]
    lib.duhl_working_set_size.restype = i64
    lib.duhl_last_error.argtypes = [p]
    lib.duhl_last_error.restype = C.c_char_p
    lib.duhl_destroy.argtypes = [p]
    lib.duhl_destroy.restype = None
    lib.duhl_probe_stream_read.argtypes = [p, p, i64, i32, C.POINTER(dbl)]
    lib.duhl_probe_scatter_add.argtypes = [p, i64, i32, C.POINTER(dbl)]
    lib.duhl_run.argtypes = [p, C.POINTER(RunOpts), C.POINTER(RunStats)]
    lib.duhl_gap_dense_static.argtypes = [i32, i64, i64, p, i64, p, p, p, dbl, dbl, dbl, p, i64, p, p, i32, p,
                                          C.c_char_p, i64]
    for name in EXPORTS:
        if name not in ("duhl_working_set_size", "duhl_last_error", "duhl_destroy"):
            getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _dptr(t, dtype):
    if t is None:
        return None
    assert isinstance(t, torch.Tensor) and t.dtype == dtype and t.is_contiguous(), (t.dtype, dtype)
    return C.c_void_p(t.data_ptr())


def gap_dense_static(model, cols, v, alpha, z, lam, target=None, eta=1.0, bound=0.0, idx=None,
                     gap_sum=None, device=0, stream=None):
    """duhl_gap_dense_static: the gap pass without a context and without any allocation.  cols:
    float32 (n, d) device tensor, row i = column a_i; v, alpha, z, target: float32 device tensors;
    idx: int32 device tensor or None; gap_sum: float64 device tensor of one element or None.  Only
    enqueues on `stream` (default: torch's current stream)."""
    lib = load()
    assert cols.dtype == torch.float32 and cols.dim() == 2 and cols.stride(1) == 1 and cols.is_cuda
    n, d = cols.shape
    if stream is None:
        stream = torch.cuda.current_stream(device)
    err = C.create_string_buffer(256)
    st = lib.duhl_gap_dense_static(model, d, n, C.c_void_p(cols.data_ptr()), cols.stride(0),
                                   _dptr(v, torch.float32), _dptr(alpha, torch.float32),
                                   _dptr(target, torch.float32), float(lam), float(eta), float(bound),
                                   _dptr(idx, torch.int32), 0 if idx is None else idx.numel(),
                                   _dptr(z, torch.float32), _dptr(gap_sum, torch.float64), device,
                                   C.c_void_p(stream.cuda_stream), err, len(err))
    if st != OK:
        raise DuhlError(st, err.value.decode())


class Duhl:
    """One problem on one GPU.  Methods are the C entry points, one to one."""

    def __init__(self, model, d, n, budget_cols, device=0, copy_stream=None):
        self.lib = load()
        self.model, self.d, self.n, self.budget = model, int(d), int(n), int(budget_cols)
        self.device = torch.device("cuda", device)
        with torch.cuda.device(self.device):
            self.compute_stream = torch.cuda.current_stream()
            self.copy_stream = copy_stream if copy_stream is not None else torch.cuda.Stream()
        self._h = C.c_void_p()
        st = self.lib.duhl_create(C.byref(self._h), model, self.d, self.n, self.budget, device,
                                  C.c_void_p(self.compute_stream.cuda_stream),
                                  C.c_void_p(self.copy_stream.cuda_stream))
        if st != OK:
            raise DuhlError(st, "duhl_create failed")
        self._keep = ()
        self._empty = None

    def _chk(self, st):
        if st != OK:
            raise DuhlError(st, self.lib.duhl_last_error(self._h).decode())

    def close(self):
        if self._h:
            self.lib.duhl_destroy(self._h)
            self._h = C.c_void_p()
            self._keep = ()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- data -----------------------------------------------------------------------------
    def set_eta(self, eta):
        self._chk(self.lib.duhl_set_eta(self._h, float(eta)))

    def set_wait_limit(self, polls):
        self._chk(self.lib.duhl_set_wait_limit(self._h, int(polls)))

    def set_data_dense(self, cols, target, lam, residency=RESIDENT_DEVICE):
        """cols: float32 (n, d) tensor, row i = column a_i (device, or pinned host memory for
        RESIDENT_HOST); row stride = leading dimension.  target: device float32."""
        assert cols.dtype == torch.float32 and cols.dim() == 2 and cols.stride(1) == 1
        assert tuple(cols.shape) == (self.n, self.d)
        if residency == RESIDENT_HOST:
            assert cols.device.type == "cpu" and cols.is_pinned()
        if residency == RESIDENT_HOST_PAGEABLE:
            assert cols.device.type == "cpu"
        self._keep = (cols, target)
        self._chk(self.lib.duhl_set_data_dense(self._h, C.c_void_p(cols.data_ptr()), cols.stride(0),
                                               residency, _dptr(target, torch.float32), float(lam)))

    def set_data_dense_chunks(self, chunks, target, lam):
        """chunks: list of pinned float32 (cols_k, d) host tensors that together hold the n columns in
        order; all but the last have the same number of rows, and all the same row stride."""
        cpc = chunks[0].shape[0]
        for k, t in enumerate(chunks):
            assert t.dtype == torch.float32 and t.dim() == 2 and t.stride(1) == 1 and t.shape[1] == self.d
            assert t.device.type == "cpu" and t.is_pinned() and t.stride(0) == chunks[0].stride(0)
            assert t.shape[0] == (cpc if k + 1 < len(chunks) else self.n - cpc * (len(chunks) - 1))
        self._keep = (list(chunks), target)
        ptrs = (C.c_void_p * len(chunks))(*[t.data_ptr() for t in chunks])
        self._chk(self.lib.duhl_set_data_dense_chunks(self._h, ptrs, len(chunks), int(cpc),
                                                      chunks[0].stride(0), _dptr(target, torch.float32),
                                                      float(lam)))

    def set_data_csr(self, rowptr, colidx, val, target, lam, residency=RESIDENT_DEVICE):
        self._keep = (rowptr, colidx, val, target)
        self._chk(self.lib.duhl_set_data_csr(self._h, _dptr(rowptr, torch.int64),
                                             _dptr(colidx, torch.int32), _dptr(val, torch.float32),
                                             residency, _dptr(target, torch.float32), float(lam)))

    # -- the hot path -----------------------------------------------------------------------
    def _list(self, t):
        """Pointer of an index list; an empty tensor (whose data pointer is NULL) still means
        "an empty list", not "no list"."""
        if t is not None and t.numel() == 0:
            if self._empty is None:
                self._empty = torch.zeros(1, dtype=torch.int32, device=self.device)
            return C.c_void_p(self._empty.data_ptr())
        return _dptr(t, torch.int32)

    def gap(self, idx=None, want_sum=True):
        out = C.c_double(0.0)
        count = 0 if idx is None else idx.numel()
        self._chk(self.lib.duhl_gap(self._h, self._list(idx), count,
                                    C.byref(out) if want_sum else None))
        return out.value if want_sum else None

    def select(self, m, P_out=None, want_stats=True, rule=SELECT_GAP, arg=0):
        nsw, rho = C.c_int64(0), C.c_double(0.0)
        self._chk(self.lib.duhl_select_rule_apply(self._h, rule, C.c_uint64(arg), int(m),
                                                  _dptr(P_out, torch.int32),
                                                  C.byref(nsw) if want_stats else None,
                                                  C.byref(rho) if want_stats else None))
        return (nsw.value, rho.value) if want_stats else None

    def host_sample_begin(self, idx, nthreads=8):
        """idx: int32 numpy array (host) of coordinates whose gaps the host threads refresh."""
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        self._chk(self.lib.duhl_host_sample_begin(self._h, idx.ctypes.data_as(C.c_void_p), idx.size,
                                                  int(nthreads)))

    def host_sample_end(self, wait_all=True):
        done = C.c_int64(0)
        self._chk(self.lib.duhl_host_sample_end(self._h, 1 if wait_all else 0, C.byref(done)))
        return done.value

    def commit_swap(self):
        self._chk(self.lib.duhl_commit_swap(self._h))

    def cd_epoch(self, mode=CD_ASYNC, order=None, seed=0, max_inflight=0):
        count = 0 if order is None else order.numel()
        self._chk(self.lib.duhl_cd_epoch(self._h, mode, self._list(order), count,
                                         C.c_uint64(seed), int(max_inflight)))

    def cd_stats(self):
        """(passes damped by the guard since the data were set, the library's bound on concurrent steps
        now, coordinate steps of the passes that were not undone, theta* of the last guarded pass)."""
        damped, now, kept, theta = C.c_int64(0), C.c_int64(0), C.c_int64(0), C.c_double(1.0)
        self._chk(self.lib.duhl_cd_stats(self._h, C.byref(damped), C.byref(now), C.byref(kept), C.byref(theta)))
        return damped.value, now.value, kept.value, theta.value

    def run(self, m, max_rounds, passes=1, mode=CD_ASYNC, gap_tol=-1.0, max_inflight=0, rule=SELECT_GAP,
            seed=0, check_every=1, sample=None, sample_per_round=0, host_threads=0, confirm=False,
            adapt_inflight=True, host_wait_all=False, max_extra_passes=0):
        """The native round loop (passes = 0: the loop chooses the passes per round from the measured cost
        of a refresh and of a pass).  sample: int32 device tensor with the coordinates whose gaps are
        refreshed window by window (None: see duhl_run); returns a dict of the statistics."""
        o = RunOpts(m=int(m), passes=int(passes), mode=mode, max_inflight=int(max_inflight), rule=rule,
                    seed=int(seed), max_rounds=int(max_rounds), gap_tol=float(gap_tol),
                    check_every=int(check_every), host_threads=int(host_threads), confirm=1 if confirm else 0,
                    adapt_inflight=1 if adapt_inflight else 0, host_wait_all=1 if host_wait_all else 0,
                    max_extra_passes=int(max_extra_passes))
        keep = None
        if sample is not None:
            assert sample.dtype == torch.int32 and sample.is_contiguous() and sample.is_cuda
            o.sample_dev = sample.data_ptr()
            o.sample_len = sample.numel()
            o.sample_per_round = int(sample_per_round)
            if host_threads > 0:
                keep = np.ascontiguousarray(sample.cpu().numpy(), dtype=np.int32)
                o.sample_host = keep.ctypes.data
        st = RunStats()
        self._chk(self.lib.duhl_run(self._h, C.byref(o), C.byref(st)))
        del keep
        return {name: getattr(st, name) for name, _ in RunStats._fields_}

    def objective(self):
        out = C.c_double(0.0)
        self._chk(self.lib.duhl_objective(self._h, C.byref(out)))
        return out.value

    def recompute_v(self):
        self._chk(self.lib.duhl_recompute_v(self._h))

    def probe_stream_read(self, tensor, reps=5):
        """Shortest time (ms) of a plain read-only streaming pass over a device tensor."""
        nbytes = tensor.numel() * tensor.element_size()
        nbytes -= nbytes % 16
        ms = C.c_double(0.0)
        self._chk(self.lib.duhl_probe_stream_read(self._h, C.c_void_p(tensor.data_ptr()), nbytes, int(reps),
                                                  C.byref(ms)))
        return ms.value

    def probe_scatter_add(self, ops, reps=3):
        """Best rate (adds per second) of fp32 atomic adds to random elements of v (adds of +0: v stays)."""
        rate = C.c_double(0.0)
        self._chk(self.lib.duhl_probe_scatter_add(self._h, int(ops), int(reps), C.byref(rate)))
        return rate.value

    def selection_threshold(self):
        """Smallest score of the last selection: the m-th largest entry of z it saw (eq. (13))."""
        out = C.c_float(0.0)
        self._chk(self.lib.duhl_selection_threshold(self._h, C.byref(out)))
        return out.value

    def resident_columns(self):
        """Columns held in device memory (host residency: device slots in use)."""
        out = C.c_int64(0)
        self._chk(self.lib.duhl_resident_columns(self._h, C.byref(out)))
        return out.value

    def swap_stats(self):
        """(columns copied, milliseconds on the copy stream) of the last committed selection."""
        cols, ms = C.c_int64(0), C.c_double(0.0)
        self._chk(self.lib.duhl_swap_stats(self._h, C.byref(cols), C.byref(ms)))
        return cols.value, ms.value

    # -- state ------------------------------------------------------------------------------
    def working_set_size(self):
        return self.lib.duhl_working_set_size(self._h)

    def _len(self, what):
        return {ALPHA: self.n, Z: self.n, SQNORM: self.n, V: self.d}.get(what, self.working_set_size())

    def get(self, what):
        n = self._len(what)
        out = np.empty(n, dtype=np.int32 if what == P else np.float32)
        self._chk(self.lib.duhl_get(self._h, what, out.ctypes.data_as(C.c_void_p), n))
        return out

    def set(self, what, arr):
        arr = np.ascontiguousarray(arr, dtype=np.float32)
        self._chk(self.lib.duhl_set(self._h, what, arr.ctypes.data_as(C.c_void_p), arr.size))

    def device_view(self, what):
        """Zero-copy torch view of a state array (float32; P: int32)."""
        ptr = C.c_void_p()
        self._chk(self.lib.duhl_device_ptr(self._h, what, C.byref(ptr)))
        n = self._len(what)
        dtype = np.int32 if what == P else np.float32

        class _Iface:
            __cuda_array_interface__ = {"shape": (n,), "typestr": np.dtype(dtype).str,
                                        "data": (ptr.value, False), "version": 2}
        return torch.as_tensor(_Iface(), device=self.device)
