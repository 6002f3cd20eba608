"""ctypes/numpy front end of the CPU oracle (``fae_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()`` and
``bench.py`` (its ``cpu_baseline`` legs and its check of steps 1 and 3 outside the timed
region); never by the product package.  Most of it marshals numpy arrays into the C
functions and loops over tables.  Three pieces of the method's arithmetic are written
here, in plain Python, because they are a few lines on scalars:
  ``t_quantile``            the Student-t quantile of Eq. 4, from the library routine
                            (pinned against printed t-table values);
  ``sampled_budget_cutoff`` the threshold scan of the Statistical Optimizer on the sampled
                            logger (Sec. 4.1.2): c = 0, 1, 2, ... until the estimated bytes fit;
  ``shuffle_scheduler``     the rate rule of Eq. 5.
``estimate_hot_rows`` scales Eq. 3 and Eq. 4 from a chunk to the table (times N).
Everything else that computes lives in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fae_oracle.c")
_LIB = os.path.join(_HERE, "libfae_oracle.so")

OK, EINVAL, ERANGE, ENOSPC = 0, -1, -2, -3


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_cutoff_eq1.restype = C.c_double
        _lib.orc_cutoff_eq1.argtypes = [C.c_double] * 3
        _lib.orc_cutoff_int.restype = C.c_uint32
        _lib.orc_cutoff_int.argtypes = [C.c_double]
        _lib.orc_count_hot.restype = C.c_int64
        _lib.orc_chunk_count.restype = C.c_int64
        _lib.orc_ci_halfwidth.restype = C.c_double
        _lib.orc_classify.restype = C.c_int64
        _lib.orc_runs.restype = C.c_int64
        _lib.orc_w0.restype = C.c_float
        _lib.orc_w0.argtypes = [C.c_uint64, C.c_int32, C.c_int64, C.c_int32, C.c_int32]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _ptr_array(arrs: Sequence[Optional[np.ndarray]]):
    out = (C.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        out[i] = None if a is None else a.ctypes.data
    return out


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"oracle {where}: error {code}")
        self.code = code


def _check(rc: int, where: str):
    if rc != OK:
        raise OracleError(rc, where)


# -- profiling ---------------------------------------------------------------------
def histogram(n_rows: int, idx: np.ndarray, cnt: Optional[np.ndarray] = None) -> np.ndarray:
    idx = _arr(idx, np.int32)
    if cnt is None:
        cnt = np.zeros(n_rows, dtype=np.uint32)
    assert cnt.dtype == np.uint32 and cnt.size == n_rows and cnt.flags.c_contiguous
    _check(lib().orc_histogram(C.c_int64(n_rows), _p(idx), C.c_int64(idx.size), _p(cnt)), "histogram")
    return cnt


def cutoff_eq1(t_percent: float, T: float, x_percent: float) -> float:
    return float(lib().orc_cutoff_eq1(t_percent, T, x_percent))


def cutoff_int(H: float) -> int:
    return int(lib().orc_cutoff_int(H))


def count_hot(cnt: np.ndarray, H: int) -> int:
    cnt = _arr(cnt, np.uint32)
    return int(lib().orc_count_hot(_p(cnt), C.c_int64(cnt.size), C.c_uint32(H)))


def budget_cutoff(dim: int, cnts: List[np.ndarray], T: Sequence[int], t_denom: int,
                  budget_bytes: int, small_table_bytes: int = 1 << 20):
    """Returns (c, H[z], n_hot[z])."""
    nt = len(cnts)
    cnts = [_arr(c, np.uint32) for c in cnts]
    rows = np.array([c.size for c in cnts], dtype=np.int64)
    Tn = np.array(T, dtype=np.int64)
    c_out = C.c_int64(0)
    H = np.zeros(nt, dtype=np.uint32)
    nh = np.zeros(nt, dtype=np.int64)
    rc = lib().orc_budget_cutoff(C.c_int32(nt), C.c_int32(dim), _p(rows), _ptr_array(cnts), _p(Tn),
                                 C.c_int64(t_denom), C.c_int64(budget_bytes),
                                 C.c_int64(small_table_bytes), C.byref(c_out), _p(H), _p(nh))
    _check(rc, "budget_cutoff")
    return int(c_out.value), H, nh


def classify(cnt: np.ndarray, H: int):
    """Returns (remap int32[R], hot_ids int32[n_hot])."""
    cnt = _arr(cnt, np.uint32)
    remap = np.empty(cnt.size, dtype=np.int32)
    hot_ids = np.empty(cnt.size, dtype=np.int32)
    n = int(lib().orc_classify(_p(cnt), C.c_int64(cnt.size), C.c_uint32(H), _p(remap), _p(hot_ids)))
    return remap, hot_ids[:n].copy()


def gather_rows(W: np.ndarray, hot_ids: np.ndarray) -> np.ndarray:
    W = _arr(W, np.float32)
    hot_ids = _arr(hot_ids, np.int32)
    out = np.empty((hot_ids.size, W.shape[1]), dtype=np.float32)
    lib().orc_gather_rows(_p(W), C.c_int32(W.shape[1]), _p(hot_ids), C.c_int64(hot_ids.size), _p(out))
    return out


def scatter_rows(W: np.ndarray, hot_ids: np.ndarray, hotW: np.ndarray) -> np.ndarray:
    """Full table with the hot rows written back (a copy; Sec. 3 (4), Sec. 6.2)."""
    W = _arr(W, np.float32).copy()
    hot_ids = _arr(hot_ids, np.int32)
    hotW = _arr(hotW, np.float32)
    assert hotW.shape == (hot_ids.size, W.shape[1])
    lib().orc_scatter_rows(_p(W), C.c_int32(W.shape[1]), _p(hot_ids), C.c_int64(hot_ids.size), _p(hotW))
    return W


def chunk_counts(cnt: np.ndarray, m: int, chunks: np.ndarray, H: int) -> np.ndarray:
    """Eq. 2 for every sampled chunk of one table's logger."""
    cnt = _arr(cnt, np.uint32)
    out = np.empty(len(chunks), dtype=np.int64)
    for i, ch in enumerate(chunks):
        out[i] = lib().orc_chunk_count(_p(cnt), C.c_int64(cnt.size), C.c_int64(m), C.c_int64(int(ch)), C.c_uint32(H))
    return out


def mean_std(Ci: np.ndarray):
    """Eq. 3: (mean, sample standard deviation) of the chunk counts."""
    Ci = _arr(Ci, np.int64)
    y, s = C.c_double(0), C.c_double(0)
    lib().orc_mean_std(_p(Ci), C.c_int64(Ci.size), C.byref(y), C.byref(s))
    return y.value, s.value


def t_quantile(confidence: float, n: int) -> float:
    """t_{alpha/2} of Student's t with n - 1 degrees of freedom (library routine)."""
    from scipy import stats
    return float(stats.t.ppf(1.0 - (1.0 - confidence) / 2.0, n - 1))


def estimate_hot_rows(cnt: np.ndarray, m: int, chunks: np.ndarray, H: int, confidence: float):
    """Sec. 4.1.2: estimated number of hot rows of one table from n sampled chunks and
    its confidence interval.  Per-chunk mean and half-width (Eq. 3, Eq. 4) are scaled by
    the number of chunks N.  Returns (estimate, half_width, ybar, s)."""
    cnt = _arr(cnt, np.uint32)
    n = len(chunks)
    N = -(-cnt.size // m)
    ybar, s = mean_std(chunk_counts(cnt, m, chunks, H))
    hw = lib().orc_ci_halfwidth(C.c_double(s), C.c_int64(n), C.c_int64(N), C.c_double(t_quantile(confidence, n)))
    return ybar * N, hw * N, ybar, s


def sampled_budget_cutoff(dim: int, cnts: List[np.ndarray], T: Sequence[int], t_denom: int, budget_bytes: int,
                          small_table_bytes: int, m: int, chunks: Sequence[Sequence[int]], c_limit: int = 1 << 20):
    """Statistical Optimizer on the sampled logger (Sec. 4.1.2, "Converging on a Threshold"):
    the budget rule of ``budget_cutoff`` with every sampled table's exact hot-row count
    replaced by its estimate ybar * N (Eq. 2, Eq. 3).  Scans c = 0, 1, 2, ... and returns the
    first (c, H[z]) whose estimated bytes fit; tables below small_table_bytes are wholly hot."""
    row_bytes = dim * 4
    for c in range(c_limit):
        total, H = 0.0, []
        for z, cnt in enumerate(cnts):
            if cnt.size * row_bytes < small_table_bytes:
                H.append(0)
                total += float(cnt.size) * float(row_bytes)
                continue
            h = min(-(-(c * int(T[z])) // int(t_denom)), 4294967295)
            H.append(h)
            ybar, _ = mean_std(chunk_counts(cnt, m, chunks[z], h))
            N = -(-cnt.size // m)
            total += ybar * float(N) * float(row_bytes)
        if total <= float(budget_bytes):
            return c, H
    raise OracleError(ENOSPC, "sampled_budget_cutoff: no threshold below c_limit fits")


def shuffle_scheduler(losses: Sequence[float], r0: float = 50.0, u: int = 4) -> List[float]:
    """Shuffle Scheduler (Sec. 5, Eq. 5): the rate after each swap, given the test loss
    measured after each swap.  Rates are the p of R(p), kept inside [1, 100].
      - loss not below the previous swap's loss      -> rate halves (not below R(1));
      - loss fell at each of the last u swaps        -> rate doubles (not above R(100)),
        and the count of successive falls starts again;
      - otherwise the rate stays.
    The first loss has nothing to be compared with and leaves the rate at r0."""
    r, falls, out = float(r0), 0, []
    for i, loss in enumerate(losses):
        if i > 0:
            if loss >= losses[i - 1]:
                r = max(r * 0.5, 1.0)
                falls = 0
            else:
                falls += 1
                if falls >= u:
                    r = min(r * 2.0, 100.0)
                    falls = 0
        out.append(r)
    return out


def w0(seed: int, table: int, row: int, dim: int, col: int) -> float:
    return float(lib().orc_w0(seed, table, row, dim, col))


def w0_rows(seed: int, table: int, rows: np.ndarray, dim: int) -> np.ndarray:
    rows = _arr(rows, np.int64)
    out = np.empty((rows.size, dim), dtype=np.float32)
    lib().orc_w0_rows(C.c_uint64(seed), C.c_int32(table), _p(rows), C.c_int64(rows.size), C.c_int32(dim), _p(out))
    return out


# -- partition ----------------------------------------------------------------------
def partition(rows: Sequence[int], n_samples: int, idx: List[np.ndarray],
              offsets: List[Optional[np.ndarray]], remap: List[np.ndarray]):
    """Returns (hot_samples, cold_samples, slots[z], hoffsets[z])."""
    nt = len(rows)
    idx = [_arr(a, np.int32) for a in idx]
    offsets = [None if o is None else _arr(o, np.int32) for o in offsets]
    remap = [_arr(r, np.int32) for r in remap]
    rows_a = np.array(rows, dtype=np.int64)
    hot = np.empty(n_samples, dtype=np.int32)
    cold = np.empty(n_samples, dtype=np.int32)
    slots = [np.empty(max(a.size, 1), dtype=np.int32) for a in idx]
    hoff = [np.empty(n_samples + 1, dtype=np.int32) for _ in range(nt)]
    nh = C.c_int64(0)
    rc = lib().orc_partition(C.c_int32(nt), _p(rows_a), C.c_int64(n_samples), _ptr_array(idx),
                             _ptr_array(offsets), _ptr_array(remap), _p(hot), _p(cold), C.byref(nh),
                             _ptr_array(slots), _ptr_array(hoff))
    _check(rc, "partition")
    n = int(nh.value)
    hoff = [h[:n + 1].copy() for h in hoff]
    slots = [s[:int(h[-1])].copy() for s, h in zip(slots, hoff)]
    return hot[:n].copy(), cold[:n_samples - n].copy(), slots, hoff


# -- forward ------------------------------------------------------------------------
def embbag_fwd(hotW: List[np.ndarray], n_samples: int, slots: List[np.ndarray],
               offsets: List[Optional[np.ndarray]], want_mag: bool = False):
    """out fp32[S][Tn][dim] (and sum|term| as fp64 of the same shape)."""
    nt = len(hotW)
    dim = hotW[0].shape[1]
    out = np.zeros((n_samples, nt, dim), dtype=np.float32)
    mag = np.zeros((n_samples, nt, dim), dtype=np.float64) if want_mag else None
    for z in range(nt):
        W = _arr(hotW[z], np.float32)
        s = _arr(slots[z], np.int32)
        o = None if offsets[z] is None else _arr(offsets[z], np.int32)
        oz = out[:, z, :]
        mz = mag[:, z, :] if want_mag else None
        # pass a pointer to the first element of the strided view
        rc = lib().orc_embbag_fwd(C.c_int64(W.shape[0]), C.c_int32(dim), _p(W), C.c_int64(n_samples),
                                  _p(s), _p(o), C.c_void_p(oz.ctypes.data), C.c_int64(nt * dim),
                                  None if mz is None else C.c_void_p(mz.ctypes.data), C.c_int64(nt * dim))
        _check(rc, "embbag_fwd")
    return (out, mag) if want_mag else out


# -- backward -----------------------------------------------------------------------
def sort_runs(slots: np.ndarray):
    """Stable order by slot, distinct slots ascending, their multiplicities."""
    slots = _arr(slots, np.int32)
    n = slots.size
    order = np.empty(max(n, 1), dtype=np.int32)
    _check(lib().orc_sort_by_slot(_p(slots), C.c_int64(n), _p(order)), "sort_by_slot")
    uniq = np.empty(max(n, 1), dtype=np.int32)
    runlen = np.empty(max(n, 1), dtype=np.int32)
    U = int(lib().orc_runs(_p(slots), _p(order), C.c_int64(n), _p(uniq), _p(runlen)))
    return order[:n], uniq[:U].copy(), runlen[:U].copy()


def bag_of(offsets: Optional[np.ndarray], n_samples: int, n_lookups: int) -> np.ndarray:
    out = np.empty(max(n_lookups, 1), dtype=np.int32)
    o = None if offsets is None else _arr(offsets, np.int32)
    lib().orc_bag_of(_p(o), C.c_int64(n_samples), _p(out))
    return out[:n_lookups]


def run_grads(order: np.ndarray, bag: np.ndarray, runlen: np.ndarray, sel: np.ndarray,
              gout: np.ndarray, table: int):
    """Summed gradient (fp64) and sum of |g| of the selected runs of one table.
    gout is fp32[S][Tn][dim]."""
    gout = _arr(gout, np.float32)
    _, nt, dim = gout.shape
    order = _arr(order, np.int32)
    bag = _arr(bag, np.int32)
    runlen = _arr(runlen, np.int32)
    sel = _arr(sel, np.int64)
    run_start = np.zeros(runlen.size + 1, dtype=np.int64)
    np.cumsum(runlen, out=run_start[1:])
    G = np.zeros((sel.size, dim), dtype=np.float64)
    Ga = np.zeros((sel.size, dim), dtype=np.float64)
    base = gout.ctypes.data + table * dim * 4
    lib().orc_run_grads(_p(order), _p(bag), _p(run_start), _p(runlen), _p(sel), C.c_int64(sel.size),
                        C.c_void_p(base), C.c_int64(nt * dim), C.c_int32(dim), _p(G), _p(Ga))
    return G, Ga


def sgd_rows(W_rows: np.ndarray, G: np.ndarray, lr: float) -> np.ndarray:
    W = _arr(W_rows, np.float32).copy()
    G = _arr(G, np.float64)
    lib().orc_sgd_rows(_p(W), _p(G), C.c_float(lr), C.c_int64(W.shape[0]), C.c_int32(W.shape[1]))
    return W


def embbag_bwd_sgd(hotW: List[np.ndarray], n_samples: int, slots: List[np.ndarray],
                   offsets: List[Optional[np.ndarray]], gout: np.ndarray, lr: float,
                   want_mag: bool = False):
    """In place on hotW[z] (fp32, C-contiguous).  Returns (uniq[z], runlen[z], mag[z])."""
    gout = _arr(gout, np.float32)
    nt = len(hotW)
    dim = hotW[0].shape[1]
    assert gout.shape == (n_samples, nt, dim)
    uniq_l, runlen_l, mag_l = [], [], []
    for z in range(nt):
        W = hotW[z]
        assert W.dtype == np.float32 and W.flags.c_contiguous
        s = _arr(slots[z], np.int32)
        o = None if offsets[z] is None else _arr(offsets[z], np.int32)
        n = s.size
        uniq = np.empty(max(n, 1), dtype=np.int32)
        runlen = np.empty(max(n, 1), dtype=np.int32)
        mag = np.zeros((max(n, 1), dim), dtype=np.float64) if want_mag else None
        nu = C.c_int64(0)
        base = gout.ctypes.data + z * dim * 4
        rc = lib().orc_embbag_bwd_sgd(C.c_int64(W.shape[0]), C.c_int32(dim), _p(W), C.c_int64(n_samples),
                                      _p(s), _p(o), C.c_int64(n), C.c_void_p(base), C.c_int64(nt * dim),
                                      C.c_float(lr), _p(uniq), _p(runlen), C.byref(nu), _p(mag))
        _check(rc, "embbag_bwd_sgd")
        U = int(nu.value)
        uniq_l.append(uniq[:U].copy())
        runlen_l.append(runlen[:U].copy())
        mag_l.append(None if mag is None else mag[:U].copy())
    return uniq_l, runlen_l, mag_l


# -- variants the paper leaves open: mean pooling, row-wise Adagrad ------------------------
POOL_SUM, POOL_MEAN = 0, 1
OPT_SGD, OPT_ROWWISE_ADAGRAD = 0, 1


def embbag_fwd_mean(hotW: List[np.ndarray], n_samples: int, slots: List[np.ndarray],
                    offsets: List[Optional[np.ndarray]], want_mag: bool = False):
    """Mean-pooled forward, same layout as ``embbag_fwd``."""
    nt = len(hotW)
    dim = hotW[0].shape[1]
    out = np.zeros((n_samples, nt, dim), dtype=np.float32)
    mag = np.zeros((n_samples, nt, dim), dtype=np.float64) if want_mag else None
    for z in range(nt):
        W = _arr(hotW[z], np.float32)
        s = _arr(slots[z], np.int32)
        o = None if offsets[z] is None else _arr(offsets[z], np.int32)
        oz = out[:, z, :]
        mz = mag[:, z, :] if want_mag else None
        rc = lib().orc_embbag_fwd_mean(C.c_int64(W.shape[0]), C.c_int32(dim), _p(W), C.c_int64(n_samples),
                                       _p(s), _p(o), C.c_void_p(oz.ctypes.data), C.c_int64(nt * dim),
                                       None if mz is None else C.c_void_p(mz.ctypes.data), C.c_int64(nt * dim))
        _check(rc, "embbag_fwd_mean")
    return (out, mag) if want_mag else out


def bag_len(offsets: Optional[np.ndarray], n_samples: int) -> np.ndarray:
    if offsets is None:
        return np.ones(n_samples, dtype=np.int32)
    return np.diff(_arr(offsets, np.int32)).astype(np.int32)


def run_grads_mean(order: np.ndarray, bag: np.ndarray, blen: np.ndarray, runlen: np.ndarray, sel: np.ndarray,
                   gout: np.ndarray, table: int):
    """``run_grads`` under mean pooling (each lookup receives its bag's gradient / bag length)."""
    gout = _arr(gout, np.float32)
    _, nt, dim = gout.shape
    order, bag, blen, runlen = (_arr(x, np.int32) for x in (order, bag, blen, runlen))
    sel = _arr(sel, np.int64)
    run_start = np.zeros(runlen.size + 1, dtype=np.int64)
    np.cumsum(runlen, out=run_start[1:])
    G = np.zeros((sel.size, dim), dtype=np.float64)
    Ga = np.zeros((sel.size, dim), dtype=np.float64)
    base = gout.ctypes.data + table * dim * 4
    lib().orc_run_grads_mean(_p(order), _p(bag), _p(blen), _p(run_start), _p(runlen), _p(sel), C.c_int64(sel.size),
                             C.c_void_p(base), C.c_int64(nt * dim), C.c_int32(dim), _p(G), _p(Ga))
    return G, Ga


def rowwise_adagrad_rows(W_rows: np.ndarray, state: np.ndarray, G: np.ndarray, lr: float, eps: float):
    """Returns (new rows, new accumulators); inputs are not modified."""
    W = _arr(W_rows, np.float32).copy()
    st = _arr(state, np.float32).copy()
    G = _arr(G, np.float64)
    lib().orc_rowwise_adagrad_rows(_p(W), _p(st), _p(G), C.c_float(lr), C.c_float(eps), C.c_int64(W.shape[0]),
                                   C.c_int32(W.shape[1]))
    return W, st


def embbag_bwd_opts(hotW: List[np.ndarray], state: Optional[List[np.ndarray]], n_samples: int,
                    slots: List[np.ndarray], offsets: List[Optional[np.ndarray]], gout: np.ndarray,
                    lr: float, eps: float = 0.0, pooling: int = POOL_SUM, optimizer: int = OPT_SGD):
    """Backward + optimizer with the chosen pooling and optimizer, in place on hotW[z] (and
    state[z] for Adagrad).  Returns per table (uniq, runlen, G fp64[U][dim], Gabs, w_old rows,
    state_old of the touched rows)."""
    res = []
    for z, W in enumerate(hotW):
        assert W.dtype == np.float32 and W.flags.c_contiguous
        s = _arr(slots[z], np.int32)
        order, uniq, runlen = sort_runs(s)
        bag = bag_of(offsets[z], n_samples, s.size)
        sel = np.arange(uniq.size)
        if pooling == POOL_MEAN:
            G, Ga = run_grads_mean(order, bag, bag_len(offsets[z], n_samples), runlen, sel, gout, z)
        else:
            G, Ga = run_grads(order, bag, runlen, sel, gout, z)
        w_old = W[uniq].copy()
        st_old = None
        if optimizer == OPT_ROWWISE_ADAGRAD:
            st_old = state[z][uniq].copy()
            W[uniq], state[z][uniq] = rowwise_adagrad_rows(w_old, st_old, G, lr, eps)
        else:
            W[uniq] = sgd_rows(w_old, G, lr)
        res.append((uniq, runlen, G, Ga, w_old, st_old))
    return res
