"""ctypes front-end of the plain CPU oracle (``skm_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
CPU-baseline leg of ``bench.py``.  The product path never imports this module
and this module never imports the product package.

Every function here is argument marshalling around one C function; the only
arithmetic done in Python is the random rotation (Algorithm 1, first line),
which is the QR factorisation of a seeded Gaussian matrix with the sign fixed
so that the triangular factor has a positive diagonal (Haar-distributed Q).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "skm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

MAX_ENTER = 32


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over points only)."""
    if force or (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Params(C.Structure):
    _fields_ = [
        ("dprime_frac", C.c_double),
        ("eps0", C.c_double),
        ("tau_group", C.c_int32),
        ("adjust_dprime", C.c_int32),
        ("adj_lo", C.c_double),
        ("adj_hi", C.c_double),
        ("adj_step", C.c_double),
        ("split_eps", C.c_double),
        ("final_assign", C.c_int32),
        ("etr", C.c_int32),
        ("nq", C.c_int32),
        ("topk", C.c_int32),
        ("probe_frac", C.c_double),
        ("etr_tol", C.c_double),
        ("etr_patience", C.c_int32),
        ("angular", C.c_int32),
        ("conv_tol", C.c_double),
    ]


class _TraceRow(C.Structure):
    _fields_ = [
        ("objective", C.c_double),
        ("prune_frac", C.c_double),
        ("recall", C.c_double),
        ("pruned_first", C.c_int64),
        ("nempty", C.c_int64),
        ("dprime", C.c_int32),
        ("pad", C.c_int32),
        ("enter", C.c_int64 * MAX_ENTER),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_rng_next.restype = C.c_uint64
        _lib.orc_rng_next.argtypes = [C.POINTER(C.c_uint64)]
        _lib.orc_rng_stream.restype = C.c_uint64
        _lib.orc_rng_stream.argtypes = [C.c_uint64, C.c_uint64]
        _lib.orc_theta_ratio.restype = C.c_double
        _lib.orc_theta_ratio.argtypes = [C.c_int32, C.c_int32, C.c_double]
        _lib.orc_dprime_init.restype = C.c_int32
        _lib.orc_dprime_init.argtypes = [C.c_int32, C.c_double]
        _lib.orc_dprime_adjust.restype = C.c_int32
        _lib.orc_dprime_adjust.argtypes = [C.c_int32, C.c_int32] + [C.c_double] * 4
        _lib.orc_hier_meso_count.restype = C.c_int32
        _lib.orc_hier_meso_count.argtypes = [C.c_int32]
        _lib.orc_hier_alloc.restype = None
        _lib.orc_hier_alloc.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        _lib.orc_nprobe.restype = C.c_int32
        _lib.orc_nprobe.argtypes = [C.c_int32, C.c_double]
        _lib.orc_recall.restype = C.c_double
        _lib.orc_split_empty.restype = C.c_int32
        _lib.orc_sample_rows.restype = C.c_int
        _lib.orc_fit.restype = C.c_int32
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


# ---------------------------------------------------------------- PRNG / init
def rng_stream(seed: int, stream: int) -> int:
    return int(lib().orc_rng_stream(C.c_uint64(seed), C.c_uint64(stream)))


def rng_draws(state: int, count: int):
    st = C.c_uint64(state)
    out = [int(lib().orc_rng_next(C.byref(st))) for _ in range(count)]
    return out, int(st.value)


def sample_rows(seed: int, n: int, k: int, stream: int = 0) -> np.ndarray:
    """k distinct row indices (Section 3.1, centroid initialisation)."""
    idx = np.empty(k, dtype=np.int64)
    rc = lib().orc_sample_rows(C.c_uint64(seed), C.c_uint64(stream), C.c_int64(n), C.c_int32(k),
                               _p(idx, C.c_int64))
    if rc != 0:
        raise ValueError("orc_sample_rows failed (k > n?)")
    return idx


# ---------------------------------------------------------------- scalars
def theta_ratio(d: int, t: int, eps0: float) -> float:
    return float(lib().orc_theta_ratio(d, t, eps0))


def dprime_init(d: int, frac: float = 0.125) -> int:
    return int(lib().orc_dprime_init(d, frac))


def dprime_adjust(d: int, dprime: int, f: float, lo=0.95, hi=0.97, step=0.20) -> int:
    return int(lib().orc_dprime_adjust(d, dprime, f, lo, hi, step))


def nprobe(k: int, probe_frac: float) -> int:
    return int(lib().orc_nprobe(k, probe_frac))


# ---------------------------------------------------------------- rotation
def random_rotation(d: int, seed: int) -> np.ndarray:
    """Haar-distributed orthogonal d x d matrix, fp32 (Algorithm 1, line 1)."""
    g = np.random.default_rng(seed).standard_normal((d, d))
    q, r = np.linalg.qr(g)
    q = q * np.sign(np.diag(r))[None, :]
    return q.astype(np.float32)


def rotate(X, R) -> np.ndarray:
    X = _f32(X)
    R = _f32(R)
    n, d = X.shape
    out = np.empty((n, d), dtype=np.float64)
    lib().orc_rotate(_p(X, C.c_float), C.c_int64(n), C.c_int32(d), _p(R, C.c_float), _p(out, C.c_double))
    return out


def unrotate(Yr, R) -> np.ndarray:
    Yr = _f64(Yr)
    R = _f32(R)
    k, d = Yr.shape
    out = np.empty((k, d), dtype=np.float64)
    lib().orc_unrotate(_p(Yr, C.c_double), C.c_int32(k), C.c_int32(d), _p(R, C.c_float), _p(out, C.c_double))
    return out


# ---------------------------------------------------------------- steps
def assign_full(Xr, Y):
    Xr = _f64(Xr)
    Y = _f64(Y)
    n, d = Xr.shape
    k = Y.shape[0]
    a = np.empty(n, dtype=np.int32)
    dist = np.empty(n, dtype=np.float64)
    lib().orc_assign_full(_p(Xr, C.c_double), C.c_int64(n), C.c_int32(d), _p(Y, C.c_double), C.c_int32(k),
                          _p(a, C.c_int32), _p(dist, C.c_double))
    return a, dist


@dataclass
class PrunedResult:
    assign: np.ndarray
    dist: np.ndarray
    pruned_first: int
    enter: np.ndarray  # pairs entering trailing block m; last entry = completed
    fate: np.ndarray | None = None


def assign_pruned(Xr, Y, prev, dprime: int, eps0: float = 2.1, G: int = 0, want_fate: bool = False) -> PrunedResult:
    Xr = _f64(Xr)
    Y = _f64(Y)
    n, d = Xr.shape
    k = Y.shape[0]
    if G <= 0:
        G = k
    prev_a = None if prev is None else _i32(prev)
    a = np.empty(n, dtype=np.int32)
    dist = np.empty(n, dtype=np.float64)
    nb = (d - dprime + 63) // 64
    enter = np.zeros(nb + 1, dtype=np.int64)
    pf = C.c_int64(0)
    fate = np.full((n, k), -1, dtype=np.int32) if want_fate else None
    lib().orc_assign_pruned(_p(Xr, C.c_double), C.c_int64(n), C.c_int32(d), _p(Y, C.c_double), C.c_int32(k),
                            _p(prev_a, C.c_int32), C.c_int32(dprime), C.c_double(eps0), C.c_int32(G),
                            _p(a, C.c_int32), _p(dist, C.c_double), C.byref(pf), _p(enter, C.c_int64),
                            _p(fate, C.c_int32))
    return PrunedResult(a, dist, int(pf.value), enter, fate)


def update(Xr, assign, Y_old):
    """Means of the assigned points; empty clusters keep Y_old's row."""
    Xr = _f64(Xr)
    n, d = Xr.shape
    Y = _f64(Y_old).copy()
    k = Y.shape[0]
    a = _i32(assign)
    counts = np.zeros(k, dtype=np.int64)
    lib().orc_update(_p(Xr, C.c_double), C.c_int64(n), C.c_int32(d), _p(a, C.c_int32), C.c_int32(k),
                     _p(Y, C.c_double), _p(counts, C.c_int64))
    return Y, counts


def split_empty(Y, counts, rng_state: int, eps: float = 1.0 / 1024.0):
    Y = _f64(Y).copy()
    counts = _i64(counts).copy()
    k, d = Y.shape
    st = C.c_uint64(rng_state)
    log = np.zeros((k, 2), dtype=np.int32)
    ns = lib().orc_split_empty(_p(Y, C.c_double), _p(counts, C.c_int64), C.c_int32(k), C.c_int32(d), C.byref(st),
                               C.c_double(eps), _p(log, C.c_int32))
    return Y, counts, log[:ns].copy(), int(st.value)


def ground_truth(X, Q, K: int) -> np.ndarray:
    X = _f32(X)
    Q = _f32(Q)
    n, d = X.shape
    nq = Q.shape[0]
    gt = np.empty((nq, K), dtype=np.int64)
    lib().orc_ground_truth(_p(X, C.c_float), C.c_int64(n), C.c_int32(d), _p(Q, C.c_float), C.c_int32(nq),
                           C.c_int32(K), _p(gt, C.c_int64))
    return gt


def recall(Qr, Y, nprobe_: int, gt, assign) -> float:
    Qr = _f64(Qr)
    Y = _f64(Y)
    gt = _i64(gt)
    a = _i32(assign)
    nq, d = Qr.shape
    k = Y.shape[0]
    return float(lib().orc_recall(_p(Qr, C.c_double), C.c_int32(nq), C.c_int32(d), _p(Y, C.c_double), C.c_int32(k),
                                  C.c_int32(nprobe_), _p(gt, C.c_int64), C.c_int32(gt.shape[1]),
                                  _p(a, C.c_int32)))


# ---------------------------------------------------------------- whole fit
@dataclass
class FitParams:
    dprime_frac: float = 0.125
    eps0: float = 2.1
    tau_group: int = 0
    adjust_dprime: bool = True
    adj_lo: float = 0.95
    adj_hi: float = 0.97
    adj_step: float = 0.20
    split_eps: float = 1.0 / 1024.0
    final_assign: bool = True
    etr: bool = False
    topk: int = 10
    probe_frac: float = 0.01
    etr_tol: float = 0.005
    etr_patience: int = 2
    angular: bool = False          # spherical k-means: unit points, centroids renormalised after every update
    conv_tol: float = 0.0          # > 0: stop after an iteration t >= 2 in which <= conv_tol * n labels changed


@dataclass
class FitResult:
    centroids: np.ndarray          # k x d, original space, fp64
    centroids_rot: np.ndarray      # k x d, rotated space, fp64
    assign: np.ndarray
    dist: np.ndarray
    iters_run: int
    trace: list = field(default_factory=list)   # dict per assignment step


def fit(X, k: int, iters: int, seed: int, params: FitParams | None = None, R=None, init_idx=None,
        queries=None, gt=None) -> FitResult:
    p = params or FitParams()
    X = _f32(X)
    n, d = X.shape
    if init_idx is None:
        init_idx = sample_rows(seed, n, k, 0)
    init_idx = _i64(init_idx)
    Rm = None if R is None else _f32(R)
    cp = _Params(p.dprime_frac, p.eps0, p.tau_group, int(p.adjust_dprime), p.adj_lo, p.adj_hi, p.adj_step,
                 p.split_eps, int(p.final_assign), int(p.etr), 0 if queries is None else int(len(queries)), p.topk,
                 p.probe_frac, p.etr_tol, p.etr_patience, int(p.angular), p.conv_tol)
    Q = None
    G = None
    if p.etr:
        Q = _f32(queries)
        G = _i64(gt if gt is not None else ground_truth(X, Q, p.topk))
    Y = np.empty((k, d), dtype=np.float64)
    Yr = np.empty((k, d), dtype=np.float64)
    a = np.empty(n, dtype=np.int32)
    dist = np.empty(n, dtype=np.float64)
    trace = (_TraceRow * (iters + 1))()
    run = lib().orc_fit(_p(X, C.c_float), C.c_int64(n), C.c_int32(d), C.c_int32(k), C.c_int32(iters),
                        C.c_uint64(seed), C.byref(cp), _p(Rm, C.c_float), _p(init_idx, C.c_int64),
                        _p(Q, C.c_float), _p(G, C.c_int64), _p(Y, C.c_double), _p(Yr, C.c_double),
                        _p(a, C.c_int32), _p(dist, C.c_double), trace)
    if run < 0:
        raise RuntimeError(f"orc_fit failed: {run}")
    rows = []
    nrows = run + (1 if p.final_assign else 0)
    for t in range(nrows):
        r = trace[t]
        rows.append(dict(objective=r.objective, prune_frac=r.prune_frac, recall=r.recall,
                         pruned_first=int(r.pruned_first), nempty=int(r.nempty), dprime=int(r.dprime),
                         enter=np.array(list(r.enter), dtype=np.int64)))
    return FitResult(Y, Yr, a, dist, int(run), rows)


def fit_sampled(X, k: int, iters: int, seed: int, sample_frac: float, params: FitParams | None = None, R=None):
    """Sampled fit (Section 4.4): Algorithm 1 on a uniform sample of round(frac * n) rows (at least k; stream 4 of
    the seed, rows kept in ascending order), then every point is assigned to the final centroids by the two-phase
    step without a previous assignment.  A composition of the steps above; returns (FitResult of the sample with
    assign/dist replaced by those of all points, sample indices)."""
    import dataclasses
    p = params or FitParams()
    X = _f32(X)
    n, d = X.shape
    s = min(max(int(np.floor(sample_frac * n + 0.5)), k), n)
    idx = np.sort(sample_rows(seed, n, s, stream=4))
    inner = fit(X[idx], k, iters, seed, dataclasses.replace(p, final_assign=False), R=R)
    last = inner.trace[-1]
    dp = dprime_init(d, p.dprime_frac)
    if inner.iters_run >= 2:
        dp = last["dprime"]
        if p.adjust_dprime and k > 1:
            dp = dprime_adjust(d, dp, last["prune_frac"], p.adj_lo, p.adj_hi, p.adj_step)
    Xr = rotate(X, R) if R is not None else X.astype(np.float64)
    fin = assign_pruned(Xr, inner.centroids_rot, None, dp, p.eps0, p.tau_group)
    inner.assign, inner.dist = fin.assign, fin.dist
    inner.trace.append(dict(objective=float(fin.dist.sum()), prune_frac=fin.pruned_first / (n * max(k - 1, 1)),
                            recall=-1.0, pruned_first=fin.pruned_first, nempty=0, dprime=dp, enter=fin.enter))
    return inner, idx


def hier_meso_count(k: int) -> int:
    return int(lib().orc_hier_meso_count(k))


def hier_alloc(sizes, k: int) -> np.ndarray:
    """Fine cluster count of every meso-cluster (Section 6; shares of k in proportion to sqrt(n_i))."""
    sizes = _i64(sizes)
    counts = np.zeros(len(sizes), dtype=np.int32)
    lib().orc_hier_alloc(_p(sizes, C.c_int64), len(sizes), k, _p(counts, C.c_int32))
    return counts


def fit_hierarchical(X, k: int, seed: int, meso_iters: int = 3, fine_iters: int = 5, params: FitParams | None = None,
                     R=None):
    """Hierarchical SuperKMeans (Section 6), composed from the steps above.  MESO: Algorithm 1 with sqrt(k) clusters
    on all (rotated) points, `meso_iters` iterations and the final assignment pass.  FINE: inside meso-cluster i
    (its points in ascending row order), Algorithm 1 with hier_alloc's count, `fine_iters` iterations, seed
    `seed + 1 + i`, no final pass.  The k fine centroids, in meso order, are the result; every point is then assigned
    to them by the two-phase step without a previous assignment.
    Returns dict(centroids, centroids_rot, assign, dist, meso_assign, meso_sizes, fine_counts, meso)."""
    import dataclasses
    p = params or FitParams()
    X = _f32(X)
    n, d = X.shape
    km = hier_meso_count(k)
    meso = fit(X, km, meso_iters, seed, dataclasses.replace(p, final_assign=True), R=R)
    Xr = rotate(X, R) if R is not None else X.astype(np.float64)
    sizes = np.bincount(meso.assign, minlength=km).astype(np.int64)
    counts = hier_alloc(sizes, k)
    Y = np.zeros((k, d), dtype=np.float64)
    off = 0
    for i in range(km):
        if counts[i] == 0:
            continue
        rows = np.nonzero(meso.assign == i)[0]
        sub = fit(Xr[rows], int(counts[i]), fine_iters, (seed + 1 + i) & 0xFFFFFFFFFFFFFFFF,
                  dataclasses.replace(p, final_assign=False), R=None)
        Y[off:off + counts[i]] = sub.centroids_rot
        off += int(counts[i])
    assert off == k
    fin = assign_pruned(Xr, Y, None, dprime_init(d, p.dprime_frac), p.eps0, p.tau_group)
    return dict(centroids=unrotate(Y, R) if R is not None else Y.copy(), centroids_rot=Y, assign=fin.assign, dist=fin.dist,
                meso_assign=meso.assign, meso_sizes=sizes, fine_counts=counts, meso=meso,
                objective=float(fin.dist.sum()), prune_frac=fin.pruned_first / (n * max(k - 1, 1)))
