"""Thin ctypes binding of ``libskm.so`` (argument marshalling only).

Every function takes torch CUDA tensors (device memory and the current stream
come from torch; no arithmetic happens here) and calls the C entry point of the
same name declared in ``include/skm.h``.  There is no CPU fallback: if the
library has not been built, or no GPU is present, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field

import torch  # loads the HIP runtime that libskm.so binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libskm.so")
MAX_BLOCKS = 32


class TraceRow(C.Structure):
    _fields_ = [
        ("objective", C.c_double), ("prune_frac", C.c_double), ("recall", C.c_double),
        ("survivors", C.c_int64), ("completed", C.c_int64), ("changed", C.c_int64), ("nempty", C.c_int64),
        ("dense_dims", C.c_int64), ("dense_pair_blocks", C.c_int64),
        ("gather_pair_blocks", C.c_int64), ("gather_pairs", C.c_int64),
        ("screen_dims", C.c_int64), ("listed_tiles", C.c_int64),
        ("dprime", C.c_int32), ("nblocks", C.c_int32),
        ("enter", C.c_int64 * MAX_BLOCKS),
        ("ms_tau", C.c_float), ("ms_gemm", C.c_float), ("ms_prune", C.c_float), ("ms_update", C.c_float),
        ("ms_etr", C.c_float), ("ms_step", C.c_float),
    ]


class Trace(C.Structure):
    _fields_ = [
        ("capacity", C.c_int32), ("rows", C.c_int32), ("iters_run", C.c_int32), ("inc_updates", C.c_int32),
        ("ms_rotate", C.c_float), ("ms_init", C.c_float), ("ms_etr_gt", C.c_float), ("ms_unrotate", C.c_float),
        ("ms_total", C.c_float), ("ms_host_total", C.c_float), ("ms_host_alloc", C.c_float), ("ms_host_free", C.c_float),
        ("row", C.POINTER(TraceRow)),
    ]


class Params(C.Structure):
    _fields_ = [
        ("dprime_frac", C.c_float), ("eps0", C.c_float), ("adjust_dprime", C.c_int32),
        ("adj_lo", C.c_float), ("adj_hi", C.c_float), ("adj_step", C.c_float), ("split_eps", C.c_float),
        ("final_assign", C.c_int32), ("block_stats", C.c_int32), ("rotate", C.c_int32),
        ("R", C.c_void_p), ("init_idx", C.c_void_p),
        ("etr", C.c_int32), ("nq", C.c_int32), ("topk", C.c_int32),
        ("probe_frac", C.c_float), ("etr_tol", C.c_float), ("etr_patience", C.c_int32),
        ("queries", C.c_void_p), ("gt", C.c_void_p),
        ("stream", C.c_void_p), ("trace", C.POINTER(Trace)), ("pair_budget", C.c_int64),
        ("dense_frac", C.c_float), ("sample_frac", C.c_float), ("angular", C.c_int32), ("full_update", C.c_int32),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_int64), ("conv_tol", C.c_float), ("screen", C.c_int32),
        ("tau_group", C.c_int32),
    ]


EXPORTS = [
    "skm_params_default", "skm_fit", "skm_fit_ex", "skm_assign", "skm_assign_ex", "skm_assign_exact", "skm_update",
    "skm_make_rotation", "skm_rotate", "skm_sample_rows", "skm_theta_ratio", "skm_dprime_init", "skm_dprime_adjust",
    "skm_strerror", "skm_last_error", "skm_version", "skm_fit_hierarchical", "skm_hier_meso_count", "skm_hier_alloc",
    "skm_fit_host", "skm_workspace_bytes", "skm_hier_workspace_bytes", "skm_debug_gemm_config",
    "skm_assign_exact_static", "skm_etr_ground_truth",
]

_lib = None


def lib():
    """Load libskm.so (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: run `python -m paper_2603_20009_amd.build` first")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float
        L.skm_params_default.argtypes = [C.POINTER(Params)]
        L.skm_params_default.restype = None
        L.skm_fit.argtypes = [vp, i64, i32, i32, i32, u64, vp, vp]
        L.skm_fit_ex.argtypes = [vp, i64, i32, i32, i32, u64, C.POINTER(Params), vp, vp, vp]
        L.skm_assign.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp]
        L.skm_assign_ex.argtypes = [vp, i64, i32, vp, i32, vp, i32, C.POINTER(Params), vp, vp]
        L.skm_assign_exact.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp]
        L.skm_assign_exact_static.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp]
        L.skm_assign_exact_static.restype = C.c_int
        L.skm_update.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp]
        L.skm_make_rotation.argtypes = [i32, u64, vp, vp]
        L.skm_rotate.argtypes = [vp, i64, i32, vp, i32, vp, vp]
        L.skm_sample_rows.argtypes = [u64, i64, i32, vp]
        L.skm_fit_hierarchical.argtypes = [vp, i64, i32, i32, i32, i32, u64, C.POINTER(Params), vp, vp, vp, vp, vp]
        L.skm_fit_host.argtypes = [vp, i64, i32, i32, i32, u64, C.POINTER(Params), i64, vp, vp, vp]
        L.skm_hier_meso_count.argtypes = [i32]
        L.skm_hier_meso_count.restype = i32
        L.skm_hier_alloc.argtypes = [vp, i32, i32, vp]
        L.skm_workspace_bytes.argtypes = [i64, i32, i32, C.POINTER(Params)]
        L.skm_workspace_bytes.restype = i64
        L.skm_hier_workspace_bytes.argtypes = [i64, i32, i32, C.POINTER(Params)]
        L.skm_hier_workspace_bytes.restype = i64
        L.skm_etr_ground_truth.argtypes = [vp, i64, i32, vp, i32, i32, vp, vp]
        L.skm_etr_ground_truth.restype = C.c_int
        L.skm_debug_gemm_config.argtypes = [i32, i32, i64]
        L.skm_debug_gemm_config.restype = None
        for f in ("skm_fit", "skm_fit_ex", "skm_assign", "skm_assign_ex", "skm_assign_exact", "skm_update",
                  "skm_make_rotation", "skm_rotate", "skm_sample_rows", "skm_fit_hierarchical", "skm_hier_alloc",
                  "skm_fit_host"):
            getattr(L, f).restype = C.c_int
        L.skm_theta_ratio.argtypes = [i32, i32, f32]
        L.skm_theta_ratio.restype = f32
        L.skm_dprime_init.argtypes = [i32, f32]
        L.skm_dprime_init.restype = i32
        L.skm_dprime_adjust.argtypes = [i32, i32, C.c_double, f32, f32, f32]
        L.skm_dprime_adjust.restype = i32
        for f in ("skm_strerror", "skm_last_error", "skm_version"):
            getattr(L, f).restype = C.c_char_p
        L.skm_strerror.argtypes = [C.c_int]
        _lib = L
    return _lib


class SkmError(RuntimeError):
    pass


def _check(rc: int):
    if rc != 0:
        L = lib()
        raise SkmError(f"libskm error {rc} ({L.skm_strerror(rc).decode()}): {L.skm_last_error().decode()}")


def _dev(t: torch.Tensor, dtype, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a CUDA tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


@dataclass
class FitOptions:
    dprime_frac: float = 0.125
    eps0: float = 2.1
    adjust_dprime: bool = True
    adj_lo: float = 0.95
    adj_hi: float = 0.97
    adj_step: float = 0.20
    split_eps: float = 1.0 / 1024.0
    final_assign: bool = True
    block_stats: bool = False
    rotate: bool = True
    R: torch.Tensor | None = None            # device d x d
    init_idx: object = None                  # host sequence of k ints
    etr: bool = False
    nq: int = 1000
    topk: int = 10
    probe_frac: float = 0.01
    etr_tol: float = 0.005
    etr_patience: int = 2
    queries: torch.Tensor | None = None      # device nq x d
    gt: torch.Tensor | None = None           # device nq x topk int64
    pair_budget: int = 0
    dense_frac: float = 0.0125
    sample_frac: float = 0.0
    angular: bool = False
    full_update: bool = False
    conv_tol: float = 0.0
    tau_group: int = 0
    screen: int = 0                          # low-precision first filter: 0 = by the previous step's prune fraction, 1 = always, -1 = never
    own_workspace: bool = False              # True: the library allocates and frees its workspace inside the call
    workspace: "torch.Tensor | None" = None  # a uint8 device tensor to lend as is (default: one of workspace_bytes())


@dataclass
class FitResult:
    centroids: torch.Tensor
    assign: torch.Tensor
    dist: torch.Tensor
    iters_run: int
    trace: list = field(default_factory=list)
    timing: dict = field(default_factory=dict)


def _row_dict(r: TraceRow) -> dict:
    return dict(objective=r.objective, prune_frac=r.prune_frac, recall=r.recall, survivors=int(r.survivors),
                completed=int(r.completed), changed=int(r.changed), nempty=int(r.nempty),
                dense_dims=int(r.dense_dims), dense_pair_blocks=int(r.dense_pair_blocks),
                gather_pair_blocks=int(r.gather_pair_blocks), gather_pairs=int(r.gather_pairs),
                screen_dims=int(r.screen_dims), listed_tiles=int(r.listed_tiles), dprime=int(r.dprime),
                nblocks=int(r.nblocks), enter=[int(v) for v in r.enter], ms_tau=r.ms_tau, ms_gemm=r.ms_gemm,
                ms_prune=r.ms_prune, ms_update=r.ms_update, ms_etr=r.ms_etr, ms_step=r.ms_step)


def _params(o: FitOptions, keep: list, trace: Trace | None) -> Params:
    p = Params()
    lib().skm_params_default(C.byref(p))
    p.dprime_frac, p.eps0 = o.dprime_frac, o.eps0
    p.adjust_dprime = int(o.adjust_dprime)
    p.adj_lo, p.adj_hi, p.adj_step, p.split_eps = o.adj_lo, o.adj_hi, o.adj_step, o.split_eps
    p.final_assign, p.block_stats, p.rotate = int(o.final_assign), int(o.block_stats), int(o.rotate)
    if o.R is not None:
        p.R = _dev(o.R, torch.float32, "R").value
    if o.init_idx is not None:
        arr = (C.c_int64 * len(o.init_idx))(*[int(v) for v in o.init_idx])
        keep.append(arr)
        p.init_idx = C.cast(arr, C.c_void_p).value
    p.etr, p.nq, p.topk = int(o.etr), o.nq, o.topk
    p.probe_frac, p.etr_tol, p.etr_patience = o.probe_frac, o.etr_tol, o.etr_patience
    if o.queries is not None:
        p.queries = _dev(o.queries, torch.float32, "queries").value
        p.nq = o.queries.shape[0]
    if o.gt is not None:
        p.gt = _dev(o.gt, torch.int64, "gt").value
    p.stream = _stream().value
    if trace is not None:
        p.trace = C.pointer(trace)
    p.pair_budget = o.pair_budget
    p.dense_frac = o.dense_frac
    p.sample_frac = o.sample_frac
    p.angular = int(o.angular)
    p.full_update = int(o.full_update)
    p.conv_tol = o.conv_tol
    p.tau_group = o.tau_group
    p.screen = o.screen
    return p


def workspace_bytes(n: int, d: int, k: int, p: Params | None = None) -> int:
    """skm_workspace_bytes: device bytes a fit / assignment call of this shape needs as workspace."""
    nbytes = int(lib().skm_workspace_bytes(n, d, k, None if p is None else C.byref(p)))
    if nbytes < 0:
        _check(nbytes)
    return nbytes


def hier_workspace_bytes(n: int, d: int, k: int, p: Params | None = None) -> int:
    """skm_hier_workspace_bytes: device bytes a hierarchical fit of this shape needs as workspace."""
    nbytes = int(lib().skm_hier_workspace_bytes(n, d, k, None if p is None else C.byref(p)))
    if nbytes < 0:
        _check(nbytes)
    return nbytes


def _lend_workspace(p: Params, o: FitOptions, n: int, d: int, k: int, device, keep: list, hierarchical: bool = False):
    """The workspace as a torch tensor (device memory is torch's business: its caching allocator hands the same block
    to the next call, so repeated fits allocate nothing)."""
    if o.own_workspace:
        return
    if o.workspace is not None:
        ws = _dev(o.workspace, torch.uint8, "workspace")
        keep.append(o.workspace)
        p.workspace = ws.value
        p.workspace_bytes = o.workspace.numel()
        return
    nbytes = hier_workspace_bytes(n, d, k, p) if hierarchical else workspace_bytes(n, d, k, p)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    keep.append(ws)
    p.workspace = ws.data_ptr()
    p.workspace_bytes = nbytes


def _new_trace(rows: int, keep: list) -> Trace:
    arr = (TraceRow * rows)()
    keep.append(arr)
    t = Trace()
    t.capacity = rows
    t.row = C.cast(arr, C.POINTER(TraceRow))
    return t


def fit(X: torch.Tensor, k: int, iters: int, seed: int, opts: FitOptions | None = None) -> FitResult:
    """skm_fit_ex: Algorithm 1 on device-resident X (n x d fp32)."""
    o = opts or FitOptions()
    n, d = X.shape
    keep: list = []
    tr = _new_trace(iters + 1, keep)
    p = _params(o, keep, tr)
    _lend_workspace(p, o, n, d, k, X.device, keep)
    cent = torch.empty((k, d), device=X.device, dtype=torch.float32)
    assign = torch.empty(n, device=X.device, dtype=torch.int32)
    dist = torch.empty(n, device=X.device, dtype=torch.float32)
    rc = lib().skm_fit_ex(_dev(X, torch.float32, "X"), n, d, k, iters, C.c_uint64(seed), C.byref(p),
                          C.c_void_p(cent.data_ptr()), C.c_void_p(assign.data_ptr()), C.c_void_p(dist.data_ptr()))
    _check(rc)
    rows = [_row_dict(tr.row[i]) for i in range(tr.rows)]
    timing = dict(ms_rotate=tr.ms_rotate, ms_init=tr.ms_init, ms_etr_gt=tr.ms_etr_gt, ms_unrotate=tr.ms_unrotate,
                  ms_total=tr.ms_total, inc_updates=int(tr.inc_updates), ms_host_total=tr.ms_host_total,
                  ms_host_alloc=tr.ms_host_alloc, ms_host_free=tr.ms_host_free)
    return FitResult(cent, assign, dist, int(tr.iters_run), rows, timing)


def fit_hierarchical(X: torch.Tensor, k: int, seed: int, meso_iters: int = 3, fine_iters: int = 5,
                     opts: FitOptions | None = None):
    """skm_fit_hierarchical (Section 6).  Returns (FitResult, meso_sizes, fine_counts); the trace holds the rows of
    the meso phase and the row of the final assignment."""
    o = opts or FitOptions()
    n, d = X.shape
    km = hier_meso_count(k)
    keep: list = []
    tr = _new_trace(meso_iters + 2, keep)
    p = _params(o, keep, tr)
    _lend_workspace(p, o, n, d, k, X.device, keep, hierarchical=True)
    cent = torch.empty((k, d), device=X.device, dtype=torch.float32)
    assign = torch.empty(n, device=X.device, dtype=torch.int32)
    dist = torch.empty(n, device=X.device, dtype=torch.float32)
    sizes = (C.c_int64 * km)()
    counts = (C.c_int32 * km)()
    rc = lib().skm_fit_hierarchical(_dev(X, torch.float32, "X"), n, d, k, meso_iters, fine_iters, C.c_uint64(seed),
                                    C.byref(p), C.c_void_p(cent.data_ptr()), C.c_void_p(assign.data_ptr()),
                                    C.c_void_p(dist.data_ptr()), C.cast(sizes, C.c_void_p), C.cast(counts, C.c_void_p))
    _check(rc)
    rows = [_row_dict(tr.row[i]) for i in range(tr.rows)]
    timing = dict(ms_meso=tr.ms_init, ms_fine=tr.ms_etr_gt, ms_total=tr.ms_total)
    return FitResult(cent, assign, dist, int(tr.iters_run), rows, timing), list(sizes), list(counts)


def fit_host(X_host: torch.Tensor, k: int, iters: int, seed: int, batch_rows: int = 0, opts: FitOptions | None = None,
             device: str = "cuda") -> FitResult:
    """skm_fit_host (Section 7.1): Algorithm 1 on points that stay in host memory (a CPU tensor, page-locked for
    copies that overlap the kernels) and pass through the device in batches of `batch_rows` rows.  The centroids come
    back on the device, the labels and distances as CPU tensors."""
    o = opts or FitOptions()
    if X_host.device.type != "cpu" or X_host.dtype != torch.float32 or not X_host.is_contiguous():
        raise ValueError("X_host must be a contiguous fp32 CPU tensor")
    n, d = X_host.shape
    keep: list = []
    tr = _new_trace(iters + 1, keep)
    p = _params(o, keep, tr)
    cent = torch.empty((k, d), device=device, dtype=torch.float32)
    assign = torch.empty(n, dtype=torch.int32, pin_memory=True)
    dist = torch.empty(n, dtype=torch.float32, pin_memory=True)
    rc = lib().skm_fit_host(C.c_void_p(X_host.data_ptr()), n, d, k, iters, C.c_uint64(seed), C.byref(p), batch_rows,
                            C.c_void_p(cent.data_ptr()), C.c_void_p(assign.data_ptr()), C.c_void_p(dist.data_ptr()))
    _check(rc)
    rows = [_row_dict(tr.row[i]) for i in range(tr.rows)]
    timing = dict(ms_init=tr.ms_init, ms_unrotate=tr.ms_unrotate, ms_total=tr.ms_total)
    return FitResult(cent, assign, dist, int(tr.iters_run), rows, timing)


def fit_default(X: torch.Tensor, k: int, iters: int, seed: int):
    """skm_fit: default parameters, default stream."""
    n, d = X.shape
    cent = torch.empty((k, d), device=X.device, dtype=torch.float32)
    assign = torch.empty(n, device=X.device, dtype=torch.int32)
    torch.cuda.synchronize()
    _check(lib().skm_fit(_dev(X, torch.float32, "X"), n, d, k, iters, C.c_uint64(seed), C.c_void_p(cent.data_ptr()),
                         C.c_void_p(assign.data_ptr())))
    return cent, assign


def assign(X: torch.Tensor, centroids: torch.Tensor, prev: torch.Tensor | None = None, dprime: int = 0,
           opts: FitOptions | None = None):
    """skm_assign_ex: one two-phase assignment step.  Returns (assign, dist, trace_row)."""
    o = opts or FitOptions()
    n, d = X.shape
    k = centroids.shape[0]
    keep: list = []
    tr = _new_trace(1, keep)
    p = _params(o, keep, tr)
    _lend_workspace(p, o, n, d, k, X.device, keep)
    a = torch.empty(n, device=X.device, dtype=torch.int32)
    dist = torch.empty(n, device=X.device, dtype=torch.float32)
    pv = None if prev is None else _dev(prev, torch.int32, "prev")
    rc = lib().skm_assign_ex(_dev(X, torch.float32, "X"), n, d, _dev(centroids, torch.float32, "centroids"), k, pv,
                             dprime, C.byref(p), C.c_void_p(a.data_ptr()), C.c_void_p(dist.data_ptr()))
    _check(rc)
    return a, dist, _row_dict(tr.row[0])


def assign_default(X: torch.Tensor, centroids: torch.Tensor, prev: torch.Tensor | None = None):
    """skm_assign: default parameters, default stream, rotation from seed 0."""
    n, d = X.shape
    k = centroids.shape[0]
    a = torch.empty(n, device=X.device, dtype=torch.int32)
    dist = torch.empty(n, device=X.device, dtype=torch.float32)
    pv = None if prev is None else _dev(prev, torch.int32, "prev")
    torch.cuda.synchronize()
    _check(lib().skm_assign(_dev(X, torch.float32, "X"), n, d, _dev(centroids, torch.float32, "centroids"), k, pv,
                            C.c_void_p(a.data_ptr()), C.c_void_p(dist.data_ptr())))
    return a, dist


def assign_exact(X: torch.Tensor, centroids: torch.Tensor):
    n, d = X.shape
    k = centroids.shape[0]
    a = torch.empty(n, device=X.device, dtype=torch.int32)
    dist = torch.empty(n, device=X.device, dtype=torch.float32)
    _check(lib().skm_assign_exact(_dev(X, torch.float32, "X"), n, d, _dev(centroids, torch.float32, "centroids"), k,
                                  _stream(), C.c_void_p(a.data_ptr()), C.c_void_p(dist.data_ptr())))
    return a, dist


def assign_exact_static(X: torch.Tensor, centroids: torch.Tensor, out=None):
    """skm_assign_exact_static: the exact step with no device allocation inside the call (outputs are the caller's)."""
    n, d = X.shape
    k = centroids.shape[0]
    a, dist = out if out is not None else (torch.empty(n, device=X.device, dtype=torch.int32),
                                           torch.empty(n, device=X.device, dtype=torch.float32))
    _check(lib().skm_assign_exact_static(_dev(X, torch.float32, "X"), n, d, _dev(centroids, torch.float32, "centroids"),
                                         k, _stream(), C.c_void_p(a.data_ptr()), C.c_void_p(dist.data_ptr())))
    return a, dist


def update(X: torch.Tensor, assign_: torch.Tensor, centroids: torch.Tensor):
    """skm_update: in-place mean update of `centroids`; returns the cluster sizes."""
    n, d = X.shape
    k = centroids.shape[0]
    counts = torch.empty(k, device=X.device, dtype=torch.int32)
    _check(lib().skm_update(_dev(X, torch.float32, "X"), n, d, _dev(assign_, torch.int32, "assign"), k, _stream(),
                            _dev(centroids, torch.float32, "centroids"), C.c_void_p(counts.data_ptr())))
    return counts


def etr_ground_truth(X: torch.Tensor, queries: torch.Tensor, topk: int) -> torch.Tensor:
    """skm_etr_ground_truth: nq x topk int64 indices of the nearest points of every query."""
    n, d = X.shape
    nq = queries.shape[0]
    gt = torch.empty((nq, topk), device=X.device, dtype=torch.int64)
    _check(lib().skm_etr_ground_truth(_dev(X, torch.float32, "X"), n, d, _dev(queries, torch.float32, "queries"), nq,
                                      topk, _stream(), C.c_void_p(gt.data_ptr())))
    return gt


def make_rotation(d: int, seed: int, device="cuda") -> torch.Tensor:
    R = torch.empty((d, d), device=device, dtype=torch.float32)
    _check(lib().skm_make_rotation(d, C.c_uint64(seed), _stream(), C.c_void_p(R.data_ptr())))
    return R


def rotate(X: torch.Tensor, R: torch.Tensor, transpose: bool = False) -> torch.Tensor:
    n, d = X.shape
    out = torch.empty((n, d), device=X.device, dtype=torch.float32)
    _check(lib().skm_rotate(_dev(X, torch.float32, "X"), n, d, _dev(R, torch.float32, "R"), int(transpose), _stream(),
                            C.c_void_p(out.data_ptr())))
    return out


def sample_rows(seed: int, n: int, k: int):
    arr = (C.c_int64 * k)()
    _check(lib().skm_sample_rows(C.c_uint64(seed), n, k, C.cast(arr, C.c_void_p)))
    return list(arr)


def hier_meso_count(k: int) -> int:
    return int(lib().skm_hier_meso_count(k))


def hier_alloc(sizes, k: int):
    km = len(sizes)
    arr = (C.c_int64 * km)(*[int(v) for v in sizes])
    out = (C.c_int32 * km)()
    _check(lib().skm_hier_alloc(C.cast(arr, C.c_void_p), km, k, C.cast(out, C.c_void_p)))
    return list(out)


def theta_ratio(d: int, t: int, eps0: float) -> float:
    return float(lib().skm_theta_ratio(d, t, eps0))


def dprime_init(d: int, frac: float = 0.125) -> int:
    return int(lib().skm_dprime_init(d, frac))


def dprime_adjust(d: int, dprime: int, f: float, lo=0.95, hi=0.97, step=0.20) -> int:
    return int(lib().skm_dprime_adjust(d, dprime, f, lo, hi, step))


def debug_gemm_config(tile256: int = -1, panel_cols: int = 0, max_tiles: int = 0):
    """skm_debug_gemm_config: force launch choices of the GEMM kernels (tests); no arguments = defaults."""
    lib().skm_debug_gemm_config(tile256, panel_cols, max_tiles)


def version() -> str:
    return lib().skm_version().decode()
