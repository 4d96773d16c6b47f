"""ctypes binding of include/lcn.h.  Same names as the C entry points;
argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblcn_hip.so")

COST_SQEUCLID, COST_EUCLID, COST_COSINE = 0, 1, 2
MODE_DENSE, MODE_SPARSE, MODE_NYSTROM, MODE_LCN = 0, 1, 2, 3
HASH_KMEANS, HASH_CROSSPOLYTOPE = 0, 1
INIT_SAMPLE, INIT_KMEANSPP, INIT_GIVEN = 0, 1, 2
F32, BF16 = 0, 1

OK, ERR_INVALID_ARG, ERR_ALLOC, ERR_DEVICE, ERR_STATE, ERR_SINGULAR, ERR_NONPOSITIVE, WARN_NO_SUPPORT, ERR_RANGE = range(9)


class LandmarkParams(ctypes.Structure):
    _fields_ = [("num_landmarks", ctypes.c_int32), ("kmeans_iters", ctypes.c_int32), ("seed", ctypes.c_uint64),
                ("ridge", ctypes.c_double), ("init", ctypes.c_int32), ("init_centroids", ctypes.c_void_p)]


class LshParams(ctypes.Structure):
    _fields_ = [("hash", ctypes.c_int32), ("num_buckets", ctypes.c_int32), ("num_rounds", ctypes.c_int32),
                ("kmeans_iters", ctypes.c_int32), ("seed", ctypes.c_uint64), ("projections", ctypes.c_void_p),
                ("branching", ctypes.c_int32 * 3), ("and_width", ctypes.c_int32)]


class Info(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("m", ctypes.c_int64), ("d", ctypes.c_int32), ("l", ctypes.c_int32),
                ("rounds", ctypes.c_int32), ("buckets", ctypes.c_int32), ("nnz_stored", ctypes.c_int64),
                ("nnz_unique", ctypes.c_int64), ("nonpositive", ctypes.c_int64), ("empty_rows", ctypes.c_int64),
                ("empty_cols", ctypes.c_int64), ("workspace_used", ctypes.c_size_t),
                ("undecided_last", ctypes.c_int64)]


class BatchDesc(ctypes.Structure):
    _fields_ = [("num_problems", ctypes.c_int32), ("x_off", ctypes.c_void_p), ("y_off", ctypes.c_void_p),
                ("lambda_", ctypes.c_void_p), ("del_cost_x", ctypes.c_void_p), ("del_cost_y", ctypes.c_void_p)]


class LcnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, lcn_status_string(status), status))


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the HIP library; there is no fallback if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("HIP library %s has not been built: run `python -m paper_2107_06876_amd.build`"
                               % _LIB_PATH)
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        lib.lcn_workspace_bytes.argtypes = [i64, i64, i32, i32, ctypes.POINTER(LandmarkParams),
                                            ctypes.POINTER(LshParams), i64, ctypes.POINTER(ctypes.c_size_t)]
        lib.lcn_build.argtypes = [vp, i64, vp, i64, i32, i32, vp, vp, ctypes.c_float, i32, i32,
                                  ctypes.POINTER(LandmarkParams), ctypes.POINTER(LshParams), vp, ctypes.c_size_t, vp,
                                  ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(vp)]
        lib.lcn_build_batched.argtypes = [vp, vp, i32, ctypes.POINTER(BatchDesc), i32, i32,
                                          ctypes.POINTER(LandmarkParams), ctypes.POINTER(LshParams), vp, ctypes.c_size_t,
                                          vp, ctypes.POINTER(ctypes.c_size_t), ctypes.POINTER(vp)]
        lib.lcn_batched_results.argtypes = [vp, vp, vp, vp, vp]
        lib.lcn_batched_get.argtypes = [vp, vp, vp, vp, vp, vp]
        lib.lcn_deletion_costs.argtypes = [vp, i64, i32, vp, vp, vp]
        lib.lcn_head_lambdas.argtypes = [ctypes.c_float, i32, vp]
        lib.lcn_calibrate.argtypes = [i32, vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_double)]
        lib.sinkhorn_run.argtypes = [vp, i32]
        lib.transport_cost.argtypes = [vp, ctypes.POINTER(ctypes.c_double)]
        lib.plan_marginals.argtypes = [vp, vp, vp, ctypes.POINTER(ctypes.c_double)]
        lib.lcn_get_scalings.argtypes = [vp, vp, vp]
        lib.lcn_set_scalings.argtypes = [vp, vp, vp]
        lib.lcn_get_landmarks.argtypes = [vp, vp]
        lib.lcn_get_buckets.argtypes = [vp, vp]
        lib.lcn_get_csr.argtypes = [vp, ctypes.POINTER(i64), vp, vp, vp]
        lib.lcn_get_factors.argtypes = [vp, vp, vp]
        lib.lcn_backward_scratch_bytes.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
        lib.lcn_backward.argtypes = [vp, vp, vp, vp, vp, vp, ctypes.c_size_t]
        lib.lcn_plan_rows.argtypes = [vp, i64, i64, vp]
        lib.lcn_get_info.argtypes = [vp, ctypes.POINTER(Info)]
        lib.lcn_last_run_timing.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32)]
        lib.lcn_destroy.argtypes = [vp]
        lib.lcn_destroy.restype = None
        lib.lcn_status_string.argtypes = [i32]
        lib.lcn_status_string.restype = ctypes.c_char_p
        for name in ("lcn_build_batched", "lcn_batched_results", "lcn_batched_get", "lcn_deletion_costs",
                     "lcn_head_lambdas", "lcn_workspace_bytes", "lcn_build", "sinkhorn_run", "transport_cost", "plan_marginals",
                     "lcn_get_scalings", "lcn_set_scalings", "lcn_get_landmarks", "lcn_get_buckets", "lcn_get_csr",
                     "lcn_get_factors", "lcn_get_info", "lcn_last_run_timing", "lcn_last_error_counts",
                     "lcn_backward_static", "lcn_calibrate"):
            getattr(lib, name).restype = i32
        _lib = lib
    return _lib


def lcn_status_string(status: int) -> str:
    return load_library().lcn_status_string(int(status)).decode()


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dev(t: torch.Tensor, dtype):
    assert t.is_cuda and t.is_contiguous() and t.dtype == dtype, "expected a contiguous %s device tensor" % dtype
    return t


class LcnHandle:
    """Owns the opaque handle and keeps the workspace tensor alive."""

    def __init__(self, raw, workspace, shape):
        self.raw = raw
        self.workspace = workspace
        self.n, self.m, self.d, self.l, self.rounds = shape
        self.device = workspace.device

    def __del__(self):
        try:
            lcn_destroy(self)
        except Exception:
            pass


def _params(landmarks, lsh, keep):
    lm = None
    if landmarks is not None:
        given = landmarks.get("init_centroids")
        if given is not None:
            given = _dev(given, torch.float32)
            keep.append(given)
        lm = LandmarkParams(int(landmarks["num_landmarks"]), int(landmarks.get("kmeans_iters", 10)),
                            int(landmarks.get("seed", 1)), float(landmarks.get("ridge", 0.0)),
                            int(landmarks.get("init", INIT_GIVEN if given is not None else INIT_SAMPLE)),
                            None if given is None else given.data_ptr())
    ls = None
    if lsh is not None:
        proj = lsh.get("projections")
        if proj is not None:
            proj = _dev(proj, torch.float32)
            keep.append(proj)
        ls = LshParams(int(lsh.get("hash", HASH_KMEANS)), int(lsh["num_buckets"]), int(lsh["num_rounds"]),
                       int(lsh.get("kmeans_iters", 10)), int(lsh.get("seed", 101)),
                       None if proj is None else proj.data_ptr())
        branching = [int(x) for x in (lsh.get("branching") or [])]
        if len(branching) > 3:
            raise ValueError("at most three levels of hierarchical k-means")
        ls.branching = (ctypes.c_int32 * 3)(*(branching + [0] * (3 - len(branching))))
        ls.and_width = int(lsh.get("and_width", 1))
    return lm, ls


def lcn_workspace_bytes(n, m, d, mode, landmarks=None, lsh=None, nnz_guess=0) -> int:
    lm, ls = _params(landmarks, lsh, [])
    out = ctypes.c_size_t(0)
    st = load_library().lcn_workspace_bytes(n, m, d, mode, None if lm is None else ctypes.byref(lm),
                                            None if ls is None else ctypes.byref(ls), int(nnz_guess),
                                            ctypes.byref(out))
    if st != OK:
        raise LcnError(st, "lcn_workspace_bytes")
    return out.value


def lcn_build(X, Y, a, b, lam, cost, mode, landmarks=None, lsh=None, workspace=None, stream=None) -> LcnHandle:
    """landmarks: dict(num_landmarks, kmeans_iters, seed, ridge, init, init_centroids); lsh: dict(hash,
    num_buckets, num_rounds, kmeans_iters, seed, projections, branching, and_width).  X, Y: float32 or
    bfloat16 device tensors.  If the workspace (a uint8 device tensor) is
    missing or too small a new one of the size the library asks for is
    allocated and the build is repeated."""
    lib = load_library()
    assert X.dtype in (torch.float32, torch.bfloat16) and Y.dtype == X.dtype
    X, Y = _dev(X, X.dtype), _dev(Y, X.dtype)
    a, b = _dev(a, torch.float32), _dev(b, torch.float32)
    n, d = X.shape
    m = Y.shape[0]
    assert Y.shape[1] == d and a.numel() == n and b.numel() == m
    keep = []
    lm, ls = _params(landmarks, lsh, keep)
    lmp = None if lm is None else ctypes.byref(lm)
    lsp = None if ls is None else ctypes.byref(ls)
    dtype = BF16 if X.dtype == torch.bfloat16 else F32
    if stream is None:
        stream = torch.cuda.current_stream(X.device).cuda_stream
    if workspace is None:
        workspace = torch.empty(lcn_workspace_bytes(n, m, d, mode, landmarks, lsh), dtype=torch.uint8,
                                device=X.device)
    for _ in range(2):
        raw = ctypes.c_void_p()
        need = ctypes.c_size_t(0)
        st = lib.lcn_build(_ptr(X), n, _ptr(Y), m, d, dtype, _ptr(a), _ptr(b), float(lam), cost, mode, lmp, lsp,
                           _ptr(workspace), workspace.numel(), ctypes.c_void_p(stream), ctypes.byref(need),
                           ctypes.byref(raw))
        if st == ERR_ALLOC and need.value > workspace.numel():
            workspace = torch.empty(need.value, dtype=torch.uint8, device=X.device)
            continue
        break
    if st != OK:
        raise LcnError(st, "lcn_build")
    h = LcnHandle(raw, workspace, (n, m, d, 0 if lm is None else lm.num_landmarks, 0 if ls is None else ls.num_rounds))
    h._keep = keep
    return h


def sinkhorn_run(h: LcnHandle, iters: int, check: bool = True) -> int:
    """Returns the status; raises on errors (a missing-support warning is returned, not raised)."""
    st = load_library().sinkhorn_run(h.raw, int(iters))
    if check and st not in (OK, WARN_NO_SUPPORT):
        raise LcnError(st, "sinkhorn_run")
    return st


def transport_cost(h: LcnHandle) -> float:
    out = ctypes.c_double(0.0)
    st = load_library().transport_cost(h.raw, ctypes.byref(out))
    if st != OK:
        raise LcnError(st, "transport_cost")
    return out.value


def plan_marginals(h: LcnHandle):
    """Returns (row marginals, column marginals, L1 residual)."""
    r = torch.empty(h.n, dtype=torch.float32, device=h.device)
    c = torch.empty(h.m, dtype=torch.float32, device=h.device)
    res = ctypes.c_double(0.0)
    st = load_library().plan_marginals(h.raw, _ptr(r), _ptr(c), ctypes.byref(res))
    if st != OK:
        raise LcnError(st, "plan_marginals")
    return r, c, res.value


def lcn_get_scalings(h: LcnHandle):
    lu = torch.empty(h.n, dtype=torch.float32, device=h.device)
    lv = torch.empty(h.m, dtype=torch.float32, device=h.device)
    st = load_library().lcn_get_scalings(h.raw, _ptr(lu), _ptr(lv))
    if st != OK:
        raise LcnError(st, "lcn_get_scalings")
    return lu, lv


def lcn_set_scalings(h: LcnHandle, log_u, log_v):
    st = load_library().lcn_set_scalings(h.raw, _ptr(_dev(log_u, torch.float32)), _ptr(_dev(log_v, torch.float32)))
    if st != OK:
        raise LcnError(st, "lcn_set_scalings")


def lcn_get_landmarks(h: LcnHandle):
    L = torch.empty((h.l, h.d), dtype=torch.float32, device=h.device)
    st = load_library().lcn_get_landmarks(h.raw, _ptr(L))
    if st != OK:
        raise LcnError(st, "lcn_get_landmarks")
    return L


def lcn_get_buckets(h: LcnHandle):
    info = lcn_get_info(h)
    out = torch.empty((info.rounds, h.n + h.m), dtype=torch.int32, device=h.device)
    st = load_library().lcn_get_buckets(h.raw, _ptr(out))
    if st != OK:
        raise LcnError(st, "lcn_get_buckets")
    return out


def lcn_get_csr(h: LcnHandle, values: bool = True):
    """Returns (rowptr int64 (n+1), colidx int32 (nnz), values float32 (nnz) or None)."""
    lib = load_library()
    rowptr = torch.empty(h.n + 1, dtype=torch.int64, device=h.device)
    nnz = ctypes.c_int64(0)
    st = lib.lcn_get_csr(h.raw, ctypes.byref(nnz), _ptr(rowptr), None, None)
    if st != OK:
        raise LcnError(st, "lcn_get_csr")
    colidx = torch.empty(max(nnz.value, 1), dtype=torch.int32, device=h.device)
    val = torch.empty(max(nnz.value, 1), dtype=torch.float32, device=h.device) if values else None
    st = lib.lcn_get_csr(h.raw, ctypes.byref(nnz), _ptr(rowptr), _ptr(colidx), _ptr(val))
    if st != OK:
        raise LcnError(st, "lcn_get_csr")
    return rowptr, colidx[:nnz.value], None if val is None else val[:nnz.value]


def lcn_get_factors(h: LcnHandle):
    U = torch.empty((h.n, h.l), dtype=torch.float32, device=h.device)
    Wt = torch.empty((h.m, h.l), dtype=torch.float32, device=h.device)
    st = load_library().lcn_get_factors(h.raw, _ptr(U), _ptr(Wt))
    if st != OK:
        raise LcnError(st, "lcn_get_factors")
    return U, Wt


def lcn_backward_scratch_bytes(h: LcnHandle) -> int:
    nbytes = ctypes.c_size_t(0)
    st = load_library().lcn_backward_scratch_bytes(h.raw, ctypes.byref(nbytes))
    if st != OK:
        raise LcnError(st, "lcn_backward_scratch_bytes")
    return int(nbytes.value)


def lcn_backward(h: LcnHandle, nnz: int = 0, factors: bool = True, pattern: bool = True):
    """Derivatives of the distance (Prop. 1): returns (gU, gWt, gsp, gnys), None for the
    parts the mode does not have.  nnz: entries of the pattern (from lcn_get_csr)."""
    has_f = factors and h.l > 0
    has_p = pattern and nnz > 0
    gU = torch.empty((h.n, h.l), dtype=torch.float32, device=h.device) if has_f else None
    gWt = torch.empty((h.m, h.l), dtype=torch.float32, device=h.device) if has_f else None
    gsp = torch.empty(nnz, dtype=torch.float32, device=h.device) if has_p else None
    gnys = torch.empty(nnz, dtype=torch.float32, device=h.device) if has_p and h.l > 0 else None
    scratch = None
    if has_p:
        scratch = torch.empty(lcn_backward_scratch_bytes(h) + 256, dtype=torch.uint8, device=h.device)
    sp = 0 if scratch is None else (scratch.data_ptr() + 255) // 256 * 256
    st = load_library().lcn_backward(h.raw, _ptr(gU), _ptr(gWt), _ptr(gsp), _ptr(gnys), ctypes.c_void_p(sp),
                                     0 if scratch is None else scratch.numel() - 256)
    if st != OK:
        raise LcnError(st, "lcn_backward")
    return gU, gWt, gsp, gnys


def lcn_backward_static(h: LcnHandle, gU=None, gWt=None, gsp=None, gnys=None) -> int:
    """lcn_backward into the caller's outputs (each may be None) with the library's own static
    scratch: the call itself allocates nothing.  Returns the status."""
    outs = [None if t is None else _dev(t, torch.float32) for t in (gU, gWt, gsp, gnys)]
    return load_library().lcn_backward_static(h.raw, *[_ptr(t) for t in outs])


def lcn_plan_rows(h: LcnHandle, i0: int, nrows: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Rows i0 .. i0 + nrows - 1 of the current transport plan as a dense (nrows, m) block."""
    if out is None:
        out = torch.empty((nrows, h.m), dtype=torch.float32, device=h.device)
    st = load_library().lcn_plan_rows(h.raw, i0, nrows, _ptr(_dev(out, torch.float32)))
    if st != OK:
        raise LcnError(st, "lcn_plan_rows")
    return out


def lcn_get_info(h: LcnHandle) -> Info:
    info = Info()
    st = load_library().lcn_get_info(h.raw, ctypes.byref(info))
    if st != OK:
        raise LcnError(st, "lcn_get_info")
    return info


def lcn_last_error_counts(h):
    """(nonpositive, empty_rows, empty_cols) accumulated over every sweep since the build; raises on
    LCN_ERR_DEVICE (a sweep gave up its bounded wait)."""
    c = [ctypes.c_int64(0) for _ in range(3)]
    st = load_library().lcn_last_error_counts(h.raw, *[ctypes.byref(x) for x in c])
    if st != OK:
        raise LcnError(st, "lcn_last_error_counts")
    return tuple(int(x.value) for x in c)


def lcn_last_run_timing(h: LcnHandle):
    ms = ctypes.c_float(0.0)
    launches = ctypes.c_int32(0)
    st = load_library().lcn_last_run_timing(h.raw, ctypes.byref(ms), ctypes.byref(launches))
    if st != OK:
        raise LcnError(st, "lcn_last_run_timing")
    return ms.value, launches.value


def lcn_destroy(h: LcnHandle):
    if getattr(h, "raw", None) is not None and h.raw.value:
        load_library().lcn_destroy(h.raw)
        h.raw = ctypes.c_void_p()


# ------------------------------------------------------------ batched problems --

class LcnBatchHandle(LcnHandle):
    def __init__(self, raw, workspace, x_off, y_off, d, l, rounds, bp):
        self.raw = raw
        self.workspace = workspace
        self.device = workspace.device
        self.x_off, self.y_off = x_off, y_off
        self.num_problems = len(x_off) - 1
        self.d, self.l, self.rounds, self.bp = d, l, rounds, bp
        self.total = int(x_off[-1] + y_off[-1])


def lcn_build_batched(X, Y, x_off, y_off, lam, cost, mode, del_cost_x=None, del_cost_y=None, landmarks=None,
                      lsh=None, workspace=None, stream=None) -> LcnBatchHandle:
    """x_off, y_off: int64 numpy arrays (P+1); lam: float32 numpy array (P); X, Y and the deletion
    costs: float32 device tensors."""
    import numpy as np
    lib = load_library()
    X, Y = _dev(X, torch.float32), _dev(Y, torch.float32)
    x_off = np.ascontiguousarray(x_off, dtype=np.int64)
    y_off = np.ascontiguousarray(y_off, dtype=np.int64)
    lam = np.ascontiguousarray(lam, dtype=np.float32)
    P = lam.shape[0]
    d = X.shape[1]
    keep = []
    lm, ls = _params(landmarks, lsh, keep)
    desc = BatchDesc(P, x_off.ctypes.data, y_off.ctypes.data, lam.ctypes.data,
                     None if del_cost_x is None else _dev(del_cost_x, torch.float32).data_ptr(),
                     None if del_cost_y is None else _dev(del_cost_y, torch.float32).data_ptr())
    if stream is None:
        stream = torch.cuda.current_stream(X.device).cuda_stream
    if workspace is None:
        workspace = torch.empty(1 << 20, dtype=torch.uint8, device=X.device)
    for _ in range(2):
        raw = ctypes.c_void_p()
        need = ctypes.c_size_t(0)
        st = lib.lcn_build_batched(_ptr(X), _ptr(Y), d, ctypes.byref(desc), cost, mode,
                                   None if lm is None else ctypes.byref(lm), None if ls is None else ctypes.byref(ls),
                                   _ptr(workspace), workspace.numel(), ctypes.c_void_p(stream), ctypes.byref(need),
                                   ctypes.byref(raw))
        if st == ERR_ALLOC and need.value > workspace.numel():
            workspace = torch.empty(need.value, dtype=torch.uint8, device=X.device)
            continue
        break
    if st != OK:
        raise LcnError(st, "lcn_build_batched")
    h = LcnBatchHandle(raw, workspace, x_off, y_off, d, 0 if lm is None else lm.num_landmarks,
                       0 if ls is None else ls.num_rounds, del_cost_x is not None)
    h._keep = keep + [X, Y, del_cost_x, del_cost_y]
    return h


def lcn_batched_results(h: LcnBatchHandle, marginals: bool = False):
    """Returns (distances (P,), residuals (P,)) as numpy arrays, plus the row and column
    marginals (device tensors) if asked."""
    import numpy as np
    dist = np.empty(h.num_problems)
    resid = np.empty(h.num_problems)
    r = torch.empty(h.total, dtype=torch.float32, device=h.device) if marginals else None
    c = torch.empty(h.total, dtype=torch.float32, device=h.device) if marginals else None
    st = load_library().lcn_batched_results(h.raw, dist.ctypes.data, resid.ctypes.data, _ptr(r), _ptr(c))
    if st != OK:
        raise LcnError(st, "lcn_batched_results")
    return (dist, resid, r, c) if marginals else (dist, resid)


def lcn_batched_get(h: LcnBatchHandle):
    """Returns dict(log_u, log_v (float64, total), landmarks (P, l, d), buckets (flat int32), kernel (P, 64, 64))."""
    P = h.num_problems
    out = dict(log_u=torch.empty(h.total, dtype=torch.float64, device=h.device),
               log_v=torch.empty(h.total, dtype=torch.float64, device=h.device),
               landmarks=torch.empty((P, max(h.l, 1), h.d), dtype=torch.float32, device=h.device),
               buckets=torch.empty(max(h.rounds, 1) * h.total, dtype=torch.int32, device=h.device),
               kernel=torch.empty((P, 64, 64), dtype=torch.float32, device=h.device))
    st = load_library().lcn_batched_get(h.raw, _ptr(out["log_u"]), _ptr(out["log_v"]), _ptr(out["landmarks"]),
                                        _ptr(out["buckets"]), _ptr(out["kernel"]))
    if st != OK:
        raise LcnError(st, "lcn_batched_get")
    return out


def lcn_deletion_costs(X, alpha, out=None, stream=None):
    """c_i = || alpha .* x_i ||_2 for every row of X (float32 device tensors); returns the float32
    device tensor of costs."""
    X, alpha = _dev(X, torch.float32), _dev(alpha, torch.float32)
    if X.dim() != 2 or alpha.numel() != X.shape[1]:
        raise ValueError("X must be (total, d) and alpha (d,)")
    if out is None:
        out = torch.empty(X.shape[0], dtype=torch.float32, device=X.device)
    if stream is None:
        stream = torch.cuda.current_stream(X.device).cuda_stream
    st = load_library().lcn_deletion_costs(_ptr(X), X.shape[0], X.shape[1], _ptr(alpha), _ptr(out),
                                           ctypes.c_void_p(stream))
    if st != OK:
        raise LcnError(st, "lcn_deletion_costs")
    return out


CAL_COPY_GBS, CAL_READ_GBS, CAL_MFMA_BF16_TFLOPS, CAL_MFMA_F64_TFLOPS, CAL_LAUNCH_US = range(5)


def lcn_calibrate(what: int, workspace) -> float:
    """One of the part's measured ceilings (see lcn.h); `workspace`: a contiguous device tensor of at
    least 64 MiB, overwritten."""
    import torch
    value = ctypes.c_double(0.0)
    stream = torch.cuda.current_stream(workspace.device).cuda_stream
    st = load_library().lcn_calibrate(int(what), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                      stream, ctypes.byref(value))
    if st != OK:
        raise LcnError(st, "lcn_calibrate")
    return value.value


def lcn_head_lambdas(lam: float, num_heads: int):
    """lambda_k = 2^(k - K/2) * lambda for k = 1 .. K as a float32 numpy array."""
    import numpy as np
    out = np.empty(max(int(num_heads), 1), dtype=np.float32)
    st = load_library().lcn_head_lambdas(float(lam), int(num_heads), out.ctypes.data)
    if st != OK:
        raise LcnError(st, "lcn_head_lambdas")
    return out
