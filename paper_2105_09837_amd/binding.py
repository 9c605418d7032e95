"""ctypes binding with the same names as the C ABI in include/pdadmm.h."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

STATUS = {0: "OK", 1: "EINVAL", 2: "ENOMEM", 3: "EHIP", 4: "EBACKTRACK", 5: "ENONFINITE"}


class VAR:
    P, W, B, Z, Q, U, TAU, THETA, PIDX, RESID, GRAD_P, GRAD_W, PROBE = range(13)


class PHASE:
    P, W, BZQU = range(3)


class PdadmmError(RuntimeError):
    def __init__(self, code: int, where: str, detail: str = ""):
        self.code = code
        self.status = STATUS.get(code, str(code))
        super().__init__(f"{where}: {self.status}" + (f" ({detail})" if detail else ""))


class _CConfig(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("n_layers", C.c_int32), ("dims", C.POINTER(C.c_int32)),
                ("rho", C.c_float), ("nu", C.c_float), ("quantize", C.c_int32),
                ("q_lo", C.c_float), ("q_hi", C.c_float), ("q_levels", C.c_int32),
                ("fista_iters", C.c_int32), ("bt_eta", C.c_float), ("tau0", C.c_float),
                ("theta0", C.c_float), ("bt_max_trials", C.c_int32), ("refresh_every", C.c_int32),
                ("leaky_slope", C.c_float), ("use_graph", C.c_int32), ("bt_probe_backoff", C.c_int32),
                ("risk_kind", C.c_int32)]


class _CObjective(C.Structure):
    _fields_ = [(n, C.c_double) for n in ("risk", "lin_pen", "act_pen", "dual_lin", "dual_quad", "F", "L_rho")]


RISK = {"ce": 0, "ls": 1}

EXPORTS = ["pdadmm_normalize_adj", "pdadmm_augment", "pdadmm_quantize", "pdadmm_gemm_nt", "pdadmm_gemm_tn",
           "pdadmm_gemm_tn_static",
           "pdadmm_workspace_bytes", "pdadmm_init", "pdadmm_grow_layers", "pdadmm_set_var", "pdadmm_get_var", "pdadmm_iterate",
           "pdadmm_step_phase", "pdadmm_sync", "pdadmm_objective", "pdadmm_residual", "pdadmm_stats", "pdadmm_plan_info",
           "pdadmm_predict",
           "pdadmm_timing", "pdadmm_timing_read", "pdadmm_last_error", "pdadmm_destroy"]


def library_path() -> str:
    return os.path.join(_HERE, "libpdadmm.so")


def exported_symbols():
    return list(EXPORTS)


def load_library():
    """Load libpdadmm.so from the package directory; raise if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise PdadmmError(3, "load_library", f"{path} is missing: run __graft_entry__.build() first; "
                                             "there is no CPU fallback")
    lib = C.CDLL(path)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    lib.pdadmm_normalize_adj.argtypes = [i32, vp, vp, vp, vp, vp]
    lib.pdadmm_augment.argtypes = [i32, i64, vp, vp, vp, vp, i32, i32, vp, vp]
    lib.pdadmm_quantize.argtypes = [vp, i64, f32, f32, i32, vp, vp, vp]
    lib.pdadmm_gemm_nt.argtypes = [i32, i32, i32, vp, i32, vp, i32, vp, i32, vp]
    lib.pdadmm_gemm_tn.argtypes = [i32, i32, i32, f32, vp, i32, vp, i32, vp, i32, i32, vp, vp]
    lib.pdadmm_gemm_tn_static.argtypes = [i32, i32, i32, f32, vp, i32, vp, i32, vp, i32, i32, vp]
    lib.pdadmm_workspace_bytes.argtypes = [C.POINTER(_CConfig)]
    lib.pdadmm_workspace_bytes.restype = C.c_size_t
    lib.pdadmm_init.argtypes = [C.POINTER(vp), C.POINTER(_CConfig), vp, C.c_size_t, vp, vp, vp,
                                C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), i32]
    lib.pdadmm_grow_layers.argtypes = [C.POINTER(vp), C.POINTER(_CConfig), vp, C.c_size_t, vp, vp, vp, vp, vp,
                                       C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), i32]
    lib.pdadmm_set_var.argtypes = [vp, i32, i32, vp]
    lib.pdadmm_get_var.argtypes = [vp, i32, i32, vp]
    lib.pdadmm_iterate.argtypes = [vp, i32]
    lib.pdadmm_step_phase.argtypes = [vp, i32]
    lib.pdadmm_sync.argtypes = [vp]
    lib.pdadmm_objective.argtypes = [vp, C.POINTER(_CObjective)]
    lib.pdadmm_residual.argtypes = [vp, C.POINTER(C.c_double), vp]
    lib.pdadmm_stats.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.pdadmm_plan_info.argtypes = [vp, vp, vp, vp, vp]
    lib.pdadmm_predict.argtypes = [vp, vp, vp, vp, vp]
    lib.pdadmm_timing.argtypes = [vp, C.c_uint32]
    lib.pdadmm_timing_read.argtypes = [vp, vp, vp, i32]
    lib.pdadmm_last_error.argtypes = [vp]
    lib.pdadmm_last_error.restype = C.c_char_p
    lib.pdadmm_destroy.argtypes = [vp]
    lib.pdadmm_destroy.restype = None
    for name in EXPORTS:
        if name not in ("pdadmm_workspace_bytes", "pdadmm_last_error", "pdadmm_destroy"):
            getattr(lib, name).restype = C.c_int
    _LIB = lib
    return lib


@dataclass
class Config:
    n_nodes: int
    dims: Sequence[int]             # n_0 .. n_L
    rho: float
    nu: float
    quantize: int = 0
    q_lo: float = -1.0
    q_hi: float = 1.0
    q_levels: int = 256
    fista_iters: int = 20
    bt_eta: float = 2.0
    tau0: float = 1.0
    theta0: float = 1.0
    bt_max_trials: int = 64
    refresh_every: int = 0
    leaky_slope: float = 0.0
    use_graph: int = 0
    bt_probe_backoff: int = 1
    risk_kind: int = 0              # 0 cross-entropy, 1 least squares (see RISK)

    def to_c(self):
        dims = (C.c_int32 * len(self.dims))(*[int(d) for d in self.dims])
        cc = _CConfig(int(self.n_nodes), len(self.dims) - 1, C.cast(dims, C.POINTER(C.c_int32)),
                      float(self.rho), float(self.nu), int(self.quantize), float(self.q_lo), float(self.q_hi),
                      int(self.q_levels), int(self.fista_iters), float(self.bt_eta), float(self.tau0),
                      float(self.theta0), int(self.bt_max_trials), int(self.refresh_every), float(self.leaky_slope), int(self.use_graph),
                      int(self.bt_probe_backoff), int(self.risk_kind))
        cc._keep = dims
        return cc


class Context:
    """Handle returned by pdadmm_init; keeps the workspace tensor alive."""

    def __init__(self, handle, cfg: Config, workspace, stream):
        self.handle = handle
        self.cfg = cfg
        self.workspace = workspace
        self.stream = stream
        self.N = int(cfg.n_nodes)
        self.L = len(cfg.dims) - 1
        self.dims = [int(d) for d in cfg.dims]

    def last_error(self) -> str:
        return load_library().pdadmm_last_error(self.handle).decode()

    def __del__(self):
        try:
            pdadmm_destroy(self)
        except Exception:
            pass


def thread_error() -> str:
    """Reason of this thread's last failed call that had no context."""
    return (load_library().pdadmm_last_error(None) or b"").decode()


def _check(code, where, ctx: Optional[Context] = None):
    if code != 0:
        raise PdadmmError(code, where, ctx.last_error() if ctx is not None and ctx.handle else thread_error())


def _ptr(t):
    """Raw address of a torch tensor or numpy array (None -> NULL)."""
    if t is None:
        return None
    if isinstance(t, np.ndarray):
        return t.ctypes.data
    return t.data_ptr()


def _stream_ptr(stream):
    if stream is None:
        return None
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _dev_f32(t, name):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise PdadmmError(1, name, "expected a contiguous float32 device tensor")


# ----------------------------------------------------------------------------- host helper
def pdadmm_normalize_adj(rowptr: np.ndarray, colidx: np.ndarray):
    """HOST: CSR pattern of A -> CSR of the renormalised adjacency (rowptr, colidx, vals)."""
    lib = load_library()
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    n = rowptr.size - 1
    nnz = int(rowptr[-1]) if n >= 0 and rowptr.size else 0
    out_rp = np.empty(n + 1, dtype=np.int32)
    out_ci = np.empty(nnz + n, dtype=np.int32)
    out_v = np.empty(nnz + n, dtype=np.float32)
    _check(lib.pdadmm_normalize_adj(n, rowptr.ctypes.data, colidx.ctypes.data, out_rp.ctypes.data,
                                    out_ci.ctypes.data, out_v.ctypes.data), "pdadmm_normalize_adj")
    return out_rp, out_ci, out_v


# ----------------------------------------------------------------------------- device calls
def pdadmm_augment(rowptr, colidx, vals, X, hops: int, out=None, stream=None):
    """DEVICE: X_aug = [X | A~X | ... | A~^hops X]. Tensors: int32, int32, float32, float32 [n, d]."""
    import torch
    lib = load_library()
    _dev_f32(X, "pdadmm_augment")
    n, d = X.shape
    if out is None:
        out = torch.empty((n, (hops + 1) * d), dtype=torch.float32, device=X.device)
    _check(lib.pdadmm_augment(n, int(colidx.numel()), _ptr(rowptr), _ptr(colidx), _ptr(vals), _ptr(X), d, hops,
                              _ptr(out), _stream_ptr(stream)), "pdadmm_augment")
    return out


def pdadmm_quantize(v, lo: float, hi: float, levels: int, want_idx=True, want_val=True, stream=None):
    import torch
    lib = load_library()
    _dev_f32(v, "pdadmm_quantize")
    idx = torch.empty(v.shape, dtype=torch.uint8 if levels <= 256 else torch.uint16, device=v.device) if want_idx else None
    val = torch.empty_like(v) if want_val else None
    _check(lib.pdadmm_quantize(_ptr(v), v.numel(), lo, hi, levels, _ptr(idx), _ptr(val), _stream_ptr(stream)),
           "pdadmm_quantize")
    return idx, val


def pdadmm_gemm_nt(A, B, out=None, stream=None):
    """C[M,N] = A[M,K] @ B[N,K]^T (2-D float32 device tensors; row strides are honoured)."""
    import torch
    lib = load_library()
    M, K = A.shape
    N = B.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    _check(lib.pdadmm_gemm_nt(M, N, K, _ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(out), out.stride(0),
                              _stream_ptr(stream)), "pdadmm_gemm_nt")
    return out


def pdadmm_gemm_tn(A, B, alpha: float = 1.0, splitk: int = 1, out=None, stream=None):
    """C[M,N] = alpha * A[K,M]^T @ B[K,N]."""
    import torch
    lib = load_library()
    K, M = A.shape
    N = B.shape[1]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    part = torch.empty((max(splitk, 1), M, out.stride(0)), dtype=torch.float32, device=A.device)
    _check(lib.pdadmm_gemm_tn(M, N, K, alpha, _ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(out), out.stride(0),
                              splitk, _ptr(part), _stream_ptr(stream)), "pdadmm_gemm_tn")
    return out


def pdadmm_gemm_tn_static(A, B, alpha: float = 1.0, splitk: int = 1, out=None, stream=None):
    """pdadmm_gemm_tn with the library's built-in scratch: the call itself allocates nothing (pass `out`)."""
    import torch
    lib = load_library()
    K, M = A.shape
    N = B.shape[1]
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=A.device)
    _check(lib.pdadmm_gemm_tn_static(M, N, K, alpha, _ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(out),
                                     out.stride(0), splitk, _stream_ptr(stream)), "pdadmm_gemm_tn_static")
    return out


def pdadmm_workspace_bytes(cfg: Config) -> int:
    return int(load_library().pdadmm_workspace_bytes(C.byref(cfg.to_c())))


def pdadmm_init(cfg: Config, X_aug, labels, W0, b0, train_mask=None, stream=None, workspace=None, aux_stream=None) -> Context:
    """Create a context. All tensors live on the GPU; the workspace tensor is allocated here with
    torch (device memory plumbing) unless one is passed in. `stream`: the stream that carries the iteration
    (None = the default stream); `aux_stream`: optional second stream for the independent parts of an iteration."""
    return _new_context(cfg, X_aug, labels, W0, b0, train_mask, stream, workspace, None, None, aux_stream)


def pdadmm_grow_layers(source: Context, from_layer, cfg: Config, X_aug, labels, W0, b0, train_mask=None, stream=None,
                       workspace=None, aux_stream=None) -> Context:
    """Deeper model from a trained one: layer l takes W, b from layer from_layer[l-1] of `source` where
    that entry is positive, else from W0[l-1], b0[l-1] (device tensors; None allowed for carried layers)."""
    return _new_context(cfg, X_aug, labels, W0, b0, train_mask, stream, workspace, source, from_layer, aux_stream)


def _new_context(cfg, X_aug, labels, W0, b0, train_mask, stream, workspace, source, from_layer, aux_stream=None) -> Context:
    import torch
    lib = load_library()
    cc = cfg.to_c()
    need = int(lib.pdadmm_workspace_bytes(C.byref(cc)))
    if need == 0:
        raise PdadmmError(1, "pdadmm_workspace_bytes", thread_error() or "invalid configuration")
    if workspace is None:
        workspace = torch.empty(need + 4096, dtype=torch.uint8, device=X_aug.device)
    base = workspace.data_ptr()
    aligned = (base + 4095) & ~4095           # the library asks for 256; 4 KiB lets its arrays start on page boundaries
    avail = workspace.numel() - (aligned - base)
    L = len(cfg.dims) - 1
    Wp = (C.c_void_p * L)(*[_ptr(w) for w in W0])
    bp = (C.c_void_p * L)(*[_ptr(b) for b in b0])
    handle = C.c_void_p()
    n_streams = 2 if aux_stream is not None else 1
    streams = (C.c_void_p * 2)(_stream_ptr(stream), _stream_ptr(aux_stream))
    if source is None:
        what = "pdadmm_init"
        code = lib.pdadmm_init(C.byref(handle), C.byref(cc), aligned, avail, _ptr(X_aug), _ptr(labels),
                               _ptr(train_mask), Wp, bp, streams, n_streams)
    else:
        what = "pdadmm_grow_layers"
        fl = np.ascontiguousarray(from_layer, dtype=np.int32)
        if fl.shape != (L,):
            raise ValueError("from_layer needs one entry per layer of the new model")
        code = lib.pdadmm_grow_layers(C.byref(handle), C.byref(cc), aligned, avail, _ptr(X_aug), _ptr(labels),
                                      _ptr(train_mask), source.handle, fl.ctypes.data, Wp, bp, streams, n_streams)
    ctx = Context(handle, cfg, workspace, stream)
    ctx.aux_stream = aux_stream
    if code != 0:
        detail = ctx.last_error() if handle else thread_error()
        raise PdadmmError(code, what, detail)
    return ctx


def _var_shape(ctx: Context, kind: int, layer: int):
    n_in, n_out = ctx.dims[layer - 1], ctx.dims[layer]
    if kind in (VAR.P, VAR.GRAD_P, VAR.PIDX):
        return (ctx.N, n_in)
    if kind in (VAR.W, VAR.GRAD_W):
        return (n_out, n_in)
    if kind == VAR.B:
        return (n_out,)
    return (ctx.N, n_out)


def pdadmm_set_var(ctx: Context, kind: int, layer: int, src) -> None:
    lib = load_library()
    if kind in (VAR.TAU, VAR.THETA):
        v = C.c_double(float(src))
        _check(lib.pdadmm_set_var(ctx.handle, kind, layer, C.addressof(v)), "pdadmm_set_var", ctx)
        return
    if kind == VAR.PROBE:
        v = (C.c_int32 * 2)(int(src[0]), int(src[1]))
        _check(lib.pdadmm_set_var(ctx.handle, kind, layer, C.addressof(v)), "pdadmm_set_var", ctx)
        return
    if isinstance(src, np.ndarray):
        src = np.ascontiguousarray(src, dtype=np.float32)
    else:
        src = src.contiguous()
    if tuple(src.shape) != _var_shape(ctx, kind, layer):
        raise PdadmmError(1, "pdadmm_set_var", f"shape {tuple(src.shape)} != {_var_shape(ctx, kind, layer)}")
    _check(lib.pdadmm_set_var(ctx.handle, kind, layer, _ptr(src)), "pdadmm_set_var", ctx)


def pdadmm_get_var(ctx: Context, kind: int, layer: int, to_host: bool = True):
    import torch
    lib = load_library()
    if kind in (VAR.TAU, VAR.THETA):
        v = C.c_double()
        _check(lib.pdadmm_get_var(ctx.handle, kind, layer, C.addressof(v)), "pdadmm_get_var", ctx)
        return v.value
    if kind == VAR.PROBE:
        v = (C.c_int32 * 2)()
        _check(lib.pdadmm_get_var(ctx.handle, kind, layer, C.addressof(v)), "pdadmm_get_var", ctx)
        return (int(v[0]), int(v[1]))
    shape = _var_shape(ctx, kind, layer)
    wide = kind == VAR.PIDX and ctx.cfg.q_levels > 256      # indices of two bytes
    if to_host:
        out = np.empty(shape, dtype=(np.uint16 if wide else np.uint8) if kind == VAR.PIDX else np.float32)
    else:
        out = torch.empty(shape, dtype=(torch.uint16 if wide else torch.uint8) if kind == VAR.PIDX else torch.float32,
                          device=ctx.workspace.device)
    _check(lib.pdadmm_get_var(ctx.handle, kind, layer, _ptr(out)), "pdadmm_get_var", ctx)
    return out


def pdadmm_iterate(ctx: Context, n_iters: int = 1) -> None:
    _check(load_library().pdadmm_iterate(ctx.handle, n_iters), "pdadmm_iterate", ctx)


def pdadmm_step_phase(ctx: Context, phase: int) -> None:
    _check(load_library().pdadmm_step_phase(ctx.handle, phase), "pdadmm_step_phase", ctx)


def pdadmm_sync(ctx: Context) -> None:
    _check(load_library().pdadmm_sync(ctx.handle), "pdadmm_sync", ctx)


def pdadmm_objective(ctx: Context) -> dict:
    o = _CObjective()
    _check(load_library().pdadmm_objective(ctx.handle, C.byref(o)), "pdadmm_objective", ctx)
    return {n: getattr(o, n) for n, _ in _CObjective._fields_}


def pdadmm_residual(ctx: Context):
    tot = C.c_double()
    per = np.zeros(max(ctx.L - 1, 1), dtype=np.float64)
    _check(load_library().pdadmm_residual(ctx.handle, C.byref(tot), per.ctypes.data), "pdadmm_residual", ctx)
    return tot.value, per[:ctx.L - 1]


def pdadmm_stats(ctx: Context, drift: bool = False) -> dict:
    L = ctx.L
    tau = np.zeros(L)
    theta = np.zeros(L)
    pt = np.zeros(L, dtype=np.int32)
    wt = np.zeros(L, dtype=np.int32)
    d = C.c_double(0.0)
    pp = np.zeros(L, dtype=np.int64)
    _check(load_library().pdadmm_stats(ctx.handle, tau.ctypes.data, theta.ctypes.data, pt.ctypes.data,
                                       wt.ctypes.data, C.addressof(d) if drift else None, pp.ctypes.data),
           "pdadmm_stats", ctx)
    return dict(tau=tau, theta=theta, p_trials=pt, w_trials=wt, r_drift=d.value if drift else None, p_products=pp)


def pdadmm_plan_info(ctx: Context) -> dict:
    fused, wts, pb = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    ws = np.zeros(ctx.L, dtype=np.int32)
    _check(load_library().pdadmm_plan_info(ctx.handle, C.addressof(fused), ws.ctypes.data, C.addressof(wts),
                                           C.addressof(pb)), "pdadmm_plan_info", ctx)
    return dict(fused_updates=int(fused.value), wgrad_split=ws, wtrial_split=int(wts.value), p_bytes=int(pb.value))


def pdadmm_predict(ctx: Context, mask=None, want_logits: bool = False) -> dict:
    """Forward pass with the current weights: predicted class per node (device int32 tensor), accuracy
    over the nodes of `mask` (device uint8 tensor or None = all) and optionally the output layer."""
    import torch
    dev = ctx.workspace.device
    pred = torch.empty(ctx.N, dtype=torch.int32, device=dev)
    logits = torch.empty((ctx.N, ctx.dims[-1]), dtype=torch.float32, device=dev) if want_logits else None
    acc = C.c_double(0.0)
    if mask is not None and not (isinstance(mask, torch.Tensor) and mask.is_cuda and mask.dtype == torch.uint8
                                 and mask.numel() == ctx.N and mask.is_contiguous()):
        raise PdadmmError(1, "pdadmm_predict", "mask must be a contiguous uint8 device tensor of N entries")
    _check(load_library().pdadmm_predict(ctx.handle, _ptr(pred), _ptr(logits), _ptr(mask), C.addressof(acc)),
           "pdadmm_predict", ctx)
    return dict(pred=pred, accuracy=acc.value, logits=logits)


TIMING_CLASSES = ["gemm_pgrad", "gemm_trial", "gemm_wgrad", "splitk_reduce", "select", "p_step", "w_step",
                  "resid_colsum", "bias", "zqu", "fista", "quant_trial", "quant_apply", "refresh"]


def pdadmm_timing(ctx: Context, class_mask: int) -> None:
    _check(load_library().pdadmm_timing(ctx.handle, class_mask), "pdadmm_timing", ctx)


def pdadmm_timing_read(ctx: Context) -> dict:
    """{class name: (milliseconds, launches)} since the last read."""
    n = len(TIMING_CLASSES)
    ms = np.zeros(n)
    cnt = np.zeros(n, dtype=np.int64)
    _check(load_library().pdadmm_timing_read(ctx.handle, ms.ctypes.data, cnt.ctypes.data, n), "pdadmm_timing_read", ctx)
    return {name: (float(ms[i]), int(cnt[i])) for i, name in enumerate(TIMING_CLASSES)}


def pdadmm_destroy(ctx: Context) -> None:
    if ctx.handle:
        load_library().pdadmm_destroy(ctx.handle)
        ctx.handle = None
