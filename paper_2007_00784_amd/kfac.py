"""ctypes binding of libkfac_hip.so: the same entry points as ``include/kfac.h``.

Argument marshalling only.  Device buffers are torch tensors (PyTorch is used for device memory and
streams, nothing else) or raw integer device addresses; every step of the path runs in the HIP
library.  Loading fails loudly if the library has not been built (``python -m
paper_2007_00784_amd.build`` or ``__graft_entry__.build()``); there is no fallback.
"""
import ctypes
import os

KFAC_OK, KFAC_EINVAL, KFAC_ENOCONV, KFAC_EHIP, KFAC_EWORKSPACE, KFAC_ESCRATCH = 0, -1, -2, -3, -4, -5
KFAC_F32, KFAC_BF16 = 0, 1
KFAC_LAYOUT_RD, KFAC_LAYOUT_NDT = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkfac_hip.so")

EXPORTS = (
    "kfac_create", "kfac_destroy", "kfac_workspace_bytes", "kfac_eig_workspace_bytes", "kfac_strerror",
    "kfac_unfold", "kfac_unfold_batched", "kfac_unfold_workspace_bytes", "kfac_update_factors", "kfac_eig", "kfac_precondition", "kfac_schedule_due",
    "kfac_profile_begin", "kfac_profile_end", "kfac_precondition_batched", "kfac_precondition_workspace_bytes",
    "kfac_update_factors_batched", "kfac_update_factors_workspace_bytes", "kfac_precondition_batched_scaled",
    "kfac_update_factors_static", "kfac_static_scratch_bytes",
    "kfac_invert_factors", "kfac_invert_workspace_bytes", "kfac_precondition_inverse",
    "kfac_precondition_inverse_batched", "kfac_precondition_inverse_workspace_bytes",
)


class kfac_precond_inv_item(ctypes.Structure):
    _fields_ = [("Ainv", ctypes.c_void_p), ("dA", ctypes.c_int), ("Ginv", ctypes.c_void_p), ("dG", ctypes.c_int),
                ("grad", ctypes.c_void_p), ("grad_dtype", ctypes.c_int)]


class kfac_conv_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in
                ("N", "C", "H", "W", "kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w", "dtype")]


class kfac_eig_opts(ctypes.Structure):
    _fields_ = [("max_sweeps", ctypes.c_int), ("tol", ctypes.c_float), ("fp32_only", ctypes.c_int),
                ("warm_start", ctypes.c_int)]


class kfac_eig_info(ctypes.Structure):
    _fields_ = [("sweeps", ctypes.c_int), ("off_norm_rel", ctypes.c_float), ("converged", ctypes.c_int)]


class kfac_kernel_stat(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 32), ("launches", ctypes.c_int), ("ms", ctypes.c_double),
                ("flops", ctypes.c_double), ("bytes", ctypes.c_double)]


class kfac_precond_item(ctypes.Structure):
    _fields_ = [("QA", ctypes.c_void_p), ("lamA", ctypes.c_void_p), ("dA", ctypes.c_int),
                ("QG", ctypes.c_void_p), ("lamG", ctypes.c_void_p), ("dG", ctypes.c_int),
                ("damping", ctypes.c_float), ("grad", ctypes.c_void_p), ("grad_dtype", ctypes.c_int),
                ("factored_damping", ctypes.c_int), ("split_f16", ctypes.c_int)]


class kfac_factor_item(ctypes.Structure):
    _fields_ = [("X", ctypes.c_void_p), ("dtype", ctypes.c_int), ("layout", ctypes.c_int),
                ("N", ctypes.c_int), ("d", ctypes.c_int), ("T", ctypes.c_int), ("append_ones", ctypes.c_int),
                ("scale", ctypes.c_float), ("decay", ctypes.c_float), ("F", ctypes.c_void_p)]


class KfacError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, kfac_strerror(code), code))


_lib = None


def lib():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libkfac_hip.so is not built: run `python -m paper_2007_00784_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    vp, i, f, sz, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t, ctypes.c_int64
    ip = ctypes.POINTER(ctypes.c_int)
    L.kfac_create.argtypes = [ctypes.POINTER(vp), i, vp, vp, sz]
    L.kfac_destroy.argtypes = [vp]
    L.kfac_workspace_bytes.argtypes = [i, i, i64]
    L.kfac_workspace_bytes.restype = sz
    L.kfac_eig_workspace_bytes.argtypes = [i, ip]
    L.kfac_eig_workspace_bytes.restype = sz
    L.kfac_strerror.argtypes = [i]
    L.kfac_strerror.restype = ctypes.c_char_p
    L.kfac_unfold.argtypes = [vp, ctypes.POINTER(kfac_conv_desc), vp, vp]
    L.kfac_unfold_batched.argtypes = [vp, i, ctypes.POINTER(kfac_conv_desc), ctypes.POINTER(vp), ctypes.POINTER(vp)]
    L.kfac_unfold_workspace_bytes.argtypes = [i]
    L.kfac_unfold_workspace_bytes.restype = sz
    L.kfac_update_factors.argtypes = [vp, vp, i, i, i, i, i, i, f, f, vp]
    L.kfac_update_factors_static.argtypes = [vp, vp, i, i, i, i, i, i, f, f, vp]
    L.kfac_static_scratch_bytes.argtypes = []
    L.kfac_static_scratch_bytes.restype = sz
    L.kfac_eig.argtypes = [vp, i, ctypes.POINTER(vp), ip, ctypes.POINTER(vp), ctypes.POINTER(vp),
                           ctypes.POINTER(kfac_eig_opts), ctypes.POINTER(kfac_eig_info)]
    L.kfac_precondition.argtypes = [vp, vp, vp, i, vp, vp, i, f, vp, i]
    L.kfac_schedule_due.argtypes = [i64, i, i, ip, ip]
    L.kfac_precondition_batched.argtypes = [vp, i, ctypes.POINTER(kfac_precond_item)]
    L.kfac_precondition_batched_scaled.argtypes = [vp, i, ctypes.POINTER(kfac_precond_item), f, f, vp]
    L.kfac_precondition_workspace_bytes.argtypes = [i, ctypes.POINTER(kfac_precond_item)]
    L.kfac_precondition_workspace_bytes.restype = sz
    L.kfac_update_factors_batched.argtypes = [vp, i, ctypes.POINTER(kfac_factor_item)]
    L.kfac_update_factors_workspace_bytes.argtypes = [i, ctypes.POINTER(kfac_factor_item)]
    L.kfac_update_factors_workspace_bytes.restype = sz
    L.kfac_invert_factors.argtypes = [vp, i, ctypes.POINTER(vp), ip, f, ctypes.POINTER(vp)]
    L.kfac_invert_workspace_bytes.argtypes = [i, ip]
    L.kfac_invert_workspace_bytes.restype = sz
    L.kfac_precondition_inverse.argtypes = [vp, vp, i, vp, i, vp, i]
    L.kfac_precondition_inverse_batched.argtypes = [vp, i, ctypes.POINTER(kfac_precond_inv_item)]
    L.kfac_precondition_inverse_workspace_bytes.argtypes = [i, ctypes.POINTER(kfac_precond_inv_item)]
    L.kfac_precondition_inverse_workspace_bytes.restype = sz
    L.kfac_profile_begin.argtypes = [vp]
    L.kfac_profile_end.argtypes = [vp, ctypes.POINTER(kfac_kernel_stat), i, ip]
    for name in EXPORTS:
        if name not in ("kfac_workspace_bytes", "kfac_eig_workspace_bytes", "kfac_strerror",
                        "kfac_precondition_workspace_bytes", "kfac_update_factors_workspace_bytes",
                        "kfac_unfold_workspace_bytes", "kfac_static_scratch_bytes", "kfac_invert_workspace_bytes",
                        "kfac_precondition_inverse_workspace_bytes"):
            getattr(L, name).restype = i
    _lib = L
    return L


def _ptr(t):
    """Device address of a torch tensor (must be contiguous) or a raw integer address."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return KFAC_F32
    if t.dtype == torch.bfloat16:
        return KFAC_BF16
    raise ValueError("unsupported dtype %s" % t.dtype)


def _check(rc, where, allow=()):
    if rc != KFAC_OK and rc not in allow:
        raise KfacError(rc, where)
    return rc


def kfac_strerror(code):
    return lib().kfac_strerror(int(code)).decode()


def kfac_workspace_bytes(max_d, max_batch_factors, max_R):
    return int(lib().kfac_workspace_bytes(int(max_d), int(max_batch_factors), int(max_R)))


def kfac_eig_workspace_bytes(dims):
    arr = (ctypes.c_int * len(dims))(*[int(x) for x in dims])
    return int(lib().kfac_eig_workspace_bytes(len(dims), arr))


def kfac_create(device, stream, workspace, workspace_bytes=None):
    """Returns an opaque context handle.  `stream` is a hipStream_t value (torch: stream.cuda_stream),
    `workspace` a uint8 torch tensor (or address) that must stay alive as long as the context."""
    h = ctypes.c_void_p()
    nbytes = workspace_bytes if workspace_bytes is not None else (workspace.numel() * workspace.element_size()
                                                                  if workspace is not None else 0)
    _check(lib().kfac_create(ctypes.byref(h), int(device), stream or None, _ptr(workspace), nbytes), "kfac_create")
    return h


def kfac_destroy(ctx):
    _check(lib().kfac_destroy(ctx), "kfac_destroy")


def kfac_unfold(ctx, x, kh, kw, stride, pad, patches):
    """x [N,C,H,W] -> patches [N, C*kh*kw, Ho*Wo] (same dtype)."""
    N, C, H, W = x.shape
    sh, sw = (stride, stride) if isinstance(stride, int) else stride
    ph, pw = (pad, pad) if isinstance(pad, int) else pad
    d = kfac_conv_desc(N, C, H, W, kh, kw, sh, sw, ph, pw, _dtype_code(x))
    _check(lib().kfac_unfold(ctx, ctypes.byref(d), _ptr(x), _ptr(patches)), "kfac_unfold")


def kfac_unfold_batched(ctx, xs, convs, patches):
    """xs: list of [N,C,H,W] device tensors; convs: list of (kh, kw, stride, pad); patches: list of outputs."""
    n = len(xs)
    descs = (kfac_conv_desc * n)()
    for j, (x, (kh, kw, stride, pad)) in enumerate(zip(xs, convs)):
        N, C, H, W = x.shape
        sh, sw = (stride, stride) if isinstance(stride, int) else stride
        ph, pw = (pad, pad) if isinstance(pad, int) else pad
        descs[j] = kfac_conv_desc(N, C, H, W, kh, kw, sh, sw, ph, pw, _dtype_code(x))
    xp = (ctypes.c_void_p * n)(*[_ptr(x) for x in xs])
    pp = (ctypes.c_void_p * n)(*[_ptr(p) for p in patches])
    _check(lib().kfac_unfold_batched(ctx, n, descs, xp, pp), "kfac_unfold_batched")


def kfac_unfold_workspace_bytes(n):
    return int(lib().kfac_unfold_workspace_bytes(int(n)))


def kfac_update_factors(ctx, X, layout, N, d, T, append_ones, scale, decay, F, dtype=None):
    code = _dtype_code(X) if dtype is None else dtype
    _check(lib().kfac_update_factors(ctx, _ptr(X), code, int(layout), int(N), int(d), int(T), int(append_ones),
                                     float(scale), float(decay), _ptr(F)), "kfac_update_factors")


def kfac_update_factors_static(ctx, X, layout, N, d, T, append_ones, scale, decay, F, dtype=None):
    """kfac_update_factors with its scratch in the library's static device array (allocates nothing)."""
    code = _dtype_code(X) if dtype is None else dtype
    _check(lib().kfac_update_factors_static(ctx, _ptr(X), code, int(layout), int(N), int(d), int(T), int(append_ones),
                                            float(scale), float(decay), _ptr(F)), "kfac_update_factors_static")


def kfac_static_scratch_bytes():
    return int(lib().kfac_static_scratch_bytes())


def _factor_items(items):
    """items: list of dicts with the arguments of kfac_update_factors (X and F may be None for sizing)."""
    arr = (kfac_factor_item * len(items))()
    for j, it in enumerate(items):
        X, F = it.get("X"), it.get("F")
        code = it.get("dtype")
        if code is None:
            code = _dtype_code(X) if X is not None else KFAC_F32
        arr[j] = kfac_factor_item(_ptr(X), int(code), int(it["layout"]), int(it["N"]), int(it["d"]), int(it["T"]),
                                  int(it["append_ones"]), float(it.get("scale", 1.0)), float(it.get("decay", 0.0)), _ptr(F))
    return arr


def factor_items(items):
    """The marshalled item array of a batch of factor updates (see precond_items)."""
    return _factor_items(items)


def kfac_update_factors_batched(ctx, items):
    """items: list of dicts(X, layout, N, d, T, append_ones, scale, decay, F[, dtype]), or the array that
    factor_items() made of such a list; all updated in one call."""
    arr = _factor_items(items) if isinstance(items, list) else items
    _check(lib().kfac_update_factors_batched(ctx, len(arr), arr), "kfac_update_factors_batched")


def kfac_update_factors_workspace_bytes(items):
    return int(lib().kfac_update_factors_workspace_bytes(len(items), _factor_items(items)))


def kfac_eig(ctx, F, Q, lam, max_sweeps=0, tol=0.0, raise_on_noconv=True, fp32_only=False, warm_start=False):
    """F, Q, lam: lists of device tensors.  Returns a list of (sweeps, off_norm_rel, converged)."""
    n = len(F)
    vp = ctypes.c_void_p
    Fa = (vp * n)(*[_ptr(t) for t in F])
    Qa = (vp * n)(*[_ptr(t) for t in Q])
    La = (vp * n)(*[_ptr(t) for t in lam])
    dims = (ctypes.c_int * n)(*[int(t.shape[0]) for t in F])
    opts = kfac_eig_opts(int(max_sweeps), float(tol), int(bool(fp32_only)), int(bool(warm_start)))
    info = (kfac_eig_info * n)()
    rc = lib().kfac_eig(ctx, n, Fa, dims, Qa, La, ctypes.byref(opts), info)
    _check(rc, "kfac_eig", allow=() if raise_on_noconv else (KFAC_ENOCONV,))
    return [(info[i].sweeps, info[i].off_norm_rel, bool(info[i].converged)) for i in range(n)]


def kfac_invert_factors(ctx, F, damping, Finv):
    """F, Finv: lists of device tensors; Finv[b] <- (F[b] + damping I)^-1."""
    n = len(F)
    vp = ctypes.c_void_p
    Fa = (vp * n)(*[_ptr(t) for t in F])
    Ia = (vp * n)(*[_ptr(t) for t in Finv])
    dims = (ctypes.c_int * n)(*[int(t.shape[0]) for t in F])
    _check(lib().kfac_invert_factors(ctx, n, Fa, dims, float(damping), Ia), "kfac_invert_factors")


def kfac_invert_workspace_bytes(dims):
    n = len(dims)
    return int(lib().kfac_invert_workspace_bytes(n, (ctypes.c_int * n)(*[int(v) for v in dims])))


def kfac_precondition_inverse(ctx, Ainv, Ginv, grad):
    dA, dG = int(Ainv.shape[0]), int(Ginv.shape[0])
    if tuple(grad.shape) != (dG, dA):
        raise ValueError("grad must be [dG, dA]")
    _check(lib().kfac_precondition_inverse(ctx, _ptr(Ainv), dA, _ptr(Ginv), dG, _ptr(grad), _dtype_code(grad)),
           "kfac_precondition_inverse")


def precond_inv_items(Ainv, Ginv, grad):
    """Marshalled array of kfac_precond_inv_item for lists of device tensors (reusable across calls)."""
    n = len(grad)
    arr = (kfac_precond_inv_item * n)()
    for j in range(n):
        dA, dG = int(Ainv[j].shape[0]), int(Ginv[j].shape[0])
        if tuple(grad[j].shape) != (dG, dA):
            raise ValueError("grad[%d] must be [dG, dA]" % j)
        arr[j] = kfac_precond_inv_item(_ptr(Ainv[j]), dA, _ptr(Ginv[j]), dG, _ptr(grad[j]), _dtype_code(grad[j]))
    return arr


def kfac_precondition_inverse_batched(ctx, Ainv=None, Ginv=None, grad=None, items=None):
    arr = items if items is not None else precond_inv_items(Ainv, Ginv, grad)
    _check(lib().kfac_precondition_inverse_batched(ctx, len(arr), arr), "kfac_precondition_inverse_batched")


def kfac_precondition(ctx, QA, lamA, QG, lamG, damping, grad):
    dA, dG = int(QA.shape[0]), int(QG.shape[0])
    if tuple(grad.shape) != (dG, dA):
        raise ValueError("grad must be [dG, dA]")
    _check(lib().kfac_precondition(ctx, _ptr(QA), _ptr(lamA), dA, _ptr(QG), _ptr(lamG), dG, float(damping),
                                   _ptr(grad), _dtype_code(grad)), "kfac_precondition")


def _precond_items(QA, lamA, QG, lamG, damping, grad, factored_damping=False, split_f16=False):
    n = len(grad)
    arr = (kfac_precond_item * n)()
    for j in range(n):
        dA, dG = int(QA[j].shape[0]), int(QG[j].shape[0])
        if tuple(grad[j].shape) != (dG, dA):
            raise ValueError("grad[%d] must be [dG, dA]" % j)
        arr[j] = kfac_precond_item(_ptr(QA[j]), _ptr(lamA[j]), dA, _ptr(QG[j]), _ptr(lamG[j]), dG, float(damping),
                                   _ptr(grad[j]), _dtype_code(grad[j]), int(bool(factored_damping)), int(bool(split_f16)))
    return arr


def precond_items(QA, lamA, QG, lamG, damping, grad, factored_damping=False, split_f16=False):
    """The marshalled item array of a batch, for callers that precondition the same buffers every iteration and
    want to marshal them once: pass it as `items=` to the batched calls below."""
    return _precond_items(QA, lamA, QG, lamG, damping, grad, factored_damping, split_f16)


def kfac_precondition_batched(ctx, QA=None, lamA=None, QG=None, lamG=None, damping=None, grad=None, factored_damping=False,
                              split_f16=False, items=None):
    """Lists of per-layer device tensors (or a marshalled `items` array); every grad[j] is preconditioned in
    place.  factored_damping: the explicit-inverse method (G + damping I)^-1 grad (A + damping I)^-1 instead
    of the eigenbasis step.  split_f16: run the GEMM chain on the split-fp16 engine."""
    arr = items if items is not None else _precond_items(QA, lamA, QG, lamG, damping, grad, factored_damping, split_f16)
    _check(lib().kfac_precondition_batched(ctx, len(arr), arr), "kfac_precondition_batched")


def kfac_precondition_batched_scaled(ctx, QA=None, lamA=None, QG=None, lamG=None, damping=None, grad=None, kappa=None, lr=None,
                                     nu=None, split_f16=False, items=None):
    """As kfac_precondition_batched, then every gradient is multiplied by the nu of Sec. V-C; nu: device tensor
    of one float32, written by the call."""
    arr = items if items is not None else _precond_items(QA, lamA, QG, lamG, damping, grad, split_f16=split_f16)
    _check(lib().kfac_precondition_batched_scaled(ctx, len(arr), arr, float(kappa), float(lr), _ptr(nu)),
           "kfac_precondition_batched_scaled")


def kfac_precondition_workspace_bytes(dims):
    """dims: list of (dA, dG)."""
    arr = (kfac_precond_item * len(dims))()
    for j, (dA, dG) in enumerate(dims):
        arr[j].dA, arr[j].dG = int(dA), int(dG)
    return int(lib().kfac_precondition_workspace_bytes(len(dims), arr))


def kfac_schedule_due(k, f_fac, f_eig):
    a, b = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().kfac_schedule_due(int(k), int(f_fac), int(f_eig), ctypes.byref(a), ctypes.byref(b)),
           "kfac_schedule_due")
    return bool(a.value), bool(b.value)


def kfac_profile_begin(ctx):
    _check(lib().kfac_profile_begin(ctx), "kfac_profile_begin")


def kfac_profile_end(ctx):
    """Returns {kernel class: dict(launches, ms, flops, bytes)} for the launches since kfac_profile_begin."""
    out = (kfac_kernel_stat * 16)()
    n = ctypes.c_int(0)
    _check(lib().kfac_profile_end(ctx, out, 16, ctypes.byref(n)), "kfac_profile_end")
    return {out[i].name.decode(): dict(launches=out[i].launches, ms=out[i].ms, flops=out[i].flops, bytes=out[i].bytes)
            for i in range(n.value)}
