"""ctypes marshalling for ``kfac_oracle.c`` (fp64 CPU oracle, test infrastructure only).

All arrays are converted to C-contiguous float64; results are new float64 arrays.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kfac_oracle.c")
_LIB = os.path.join(_HERE, "libkfac_oracle.so")
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)
_i = ctypes.c_int
_i64 = ctypes.c_int64
_d = ctypes.c_double


def build(force=True):
    """Compile the oracle with gcc (plain C99 + OpenMP, no fast-math)."""
    global _lib
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=gnu99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        _lib = None
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        build(force=True)
    lib = ctypes.CDLL(_LIB)
    lib.oracle_num_threads.restype = _i
    lib.oracle_kron.argtypes = [_dp, _i, _i, _dp, _i, _i, _dp]
    lib.oracle_unfold.argtypes = [_dp, _i, _i, _i, _i, _i, _i, _i, _i, _i, _i, _dp]
    lib.oracle_gram.argtypes = [_dp, _i64, _i, _i, _d, _dp]
    lib.oracle_gram_entry.argtypes = [_dp, _i64, _i, _i, _d, _i, _i]
    lib.oracle_gram_entry.restype = _d
    lib.oracle_conv_factor_entry.argtypes = [_dp, _i, _i, _i, _i, _i, _i, _i, _i, _i, _i, _d, _i, _i]
    lib.oracle_conv_factor_entry.restype = _d
    lib.oracle_ema.argtypes = [_dp, _dp, _i64, _d]
    for name in ("oracle_eigh", "oracle_eigh_jacobi", "oracle_eigh_tridiag"):
        getattr(lib, name).argtypes = [_dp, _i, _dp, _dp]
        getattr(lib, name).restype = _i
    lib.oracle_precondition.argtypes = [_dp, _dp, _i, _dp, _dp, _i, _d, _dp, _dp]
    lib.oracle_bruteforce.argtypes = [_dp, _i, _dp, _i, _d, _dp, _dp]
    lib.oracle_bruteforce.restype = _i
    lib.oracle_spd_solve.argtypes = [_dp, _i, _dp, _i, _dp]
    lib.oracle_spd_solve.restype = _i
    lib.oracle_schedule.argtypes = [_i64, _i, _i, ctypes.POINTER(_i), ctypes.POINTER(_i)]
    lib.oracle_precondition_inverse.argtypes = [_dp, _i, _dp, _i, _d, _dp, _dp]
    lib.oracle_grad_scale.argtypes = [_i, ctypes.POINTER(_i64), _dp, _dp, _d, _d]
    lib.oracle_grad_scale.restype = _d
    _lib = lib
    return lib


def _c(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(_dp)


def num_threads():
    return int(_load().oracle_num_threads())


def kron(A, B):
    A, B = _c(A), _c(B)
    m, n = A.shape
    p, q = B.shape
    out = np.empty((m * p, n * q))
    _load().oracle_kron(_p(A), m, n, _p(B), p, q, _p(out))
    return out


def conv_out_hw(H, W, kh, kw, sh, sw, ph, pw):
    return (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1


def unfold(x, kh, kw, sh, sw, ph, pw):
    """x [N,C,H,W] -> P [N*Ho*Wo, C*kh*kw]."""
    x = _c(x)
    N, C, H, W = x.shape
    Ho, Wo = conv_out_hw(H, W, kh, kw, sh, sw, ph, pw)
    P = np.empty((N * Ho * Wo, C * kh * kw))
    _load().oracle_unfold(_p(x), N, C, H, W, kh, kw, sh, sw, ph, pw, _p(P))
    return P


def gram(X, append_ones, scale):
    """X [R,d] -> scale * [X|1]^T [X|1]."""
    X = _c(X)
    R, d = X.shape
    D = d + (1 if append_ones else 0)
    F = np.empty((D, D))
    _load().oracle_gram(_p(X), R, d, int(bool(append_ones)), float(scale), _p(F))
    return F


def gram_entry(X, append_ones, scale, i, j):
    X = _c(X)
    R, d = X.shape
    return float(_load().oracle_gram_entry(_p(X), R, d, int(bool(append_ones)), float(scale), int(i), int(j)))


def conv_factor_entry(x, kh, kw, sh, sw, ph, pw, scale, i, j):
    """Entry (i, j) of scale * [P|1]^T [P|1] for the unfold P of x, straight from the definition."""
    x = _c(x)
    N, C, H, W = x.shape
    return float(_load().oracle_conv_factor_entry(_p(x), N, C, H, W, kh, kw, sh, sw, ph, pw, float(scale), int(i), int(j)))


def ema(F, Fb, xi):
    """Returns xi*F + (1-xi)*Fb."""
    out = _c(F).copy()
    Fb = _c(Fb)
    assert out.shape == Fb.shape
    _load().oracle_ema(_p(out), _p(Fb), out.size, float(xi))
    return out


def _eig_call(name, F):
    F = _c(F)
    n = F.shape[0]
    assert F.shape == (n, n)
    Q = np.empty((n, n))
    lam = np.empty(n)
    rc = getattr(_load(), name)(_p(F), n, _p(Q), _p(lam))
    if rc < 0:
        raise RuntimeError("%s did not converge" % name)
    return lam, Q


def eigh(F):
    """Returns (lam ascending, Q with eigenvectors in columns)."""
    return _eig_call("oracle_eigh", F)


def eigh_jacobi(F):
    return _eig_call("oracle_eigh_jacobi", F)


def eigh_tridiag(F):
    return _eig_call("oracle_eigh_tridiag", F)


def precondition(QA, lamA, QG, lamG, gamma, grad):
    QA, lamA, QG, lamG, grad = _c(QA), _c(lamA), _c(QG), _c(lamG), _c(grad)
    dA, dG = QA.shape[0], QG.shape[0]
    assert grad.shape == (dG, dA)
    out = np.empty((dG, dA))
    _load().oracle_precondition(_p(QA), _p(lamA), dA, _p(QG), _p(lamG), dG, float(gamma), _p(grad), _p(out))
    return out


def bruteforce(G, A, gamma, grad):
    G, A, grad = _c(G), _c(A), _c(grad)
    dG, dA = G.shape[0], A.shape[0]
    assert grad.shape == (dG, dA)
    out = np.empty((dG, dA))
    rc = _load().oracle_bruteforce(_p(G), dG, _p(A), dA, float(gamma), _p(grad), _p(out))
    if rc < 0:
        raise RuntimeError("damped Kronecker product not positive definite")
    return out


def spd_solve(A, B):
    A, B = _c(A), _c(B)
    n, m = B.shape
    X = np.empty((n, m))
    rc = _load().oracle_spd_solve(_p(A), n, _p(B), m, _p(X))
    if rc < 0:
        raise RuntimeError("matrix not positive definite")
    return X


def precondition_inverse(G, A, gamma, grad):
    """(G + gamma I)^-1 grad (A + gamma I)^-1 by Cholesky solves (the explicit-inverse method of Sec. II-C)."""
    G, A, grad = _c(G), _c(A), _c(grad)
    dG, dA = G.shape[0], A.shape[0]
    assert grad.shape == (dG, dA)
    out = np.empty((dG, dA))
    rc = _load().oracle_precondition_inverse(_p(G), dG, _p(A), dA, float(gamma), _p(grad), _p(out))
    if rc < 0:
        raise RuntimeError("damped factor not positive definite")
    return out


def grad_scale(precond, grad, kappa, alpha):
    """nu of Sec. V-C for lists of per-layer preconditioned and original gradients."""
    assert len(precond) == len(grad)
    sizes = (_i64 * len(grad))(*[int(np.asarray(g).size) for g in grad])
    P = _c(np.concatenate([np.asarray(p, dtype=np.float64).ravel() for p in precond])) if len(grad) else _c(np.zeros(1))
    G = _c(np.concatenate([np.asarray(g, dtype=np.float64).ravel() for g in grad])) if len(grad) else _c(np.zeros(1))
    return float(_load().oracle_grad_scale(len(grad), sizes, _p(P), _p(G), float(kappa), float(alpha)))


def schedule(k, f_fac, f_eig):
    a, b = _i(0), _i(0)
    _load().oracle_schedule(int(k), int(f_fac), int(f_eig), ctypes.byref(a), ctypes.byref(b))
    return bool(a.value), bool(b.value)
