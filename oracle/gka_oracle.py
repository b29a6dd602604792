"""ctypes loader for oracle/gka_oracle.c (plain C, fp64, OpenMP over (batch, head) pairs).

Test infrastructure: the functions here define the expected results of the GKA forward path
(paper Section 4.1, Eq. (CH) and Algorithm 1).  Nothing in the product library may call them.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gka_oracle.c")
_SANITIZED = bool(os.environ.get("GKA_ORACLE_SANITIZED"))      # the CPU tests' sanitizer run sets this
_LIB = os.path.join(_HERE, "libgka_oracle_san.so" if _SANITIZED else "libgka_oracle.so")

SOLVER_CHEBYSHEV = 0
SOLVER_CHOLESKY = 1

_lib = None


def build(force=False):
    """Compile the oracle with gcc (no BLAS; -O2; OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        if _SANITIZED:
            # AddressSanitizer + UndefinedBehaviorSanitizer build; the process must preload gcc's libasan.so
            cmd[1:2] = ["-O1", "-g", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=all",
                        "-fno-omit-frame-pointer"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ci, cd = ctypes.c_int, ctypes.c_double
        lib.gka_oracle_omega_schedule.argtypes = [cd, cd, ci, dp]
        lib.gka_oracle_omega_schedule.restype = None
        lib.gka_oracle_chebyshev.argtypes = [ci, dp, dp, cd, cd, ci, dp, dp]
        lib.gka_oracle_chebyshev.restype = None
        lib.gka_oracle_cholesky_solve.argtypes = [ci, dp, dp, dp]
        lib.gka_oracle_cholesky_solve.restype = ci
        lib.gka_oracle_forward.argtypes = [ci] * 5 + [dp] * 7 + [cd, ci, ci] + [dp] * 7
        lib.gka_oracle_forward.restype = ci
        lib.gka_oracle_decode_step.argtypes = [ci] * 4 + [dp] * 9 + [cd, ci, ci] + [dp] * 2
        lib.gka_oracle_decode_step.restype = ci
        lib.gka_oracle_num_threads.argtypes = []
        lib.gka_oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def _f64(a, shape=None):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.float64))
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _ptr(a):
    if a is None:
        return None
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def num_threads():
    return int(_load().gka_oracle_num_threads())


def omega_schedule(L, mu, r):
    """omega_0..omega_r of Algorithm 1's weight schedule."""
    out = np.empty(r + 1, dtype=np.float64)
    _load().gka_oracle_omega_schedule(float(L), float(mu), int(r), _ptr(out))
    return out


def chebyshev(A, q, L, mu, r):
    """Algorithm 1 on the (already regularised) matrix A."""
    A = _f64(A)
    D = A.shape[0]
    q = _f64(q, (D,))
    xi = np.empty(D, dtype=np.float64)
    work = np.empty(3 * D, dtype=np.float64)
    _load().gka_oracle_chebyshev(D, _ptr(A), _ptr(q), float(L), float(mu), int(r), _ptr(xi), _ptr(work))
    return xi


def cholesky_solve(A, q):
    A = _f64(A).copy()
    D = A.shape[0]
    q = _f64(q, (D,))
    x = np.empty(D, dtype=np.float64)
    rc = _load().gka_oracle_cholesky_solve(D, _ptr(A), _ptr(q), _ptr(x))
    if rc:
        raise np.linalg.LinAlgError("matrix not positive definite")
    return x


def forward(q, k, v, gate, lam, n_iter, *, beta=None, alpha=None, lambda_scale=0.0, solver=SOLVER_CHEBYSHEV,
            H_init=None, U_init=None, return_state=False, return_fro=False, return_xhat=False):
    """Eq. (CH) over whole sequences.

    q, k: [B,T,H,d_k]; v: [B,T,H,d_v]; gate, lam, beta, alpha: [B,T,H] (lam None -> lambda_scale*||H_t||_F;
    beta: write gate of the beta-augmented recurrence; alpha: readout of alpha*xhat + (1-alpha)*q; None = 1).
    Returns y [B,T,H,d_v] (float64) and, on request, a dict with H_final, U_final, fro, xhat.
    """
    q = _f64(q)
    B, T, H, d_k = q.shape
    k = _f64(k, (B, T, H, d_k))
    v = _f64(v)
    d_v = v.shape[-1]
    v = _f64(v, (B, T, H, d_v))
    gate = _f64(gate, (B, T, H))
    lam = None if lam is None else _f64(lam, (B, T, H))
    beta = None if beta is None else _f64(beta, (B, T, H))
    alpha = None if alpha is None else _f64(alpha, (B, T, H))
    H_init = None if H_init is None else _f64(H_init, (B, H, d_k, d_k))
    U_init = None if U_init is None else _f64(U_init, (B, H, d_v, d_k))
    y = np.empty((B, T, H, d_v), dtype=np.float64)
    extra = {}
    Hf = Uf = fro = xhat = None
    if return_state:
        Hf = np.empty((B, H, d_k, d_k), dtype=np.float64)
        Uf = np.empty((B, H, d_v, d_k), dtype=np.float64)
        extra["H_final"], extra["U_final"] = Hf, Uf
    if return_fro:
        fro = np.empty((B, T, H), dtype=np.float64)
        extra["fro"] = fro
    if return_xhat:
        xhat = np.empty((B, T, H, d_k), dtype=np.float64)
        extra["xhat"] = xhat
    rc = _load().gka_oracle_forward(B, T, H, d_k, d_v, _ptr(q), _ptr(k), _ptr(v), _ptr(gate), _ptr(lam),
                                    _ptr(beta), _ptr(alpha), float(lambda_scale), int(n_iter), int(solver),
                                    _ptr(H_init), _ptr(U_init), _ptr(y), _ptr(Hf), _ptr(Uf), _ptr(fro),
                                    _ptr(xhat))
    if rc:
        raise RuntimeError(f"gka_oracle_forward failed with code {rc}")
    if extra:
        return y, extra
    return y


def decode_step(H_state, U_state, q, k, v, gate, lam, n_iter, *, beta=None, alpha=None, lambda_scale=0.0,
                solver=SOLVER_CHEBYSHEV, return_fro=False):
    """One recurrent step on float64 states [B,H,d,d], updated IN PLACE. q,k,v: [B,H,d]."""
    if H_state.dtype != np.float64 or not H_state.flags.c_contiguous:
        raise ValueError("H_state must be contiguous float64")
    if U_state.dtype != np.float64 or not U_state.flags.c_contiguous:
        raise ValueError("U_state must be contiguous float64")
    B, H, d_k, _ = H_state.shape
    d_v = U_state.shape[2]
    q = _f64(q, (B, H, d_k))
    k = _f64(k, (B, H, d_k))
    v = _f64(v, (B, H, d_v))
    gate = _f64(gate, (B, H))
    lam = None if lam is None else _f64(lam, (B, H))
    beta = None if beta is None else _f64(beta, (B, H))
    alpha = None if alpha is None else _f64(alpha, (B, H))
    y = np.empty((B, H, d_v), dtype=np.float64)
    fro = np.empty((B, H), dtype=np.float64) if return_fro else None
    rc = _load().gka_oracle_decode_step(B, H, d_k, d_v, _ptr(H_state), _ptr(U_state), _ptr(q), _ptr(k),
                                        _ptr(v), _ptr(gate), _ptr(lam), _ptr(beta), _ptr(alpha), float(lambda_scale),
                                        int(n_iter), int(solver), _ptr(y), _ptr(fro))
    if rc:
        raise RuntimeError(f"gka_oracle_decode_step failed with code {rc}")
    if return_fro:
        return y, fro
    return y
