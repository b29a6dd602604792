"""fp64 CPU oracle for the latent-sketching variant of the GKA layer (Appendix "Latent Sketching for Approximate
Solutions").

TEST INFRASTRUCTURE ONLY, like the rest of this package: nothing in the product library may import it.

What the appendix states: the normal equations of the layer are projected down into a low-dimensional subspace,
solved there, and the solution is projected back up, which takes the solver's cost from O(D^2 r) to O(d^2 r). It
gives no formulas. The reading taken here, with a sketch matrix S (d_s x D, rows = directions of the subspace) that
the caller provides:

    (H_t + lambda_t I) x = q_t       becomes       (S H_t S^T + lambda_t I) z = S q_t,
    z_t = CH(S H_t S^T + lambda_t I, S q_t, r)     (Algorithm 1 in d_s dimensions),
    xhat_t = S^T z_t,                y_t = U_t xhat_t                          (Eq. (CH) for the rest),

with S H_t S^T = sum_i eta_{t,i} (S k_i)(S k_i)^T, i.e. the same gated recurrence on the sketched keys, and the
bounds of Section 4.1 taken in the subspace: L = ||S H_t S^T||_F + lambda_t, mu = lambda_t (lambda_t given, or
lambda_t = a ||S H_t S^T||_F). U_t is the full state of Eq. (CH). No renormalisation of the sketched keys.

Written as the per-token recurrence, one state update and one solve per token; the solver is the forward oracle's
Algorithm 1 (or its direct solve).

Pins (tests/test_oracle_sketch_pins.py): S = I gives the forward oracle; keys inside the row space of an orthonormal
S give the unsketched layer exactly, also with truncated iterations (the Chebyshev polynomial acts on the subspace
and its complement separately, and U_t annihilates the complement); the explicit weighted sums with a direct solve;
rows of zeros appended to S change nothing.
"""
import numpy as np

from . import gka_oracle as _fwd

SOLVER_CHEBYSHEV = _fwd.SOLVER_CHEBYSHEV
SOLVER_CHOLESKY = _fwd.SOLVER_CHOLESKY


def forward_sketched_pair(q, k, v, gate, lam, S, n_iter, *, beta=None, lambda_scale=0.0, solver=SOLVER_CHEBYSHEV,
                          return_extra=False):
    """One (batch, head) pair. q, k: [T,D]; v: [T,d_v]; gate, lam, beta: [T] (lam None: lambda_t =
    lambda_scale ||S H_t S^T||_F); S: [d_s,D]. Returns y [T,d_v] (and z, xhat, fro if asked)."""
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    gate = np.asarray(gate, dtype=np.float64)
    S = np.asarray(S, dtype=np.float64)
    T, D = q.shape
    d_s = S.shape[0]
    beta = np.ones(T) if beta is None else np.asarray(beta, dtype=np.float64)
    rule = lam is None
    if not rule:
        lam = np.asarray(lam, dtype=np.float64)
    Hs = np.zeros((d_s, d_s))
    U = np.zeros((v.shape[1], D))
    y = np.empty((T, v.shape[1])); z = np.empty((T, d_s)); xhat = np.empty((T, D)); fro = np.empty(T)
    for t in range(T):
        ks = S @ k[t]
        Hs = gate[t] * Hs + beta[t] * np.outer(ks, ks)
        U = gate[t] * U + beta[t] * np.outer(v[t], k[t])
        fro[t] = np.sqrt(np.sum(Hs * Hs))
        lam_t = lambda_scale * fro[t] if rule else lam[t]
        A = Hs + lam_t * np.eye(d_s)
        rhs = S @ q[t]
        if solver == SOLVER_CHOLESKY:
            z[t] = _fwd.cholesky_solve(A, rhs)
        else:
            z[t] = _fwd.chebyshev(A, rhs, fro[t] + lam_t, lam_t, n_iter)
        xhat[t] = S.T @ z[t]
        y[t] = U @ xhat[t]
    if return_extra:
        return y, {"z": z, "xhat": xhat, "fro": fro}
    return y


def forward_sketched(q, k, v, gate, lam, S, n_iter, *, beta=None, lambda_scale=0.0, solver=SOLVER_CHEBYSHEV):
    """All pairs. q, k: [B,T,H,D]; v: [B,T,H,d_v]; gate, lam, beta: [B,T,H]; S: [d_s,D] (shared) or [H,d_s,D]
    (one sketch per head). Returns y [B,T,H,d_v]."""
    q = np.asarray(q, dtype=np.float64)
    B, T, H, _ = q.shape
    S = np.asarray(S, dtype=np.float64)
    y = np.empty(np.asarray(v).shape, dtype=np.float64)
    for b in range(B):
        for h in range(H):
            sel = lambda a: None if a is None else np.asarray(a)[b, :, h]
            Sh = S if S.ndim == 2 else S[h]
            y[b, :, h] = forward_sketched_pair(q[b, :, h], sel(k), sel(v), sel(gate), sel(lam), Sh, n_iter,
                                               beta=sel(beta), lambda_scale=lambda_scale, solver=solver)
    return y
