"""fp64 CPU oracle for the backward pass of the GKA layer (Section 4.2.2 "Backward Pass", Appendix B.2).

TEST INFRASTRUCTURE ONLY, like the rest of this package: nothing in the product library may import it. It exists
ahead of any GPU backward kernel, as the definition such a kernel will be checked against.

What it computes. The forward pass, per (batch, head) pair and token t (Section 4.1, Eq. (CH), with the optional
write gate beta of the Remark there and the alpha-connection of Section 4.3):

    H_t = gamma_t H_{t-1} + beta_t k_t k_t^T,     U_t = gamma_t U_{t-1} + beta_t v_t k_t^T,
    x_t = solve(H_t + lambda_t I, q_t),           y_t = U_t (alpha_t x_t + (1 - alpha_t) q_t),

with lambda_t given per token or lambda_t = a ||H_t||_F. Given dy_t = dL/dy_t it returns dL/d(q, k, v, gamma, beta,
alpha, lambda or nothing, H_init, U_init) by implicit differentiation (Section 4.2.2): x_t is treated as the exact
solution of its linear system, so that

    p_t := dL/dq_t through the solve = solve(H_t + lambda_t I, dL/dx_t),
    dL/d(H_t + lambda_t I) = -p_t x_t^T,          dL/dlambda_t = -x_t^T p_t            (Appendix B.2),

and with the rule lambda_t = a ||H_t||_F the partial gradient at H_t is -p_t x_t^T - a (x_t^T p_t) H_t / ||H_t||_F
(Appendix B.2, Eq. (dH_t-implicit)). Both solves use the same solver: Algorithm 1 with r passes (the paper's
approximate gradients, dq_t = CH(H_t + lambda_t I, dx_t, r)) or a direct solve (the exact gradients of the exact
layer, which finite differences can check). The gradients at the states are accumulated by the reverse recurrences
of Section 4.2.2 (Eq. (Ai), Eq. (Bi)) in their plain form: one d x d accumulator per state, one token at a time; no
chunking. Sign of the w_t H_t term: the Lemma of Section 4.2.2 and Appendix B.2 print opposite signs; the one used
here (minus, as in the Lemma) is the one the finite-difference pin confirms.

Pins (tests/test_oracle_backward_pins.py): central finite differences of the exact layer for every returned
gradient, with and without each optional input; the Lemma's explicit double sum for dk; the linearity lemma of
Appendix B.2 (Algorithm 1 is linear and symmetric in its right-hand side, so the gradient at q through r passes is
exactly r passes on the incoming gradient) by finite differences through the truncated iteration.
"""
import numpy as np

from . import gka_oracle as _fwd

SOLVER_CHEBYSHEV = _fwd.SOLVER_CHEBYSHEV
SOLVER_CHOLESKY = _fwd.SOLVER_CHOLESKY


def _solve(A_reg, rhs, fro, lam, n_iter, solver):
    """x with (H + lam I) x = rhs: Algorithm 1 with L = ||H||_F + lam, mu = lam, or the direct solve."""
    if solver == SOLVER_CHOLESKY:
        return _fwd.cholesky_solve(A_reg, rhs)
    return _fwd.chebyshev(A_reg, rhs, fro + lam, lam, n_iter)


def backward_pair(q, k, v, gate, lam, dy, n_iter, *, beta=None, alpha=None, lambda_scale=0.0,
                  solver=SOLVER_CHEBYSHEV, H_init=None, U_init=None):
    """One (batch, head) pair. q, k: [T,d_k]; v, dy: [T,d_v]; gate, lam, beta, alpha: [T] (lam None: the rule
    lambda_t = lambda_scale ||H_t||_F). Returns a dict of float64 gradients and the forward output y."""
    q, k, v, dy = (np.asarray(a, dtype=np.float64) for a in (q, k, v, dy))
    gate = np.asarray(gate, dtype=np.float64)
    T, d_k = q.shape
    d_v = v.shape[1]
    beta = np.ones(T) if beta is None else np.asarray(beta, dtype=np.float64)
    alpha = np.ones(T) if alpha is None else np.asarray(alpha, dtype=np.float64)
    rule = lam is None
    if not rule:
        lam = np.asarray(lam, dtype=np.float64)
    H0 = np.zeros((d_k, d_k)) if H_init is None else np.asarray(H_init, dtype=np.float64)
    U0 = np.zeros((d_v, d_k)) if U_init is None else np.asarray(U_init, dtype=np.float64)

    # ---- forward, every state kept (Eq. (CH))
    Hs = np.empty((T + 1, d_k, d_k)); Us = np.empty((T + 1, d_v, d_k))
    Hs[0], Us[0] = H0, U0
    x = np.empty((T, d_k)); y = np.empty((T, d_v)); fro = np.empty(T); lam_t = np.empty(T)
    for t in range(T):
        Hs[t + 1] = gate[t] * Hs[t] + beta[t] * np.outer(k[t], k[t])
        Us[t + 1] = gate[t] * Us[t] + beta[t] * np.outer(v[t], k[t])
        fro[t] = np.sqrt(np.sum(Hs[t + 1] ** 2))
        lam_t[t] = lambda_scale * fro[t] if rule else lam[t]
        x[t] = _solve(Hs[t + 1] + lam_t[t] * np.eye(d_k), q[t], fro[t], lam_t[t], n_iter, solver)
        y[t] = Us[t + 1] @ (alpha[t] * x[t] + (1.0 - alpha[t]) * q[t])

    # ---- backward: reverse walk with the accumulated gradients at H_t and U_t
    dq = np.empty_like(q); dk = np.empty_like(k); dv = np.empty_like(v)
    dgate = np.empty(T); dbeta = np.empty(T); dalpha = np.empty(T); dlam = np.empty(T)
    accH = np.zeros((d_k, d_k))            # dL/dH_t, everything downstream of H_t included
    accU = np.zeros((d_v, d_k))
    for t in range(T - 1, -1, -1):
        Ht, Ut = Hs[t + 1], Us[t + 1]
        xt = alpha[t] * x[t] + (1.0 - alpha[t]) * q[t]             # operand of the readout
        dxt = Ut.T @ dy[t]
        dalpha[t] = dxt @ (x[t] - q[t])
        p = _solve(Ht + lam_t[t] * np.eye(d_k), alpha[t] * dxt, fro[t], lam_t[t], n_iter, solver)
        dq[t] = p + (1.0 - alpha[t]) * dxt
        dlam[t] = -(x[t] @ p)
        local_H = -np.outer(p, x[t])
        if rule:                                                   # lambda_t = a ||H_t||_F
            local_H = local_H + dlam[t] * lambda_scale * Ht / fro[t]
        if t + 1 < T:
            accH = gate[t + 1] * accH
            accU = gate[t + 1] * accU
        accH = accH + local_H
        accU = accU + np.outer(dy[t], xt)
        dk[t] = beta[t] * ((accH + accH.T) @ k[t] + accU.T @ v[t])
        dv[t] = beta[t] * (accU @ k[t])
        dbeta[t] = k[t] @ accH @ k[t] + v[t] @ accU @ k[t]
        dgate[t] = np.sum(accH * Hs[t]) + np.sum(accU * Us[t])
    out = {"y": y, "dq": dq, "dk": dk, "dv": dv, "dgate": dgate, "dbeta": dbeta, "dalpha": dalpha,
           "dH_init": gate[0] * accH, "dU_init": gate[0] * accU, "x": x, "lam": lam_t, "fro": fro}
    if not rule:
        out["dlam"] = dlam
    return out


def backward(q, k, v, gate, lam, dy, n_iter, *, beta=None, alpha=None, lambda_scale=0.0, solver=SOLVER_CHEBYSHEV,
             H_init=None, U_init=None):
    """All pairs. q, k: [B,T,H,d_k]; v, dy: [B,T,H,d_v]; gate, lam, beta, alpha: [B,T,H]; states [B,H,d,d].
    Returns a dict of arrays in the same layouts (dgate, dlam, dbeta, dalpha: [B,T,H])."""
    q = np.asarray(q, dtype=np.float64)
    B, T, H, _ = q.shape
    res = None
    for b in range(B):
        for h in range(H):
            sel = lambda a: None if a is None else np.asarray(a)[b, :, h]
            st = lambda a: None if a is None else np.asarray(a)[b, h]
            r = backward_pair(q[b, :, h], sel(k), sel(v), sel(gate), sel(lam), sel(dy), n_iter, beta=sel(beta),
                              alpha=sel(alpha), lambda_scale=lambda_scale, solver=solver, H_init=st(H_init),
                              U_init=st(U_init))
            if res is None:
                res = {}
                for name, a in r.items():
                    if name in ("dH_init", "dU_init"):
                        res[name] = np.empty((B, H) + a.shape)
                    else:
                        res[name] = np.empty((B, T, H) + a.shape[1:])
            for name, a in r.items():
                if name in ("dH_init", "dU_init"):
                    res[name][b, h] = a
                else:
                    res[name][b, :, h] = a
    return res
