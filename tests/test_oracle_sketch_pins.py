"""Pins of the latent-sketching oracle (oracle/gka_sketch_oracle.py): special cases that reduce to the forward
oracle, and the definition written out with explicit sums. CPU only."""
import numpy as np

import oracle
from oracle import gka_sketch_oracle as sk


def _case(seed, T=12, D=8, d_v=5):
    rng = np.random.default_rng(seed)
    nrm = lambda a: a / np.linalg.norm(a, axis=-1, keepdims=True)
    return dict(q=nrm(rng.standard_normal((T, D))), k=nrm(rng.standard_normal((T, D))),
                v=rng.standard_normal((T, d_v)), gate=1 / (1 + np.exp(-(rng.standard_normal(T) + 2.0))),
                lam=np.log1p(np.exp(rng.standard_normal(T))) + 0.05,
                beta=1 / (1 + np.exp(-(rng.standard_normal(T) + 1.0))))


def _full(c, n_iter, lam, a, solver, beta=None, d_v_pad=None):
    """The unsketched layer from the forward oracle (which wants d_v = d_k: v is padded with zero columns)."""
    T, D = c["q"].shape
    v = np.zeros((T, D)); v[:, :c["v"].shape[1]] = c["v"]
    y = oracle.forward(c["q"][None, :, None], c["k"][None, :, None], v[None, :, None], c["gate"][None, :, None],
                       None if lam is None else lam[None, :, None], n_iter, lambda_scale=a, solver=solver,
                       beta=None if beta is None else beta[None, :, None])
    return y[0, :, 0, :c["v"].shape[1]]


def test_identity_sketch_is_the_layer():
    c = _case(1)
    D = c["q"].shape[1]
    for solver, r in ((sk.SOLVER_CHEBYSHEV, 5), (sk.SOLVER_CHOLESKY, 0)):
        for lam, a in ((c["lam"], 0.0), (None, 0.07)):
            y = sk.forward_sketched_pair(c["q"], c["k"], c["v"], c["gate"], lam, np.eye(D), r, beta=c["beta"],
                                         lambda_scale=a, solver=solver)
            np.testing.assert_allclose(y, _full(c, r, lam, a, solver, beta=c["beta"]), rtol=1e-11, atol=1e-13)


def test_keys_inside_the_subspace_lose_nothing():
    """Keys in the row space of an orthonormal S: H_t = S^T (S H_t S^T) S has the same Frobenius norm, Algorithm 1's
    polynomial acts on the subspace and its complement separately, and U_t (built from the same keys) annihilates
    the complement, so the sketched output equals the unsketched one, pass for pass."""
    rng = np.random.default_rng(3)
    T, D, d_s = 14, 10, 4
    Q, _ = np.linalg.qr(rng.standard_normal((D, d_s)))
    S = Q.T                                                  # orthonormal rows
    c = _case(4, T=T, D=D)
    coeff = rng.standard_normal((T, d_s))
    c["k"] = coeff @ S
    c["k"] /= np.linalg.norm(c["k"], axis=1, keepdims=True)
    for solver, r in ((sk.SOLVER_CHEBYSHEV, 3), (sk.SOLVER_CHEBYSHEV, 9), (sk.SOLVER_CHOLESKY, 0)):
        for lam, a in ((c["lam"], 0.0), (None, 0.05)):
            y = sk.forward_sketched_pair(c["q"], c["k"], c["v"], c["gate"], lam, S, r, lambda_scale=a, solver=solver)
            np.testing.assert_allclose(y, _full(c, r, lam, a, solver), rtol=1e-9, atol=1e-11)
    # and a sketch that misses part of the keys does change the output (the test can tell)
    c2 = _case(5, T=T, D=D)
    y = sk.forward_sketched_pair(c2["q"], c2["k"], c2["v"], c2["gate"], c2["lam"], S, 0, solver=sk.SOLVER_CHOLESKY)
    assert np.abs(y - _full(c2, 0, c2["lam"], 0.0, sk.SOLVER_CHOLESKY)).max() > 1e-2


def test_definition_with_explicit_sums():
    """y_t = U_t S^T (S H_t S^T + lambda_t I)^{-1} S q_t with H_t, U_t as the explicit weighted sums of Section 4.1
    (eta_{t,i} = prod_{j=i+1..t} gamma_j) and numpy's solver."""
    c = _case(7, T=9, D=7, d_v=4)
    rng = np.random.default_rng(8)
    S = rng.standard_normal((3, 7)) / np.sqrt(7)
    y, ex = sk.forward_sketched_pair(c["q"], c["k"], c["v"], c["gate"], c["lam"], S, 0, beta=c["beta"],
                                     solver=sk.SOLVER_CHOLESKY, return_extra=True)
    T = c["q"].shape[0]
    for t in range(T):
        H = np.zeros((7, 7)); U = np.zeros((4, 7))
        for i in range(t + 1):
            eta = np.prod(c["gate"][i + 1:t + 1])
            H += eta * c["beta"][i] * np.outer(c["k"][i], c["k"][i])
            U += eta * c["beta"][i] * np.outer(c["v"][i], c["k"][i])
        Hs = S @ H @ S.T
        z = np.linalg.solve(Hs + c["lam"][t] * np.eye(3), S @ c["q"][t])
        np.testing.assert_allclose(ex["fro"][t], np.linalg.norm(Hs), rtol=1e-12)
        np.testing.assert_allclose(ex["z"][t], z, rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(y[t], U @ (S.T @ z), rtol=1e-10, atol=1e-13)


def test_truncated_iteration_is_algorithm_1_in_the_subspace():
    """z_t against the forward oracle run on the sketched keys and queries as a d_s-dimensional layer (its xhat)."""
    c = _case(9, T=10, D=8)
    rng = np.random.default_rng(10)
    S = rng.standard_normal((4, 8)) / np.sqrt(8)
    r = 4
    _, ex = sk.forward_sketched_pair(c["q"], c["k"], c["v"], c["gate"], None, S, r, lambda_scale=0.1,
                                     return_extra=True)
    qs, ks = c["q"] @ S.T, c["k"] @ S.T
    _, fx = oracle.forward(qs[None, :, None], ks[None, :, None], np.zeros_like(qs)[None, :, None],
                           c["gate"][None, :, None], None, r, lambda_scale=0.1, return_xhat=True, return_fro=True)
    np.testing.assert_allclose(ex["z"], fx["xhat"][0, :, 0], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(ex["fro"], fx["fro"][0, :, 0], rtol=1e-12)


def test_zero_rows_of_the_sketch_change_nothing():
    c = _case(11)
    rng = np.random.default_rng(12)
    S = rng.standard_normal((3, 8)) / np.sqrt(8)
    Sp = np.vstack([S, np.zeros((5, 8))])
    for lam, a in ((c["lam"], 0.0), (None, 0.05)):
        y0 = sk.forward_sketched_pair(c["q"], c["k"], c["v"], c["gate"], lam, S, 6, lambda_scale=a)
        y1 = sk.forward_sketched_pair(c["q"], c["k"], c["v"], c["gate"], lam, Sp, 6, lambda_scale=a)
        np.testing.assert_allclose(y1, y0, rtol=1e-12, atol=1e-14)


def test_batched_wrapper_layouts():
    rng = np.random.default_rng(13)
    B, T, H, D = 2, 6, 3, 8
    cs = [[_case(50 + b * H + h, T=T, D=D, d_v=D) for h in range(H)] for b in range(B)]
    stack = lambda n: np.stack([np.stack([cs[b][h][n] for h in range(H)], axis=1) for b in range(B)])
    S = rng.standard_normal((H, 4, D)) / np.sqrt(D)
    y = sk.forward_sketched(stack("q"), stack("k"), stack("v"), stack("gate"), stack("lam"), S, 5, beta=stack("beta"))
    one = sk.forward_sketched_pair(cs[1][2]["q"], cs[1][2]["k"], cs[1][2]["v"], cs[1][2]["gate"], cs[1][2]["lam"],
                                   S[2], 5, beta=cs[1][2]["beta"])
    np.testing.assert_array_equal(y[1, :, 2], one)
    y2 = sk.forward_sketched(stack("q"), stack("k"), stack("v"), stack("gate"), stack("lam"), S[0], 5)
    one2 = sk.forward_sketched_pair(cs[0][1]["q"], cs[0][1]["k"], cs[0][1]["v"], cs[0][1]["gate"], cs[0][1]["lam"],
                                    S[0], 5)
    np.testing.assert_array_equal(y2[0, :, 1], one2)
