"""Pins of the backward oracle (oracle/gka_backward_oracle.py): finite differences of the exact layer, the explicit
double sum of the Lemma of Section 4.2.2, and the linearity lemma of Appendix B.2. CPU only."""
import numpy as np
import pytest

import oracle
from oracle import gka_backward_oracle as bwd


def _case(seed, T=7, d_k=5, d_v=4, with_state=True):
    rng = np.random.default_rng(seed)
    nrm = lambda a: a / np.linalg.norm(a, axis=-1, keepdims=True)
    c = dict(q=nrm(rng.standard_normal((T, d_k))), k=nrm(rng.standard_normal((T, d_k))),
             v=rng.standard_normal((T, d_v)), gate=1 / (1 + np.exp(-(rng.standard_normal(T) + 2.0))),
             lam=np.log1p(np.exp(rng.standard_normal(T))) + 0.05, dy=rng.standard_normal((T, d_v)),
             beta=1 / (1 + np.exp(-(rng.standard_normal(T) + 1.0))), alpha=1 / (1 + np.exp(-(rng.standard_normal(T) + 1.0))))
    if with_state:
        A = rng.standard_normal((d_k, d_k))
        c["H_init"] = A @ A.T / d_k
        c["U_init"] = rng.standard_normal((d_v, d_k))
    return c


def _loss(c, names, n_iter, solver, lambda_scale):
    """sum_t <dy_t, y_t> of the forward oracle (the C one, not the backward module's own forward)."""
    g = lambda n: None if n not in names else c[n][None, :, None]
    st = lambda n: None if n not in c else c[n][None, None]
    y = oracle.forward(c["q"][None, :, None], c["k"][None, :, None], c["v"][None, :, None], c["gate"][None, :, None],
                       g("lam"), n_iter, beta=g("beta"), alpha=g("alpha"), lambda_scale=lambda_scale, solver=solver,
                       H_init=st("H_init"), U_init=st("U_init"))
    return float(np.sum(y[0, :, 0] * c["dy"]))


def _fd(c, name, names, n_iter, solver, lambda_scale, h=1e-6):
    base = c[name]
    g = np.empty_like(base)
    it = np.nditer(base, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        cp, cm = dict(c), dict(c)
        cp[name] = base.copy(); cp[name][i] += h
        cm[name] = base.copy(); cm[name][i] -= h
        if name == "H_init" and i[0] != i[1]:            # H stays symmetric: both mirror images move together
            cp[name][i[::-1]] += h
            cm[name][i[::-1]] -= h
        g[i] = (_loss(cp, names, n_iter, solver, lambda_scale) - _loss(cm, names, n_iter, solver, lambda_scale)) / (2 * h)
    return g


VARIANTS = {
    "plain": ("lam",),
    "rule": (),
    "beta": ("lam", "beta"),
    "alpha": ("lam", "alpha"),
    "all": ("beta", "alpha"),
}


@pytest.mark.parametrize("variant", sorted(VARIANTS))
def test_exact_gradients_match_finite_differences(variant):
    """With the direct solve the implicit-differentiation gradients are the gradients of the layer: every one of
    them against central differences of the forward oracle. H_init is perturbed along symmetric directions (an
    element and its mirror image together), so its reference is G + G^T - diag(G) of the returned gradient G."""
    names = VARIANTS[variant]
    a = 0.0 if "lam" in names else 0.07
    c = _case(11 + len(variant))
    r = bwd.backward_pair(c["q"], c["k"], c["v"], c["gate"], c["lam"] if "lam" in names else None, c["dy"], 0,
                          beta=c["beta"] if "beta" in names else None, alpha=c["alpha"] if "alpha" in names else None,
                          lambda_scale=a, solver=bwd.SOLVER_CHOLESKY, H_init=c["H_init"], U_init=c["U_init"])
    checks = [("q", "dq"), ("k", "dk"), ("v", "dv"), ("gate", "dgate"), ("U_init", "dU_init"), ("H_init", "dH_init")]
    checks += [(n, "d" + n) for n in names]
    for name, gname in checks:
        fd = _fd(c, name, names, 0, oracle.SOLVER_CHOLESKY, a)
        got = r[gname]
        if name == "H_init":                             # derivative along symmetric directions
            got = got + got.T - np.diag(np.diag(got))
        scale = max(np.abs(fd).max(), 1e-3)
        assert np.abs(got - fd).max() <= 2e-6 * scale + 1e-7, (variant, name, np.abs(got - fd).max(), scale)


def test_forward_of_backward_module_matches_forward_oracle():
    c = _case(5)
    for solver, r_ in ((bwd.SOLVER_CHEBYSHEV, 6), (bwd.SOLVER_CHOLESKY, 0)):
        r = bwd.backward_pair(c["q"], c["k"], c["v"], c["gate"], None, c["dy"], r_, beta=c["beta"], alpha=c["alpha"],
                              lambda_scale=0.1, solver=solver, H_init=c["H_init"], U_init=c["U_init"])
        y = oracle.forward(c["q"][None, :, None], c["k"][None, :, None], c["v"][None, :, None],
                           c["gate"][None, :, None], None, r_, beta=c["beta"][None, :, None],
                           alpha=c["alpha"][None, :, None], lambda_scale=0.1, solver=solver,
                           H_init=c["H_init"][None, None], U_init=c["U_init"][None, None])[0, :, 0]
        np.testing.assert_allclose(r["y"], y, rtol=1e-12, atol=1e-13)


def test_dk_equals_the_lemmas_double_sum():
    """Lemma of Section 4.2.2: dk_i = sum_{t>=i} M[i,t] (-dq_t x_t^T - x_t dq_t^T - w_t H_t) k_i with
    w_t = 2 a x_t^T dq_t / ||H_t||_F, evaluated term by term (beta = 1, no alpha-connection, zero initial state),
    plus the readout's own path through U_t; here against the reverse recurrences, with the truncated solver."""
    c = _case(23, T=9, with_state=False)
    a, n_iter = 0.05, 4
    r = bwd.backward_pair(c["q"], c["k"], c["v"], c["gate"], None, c["dy"], n_iter, lambda_scale=a)
    T, d = c["q"].shape
    # states and masks written out directly
    logg = np.log(c["gate"])
    M = np.zeros((T, T))
    for i in range(T):
        for t in range(i, T):
            M[i, t] = np.exp(np.sum(logg[i + 1:t + 1]))
    Ht = [sum(M[j, t] * np.outer(c["k"][j], c["k"][j]) for j in range(t + 1)) for t in range(T)]
    Ut = [sum(M[j, t] * np.outer(c["v"][j], c["k"][j]) for j in range(t + 1)) for t in range(T)]
    x, p = r["x"], r["dq"]                                         # alpha = 1: dq_t is the solve's gradient
    for i in range(T):
        acc = np.zeros(d)
        for t in range(i, T):
            w = 2 * a * (x[t] @ p[t]) / np.sqrt(np.sum(Ht[t] ** 2))
            acc += M[i, t] * ((-np.outer(p[t], x[t]) - np.outer(x[t], p[t]) - w * Ht[t]) @ c["k"][i])
            acc += M[i, t] * x[t] * (c["dy"][t] @ c["v"][i])       # through U_t: y_t = U_t x_t
        np.testing.assert_allclose(r["dk"][i], acc, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(r["y"], np.stack([Ut[t] @ x[t] for t in range(T)]), rtol=1e-11, atol=1e-12)


def test_gradient_at_q_through_truncated_iteration_is_the_same_iteration():
    """Appendix B.2 (linearity lemma): r passes of Algorithm 1 are a symmetric linear map of the right-hand side, so
    differentiating through them at q gives exactly r passes on the incoming gradient: finite differences of the
    truncated forward (r = 3, far from converged) against the oracle's dq."""
    c = _case(31, T=6)
    n_iter = 3
    r = bwd.backward_pair(c["q"], c["k"], c["v"], c["gate"], c["lam"], c["dy"], n_iter, H_init=c["H_init"],
                          U_init=c["U_init"])
    fd = _fd(c, "q", ("lam",), n_iter, oracle.SOLVER_CHEBYSHEV, 0.0)
    assert np.abs(r["dq"] - fd).max() <= 2e-6 * np.abs(fd).max()
    # and it differs from the exact-solve gradient, i.e. the test can tell the two apart
    e = bwd.backward_pair(c["q"], c["k"], c["v"], c["gate"], c["lam"], c["dy"], 0, solver=bwd.SOLVER_CHOLESKY,
                          H_init=c["H_init"], U_init=c["U_init"])
    assert np.abs(e["dq"] - fd).max() > 1e-3 * np.abs(fd).max()


def test_batched_wrapper_layouts():
    rng = np.random.default_rng(2)
    B, T, H, d = 2, 5, 3, 4
    cs = [[_case(100 + b * H + h, T=T, d_k=d, d_v=d) for h in range(H)] for b in range(B)]
    stack = lambda n: np.stack([np.stack([cs[b][h][n] for h in range(H)], axis=1) for b in range(B)])
    st = lambda n: np.stack([np.stack([cs[b][h][n] for h in range(H)]) for b in range(B)])
    r = bwd.backward(stack("q"), stack("k"), stack("v"), stack("gate"), stack("lam"), stack("dy"), 5,
                     beta=stack("beta"), H_init=st("H_init"), U_init=st("U_init"))
    one = bwd.backward_pair(cs[1][2]["q"], cs[1][2]["k"], cs[1][2]["v"], cs[1][2]["gate"], cs[1][2]["lam"],
                            cs[1][2]["dy"], 5, beta=cs[1][2]["beta"], H_init=cs[1][2]["H_init"],
                            U_init=cs[1][2]["U_init"])
    for name in ("dq", "dk", "dv", "dgate", "dlam", "dbeta", "y"):
        np.testing.assert_array_equal(r[name][1, :, 2], one[name])
    np.testing.assert_array_equal(r["dH_init"][1, 2], one["dH_init"])
    assert r["dq"].shape == (B, T, H, d) and r["dgate"].shape == (B, T, H) and r["dU_init"].shape == (B, H, d, d)
