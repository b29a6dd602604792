"""Pins for the fp64 CPU oracle: each test fixes the oracle to something other than itself
(values the paper prints, closed forms, a library solve, brute force on tiny inputs)."""
import os

import numpy as np
import pytest

import oracle
from oracle import chunked

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_inputs(rng, B, T, H, d, d_v=None, gate_lo=0.5, normalise=True):
    d_v = d if d_v is None else d_v
    q = rng.standard_normal((B, T, H, d))
    k = rng.standard_normal((B, T, H, d))
    if normalise:
        q /= np.linalg.norm(q, axis=-1, keepdims=True)
        k /= np.linalg.norm(k, axis=-1, keepdims=True)
    v = rng.standard_normal((B, T, H, d_v))
    gate = rng.uniform(gate_lo, 1.0, (B, T, H))
    lam = rng.uniform(0.05, 1.0, (B, T, H))
    return q, k, v, gate, lam


def _cheb_T(n, x):
    """Chebyshev polynomial of the first kind T_n(x) for real x (any magnitude)."""
    x = np.asarray(x, dtype=np.float64)
    out = np.empty_like(x)
    inside = np.abs(x) <= 1.0
    out[inside] = np.cos(n * np.arccos(x[inside]))
    xo = x[~inside]
    out[~inside] = np.sign(xo) ** n * np.cosh(n * np.arccosh(np.abs(xo)))
    return out


# --------------------------------------------------------------------------------------------
# omega schedule: printed constants (Appendix B.1 Remark) and the two lemmas before it
# --------------------------------------------------------------------------------------------

def _read_printed_constants():
    rows = []
    with open(os.path.join(GOLDEN, "remark_kappa51.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, power, value = line.split()
            rows.append((name, int(power), float(value), value))
    return rows


def _printed_tolerance(text):
    # half a unit in the last printed digit, doubled because the paper writes "approximately"
    if "e" in text:
        mant, exp = text.split("e")
        digits = len(mant.split(".")[1]) if "." in mant else 0
        return 10.0 ** (int(exp) - digits)
    digits = len(text.split(".")[1]) if "." in text else 0
    return 10.0 ** (-digits)


def test_omega_fixed_point_matches_printed_rate():
    """The fixed point omega* of the oracle's schedule gives 1 - sqrt(1 - rho^2) = rho^2 omega*/2,
    which the omega-rate lemma shows equals R; the Remark prints R and its powers for kappa = 51."""
    L, mu = 1.02, 0.02
    om = oracle.omega_schedule(L, mu, 400)
    rho = (L - mu) / (L + mu)
    R_from_oracle = rho * rho * om[-1] / 2.0
    kappa = L / mu
    Ra = (np.sqrt(kappa) - 1) / (np.sqrt(kappa) + 1)
    for name, power, value, text in _read_printed_constants():
        base = R_from_oracle if name == "R" else Ra
        assert abs(base ** power - value) <= _printed_tolerance(text), (name, power, base ** power)
    # and R factorises as the lemma states
    assert abs(R_from_oracle - (kappa - 1) / (kappa + 1) * Ra) < 1e-12


@pytest.mark.parametrize("seed", range(5))
def test_omega_lemmas(seed):
    rng = np.random.default_rng(seed)
    mu = 10 ** rng.uniform(-3, 0)
    L = mu * (1.0 + 10 ** rng.uniform(-2, 4))
    r = 40
    om = oracle.omega_schedule(L, mu, r)
    rho = (L - mu) / (L + mu)
    star = 2 * (1 - np.sqrt(1 - rho ** 2)) / rho ** 2
    assert om[0] == 2.0
    assert np.all(np.diff(om) <= 1e-15)                      # non-increasing
    assert np.all(om >= star - 1e-12) and star > 1.0          # bounded below by omega*_1 > 1
    assert np.all((4 - rho ** 2 * om >= 2 - 1e-12) & (4 - rho ** 2 * om <= 4))
    kappa = L / mu
    R = (kappa - 1) / (kappa + 1) * (np.sqrt(kappa) - 1) / (np.sqrt(kappa) + 1)
    i = np.arange(r + 1)
    assert np.all(om - star <= R ** i * (2.0 - star) * (1 + 1e-9) + 1e-15)


def test_omega_equal_bounds():
    # L == mu: rho = 0, every omega_i (i >= 1) is 1
    om = oracle.omega_schedule(0.7, 0.7, 5)
    assert om[0] == 2.0 and np.all(om[1:] == 1.0)


# --------------------------------------------------------------------------------------------
# Algorithm 1: closed form through Chebyshev polynomials on an eigen-decomposed matrix
# --------------------------------------------------------------------------------------------

@pytest.mark.parametrize("r", [0, 1, 2, 3, 7, 10, 16, 30])
def test_chebyshev_closed_form(r):
    """For an eigenvalue h in [mu, L] the r-th iterate has component
    (1 - T_{r+1}(z) / T_{r+1}(sigma)) q_h / h,  z = (L + mu - 2h)/(L - mu), sigma = (L + mu)/(L - mu):
    the textbook Chebyshev semi-iteration residual polynomial."""
    rng = np.random.default_rng(100 + r)
    D = 12
    mu, L = 0.3, 4.0
    h = np.concatenate([[mu, L], rng.uniform(mu, L, D - 2)])
    Qm, _ = np.linalg.qr(rng.standard_normal((D, D)))
    A = (Qm * h) @ Qm.T
    q = rng.standard_normal(D)
    xi = oracle.chebyshev(A, q, L, mu, r)
    z = (L + mu - 2 * h) / (L - mu)
    sigma = (L + mu) / (L - mu)
    factor = 1.0 - _cheb_T(r + 1, z) / _cheb_T(r + 1, np.array([sigma]))[0]
    expected = Qm @ (factor * (Qm.T @ q) / h)
    np.testing.assert_allclose(xi, expected, rtol=0, atol=1e-12 * np.abs(expected).max())


def test_chebyshev_r0_is_first_gradient_step():
    A = np.diag([1.0, 2.0, 3.0])
    q = np.array([1.0, -2.0, 0.5])
    np.testing.assert_allclose(oracle.chebyshev(A, q, 3.0, 1.0, 0), 2 * q / 4.0, rtol=1e-15)


def test_chebyshev_converges_to_direct_solve_within_bound():
    """||xi_r - x*|| <= ||x*|| / T_{r+1}(1/rho) <= 2 c^{r+1} ||x*||, c = (sqrt(kappa)-1)/(sqrt(kappa)+1)."""
    rng = np.random.default_rng(7)
    D = 16
    B = rng.standard_normal((D, D))
    Hm = B @ B.T / D
    lam = 0.05
    A = Hm + lam * np.eye(D)
    fro = np.linalg.norm(Hm, "fro")
    L, mu = fro + lam, lam
    q = rng.standard_normal(D)
    xstar = np.linalg.solve(A, q)
    rho = (L - mu) / (L + mu)
    kappa = L / mu
    c = (np.sqrt(kappa) - 1) / (np.sqrt(kappa) + 1)
    prev = None
    for r in range(0, 80):
        err = np.linalg.norm(oracle.chebyshev(A, q, L, mu, r) - xstar)
        bound = np.linalg.norm(xstar) / _cheb_T(r + 1, np.array([1 / rho]))[0]
        assert err <= bound * (1 + 1e-9) + 1e-13
        assert bound <= 2 * c ** (r + 1) * np.linalg.norm(xstar) * (1 + 1e-12)
        prev = err
    assert np.linalg.norm(oracle.chebyshev(A, q, L, mu, 400) - xstar) <= 1e-12 * np.linalg.norm(xstar)
    assert prev < 1e-3 * np.linalg.norm(xstar)


def test_cholesky_solver_matches_library():
    rng = np.random.default_rng(3)
    D = 9
    B = rng.standard_normal((D, D))
    A = B @ B.T + 0.1 * np.eye(D)
    q = rng.standard_normal(D)
    np.testing.assert_allclose(oracle.cholesky_solve(A, q), np.linalg.solve(A, q), rtol=1e-10)
    with pytest.raises(np.linalg.LinAlgError):
        oracle.cholesky_solve(-np.eye(3), np.ones(3))


# --------------------------------------------------------------------------------------------
# The layer: brute-force weighted ridge regression, single-token closed form, KF recursion
# --------------------------------------------------------------------------------------------

def test_forward_direct_equals_bruteforce_ridge_regression():
    """With the exact solver the layer output is S_t q_t with S_t the minimiser of
    lambda ||S||_F^2 + sum_i eta_{t,i} ||S k_i - v_i||^2, eta_{t,i} = prod_{j=i+1..t} gamma_j
    (Eq. (rls) with the gating weights of Section 4.1). Solve that by least squares on the stacked system."""
    rng = np.random.default_rng(11)
    B, T, H, d, d_v = 2, 7, 2, 5, 3
    q, k, v, gate, lam = _rand_inputs(rng, B, T, H, d, d_v)
    y = oracle.forward(q, k, v, gate, lam, 0, solver=oracle.SOLVER_CHOLESKY)
    for b in range(B):
        for h in range(H):
            for t in range(T):
                eta = np.array([np.prod(gate[b, i + 1:t + 1, h]) for i in range(t + 1)])
                Kw = np.sqrt(eta)[:, None] * k[b, :t + 1, h]
                Vw = np.sqrt(eta)[:, None] * v[b, :t + 1, h]
                Aug = np.vstack([Kw, np.sqrt(lam[b, t, h]) * np.eye(d)])
                Rhs = np.vstack([Vw, np.zeros((d, d_v))])
                St, *_ = np.linalg.lstsq(Aug, Rhs, rcond=None)      # S^T
                np.testing.assert_allclose(y[b, t, h], St.T @ q[b, t, h], rtol=1e-8, atol=1e-10)


@pytest.mark.parametrize("r", [0, 1, 4, 9])
def test_single_token_closed_form(r):
    """T = 1, ||k|| = 1: H_1 = k k^T, ||H_1||_F = 1, L = 1 + lambda is the top eigenvalue, so
    y_1 = v (k^T q) (1 - (-1)^{r+1} / T_{r+1}(1 + 2 lambda)) / (1 + lambda)."""
    rng = np.random.default_rng(20 + r)
    d = 6
    k = rng.standard_normal(d); k /= np.linalg.norm(k)
    q = rng.standard_normal(d)
    v = rng.standard_normal(d)
    lam = 0.37
    y = oracle.forward(q.reshape(1, 1, 1, d), k.reshape(1, 1, 1, d), v.reshape(1, 1, 1, d),
                       np.full((1, 1, 1), 0.9), np.full((1, 1, 1), lam), r)
    Tn = _cheb_T(r + 1, np.array([1 + 2 * lam]))[0]
    expected = v * (k @ q) * (1 - (-1) ** (r + 1) / Tn) / (1 + lam)
    np.testing.assert_allclose(y.reshape(d), expected, rtol=1e-12, atol=1e-14)


def test_ungated_constant_lambda_equals_kalman_recursion():
    """gamma = 1 and constant lambda: Eq. (KF) with eta_t = 1 and Phi updated by the Woodbury identity."""
    rng = np.random.default_rng(5)
    T, d, d_v = 12, 6, 4
    q, k, v, _, _ = _rand_inputs(rng, 1, T, 1, d, d_v)
    lam = 0.2
    y = oracle.forward(q, k, v, np.ones((1, T, 1)), np.full((1, T, 1), lam), 0, solver=oracle.SOLVER_CHOLESKY)
    S = np.zeros((d_v, d))
    Phi = np.eye(d) / lam
    for t in range(T):
        kt, vt = k[0, t, 0], v[0, t, 0]
        denom = 1.0 + kt @ Phi @ kt
        S = S - np.outer(S @ kt - vt, kt @ Phi) / denom
        Phi = Phi - np.outer(Phi @ kt, kt @ Phi) / denom
        np.testing.assert_allclose(y[0, t, 0], S @ q[0, t, 0], rtol=1e-9, atol=1e-11)


def test_forward_chebyshev_matches_explicit_per_token_solve():
    """The forward's Chebyshev path = Algorithm 1 applied to the explicitly rebuilt H_t + lambda_t I
    (rebuilt here from the definition of eta_{t,i}, not from the recurrence), with L, mu of Section 4.1."""
    rng = np.random.default_rng(13)
    B, T, H, d, d_v, r = 1, 9, 2, 5, 4, 6
    q, k, v, gate, lam = _rand_inputs(rng, B, T, H, d, d_v)
    y, ex = oracle.forward(q, k, v, gate, lam, r, return_fro=True, return_xhat=True)
    for h in range(H):
        for t in range(T):
            eta = np.array([np.prod(gate[0, i + 1:t + 1, h]) for i in range(t + 1)])
            Ht = (k[0, :t + 1, h].T * eta) @ k[0, :t + 1, h]
            Ut = (v[0, :t + 1, h].T * eta) @ k[0, :t + 1, h]
            fro = np.linalg.norm(Ht, "fro")
            assert abs(ex["fro"][0, t, h] - fro) < 1e-12
            l = lam[0, t, h]
            # closed form via eigen-decomposition (independent of the oracle's recurrence)
            hv, Qm = np.linalg.eigh(Ht + l * np.eye(d))
            L, mu = fro + l, l
            z = (L + mu - 2 * hv) / (L - mu)
            sigma = (L + mu) / (L - mu)
            fac = 1 - _cheb_T(r + 1, z) / _cheb_T(r + 1, np.array([sigma]))[0]
            xhat = Qm @ (fac * (Qm.T @ q[0, t, h]) / hv)
            np.testing.assert_allclose(ex["xhat"][0, t, h], xhat, rtol=0, atol=1e-11 * np.abs(xhat).max())
            np.testing.assert_allclose(y[0, t, h], Ut @ xhat, rtol=0, atol=1e-10 * (np.abs(Ut @ xhat).max() + 1))


def test_paper_lambda_rule_and_condition_bound():
    """lambda = None selects lambda_t = a ||H_t||_F; then kappa_t <= (a + 1)/a (Eq. (kappa-ub))
    and lambda_max(H_t) <= ||H_t||_F always."""
    rng = np.random.default_rng(17)
    B, T, H, d = 1, 10, 1, 6
    q, k, v, gate, _ = _rand_inputs(rng, B, T, H, d)
    a = 0.02
    y, ex = oracle.forward(q, k, v, gate, None, 30, lambda_scale=a, return_fro=True, return_state=True)
    y_explicit = oracle.forward(q, k, v, gate, a * ex["fro"], 30)
    np.testing.assert_allclose(y, y_explicit, rtol=1e-13, atol=1e-15)
    Hs = np.zeros((d, d))
    for t in range(T):
        Hs = gate[0, t, 0] * Hs + np.outer(k[0, t, 0], k[0, t, 0])
        ev = np.linalg.eigvalsh(Hs)
        fro = ex["fro"][0, t, 0]
        assert ev[-1] <= fro * (1 + 1e-12)
        kappa = (ev[-1] + a * fro) / (max(ev[0], 0.0) + a * fro)
        assert kappa <= (a + 1) / a * (1 + 1e-12)
    np.testing.assert_allclose(ex["H_final"][0, 0], Hs, rtol=1e-12, atol=1e-14)


def test_huge_lambda_limit_is_scaled_linear_attention():
    # lambda -> infinity: (H + lambda I)^{-1} q -> q / lambda, so lambda * y_t -> U_t q_t.
    # Any r >= 1 reproduces it: kappa -> 1.
    rng = np.random.default_rng(23)
    B, T, H, d = 1, 6, 1, 4
    q, k, v, gate, _ = _rand_inputs(rng, B, T, H, d)
    lam = np.full((B, T, H), 1e9)
    y = oracle.forward(q, k, v, gate, lam, 3)
    U = np.zeros((d, d))
    for t in range(T):
        U = gate[0, t, 0] * U + np.outer(v[0, t, 0], k[0, t, 0])
        np.testing.assert_allclose(1e9 * y[0, t, 0], U @ q[0, t, 0], rtol=1e-6, atol=1e-8)


def test_beta_gate_reduces_to_plain_and_scales_writes():
    rng = np.random.default_rng(29)
    B, T, H, d = 1, 8, 2, 5
    q, k, v, gate, lam = _rand_inputs(rng, B, T, H, d)
    y0 = oracle.forward(q, k, v, gate, lam, 5)
    y1 = oracle.forward(q, k, v, gate, lam, 5, beta=np.ones((B, T, H)))
    np.testing.assert_array_equal(y0, y1)
    beta = rng.uniform(0.2, 1.0, (B, T, H))
    # beta_t k k^T = (sqrt(beta) k)(sqrt(beta) k)^T and beta_t v k^T = (sqrt(beta) v)(sqrt(beta) k)^T
    sb = np.sqrt(beta)[..., None]
    y2 = oracle.forward(q, k, v, gate, lam, 5, beta=beta)
    y3 = oracle.forward(q, sb * k, sb * v, gate, lam, 5)
    np.testing.assert_allclose(y2, y3, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("r", [0, 3, 8])
def test_single_token_closed_form_with_gates(r):
    """T = 1, ||k|| = 1, write gate beta, alpha-connection: H_1 = beta k k^T, ||H_1||_F = beta, L = beta + lambda is
    the top eigenvalue, 1/rho = (beta + 2 lambda) / beta, and along k
    xhat = (k^T q)(1 - (-1)^{r+1} / T_{r+1}(1/rho)) / (beta + lambda); y_1 = beta v k^T (alpha xhat + (1 - alpha) q)."""
    rng = np.random.default_rng(120 + r)
    d = 6
    k = rng.standard_normal(d); k /= np.linalg.norm(k)
    q = rng.standard_normal(d)
    v = rng.standard_normal(d)
    lam, beta, alpha = 0.21, 0.6, 0.3
    one = lambda x: np.full((1, 1, 1), x)
    y = oracle.forward(q.reshape(1, 1, 1, d), k.reshape(1, 1, 1, d), v.reshape(1, 1, 1, d), one(0.8), one(lam), r,
                       beta=one(beta), alpha=one(alpha))
    Tn = _cheb_T(r + 1, np.array([(beta + 2 * lam) / beta]))[0]
    xk = (k @ q) * (1 - (-1) ** (r + 1) / Tn) / (beta + lam)
    expected = beta * v * (alpha * xk + (1 - alpha) * (k @ q))
    np.testing.assert_allclose(y.reshape(d), expected, rtol=1e-12, atol=1e-14)
    # the paper's lambda rule on the same token: lambda = a ||H_1||_F = a beta
    a = 0.35
    y2 = oracle.forward(q.reshape(1, 1, 1, d), k.reshape(1, 1, 1, d), v.reshape(1, 1, 1, d), one(0.8), None, r,
                        beta=one(beta), alpha=one(alpha), lambda_scale=a)
    Tn2 = _cheb_T(r + 1, np.array([1 + 2 * a]))[0]
    xk2 = (k @ q) * (1 - (-1) ** (r + 1) / Tn2) / (beta * (1 + a))
    np.testing.assert_allclose(y2.reshape(d), beta * v * (alpha * xk2 + (1 - alpha) * (k @ q)), rtol=1e-12, atol=1e-14)


def test_alpha_connection_interpolates_between_solve_and_linear_attention():
    """y(alpha) = alpha * y(alpha = 1) + (1 - alpha) * U_t q_t, with U_t q_t summed directly from its definition
    (gated linear attention), and alpha = 1 is the plain recurrence."""
    rng = np.random.default_rng(31)
    B, T, H, d = 1, 9, 2, 5
    q, k, v, gate, lam = _rand_inputs(rng, B, T, H, d)
    beta = rng.uniform(0.3, 1.0, (B, T, H))
    alpha = rng.uniform(0.0, 1.0, (B, T, H))
    y1 = oracle.forward(q, k, v, gate, lam, 6, beta=beta)
    np.testing.assert_array_equal(y1, oracle.forward(q, k, v, gate, lam, 6, beta=beta, alpha=np.ones((B, T, H))))
    ya = oracle.forward(q, k, v, gate, lam, 6, beta=beta, alpha=alpha)
    for h in range(H):
        for t in range(T):
            lin = np.zeros(d)
            for j in range(t + 1):
                decay = np.prod(gate[0, j + 1:t + 1, h])
                lin += decay * beta[0, j, h] * v[0, j, h] * (k[0, j, h] @ q[0, t, h])
            want = alpha[0, t, h] * y1[0, t, h] + (1 - alpha[0, t, h]) * lin
            np.testing.assert_allclose(ya[0, t, h], want, rtol=1e-11, atol=1e-13)
    # decode step: same readout
    Hs = np.zeros((B, H, d, d)); Us = np.zeros((B, H, d, d))
    for t in range(T):
        yd = oracle.decode_step(Hs, Us, q[:, t], k[:, t], v[:, t], gate[:, t], lam[:, t], 6, beta=beta[:, t],
                                alpha=alpha[:, t])
        np.testing.assert_allclose(yd, ya[:, t], rtol=1e-12, atol=1e-14)


# --------------------------------------------------------------------------------------------
# Chunk identities of Section 4.2.1 against the step-by-step recurrence
# --------------------------------------------------------------------------------------------

@pytest.mark.parametrize("C", [1, 8, 24])
def test_chunk_identities(C):
    rng = np.random.default_rng(31 + C)
    d, T0 = 6, 5
    T = T0 + C
    q, k, v, gate, lam = _rand_inputs(rng, 1, T, 1, d)
    # state after T0 tokens = initial state of the chunk
    _, ex0 = oracle.forward(q[:, :T0], k[:, :T0], v[:, :T0], gate[:, :T0], lam[:, :T0], 0, return_state=True)
    H0, U0 = ex0["H_final"][0, 0], ex0["U_final"][0, 0]
    Kc, Vc, gc = k[0, T0:, 0], v[0, T0:, 0], gate[0, T0:, 0]
    # per-token states of the chunk from the step-by-step oracle
    states = []
    for c in range(1, C + 1):
        _, exc = oracle.forward(q[:, :T0 + c], k[:, :T0 + c], v[:, :T0 + c], gate[:, :T0 + c], lam[:, :T0 + c], 0,
                                return_state=True, return_fro=True)
        states.append((exc["H_final"][0, 0], exc["U_final"][0, 0], exc["fro"][0, -1, 0]))
    Hc_unrolled = chunked.unrolled_states(H0, Kc, gc)
    fro_chunk = chunked.frobenius_norms(H0, Kc, gc)
    Xi = rng.standard_normal((C, d))
    mv = chunked.chunk_matvec(H0, Kc, gc, Xi)
    for c in range(C):
        np.testing.assert_allclose(Hc_unrolled[c], states[c][0], rtol=1e-12, atol=1e-14)
        assert abs(fro_chunk[c] - states[c][2]) <= 1e-12 * states[c][2]
        np.testing.assert_allclose(mv[c], states[c][0] @ Xi[c], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(chunked.chunk_end_state(H0, Kc, Kc, gc), states[-1][0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(chunked.chunk_end_state(U0, Vc, Kc, gc), states[-1][1], rtol=1e-12, atol=1e-14)


def test_decay_mask_convention():
    # token j's own outer product has weight 1 at time j; gamma_c multiplies what came before c
    gamma = np.array([0.5, 0.25, 0.8])
    zeta, M = chunked.decay_mask(gamma)
    np.testing.assert_allclose(zeta, [0.5, 0.125, 0.1])
    np.testing.assert_allclose(M, [[1, 0.25, 0.2], [0, 1, 0.8], [0, 0, 1]])


# --------------------------------------------------------------------------------------------
# State hand-off: split sequences and recurrent decoding
# --------------------------------------------------------------------------------------------

def test_split_sequence_and_decode_handoff():
    rng = np.random.default_rng(41)
    B, T, H, d, d_v, r = 2, 11, 2, 5, 3, 4
    q, k, v, gate, lam = _rand_inputs(rng, B, T, H, d, d_v)
    y_full, ex_full = oracle.forward(q, k, v, gate, lam, r, return_state=True)
    T1 = 6
    y_a, ex_a = oracle.forward(q[:, :T1], k[:, :T1], v[:, :T1], gate[:, :T1], lam[:, :T1], r, return_state=True)
    y_b, ex_b = oracle.forward(q[:, T1:], k[:, T1:], v[:, T1:], gate[:, T1:], lam[:, T1:], r,
                               H_init=ex_a["H_final"], U_init=ex_a["U_final"], return_state=True)
    np.testing.assert_allclose(np.concatenate([y_a, y_b], axis=1), y_full, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(ex_b["H_final"], ex_full["H_final"], rtol=1e-13)
    # decode steps from the prefill state
    Hs, Us = ex_a["H_final"].copy(), ex_a["U_final"].copy()
    for t in range(T1, T):
        y_t = oracle.decode_step(Hs, Us, q[:, t], k[:, t], v[:, t], gate[:, t], lam[:, t], r)
        np.testing.assert_allclose(y_t, y_full[:, t], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(Us, ex_full["U_final"], rtol=1e-13)


def test_initial_state_is_decayed_by_first_gate():
    # gamma_0 multiplies H_init: with k_0 = 0 the state after one token is gamma_0 * H_init
    d = 4
    Hi = np.eye(d)[None, None] * 2.0
    Ui = np.arange(d * d, dtype=float).reshape(1, 1, d, d)
    z = np.zeros((1, 1, 1, d))
    _, ex = oracle.forward(z + 1.0, z, z, np.full((1, 1, 1), 0.25), np.full((1, 1, 1), 1.0), 2,
                           H_init=Hi, U_init=Ui, return_state=True)
    np.testing.assert_allclose(ex["H_final"], 0.25 * Hi)
    np.testing.assert_allclose(ex["U_final"], 0.25 * Ui)


def test_zero_gate_resets_the_state():
    """A gate of exactly 0 discards the past: two sequences concatenated with gamma = 0 at the seam give the outputs
    of the two sequences run separately (packed variable-length batches rest on this)."""
    rng = np.random.default_rng(41)
    B, T, H, d = 1, 11, 2, 4
    q, k, v, gate, lam = _rand_inputs(rng, B, T, H, d)
    cut = 6
    gate[:, cut] = 0.0
    y = oracle.forward(q, k, v, gate, lam, 5)
    ya = oracle.forward(q[:, :cut], k[:, :cut], v[:, :cut], gate[:, :cut], lam[:, :cut], 5)
    gb = gate[:, cut:].copy(); gb[:, 0] = 0.7
    yb = oracle.forward(q[:, cut:], k[:, cut:], v[:, cut:], gb, lam[:, cut:], 5)
    np.testing.assert_allclose(y[:, :cut], ya, rtol=0, atol=0)
    np.testing.assert_allclose(y[:, cut:], yb, rtol=1e-13, atol=1e-15)
