"""Mutation check of the oracle's pins, on the CPU: a plausible mistake is planted in a COPY of one oracle source
(a wrong weight schedule, sign, index, transposed operand, a missing gate ...), and the pin tests of that oracle are
run on the copy in a child process: every planted mistake must make at least one pin fail. The working tree is never
modified; the GPU is not involved."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (file under oracle/, pin test file, [(label, text, replacement)])
FORWARD = ("gka_oracle.c", "tests/test_oracle_pins.py", [
    ("weight schedule 4 -> 3", "omega = 4.0 / (4.0 - rho * rho * omega);\n        omega_out[i]",
     "omega = 4.0 / (3.0 - rho * rho * omega);\n        omega_out[i]"),
    ("solver's schedule uses rho, not rho^2", "omega = 4.0 / (4.0 - rho * rho * omega);\n        richardson_map",
     "omega = 4.0 / (4.0 - rho * omega);\n        richardson_map"),
    ("omega_0 = 1", "double omega = 2.0;\n    memset(older", "double omega = 1.0;\n    memset(older"),
    ("step 1 / (L + mu)", "const double tau = 2.0 / (L + mu);", "const double tau = 1.0 / (L + mu);"),
    ("residual sign", "out[a] = x[a] + tau * (q[a] - Ax);", "out[a] = x[a] - tau * (q[a] - Ax);"),
    ("right-hand side sign", "out[a] = x[a] + tau * (q[a] - Ax);", "out[a] = x[a] + tau * (-q[a] - Ax);"),
    ("extrapolation from the newer iterate", "mapped[a] = older[a] + omega * (mapped[a] - older[a]);",
     "mapped[a] = newer[a] + omega * (mapped[a] - newer[a]);"),
    ("extrapolation weight omega - 1", "mapped[a] = older[a] + omega * (mapped[a] - older[a]);",
     "mapped[a] = older[a] + (omega - 1.0) * (mapped[a] - older[a]);"),
    ("shifted operand in A x", "Ax += A[(size_t)a * D + b] * x[b];", "Ax += A[(size_t)a * D + b] * x[(b + 1) % D];"),
    ("one pass too many", "for (int i = 1; i <= r; ++i) {\n        omega = 4.0 / (4.0 - rho * rho * omega);\n        richardson_map",
     "for (int i = 0; i <= r; ++i) {\n        omega = 4.0 / (4.0 - rho * rho * omega);\n        richardson_map"),
    ("beta dropped in H", "gamma * Hs[(size_t)i * d_k + j] + beta * k[i] * k[j]",
     "gamma * Hs[(size_t)i * d_k + j] + k[i] * k[j]"),
    ("beta dropped in U", "gamma * Us[(size_t)i * d_k + j] + beta * v[i] * k[j]",
     "gamma * Us[(size_t)i * d_k + j] + v[i] * k[j]"),
    ("U stores k v^T", "beta * v[i] * k[j];", "beta * v[j % d_v] * k[i % d_k];"),
    ("gamma not applied to U", "Us[(size_t)i * d_k + j] = gamma * Us[(size_t)i * d_k + j]",
     "Us[(size_t)i * d_k + j] = Us[(size_t)i * d_k + j]"),
    ("gamma applied after the write", "double h = gamma * Hs[(size_t)i * d_k + j] + beta * k[i] * k[j];",
     "double h = gamma * (Hs[(size_t)i * d_k + j] + beta * k[i] * k[j]);"),
    ("L without lambda", "double L = fro + lambda;", "double L = fro;"),
    ("mu = lambda / 2", "double mu = lambda;", "double mu = 0.5 * lambda;"),
    ("lambda not on the diagonal", "(i == j ? lambda : 0.0)", "0.0"),
    ("alpha swapped", "xi[j] = alpha * xi[j] + (1.0 - alpha) * q[j]", "xi[j] = (1.0 - alpha) * xi[j] + alpha * q[j]"),
    ("norm without the square root", "double fro = sqrt(fro2);", "double fro = fro2;"),
    ("rule uses the squared norm", "a * fro;", "a * fro2;"),
    ("readout with U^T", "s += Us[(size_t)i * d_k + j] * xi[j];", "s += Us[(size_t)j * d_k + i] * xi[j];"),
    ("decode ignores beta", "gate[p], beta ? beta[p] : 1.0,", "gate[p], 1.0,"),
    ("wrong head in the token index", "size_t tok = ((size_t)b * T + t) * H + h;",
     "size_t tok = ((size_t)b * T + t) * H + (H - 1 - h);"),
])
BACKWARD = ("gka_backward_oracle.py", "tests/test_oracle_backward_pins.py", [
    ("sign of the rule's term", "local_H = local_H + dlam[t] * lambda_scale * Ht / fro[t]",
     "local_H = local_H - dlam[t] * lambda_scale * Ht / fro[t]"),
    ("sign of dlambda", "dlam[t] = -(x[t] @ p)", "dlam[t] = (x[t] @ p)"),
    ("gate index of the H accumulator", "accH = gate[t + 1] * accH", "accH = gate[t] * accH"),
    ("gate index of the U accumulator", "accU = gate[t + 1] * accU", "accU = gate[t] * accU"),
    ("dk without the U term", "dk[t] = beta[t] * ((accH + accH.T) @ k[t] + accU.T @ v[t])",
     "dk[t] = beta[t] * ((accH + accH.T) @ k[t])"),
    ("dk without symmetrisation", "dk[t] = beta[t] * ((accH + accH.T) @ k[t] + accU.T @ v[t])",
     "dk[t] = beta[t] * (2 * accH @ k[t] + accU.T @ v[t])"),
    ("dv without beta", "dv[t] = beta[t] * (accU @ k[t])", "dv[t] = (accU @ k[t])"),
    ("dbeta without the U term", "dbeta[t] = k[t] @ accH @ k[t] + v[t] @ accU @ k[t]", "dbeta[t] = k[t] @ accH @ k[t]"),
    ("dgate with the states after the token", "dgate[t] = np.sum(accH * Hs[t]) + np.sum(accU * Us[t])",
     "dgate[t] = np.sum(accH * Hs[t + 1]) + np.sum(accU * Us[t + 1])"),
    ("dq without the alpha path", "dq[t] = p + (1.0 - alpha[t]) * dxt", "dq[t] = p"),
    ("dalpha without q", "dalpha[t] = dxt @ (x[t] - q[t])", "dalpha[t] = dxt @ x[t]"),
    ("second solve without alpha", "p = _solve(Ht + lam_t[t] * np.eye(d_k), alpha[t] * dxt",
     "p = _solve(Ht + lam_t[t] * np.eye(d_k), dxt"),
    ("H gradient from the mixed operand", "local_H = -np.outer(p, x[t])", "local_H = -np.outer(p, xt)"),
    ("U gradient from the unmixed operand", "accU = accU + np.outer(dy[t], xt)", "accU = accU + np.outer(dy[t], x[t])"),
    ("dH_init without the first gate", '"dH_init": gate[0] * accH', '"dH_init": accH'),
    ("dxt with U instead of U^T", "dxt = Ut.T @ dy[t]", "dxt = Ut @ dy[t]"),
])
SKETCH = ("gka_sketch_oracle.py", "tests/test_oracle_sketch_pins.py", [
    ("beta dropped in the sketched H", "beta[t] * np.outer(ks, ks)", "np.outer(ks, ks)"),
    ("beta dropped in U", "U = gate[t] * U + beta[t] * np.outer(v[t], k[t])", "U = gate[t] * U + np.outer(v[t], k[t])"),
    ("gate dropped", "Hs = gate[t] * Hs", "Hs = Hs"),
    ("L without lambda", "fro[t] + lam_t, lam_t, n_iter", "fro[t], lam_t, n_iter"),
    ("rule uses the squared norm", "lambda_scale * fro[t] if rule", "lambda_scale * fro[t] ** 2 if rule"),
    ("right-hand side from k", "rhs = S @ q[t]", "rhs = S @ k[t]"),
    ("up-projection by the pseudo-inverse", "xhat[t] = S.T @ z[t]", "xhat[t] = np.linalg.pinv(S) @ z[t]"),
    ("lambda = 1 on the diagonal", "A = Hs + lam_t * np.eye(d_s)", "A = Hs + np.eye(d_s)"),
    ("norm of absolute values", "fro[t] = np.sqrt(np.sum(Hs * Hs))", "fro[t] = np.sqrt(np.sum(np.abs(Hs)))"),
    ("sketched keys renormalised", "ks = S @ k[t]", "ks = S @ k[t] / np.linalg.norm(S @ k[t])"),
])

GROUPS = {"forward": FORWARD, "backward": BACKWARD, "sketch": SKETCH}
WORKERS = 6                          # child processes at a time, each in a sandbox of its own


def make_sandbox(root):
    """A copy of the oracle, the input generators and the tests (no built libraries, no kernels)."""
    skip = shutil.ignore_patterns("*.so", "_build", "csrc", "__pycache__", "*.o")
    for d in ("oracle", "tests", "paper_2511_21016_amd"):
        shutil.copytree(os.path.join(ROOT, d), os.path.join(root, d), ignore=skip)
    return root


def run_mutant(box, source, pins, label, text, replacement):
    """Plant one mistake in the sandbox's copy of oracle/<source>, run the pins there; returns None if a pin failed,
    else a description of the survivor."""
    original = open(os.path.join(ROOT, "oracle", source)).read()
    if text not in original:
        return f"'{label}': the mutation's anchor text is gone from oracle/{source} (update this test)"
    path = os.path.join(box, "oracle", source)
    with open(path, "w") as f:
        f.write(original.replace(text, replacement, 1))
    lib = os.path.join(box, "oracle", "libgka_oracle.so")
    if os.path.exists(lib):
        os.unlink(lib)                   # the C oracle is rebuilt from the mutated source
    env = {k: v for k, v in os.environ.items() if k not in ("GKA_ORACLE_SANITIZED", "GKA_LIBRARY")}
    env["OMP_NUM_THREADS"] = "1"
    pr = subprocess.run([sys.executable, "-m", "pytest", pins, "-x", "-q", "-p", "no:cacheprovider"], cwd=box, env=env,
                        stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)
    with open(path, "w") as f:
        f.write(original)
    if pr.returncode == 1 and " failed" in pr.stdout:
        return None
    return f"'{label}' survived the pins of oracle/{source} (exit {pr.returncode}):\n" + pr.stdout[-800:]


@pytest.mark.parametrize("group", sorted(GROUPS))
def test_every_planted_mistake_fails_a_pin(group, tmp_path):
    import concurrent.futures
    import queue
    source, pins, mutants = GROUPS[group]
    boxes = queue.Queue()
    for i in range(min(WORKERS, len(mutants))):
        boxes.put(make_sandbox(str(tmp_path / f"box{i}")))

    def job(m):
        box = boxes.get()
        try:
            return run_mutant(box, source, pins, *m)
        finally:
            boxes.put(box)

    with concurrent.futures.ThreadPoolExecutor(max_workers=WORKERS) as pool:
        survivors = [r for r in pool.map(job, mutants) if r is not None]
    assert not survivors, "\n".join(survivors)
