"""GPU parity: gka_decode_step against the oracle's recurrent step."""
import numpy as np
import pytest

import oracle
from paper_2511_21016_amd import binding, synth
from gka_testutil import pair_rel_err, to_device, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d,dtype", [(64, "f32"), (128, "f32"), (128, "bf16"), (64, "bf16")])
def test_decode_steps_from_oracle_prefill(d, dtype):
    import torch
    base = synth.CFG5 if dtype == "bf16" else synth.CFG1
    w = base.scaled(B=3, H=2, T=40, d=d, n_iter=6, seed=31 + d)
    x = synth.make_inputs(w)
    _, ex = oracle.forward(x["q"], x["k"], x["v"], x["gate"], x["lam"], w.n_iter, return_state=True)
    Hs, Us = ex["H_final"].copy(), ex["U_final"].copy()
    Hd = to_device(Hs.astype(np.float32), "f32")
    Ud = to_device(Us.astype(np.float32), "f32")
    Hs, Us = to_host(Hd), to_host(Ud)            # oracle continues from the exact fp32 states
    n_steps = 12
    steps = synth.make_decode_tokens(w, n_steps)
    tol = 2e-2 if dtype == "bf16" else 1e-4
    for s in range(n_steps):
        q, k, v = (to_device(steps[n][s], dtype) for n in ("q", "k", "v"))
        gate, lam = to_device(steps["gate"][s], "f32"), to_device(steps["lam"][s], "f32")
        o = binding.gka_decode_step(Hd, Ud, q, k, v, gate, lam, w.n_iter)
        torch.cuda.synchronize()
        ref = oracle.decode_step(Hs, Us, steps["q"][s], steps["k"][s], steps["v"][s], steps["gate"][s],
                                 steps["lam"][s], w.n_iter)
        y = to_host(o)
        err = np.abs(y - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
        assert err.max() <= tol, (s, err.max())
    np.testing.assert_allclose(to_host(Hd), Hs, rtol=0, atol=1e-5 * np.abs(Hs).max())
    np.testing.assert_allclose(to_host(Ud), Us, rtol=0, atol=1e-5 * np.abs(Us).max())


@pytest.mark.parametrize("d,dtype", [(128, "f32"), (64, "bf16")])
def test_decode_layer_variants(d, dtype):
    """Write gate, alpha-connection and lambda = a ||H||_F together, stepping from zero states."""
    import torch
    base = synth.CFG5 if dtype == "bf16" else synth.CFG1
    w = base.scaled(B=2, H=3, T=1, d=d, n_iter=7, seed=77 + d)
    n_steps = 10
    steps = synth.make_decode_tokens(w, n_steps)
    gates = synth.make_gates(w, T=n_steps)                      # [B, n_steps, H]
    Hs = np.zeros((w.B, w.H, d, d)); Us = np.zeros((w.B, w.H, d, d))
    Hd, Ud = to_device(Hs.astype(np.float32), "f32"), to_device(Us.astype(np.float32), "f32")
    tol = 2e-2 if dtype == "bf16" else 1e-4
    for s in range(n_steps):
        q, k, v = (to_device(steps[n][s], dtype) for n in ("q", "k", "v"))
        beta, alpha = np.ascontiguousarray(gates["beta"][:, s]), np.ascontiguousarray(gates["alpha"][:, s])
        o = binding.gka_decode_step(Hd, Ud, q, k, v, to_device(steps["gate"][s], "f32"), None, w.n_iter,
                                    beta=to_device(beta, "f32"), alpha=to_device(alpha, "f32"), lambda_scale=0.05)
        torch.cuda.synchronize()
        ref = oracle.decode_step(Hs, Us, steps["q"][s], steps["k"][s], steps["v"][s], steps["gate"][s], None,
                                 w.n_iter, beta=beta, alpha=alpha, lambda_scale=0.05)
        y = to_host(o)
        err = np.abs(y - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
        assert err.max() <= tol, (s, err.max())
    np.testing.assert_allclose(to_host(Hd), Hs, rtol=0, atol=2e-5 * np.abs(Hs).max())
