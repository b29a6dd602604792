"""GPU parity: gka_forward_sketched (through the C ABI) against the latent-sketching oracle on identical seeded
inputs."""
import numpy as np
import pytest

from oracle import gka_sketch_oracle as sk
from paper_2511_21016_amd import binding, synth
from gka_testutil import pair_rel_err, to_device, to_host, upload_inputs

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


def _sketch(rng, shape):
    """Gaussian sketch with unit-norm rows in expectation (float32, not bf16-representable on purpose)."""
    return (rng.standard_normal(shape) / np.sqrt(shape[-1])).astype(np.float32)


@pytest.mark.parametrize("d,d_s,T,per_head,rule,with_beta", [(128, 32, 200, False, False, False),
                                                             (128, 64, 333, True, True, True),
                                                             (128, 17, 64, False, True, False),
                                                             (64, 32, 150, True, False, True),
                                                             (128, 32, 1100, False, False, True)])
def test_sketched_forward_against_oracle(d, d_s, T, per_head, rule, with_beta):
    import torch
    w = synth.CFG2.scaled(B=2, H=2, T=T, d=d, n_iter=8, seed=3100 + d + d_s + T)
    x = synth.make_inputs(w)
    rng = np.random.default_rng(w.seed + 9)
    S = _sketch(rng, (w.H, d_s, d) if per_head else (d_s, d))
    beta = synth.make_gates(w)["beta"] if with_beta else None
    a = 0.05 if rule else 0.0
    dev = upload_inputs(x, w.dtype)
    out = binding.gka_forward_sketched(dev["q"], dev["k"], dev["v"], dev["gate"], None if rule else dev["lam"],
                                       to_device(S, "f32"), w.n_iter, lambda_scale=a,
                                       beta=None if beta is None else to_device(beta, "f32"))
    torch.cuda.synchronize()
    ref = sk.forward_sketched(x["q"], x["k"], x["v"], x["gate"], None if rule else x["lam"], S, w.n_iter, beta=beta,
                              lambda_scale=a)
    err = pair_rel_err(to_host(out), ref)
    print("sketch", d, d_s, T, per_head, rule, with_beta, err)
    # The sketched keys S k_t are an intermediate tensor of the bf16 path, stored in bf16. Solve and readout both work
    # on those stored keys (the readout runs in the sketched space), so the output is the exact layer of slightly
    # perturbed keys and stays inside the forward tolerance, also with the rule's kappa = (1 + a) / a = 21.
    assert err <= TOL_BF16, err


def test_identity_sketch_matches_the_unsketched_forward():
    """d = 64 with S = I: the sketched path (projections, solve, separate readout) against gka_forward itself."""
    import torch
    w = synth.CFG2.scaled(B=1, H=2, T=300, d=64, n_iter=8, seed=77)
    x = synth.make_inputs(w)
    dev = upload_inputs(x, w.dtype)
    S = np.eye(64, dtype=np.float32)
    out = binding.gka_forward_sketched(dev["q"], dev["k"], dev["v"], dev["gate"], dev["lam"], to_device(S, "f32"),
                                       w.n_iter)
    plain = binding.gka_forward(dev["q"], dev["k"], dev["v"], dev["gate"], dev["lam"], w.n_iter)
    torch.cuda.synchronize()
    assert pair_rel_err(to_host(out), to_host(plain).astype(np.float64)) <= TOL_BF16


@pytest.mark.parametrize("i", range(8))
def test_sketched_forward_random_shapes(i):
    """Odd shapes: single tokens, partial chunks, one head, sketch dimensions from 1 to 64."""
    import torch
    rng = np.random.default_rng(5000 + i)
    B, H = int(rng.integers(1, 4)), int(rng.integers(1, 6))
    T = int(rng.choice([1, 2, 63, 64, 65, 129, 300, 700]))
    d = int(rng.choice([64, 128]))
    d_s = int(rng.choice([1, 5, 16, 31, 32, 33, 64]))
    rule = bool(rng.integers(0, 2))
    per_head = bool(rng.integers(0, 2))
    with_beta = bool(rng.integers(0, 2))
    w = synth.CFG2.scaled(B=B, H=H, T=T, d=d, n_iter=int(rng.integers(0, 12)), seed=5100 + i)
    x = synth.make_inputs(w)
    S = _sketch(rng, (H, d_s, d) if per_head else (d_s, d))
    beta = synth.make_gates(w)["beta"] if with_beta else None
    a = 0.05 if rule else 0.0
    dev = upload_inputs(x, w.dtype)
    out = binding.gka_forward_sketched(dev["q"], dev["k"], dev["v"], dev["gate"], None if rule else dev["lam"],
                                       to_device(S, "f32"), w.n_iter, lambda_scale=a,
                                       beta=None if beta is None else to_device(beta, "f32"))
    torch.cuda.synchronize()
    ref = sk.forward_sketched(x["q"], x["k"], x["v"], x["gate"], None if rule else x["lam"], S, w.n_iter, beta=beta,
                              lambda_scale=a)
    err = pair_rel_err(to_host(out), ref)
    print("sketch random", i, dict(B=B, H=H, T=T, d=d, d_s=d_s, rule=rule, per_head=per_head, beta=with_beta,
                                   n_iter=w.n_iter), err)
    assert err <= TOL_BF16, err


@pytest.mark.parametrize("T,n_iter,d_s", [(1, 8, 32), (2, 0, 32), (17, 1, 8), (64, 3, 32), (65, 8, 24), (191, 12, 32)])
def test_small_sketch_degenerate_sizes(T, n_iter, d_s):
    """The kernels of the solve in at most 32 sketched dimensions at the ends of their ranges: single tokens, no pass
    or one, a chunk exactly full, one token beyond it."""
    import torch
    w = synth.CFG2.scaled(B=1, H=3, T=T, d=128, n_iter=n_iter, seed=4400 + 7 * T + n_iter)
    x = synth.make_inputs(w)
    S = _sketch(np.random.default_rng(w.seed + 9), (d_s, 128))
    dev = upload_inputs(x, w.dtype)
    out = binding.gka_forward_sketched(dev["q"], dev["k"], dev["v"], dev["gate"], dev["lam"], to_device(S, "f32"), n_iter)
    torch.cuda.synchronize()
    ref = sk.forward_sketched(x["q"], x["k"], x["v"], x["gate"], x["lam"], S, n_iter)
    y = to_host(out)
    assert np.isfinite(y).all()
    # (a single token has no other token of its pair to be normalised with: all pairs together)
    err = float(np.abs(y - ref).max() / np.abs(ref).max()) if T < 4 else pair_rel_err(y, ref)
    print("small sketch", T, n_iter, d_s, err)
    assert err <= TOL_BF16, err


def test_small_sketch_packed_sequences_and_slow_decay():
    """Gates of 0 inside chunks (packed sequences: the state is wiped) and gates close to 1 over many chunks (the
    states before the chunks carry far): both through the chunk-delta, state-scan and solve kernels."""
    import torch
    w = synth.CFG2.scaled(B=2, H=2, T=1500, d=128, n_iter=8, seed=5151)
    x = synth.make_inputs(w)
    rng = np.random.default_rng(w.seed + 1)
    gate = (1.0 - 10.0 ** rng.uniform(-4.0, -2.0, size=x["gate"].shape)).astype(np.float32)   # 0.99 .. 0.9999
    for b in range(w.B):
        for start in (0, 1, 63, 64, 200, 777, 1499):
            gate[b, start, :] = 0.0
    S = _sketch(np.random.default_rng(w.seed + 9), (w.H, 32, 128))
    beta = synth.make_gates(w)["beta"]
    dev = upload_inputs(x, w.dtype)
    out = binding.gka_forward_sketched(dev["q"], dev["k"], dev["v"], to_device(gate, "f32"), dev["lam"],
                                       to_device(S, "f32"), w.n_iter, beta=to_device(beta, "f32"))
    torch.cuda.synchronize()
    ref = sk.forward_sketched(x["q"], x["k"], x["v"], gate, x["lam"], S, w.n_iter, beta=beta)
    y = to_host(out)
    assert np.isfinite(y).all()
    err = pair_rel_err(y, ref)
    print("small sketch packed / slow decay", err)
    assert err <= TOL_BF16, err


def test_small_and_padded_sketch_solves_agree():
    """d_s = 32 runs on the 32-dimensional kernels, d_s = 33 with a zero last row on the 64-dimensional ones: two
    device implementations of the same operator."""
    import torch
    w = synth.CFG2.scaled(B=1, H=4, T=600, d=128, n_iter=8, seed=6262)
    x = synth.make_inputs(w)
    S32 = _sketch(np.random.default_rng(w.seed + 9), (32, 128))
    S33 = np.concatenate([S32, np.zeros((1, 128), np.float32)], axis=0)
    dev = upload_inputs(x, w.dtype)
    y32 = binding.gka_forward_sketched(dev["q"], dev["k"], dev["v"], dev["gate"], dev["lam"], to_device(S32, "f32"), 8)
    y33 = binding.gka_forward_sketched(dev["q"], dev["k"], dev["v"], dev["gate"], dev["lam"], to_device(S33, "f32"), 8)
    torch.cuda.synchronize()
    err = pair_rel_err(to_host(y32), to_host(y33).astype(np.float64))
    print("small vs padded sketch", err)
    assert err <= TOL_BF16, err
