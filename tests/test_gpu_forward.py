"""GPU parity: gka_forward (through the C ABI) against the fp64 oracle on identical seeded inputs."""
import numpy as np
import pytest

import oracle
from paper_2511_21016_amd import binding, synth
from gka_testutil import pair_rel_err, to_device, to_host, upload_inputs

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4     # max relative error, fp32 configurations
TOL_BF16 = 2e-2    # max relative error, bf16 configurations


def run_forward(w, x, compute=None, **kw):
    import torch
    dev = upload_inputs(x, w.dtype)
    out = binding.gka_forward(dev["q"], dev["k"], dev["v"], dev["gate"], dev["lam"], w.n_iter, compute=compute,
                              chunk=w.chunk, **kw)
    torch.cuda.synchronize()
    return out


def oracle_forward(w, x, **kw):
    return oracle.forward(x["q"], x["k"], x["v"], x["gate"], x["lam"], w.n_iter, **kw)


def test_cfg1_tiny_f32():
    w = synth.CFG1
    x = synth.make_inputs(w)
    o, ex = run_forward(w, x, return_fro=True, return_state=True)
    ref, rex = oracle_forward(w, x, return_fro=True, return_state=True)
    assert np.abs(to_host(ex["fro"]) - rex["fro"]).max() <= 1e-5 * rex["fro"].max()
    assert pair_rel_err(to_host(o), ref) <= TOL_F32
    np.testing.assert_allclose(to_host(ex["H_final"]), rex["H_final"], rtol=0, atol=1e-5 * np.abs(rex["H_final"]).max())
    np.testing.assert_allclose(to_host(ex["U_final"]), rex["U_final"], rtol=0, atol=1e-5 * np.abs(rex["U_final"]).max())


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("T", [1, 37, 64, 200])
@pytest.mark.parametrize("n_iter", [0, 1, 5])
def test_f32_small_shapes(d, T, n_iter):
    w = synth.CFG1.scaled(B=2, H=3, T=T, d=d, n_iter=n_iter, seed=100 + T + d + n_iter)
    x = synth.make_inputs(w)
    o, ex = run_forward(w, x, return_fro=True)
    ref, rex = oracle_forward(w, x, return_fro=True)
    assert np.abs(to_host(ex["fro"]) - rex["fro"]).max() <= 1e-5 * rex["fro"].max()
    assert pair_rel_err(to_host(o), ref) <= TOL_F32


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("T", [50, 256, 333])
def test_bf16_small_shapes(d, T):
    w = synth.CFG2.scaled(B=2, H=2, T=T, d=d, seed=200 + T + d)
    x = synth.make_inputs(w)
    o, ex = run_forward(w, x, return_fro=True)
    ref, rex = oracle_forward(w, x, return_fro=True)
    assert np.abs(to_host(ex["fro"]) - rex["fro"]).max() <= 5e-3 * rex["fro"].max()
    assert pair_rel_err(to_host(o), ref) <= TOL_BF16


@pytest.mark.parametrize("d", [64, 128])
def test_bf16_io_f32_compute(d):
    w = synth.CFG4.scaled(B=1, H=2, T=300, d=d)
    x = synth.make_inputs(w)
    o = run_forward(w, x, compute=binding.GKA_COMPUTE_F32)
    ref = oracle_forward(w, x)
    assert pair_rel_err(to_host(o), ref) <= TOL_BF16


def test_initial_and_final_state_handoff():
    """forward(T) == forward(T1) followed by forward(T - T1) started from the returned state."""
    w = synth.CFG1.scaled(B=1, H=2, T=300, d=64, n_iter=6, seed=7)
    x = synth.make_inputs(w)
    T1 = 130
    xa = {n: a[:, :T1] for n, a in x.items()}
    xb = {n: np.ascontiguousarray(a[:, T1:]) for n, a in x.items()}
    xa = {n: np.ascontiguousarray(a) for n, a in xa.items()}
    o_full, ex_full = run_forward(w, x, return_state=True)
    o_a, ex_a = run_forward(w.scaled(T=T1), xa, return_state=True)
    o_b, ex_b = run_forward(w.scaled(T=w.T - T1), xb, H_init=ex_a["H_final"], U_init=ex_a["U_final"], return_state=True)
    ref = oracle_forward(w, x)
    y = np.concatenate([to_host(o_a), to_host(o_b)], axis=1)
    assert pair_rel_err(y, ref) <= TOL_F32
    assert pair_rel_err(to_host(o_full), ref) <= TOL_F32
    np.testing.assert_allclose(to_host(ex_b["H_final"]), to_host(ex_full["H_final"]), rtol=0, atol=1e-5)


@pytest.mark.parametrize("compute", ["bf16", "f32"])
def test_multi_slab_with_state_carry(compute):
    """The sequence is processed as several chunk slabs (states carried between launches), with a ragged tail
    and non-zero initial states; final states are checked too."""
    w = synth.CFG2.scaled(B=8, H=16, T=1000, seed=77)
    x = synth.make_inputs(w)
    cm = binding.GKA_COMPUTE_BF16 if compute == "bf16" else binding.GKA_COMPUTE_F32
    params = binding.make_params(w.B, w.H, w.T, w.d, w.n_iter, binding.GKA_BF16, cm)
    one_slab = binding.forward_workspace_bytes(params)
    # a workspace budget small enough that this problem is cut into slabs of four chunks (two-phase kernels)
    slab = dict(slab_state_bytes=48 << 20, path=binding.GKA_PATH_TWO_PHASE)
    params = binding.make_params(w.B, w.H, w.T, w.d, w.n_iter, binding.GKA_BF16, cm, slab_state_bytes=48 << 20)
    assert binding.forward_workspace_bytes(params) < one_slab // 2
    rng = np.random.default_rng(5)
    A = rng.standard_normal((w.B, w.H, w.d, 8)).astype(np.float32)
    Hi = np.einsum("bhik,bhjk->bhij", A, A).astype(np.float32) / 8
    Ui = rng.standard_normal((w.B, w.H, w.d, w.d)).astype(np.float32) * 0.1
    cmode = binding.GKA_COMPUTE_BF16 if compute == "bf16" else binding.GKA_COMPUTE_F32
    o, ex = run_forward(w, x, compute=cmode, H_init=to_device(Hi, "f32"), U_init=to_device(Ui, "f32"),
                        return_state=True, **slab)
    ref, rex = oracle_forward(w, x, H_init=Hi, U_init=Ui, return_state=True)
    err = pair_rel_err(to_host(o), ref)
    assert err <= TOL_BF16, err
    tol_state = 5e-3 if compute == "bf16" else 2e-5
    assert np.abs(to_host(ex["H_final"]) - rex["H_final"]).max() <= tol_state * np.abs(rex["H_final"]).max()
    assert np.abs(to_host(ex["U_final"]) - rex["U_final"]).max() <= tol_state * np.abs(rex["U_final"]).max()


@pytest.mark.parametrize("compute", ["bf16", "f32"])
@pytest.mark.parametrize("d", [64, 128])
def test_explicit_strides_head_major_layout(compute, d):
    """q, k, v, o stored [B,H,T,d] (heads outermost) and passed through the stride arguments of the C ABI."""
    import torch
    w = synth.CFG2.scaled(B=2, H=3, T=200, d=d, seed=11)
    x = synth.make_inputs(w)
    dev = {n: to_device(np.ascontiguousarray(np.transpose(x[n], (0, 2, 1, 3))), "bf16") for n in ("q", "k", "v")}
    gate, lam = to_device(x["gate"], "f32"), to_device(x["lam"], "f32")
    o = torch.zeros_like(dev["v"])
    cm = binding.GKA_COMPUTE_BF16 if compute == "bf16" else binding.GKA_COMPUTE_F32
    params = binding.make_params(w.B, w.H, w.T, w.d, w.n_iter, binding.GKA_BF16, cm,
                                 strides=(w.H * w.T * w.d, w.d, w.T * w.d))
    ws = torch.empty(binding.forward_workspace_bytes(params), dtype=torch.uint8, device="cuda")
    st = binding.forward_raw(params, dev["q"].data_ptr(), dev["k"].data_ptr(), dev["v"].data_ptr(), gate.data_ptr(),
                             lam.data_ptr(), o.data_ptr(), workspace=ws.data_ptr(), workspace_bytes=ws.numel(),
                             stream=torch.cuda.current_stream().cuda_stream)
    assert st == binding.GKA_OK
    torch.cuda.synchronize()
    ref = oracle_forward(w, x)
    y = np.transpose(to_host(o), (0, 2, 1, 3))
    assert pair_rel_err(y, ref) <= TOL_BF16


VARIANTS = {
    "beta": dict(beta=True),
    "alpha": dict(alpha=True),
    "lambda_rule": dict(rule=True),
    "all": dict(beta=True, alpha=True, rule=True),
}


@pytest.mark.parametrize("which", sorted(VARIANTS))
@pytest.mark.parametrize("dtype,compute,d", [("f32", "f32", 64), ("f32", "f32", 128), ("bf16", "bf16", 128),
                                             ("bf16", "bf16", 64), ("bf16", "f32", 128)])
def test_layer_variants(which, dtype, compute, d):
    """Write gate beta_t, alpha-connection and the rule lambda_t = a ||H_t||_F (a = 0.02, the paper's default),
    one at a time and together, on a ragged multi-chunk sequence."""
    import torch
    sel = VARIANTS[which]
    base = synth.CFG1 if dtype == "f32" else synth.CFG2
    w = base.scaled(B=2, H=2, T=300, d=d, n_iter=8, seed=50 + d)
    x = synth.make_inputs(w)
    gates = synth.make_gates(w)
    beta = gates["beta"] if sel.get("beta") else None
    alpha = gates["alpha"] if sel.get("alpha") else None
    # a few tokens write nothing at all
    if beta is not None:
        beta = beta.copy()
        beta[:, 5::37] = 0.0
    a = 0.02 if sel.get("rule") else 0.0
    dev = upload_inputs(x, w.dtype)
    cm = binding.GKA_COMPUTE_BF16 if compute == "bf16" else binding.GKA_COMPUTE_F32
    o, ex = binding.gka_forward(dev["q"], dev["k"], dev["v"], dev["gate"], None if a else dev["lam"], w.n_iter,
                                compute=cm, beta=None if beta is None else to_device(beta, "f32"),
                                alpha=None if alpha is None else to_device(alpha, "f32"), lambda_scale=a,
                                return_fro=True, return_state=True)
    torch.cuda.synchronize()
    ref, rex = oracle.forward(x["q"], x["k"], x["v"], x["gate"], None if a else x["lam"], w.n_iter, beta=beta,
                              alpha=alpha, lambda_scale=a, return_fro=True, return_state=True)
    tol = TOL_F32 if compute == "f32" and dtype == "f32" else TOL_BF16
    err = pair_rel_err(to_host(o), ref)
    assert err <= tol, err
    ftol = 1e-5 if dtype == "f32" else 5e-3
    assert np.abs(to_host(ex["fro"]) - rex["fro"]).max() <= ftol * rex["fro"].max()
    stol = 2e-5 if compute == "f32" else 5e-3
    assert np.abs(to_host(ex["U_final"]) - rex["U_final"]).max() <= stol * np.abs(rex["U_final"]).max()


@pytest.mark.parametrize("dtype,compute,lam_min", [("f32", "f32", 1e-4), ("bf16", "f32", 1e-4), ("bf16", "bf16", 1e-2)])
def test_degenerate_values(dtype, compute, lam_min):
    """Zero keys (H_t stays 0 for a while), zero queries and values, gates of exactly 1 and gates so small that the
    whole past is forgotten within a token, lambda over many decades, many passes: finite outputs and parity.
    With bf16 operands lambda starts at 1e-2: below that the first tokens (rank-one H_t) have |xhat| a thousand times
    |y|, which is the regime the fp32-operand mode exists for."""
    base = synth.CFG1 if dtype == "f32" else synth.CFG2
    w = base.scaled(B=1, H=4, T=200, d=64, n_iter=40, seed=91)
    x = {n: a.copy() for n, a in synth.make_inputs(w).items()}
    x["k"][:, :70, 0] = 0.0                    # head 0: nothing written for the first 70 tokens
    x["q"][:, 100:110, 1] = 0.0
    x["v"][:, 120:130, 1] = 0.0
    x["gate"][:, :, 2] = 1.0                   # head 2: no forgetting
    x["gate"][:, 50::17, 3] = 1e-30            # head 3: hard resets (log2 below the documented floor of exp(-100))
    x["gate"][:, 90, 3] = 0.999
    lam = np.geomspace(lam_min, 1e4, w.T).astype(np.float32)
    x["lam"][:] = lam[None, :, None]
    cm = binding.GKA_COMPUTE_BF16 if compute == "bf16" else binding.GKA_COMPUTE_F32
    o, ex = run_forward(w, x, compute=cm, return_fro=True)
    y = to_host(o)
    assert np.isfinite(y).all()
    ref, rex = oracle_forward(w, x, return_fro=True)
    err = pair_rel_err(y, ref)
    assert err <= (TOL_F32 if dtype == "f32" else TOL_BF16), err
    assert np.abs(to_host(ex["fro"]) - rex["fro"]).max() <= (1e-5 if dtype == "f32" else 5e-3) * rex["fro"].max()


def test_more_pairs_than_one_batch():
    """More (batch, head) pairs than the library processes per launch (1024): the pair-batch loop with non-zero
    initial states and returned final states, ragged T."""
    w = synth.CFG2.scaled(B=41, H=32, T=100, d=64, n_iter=6, seed=123)
    x = synth.make_inputs(w)
    rng = np.random.default_rng(6)
    A = rng.standard_normal((w.B, w.H, w.d, 4)).astype(np.float32)
    Hi = np.einsum("bhik,bhjk->bhij", A, A).astype(np.float32) / 4
    Ui = rng.standard_normal((w.B, w.H, w.d, w.d)).astype(np.float32) * 0.1
    o, ex = run_forward(w, x, H_init=to_device(Hi, "f32"), U_init=to_device(Ui, "f32"), return_state=True)
    ref, rex = oracle_forward(w, x, H_init=Hi, U_init=Ui, return_state=True)
    assert pair_rel_err(to_host(o), ref) <= TOL_BF16
    assert np.abs(to_host(ex["H_final"]) - rex["H_final"]).max() <= 5e-3 * np.abs(rex["H_final"]).max()
    assert np.abs(to_host(ex["U_final"]) - rex["U_final"]).max() <= 5e-3 * np.abs(rex["U_final"]).max()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_packed_variable_length_sequences(dtype):
    """Sequences of different lengths concatenated along T, the gate of every sequence's first token set to 0 (the
    library treats it as exp(-100), which wipes the state): every sequence must come out as if it had been run alone
    from zero states, whatever the chunk boundaries."""
    base = synth.CFG1 if dtype == "f32" else synth.CFG2
    lengths = [70, 1, 130, 63, 64, 56]
    w = base.scaled(B=1, H=3, T=sum(lengths), d=64, n_iter=6, seed=19)
    x = {n: a.copy() for n, a in synth.make_inputs(w).items()}
    starts = np.cumsum([0] + lengths[:-1])
    x["gate"][:, starts] = 0.0
    o = run_forward(w, x)
    y = to_host(o)
    assert np.isfinite(y).all()
    tol = TOL_F32 if dtype == "f32" else TOL_BF16
    for s0, n in zip(starts, lengths):
        part = {name: np.ascontiguousarray(a[:, s0:s0 + n]) for name, a in x.items()}
        part["gate"][:, 0] = 0.5                 # irrelevant: the sequence starts from zero states
        ref = oracle.forward(part["q"], part["k"], part["v"], part["gate"], part["lam"], w.n_iter)
        err = pair_rel_err(y[:, s0:s0 + n], ref)
        assert err <= tol, (s0, n, err)


def _random_case(i):
    """Seeded draw of one configuration: shape, dtypes, variants, initial state."""
    rng = np.random.default_rng(9000 + i)
    dtype, compute = [("f32", "f32"), ("bf16", "bf16"), ("bf16", "f32")][int(rng.integers(3))]
    return dict(B=int(rng.integers(1, 4)), H=int(rng.integers(1, 5)), T=int(rng.integers(1, 300)),
                d=int(rng.choice([64, 128])), n_iter=int(rng.integers(0, 13)), dtype=dtype, compute=compute,
                beta=bool(rng.integers(2)), alpha=bool(rng.integers(2)), rule=bool(rng.integers(2)),
                init=bool(rng.integers(2)), seed=9000 + i)


@pytest.mark.parametrize("i", range(24))
def test_random_configurations(i):
    """24 seeded random draws over shapes (ragged T included), dtypes, compute modes, layer variants and initial
    states: output and final states against the oracle."""
    import torch
    c = _random_case(i)
    base = synth.CFG2 if c["dtype"] == "bf16" else synth.CFG1
    w = base.scaled(B=c["B"], H=c["H"], T=c["T"], d=c["d"], n_iter=c["n_iter"], seed=c["seed"])
    x = synth.make_inputs(w)
    gates = synth.make_gates(w)
    kw, okw = {}, {}
    if c["beta"]:
        kw["beta"], okw["beta"] = to_device(gates["beta"], "f32"), gates["beta"]
    if c["alpha"]:
        kw["alpha"], okw["alpha"] = to_device(gates["alpha"], "f32"), gates["alpha"]
    lam_h = x["lam"]
    if c["rule"]:
        kw["lambda_scale"] = okw["lambda_scale"] = 0.05
        lam_h = None
    if c["init"]:
        rng = np.random.default_rng(c["seed"] + 1)
        A = rng.standard_normal((w.B, w.H, w.d, w.d)).astype(np.float32) / np.sqrt(w.d)
        H0 = np.ascontiguousarray(A @ np.transpose(A, (0, 1, 3, 2)))
        H0 = (0.5 * (H0 + np.transpose(H0, (0, 1, 3, 2)))).astype(np.float32)      # exactly symmetric in fp32
        U0 = rng.standard_normal((w.B, w.H, w.d, w.d)).astype(np.float32)
        kw["H_init"], kw["U_init"] = to_device(H0, "f32"), to_device(U0, "f32")
        okw["H_init"], okw["U_init"] = H0.astype(np.float64), U0.astype(np.float64)
    dev = upload_inputs(x, w.dtype)
    cm = binding.GKA_COMPUTE_BF16 if c["compute"] == "bf16" else binding.GKA_COMPUTE_F32
    o, ex = binding.gka_forward(dev["q"], dev["k"], dev["v"], dev["gate"], None if c["rule"] else dev["lam"],
                                w.n_iter, compute=cm, return_state=True, **kw)
    torch.cuda.synchronize()
    ref, rex = oracle.forward(x["q"], x["k"], x["v"], x["gate"], lam_h, w.n_iter, return_state=True, **okw)
    tol = TOL_BF16 if c["compute"] == "bf16" else (TOL_F32 if c["dtype"] == "f32" else TOL_BF16)
    assert pair_rel_err(to_host(o), ref) <= tol, c
    st_tol = 2e-2 if c["compute"] == "bf16" else 2e-5
    for name in ("H_final", "U_final"):
        np.testing.assert_allclose(to_host(ex[name]), rex[name], rtol=0, atol=st_tol * np.abs(rex[name]).max(),
                                   err_msg=str(c))


@pytest.mark.parametrize("dtype,compute,d", [("f32", "f32", 64), ("f32", "f32", 128), ("bf16", "bf16", 128),
                                             ("bf16", "bf16", 64), ("bf16", "f32", 128)])
def test_solve_result_output(dtype, compute, d):
    """xhat_out: the solve's result before the readout, against the oracle's; with the alpha-connection on, so that
    the output is seen to be taken before the mix; and the output o is unchanged by asking for it."""
    import torch
    base = synth.CFG2 if dtype == "bf16" else synth.CFG1
    w = base.scaled(B=2, H=2, T=150, d=d, n_iter=7, seed=606 + d)
    x = synth.make_inputs(w)
    gates = synth.make_gates(w)
    dev = upload_inputs(x, w.dtype)
    cm = binding.GKA_COMPUTE_BF16 if compute == "bf16" else binding.GKA_COMPUTE_F32
    alpha = to_device(gates["alpha"], "f32")
    # (the two-phase kernels in both calls: they are the ones that write xhat)
    o, ex = binding.gka_forward(dev["q"], dev["k"], dev["v"], dev["gate"], dev["lam"], w.n_iter, compute=cm,
                                alpha=alpha, return_xhat=True)
    o2 = binding.gka_forward(dev["q"], dev["k"], dev["v"], dev["gate"], dev["lam"], w.n_iter, compute=cm, alpha=alpha,
                             path=binding.GKA_PATH_TWO_PHASE)
    torch.cuda.synchronize()
    assert torch.equal(o, o2)
    ref, rex = oracle.forward(x["q"], x["k"], x["v"], x["gate"], x["lam"], w.n_iter, alpha=gates["alpha"],
                              return_xhat=True)
    tol = TOL_BF16 if compute == "bf16" else 1e-4
    assert pair_rel_err(to_host(ex["xhat"]), rex["xhat"]) <= tol
    assert pair_rel_err(to_host(o), ref) <= (TOL_F32 if dtype == "f32" else TOL_BF16)


@pytest.mark.parametrize("dtype,compute,d", [("f32", "f32", 64), ("bf16", "f32", 128), ("bf16", "bf16", 128)])
def test_slow_decay_over_many_segments(dtype, compute, d):
    """Gates of about 0.999: after 1300 tokens the first token still weighs e^-2, so every state that the segmented
    chunk scan carries from segment to segment (and the decays it carries them with) shows in the outputs and in
    the final states. The other configurations forget within a chunk or two."""
    base = synth.CFG2 if dtype == "bf16" else synth.CFG1
    w = base.scaled(B=1, H=2, T=1300, d=d, n_iter=8, gate_mean=7.0, seed=4242 + d)
    x = synth.make_inputs(w)
    assert np.prod(x["gate"].astype(np.float64), axis=1).min() > 0.02
    cm = binding.GKA_COMPUTE_BF16 if compute == "bf16" else binding.GKA_COMPUTE_F32
    o, ex = run_forward(w, x, compute=cm, return_state=True)
    ref, rex = oracle_forward(w, x, return_state=True)
    err = pair_rel_err(to_host(o), ref)
    print("slow decay", dtype, compute, d, err)
    assert err <= (TOL_F32 if dtype == "f32" else TOL_BF16), err
    tol_state = 5e-3 if compute == "bf16" else 2e-5
    assert np.abs(to_host(ex["H_final"]) - rex["H_final"]).max() <= tol_state * np.abs(rex["H_final"]).max()
    assert np.abs(to_host(ex["U_final"]) - rex["U_final"]).max() <= tol_state * np.abs(rex["U_final"]).max()
