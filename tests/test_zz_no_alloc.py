"""gka_forward_static (the entry point for callers that cannot allocate: its kernels' scratch lives in a fixed device
array) against gka_forward on the same inputs, through the C ABI: the outputs, ||H_t||_F and the final states must be
bit-identical (the same kernels, the same launch plan) and meet the oracle; two calls in a row, the second on a smaller
problem that leaves most of the array holding the first call's contents. Also the refusals, which launch nothing."""
import numpy as np
import pytest

import oracle
from paper_2511_21016_amd import binding, synth
from gka_testutil import pair_rel_err, to_host, upload_inputs

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2


def both_entry_points(w, x, walk):
    import torch
    dev = upload_inputs(x, w.dtype)
    ref, ex = binding.gka_forward(dev["q"], dev["k"], dev["v"], dev["gate"], dev["lam"], w.n_iter,
                                  path=binding.GKA_PATH_FUSED, walk_chunks=walk, return_fro=True, return_state=True)
    torch.cuda.synchronize()
    params = binding.make_params(w.B, w.H, w.T, w.d, w.n_iter, binding.GKA_BF16, binding.GKA_COMPUTE_BF16,
                                 walk_chunks=walk)
    o = torch.full_like(dev["v"], float("nan"))
    fro = torch.full((w.B, w.T, w.H), float("nan"), dtype=torch.float32, device="cuda")
    Hf = torch.full((w.B, w.H, w.d, w.d), float("nan"), dtype=torch.float32, device="cuda")
    Uf = torch.full_like(Hf, float("nan"))
    before = torch.cuda.memory_allocated()
    st = binding.forward_static_raw(params, dev["q"].data_ptr(), dev["k"].data_ptr(), dev["v"].data_ptr(),
                                    dev["gate"].data_ptr(), dev["lam"].data_ptr(), o.data_ptr(), None, None,
                                    Hf.data_ptr(), Uf.data_ptr(), fro.data_ptr(),
                                    torch.cuda.current_stream().cuda_stream)
    assert st == binding.GKA_OK, binding.status_string(st)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(o, ref)
    assert torch.equal(fro, ex["fro"])
    assert torch.equal(Hf, ex["H_final"]) and torch.equal(Uf, ex["U_final"])
    return to_host(o)


def test_static_scratch_matches_gka_forward_on_two_calls_in_a_row():
    # 3 pairs x 6 segments of 4 chunks (the last ragged), then 2 pairs x 2 segments: the second call's scratch is a
    # prefix of what the first one left behind
    for (B, H, T, walk, seed) in [(1, 3, 1450, 4, 91), (2, 1, 200, 2, 92)]:
        w = synth.CFG2.scaled(B=B, H=H, T=T, n_iter=10, seed=seed)
        x = synth.make_inputs(w)
        y = both_entry_points(w, x, walk)
        want = oracle.forward(x["q"], x["k"], x["v"], x["gate"], x["lam"], w.n_iter)
        assert pair_rel_err(y, want) <= TOL_BF16


def test_static_scratch_refusals():
    import torch
    t = torch.zeros(64, dtype=torch.float32, device="cuda")
    p = t.data_ptr()
    # 342 workgroups (one segment each): one more than the array holds
    big = binding.make_params(342, 1, 64, 128, 10, binding.GKA_BF16, binding.GKA_COMPUTE_BF16)
    assert binding.forward_static_raw(big, p, p, p, p, p, p) == binding.GKA_ERR_STATIC_SCRATCH
    assert "scratch" in binding.status_string(binding.GKA_ERR_STATIC_SCRATCH)
    # shapes and modes the fused kernels do not cover
    f32 = binding.make_params(1, 1, 64, 128, 10, binding.GKA_F32, binding.GKA_COMPUTE_F32)
    assert binding.forward_static_raw(f32, p, p, p, p, p, p) == binding.GKA_ERR_UNSUPPORTED
    d64 = binding.make_params(1, 1, 64, 64, 10, binding.GKA_BF16, binding.GKA_COMPUTE_BF16)
    assert binding.forward_static_raw(d64, p, p, p, p, p, p) == binding.GKA_ERR_UNSUPPORTED
    two = binding.make_params(1, 1, 64, 128, 10, binding.GKA_BF16, binding.GKA_COMPUTE_BF16,
                              path=binding.GKA_PATH_TWO_PHASE)
    assert binding.forward_static_raw(two, p, p, p, p, p, p) == binding.GKA_ERR_UNSUPPORTED
    # the solve's result as an output is not something the fused kernels write
    xh = binding.make_params(1, 1, 64, 128, 10, binding.GKA_BF16, binding.GKA_COMPUTE_BF16, xhat_out=p)
    assert binding.forward_static_raw(xh, p, p, p, p, p, p) == binding.GKA_ERR_UNSUPPORTED
    assert binding.forward_static_raw(None, p, p, p, p, p, p) == binding.GKA_ERR_NULL
