"""The library under HIP graph capture: gka_forward_static (the entry point without allocations or a workspace) followed
by a decode step on the states it leaves, recorded once and replayed several times with eager work and synchronisations
in between. Every replay must reproduce the eager results bit for bit. (The library enqueues kernels only: no
allocation, no synchronisation, no memset or copy nodes.)"""
import numpy as np
import pytest

from paper_2511_21016_amd import binding, synth
from gka_testutil import to_device, upload_inputs

pytestmark = pytest.mark.gpu


def test_forward_static_and_decode_step_replayed_from_a_graph():
    import torch
    w = synth.CFG2.scaled(B=2, H=4, T=600, n_iter=8, seed=4242)
    x = synth.make_inputs(w)
    dev = upload_inputs(x, w.dtype)
    step = synth.make_decode_tokens(w, 1)
    q1, k1, v1 = (to_device(step[n][0], w.dtype) for n in ("q", "k", "v"))
    g1, l1 = to_device(step["gate"][0], "f32"), to_device(step["lam"][0], "f32")
    params = binding.make_params(w.B, w.H, w.T, w.d, w.n_iter, binding.GKA_BF16, binding.GKA_COMPUTE_BF16)
    params1 = binding.make_params(w.B, w.H, 1, w.d, w.n_iter, binding.GKA_BF16, binding.GKA_COMPUTE_F32)

    def buffers():
        f32 = dict(dtype=torch.float32, device="cuda")
        return dict(o=torch.empty_like(dev["v"]), fro=torch.empty((w.B, w.T, w.H), **f32),
                    H=torch.empty((w.B, w.H, w.d, w.d), **f32), U=torch.empty((w.B, w.H, w.d, w.d), **f32),
                    o1=torch.empty_like(v1))

    def enqueue(b):
        stream = torch.cuda.current_stream().cuda_stream
        st = binding.forward_static_raw(params, dev["q"].data_ptr(), dev["k"].data_ptr(), dev["v"].data_ptr(),
                                        dev["gate"].data_ptr(), dev["lam"].data_ptr(), b["o"].data_ptr(), None, None,
                                        b["H"].data_ptr(), b["U"].data_ptr(), b["fro"].data_ptr(), stream)
        assert st == binding.GKA_OK, binding.status_string(st)
        st = binding.decode_step_raw(params1, b["H"].data_ptr(), b["U"].data_ptr(), q1.data_ptr(), k1.data_ptr(),
                                     v1.data_ptr(), g1.data_ptr(), l1.data_ptr(), b["o1"].data_ptr(), stream)
        assert st == binding.GKA_OK, binding.status_string(st)

    want = buffers()
    enqueue(want)                                # eager; also the first call on this device (scratch address, attributes)
    torch.cuda.synchronize()

    got = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue(got)
    torch.cuda.synchronize()

    other = upload_inputs(synth.make_inputs(w.scaled(seed=4243)), w.dtype)
    for replay in range(3):
        for t in got.values():
            t.copy_(torch.full_like(t, float("nan")))           # (a copy kernel, outside the graph)
        # eager work of the program between the replays
        binding.gka_forward(other["q"], other["k"], other["v"], other["gate"], other["lam"], w.n_iter)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in want:
            assert torch.equal(got[name], want[name]), (replay, name)
    assert np.isfinite(got["o1"].float().cpu().numpy()).all()
