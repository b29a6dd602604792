"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and rejects bad
arguments on the host before any launch (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2511_21016_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_21016_amd import build
        build.build_library(verbose=False)
    return binding.load_library()


def test_header_symbols_are_exported(lib):
    header = open(os.path.join(ROOT, "include", "gka.h")).read()
    declared = set(re.findall(r"\b(gka_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert binding.version() >= 100
    for s in range(7):
        assert binding.status_string(s)
    assert binding.status_string(binding.GKA_OK) == "ok"


def _p(**kw):
    base = dict(B=2, H=2, T=100, d=128, n_iter=4, io_dtype=binding.GKA_BF16, compute=binding.GKA_COMPUTE_BF16)
    base.update(kw)
    return binding.make_params(**base)


def test_workspace_query(lib):
    assert binding.forward_workspace_bytes(_p()) > 0
    assert binding.forward_workspace_bytes(_p()) % 256 == 0
    # two chunks of a longer sequence need more scratch
    assert binding.forward_workspace_bytes(_p(T=1000)) > binding.forward_workspace_bytes(_p(T=100))
    assert binding.forward_workspace_bytes(_p(d=96)) == 0
    # d = 16, 32 with bf16 operands: chunk-wise kernels with materialised d x d chunk states (two chunks of four
    # pairs: deltas and states of H and U, and the chunks' decays)
    assert binding.forward_workspace_bytes(_p(d=16)) == 4 * (2 * 4 * 16 * 16 * 4) + 256
    assert binding.forward_workspace_bytes(_p(d=32)) == 4 * (2 * 4 * 32 * 32 * 4) + 256
    # the token-by-token path keeps the states in registers; only d = 256 streams U through memory
    assert binding.forward_workspace_bytes(_p(d=16, path=binding.GKA_PATH_RECURRENT)) == 256
    assert binding.forward_workspace_bytes(_p(d=16, io_dtype=binding.GKA_F32, compute=binding.GKA_COMPUTE_F32)) == 256
    assert binding.forward_workspace_bytes(_p(path=binding.GKA_PATH_RECURRENT)) == 256
    assert binding.forward_workspace_bytes(_p(d=256)) == 256 + 4 * 256 * 256 * 4
    assert binding.forward_workspace_bytes(_p(T=0)) == 0


def test_argument_errors_are_reported_before_any_launch(lib):
    fake = 0x1000  # never dereferenced: every case below fails validation on the host
    ok_ws = binding.forward_workspace_bytes(_p())

    def fwd(p, q=fake, gate=fake, ws=0x100000, ws_bytes=ok_ws, H_init=None, U_init=None):
        return binding.forward_raw(p, q, fake, fake, gate, fake, fake, H_init=H_init, U_init=U_init,
                                   workspace=ws, workspace_bytes=ws_bytes)

    assert fwd(_p(B=0)) == binding.GKA_ERR_SHAPE
    assert fwd(_p(n_iter=-1)) == binding.GKA_ERR_SHAPE
    assert fwd(_p(d=96)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(chunk=32)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(d_v=64)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(io_dtype=binding.GKA_F32)) == binding.GKA_ERR_UNSUPPORTED     # f32 tensors need f32 compute
    assert fwd(_p(io_dtype=7)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(phase=3)) == binding.GKA_ERR_UNSUPPORTED
    # a single phase needs the whole problem in one batch of pairs: this one is far too large for that
    big = _p(B=64, H=32, T=32768, phase=binding.GKA_PHASE_SOLVE)
    assert binding.forward_raw(big, fake, fake, fake, fake, fake, fake, workspace=0x100000,
                               workspace_bytes=binding.forward_workspace_bytes(big)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(strides=(1, -1, 1))) == binding.GKA_ERR_SHAPE
    # bf16 operands: strides in units of 16 bytes, token stride below 2^23 elements
    assert fwd(_p(strides=(64 * 130 * 4, 4 * 130, 132))) == binding.GKA_ERR_SHAPE
    assert fwd(_p(strides=(1 << 40, 1 << 23, 128))) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(), q=None) == binding.GKA_ERR_NULL
    assert fwd(_p(), gate=None) == binding.GKA_ERR_NULL
    # lambda may be NULL only together with the rule lambda_t = lambda_scale ||H_t||_F
    assert binding.forward_raw(_p(), fake, fake, fake, fake, None, fake, workspace=0x100000,
                               workspace_bytes=ok_ws) == binding.GKA_ERR_NULL
    assert fwd(_p(lambda_scale=-1.0)) == binding.GKA_ERR_SHAPE
    assert fwd(_p(state_layout=2)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(state_layout=binding.GKA_STATE_H_LOWER_BLOCKS), ws=None) == binding.GKA_ERR_WORKSPACE   # valid layout
    assert fwd(_p(), H_init=fake) == binding.GKA_ERR_NULL                        # H_init without U_init
    # head dimension 256, and 16 and 32 with float32 operands, run token by token only; that path has no phases and
    # no split operands; the chunk-wise kernels of 16 and 32 have no phases either
    assert fwd(_p(d=16, path=binding.GKA_PATH_TWO_PHASE, io_dtype=binding.GKA_F32,
                  compute=binding.GKA_COMPUTE_F32)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(d=16, path=binding.GKA_PATH_FUSED)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(d=16, compute=binding.GKA_COMPUTE_BF16_SPLIT, path=binding.GKA_PATH_TWO_PHASE)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(d=256, path=binding.GKA_PATH_FUSED)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(d=256, state_layout=binding.GKA_STATE_H_LOWER_BLOCKS)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(d=32, phase=binding.GKA_PHASE_STATES)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(path=binding.GKA_PATH_RECURRENT, phase=binding.GKA_PHASE_SOLVE)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(path=binding.GKA_PATH_RECURRENT, compute=binding.GKA_COMPUTE_BF16_SPLIT)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(path=4)) == binding.GKA_ERR_UNSUPPORTED
    assert fwd(_p(d=16), ws=None) == binding.GKA_ERR_WORKSPACE                   # a valid shape
    assert fwd(_p(), ws=None) == binding.GKA_ERR_WORKSPACE
    assert fwd(_p(), ws_bytes=ok_ws - 1) == binding.GKA_ERR_WORKSPACE
    assert fwd(_p(), ws=0x100010) == binding.GKA_ERR_WORKSPACE                   # misaligned
    assert binding.decode_step_raw(_p(), None, fake, fake, fake, fake, fake, fake, fake) == binding.GKA_ERR_NULL
    assert binding.decode_step_raw(_p(d=48), fake, fake, fake, fake, fake, fake, fake, fake) == binding.GKA_ERR_UNSUPPORTED
    assert binding.decode_step_raw(_p(d=256, state_layout=binding.GKA_STATE_H_LOWER_BLOCKS), fake, fake, fake, fake,
                                   fake, fake, fake, fake) == binding.GKA_ERR_UNSUPPORTED
    assert binding.decode_tokens_raw(_p(), None, fake, fake, fake, fake, fake, fake, fake) == binding.GKA_ERR_NULL
    assert binding.decode_tokens_raw(_p(T=0), fake, fake, fake, fake, fake, fake, fake, fake) == binding.GKA_ERR_SHAPE
    assert binding.decode_tokens_raw(_p(strides=(1 << 20, 2048, 128)), fake, fake, fake, fake, fake, fake, fake,
                                     fake) == binding.GKA_ERR_UNSUPPORTED
    assert binding.decode_tokens_raw(None, fake, fake, fake, fake, fake, fake, fake, fake) == binding.GKA_ERR_NULL
    # backward: workspace query and argument checks
    bws = binding.backward_workspace_bytes(_p())
    assert bws > ok_ws and bws % 256 == 0
    # strided inputs are packed into four more tensors at the head of the workspace
    assert binding.backward_workspace_bytes(_p(strides=(1 << 20, 2048, 128))) == bws + 4 * 2 * 100 * 2 * 128 * 2
    assert binding.backward_workspace_bytes(_p(strides=(1 << 20, 2048, 132))) == 0       # rows not 16-byte aligned
    bw = lambda p, **kw: binding.backward_raw(p, *[kw.get(n, fake) for n in ("q", "k", "v", "gate", "lam", "dy", "dq",
                                                                            "dk", "dv", "dgate")],
                                              workspace=kw.get("ws", 0x100000), workspace_bytes=kw.get("ws_bytes", bws))
    assert bw(_p(), dy=None) == binding.GKA_ERR_NULL
    assert bw(_p(), lam=None) == binding.GKA_ERR_NULL                 # no lambda and no rule (lambda_scale = 0)
    assert bw(_p(strides=(1 << 20, 2048, 132))) == binding.GKA_ERR_SHAPE
    assert bw(_p(strides=(1 << 20, 2048, 128))) == binding.GKA_ERR_WORKSPACE        # valid: needs the larger workspace
    assert bw(_p(), ws_bytes=bws - 1) == binding.GKA_ERR_WORKSPACE
    assert bw(_p(d=96)) == binding.GKA_ERR_UNSUPPORTED
    assert bw(_p(d=16)) == binding.GKA_ERR_UNSUPPORTED                # the backward pass runs on the chunk-wise kernels
    assert bw(_p(path=binding.GKA_PATH_RECURRENT)) == binding.GKA_ERR_UNSUPPORTED
    # latent sketching: workspace query and argument checks
    sws = binding.forward_sketched_workspace_bytes(_p(), 32)
    assert sws > 0 and sws % 256 == 0
    assert binding.forward_sketched_workspace_bytes(_p(), 65) == 0
    assert binding.forward_sketched_workspace_bytes(_p(io_dtype=binding.GKA_F32, compute=binding.GKA_COMPUTE_F32), 32) == 0
    sk = lambda p, d_s=32, **kw: binding.forward_sketched_raw(
        p, *[kw.get(n, fake) for n in ("q", "k", "v", "gate", "lam", "S")], d_s, 0, kw.get("o", fake),
        workspace=kw.get("ws", 0x100000), workspace_bytes=kw.get("ws_bytes", sws))
    assert sk(_p(), S=None) == binding.GKA_ERR_NULL
    assert sk(_p(), lam=None) == binding.GKA_ERR_NULL
    assert sk(_p(), d_s=0) == binding.GKA_ERR_SHAPE
    assert sk(_p(), d_s=65) == binding.GKA_ERR_SHAPE
    assert sk(_p(alpha=fake)) == binding.GKA_ERR_UNSUPPORTED
    assert sk(_p(compute=binding.GKA_COMPUTE_F32)) == binding.GKA_ERR_UNSUPPORTED
    assert sk(_p(strides=(1 << 20, 2048, 128))) == binding.GKA_ERR_UNSUPPORTED
    assert sk(_p(), ws_bytes=sws - 1) == binding.GKA_ERR_WORKSPACE
    assert sk(_p(d=256)) == binding.GKA_ERR_UNSUPPORTED
    assert binding.forward_raw(None, fake, fake, fake, fake, fake, fake) == binding.GKA_ERR_NULL
