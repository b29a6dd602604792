"""Thin ctypes binding of libgka (include/gka.h). Argument marshalling only: every step of the path
runs in the library's HIP kernels. PyTorch is used for device memory and streams, nothing else.

The library must have been built (python -m paper_2511_21016_amd.build, or __graft_entry__.build());
loading fails loudly otherwise. There is no CPU fallback.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# GKA_LIBRARY: another build of the same library (the CPU tests use it to load the copy whose host code was compiled
# with sanitizers).
LIB_PATH = os.environ.get("GKA_LIBRARY") or os.path.join(_HERE, "libgka.so")

(GKA_OK, GKA_ERR_NULL, GKA_ERR_SHAPE, GKA_ERR_UNSUPPORTED, GKA_ERR_WORKSPACE, GKA_ERR_LAUNCH,
 GKA_ERR_STATIC_SCRATCH) = range(7)
GKA_STATIC_SCRATCH_BYTES = 64 << 20
GKA_F32, GKA_BF16 = 0, 1
GKA_COMPUTE_F32, GKA_COMPUTE_BF16, GKA_COMPUTE_BF16_SPLIT = 0, 1, 2
GKA_PHASE_ALL, GKA_PHASE_STATES, GKA_PHASE_SOLVE = 0, 1, 2
GKA_STATE_FULL, GKA_STATE_H_LOWER_BLOCKS = 0, 1
GKA_PATH_AUTO, GKA_PATH_TWO_PHASE, GKA_PATH_FUSED, GKA_PATH_RECURRENT = 0, 1, 2, 3

EXPORTED_SYMBOLS = (
    "gka_forward_workspace_bytes",
    "gka_forward",
    "gka_forward_static",
    "gka_forward_profile",
    "gka_decode_step",
    "gka_decode_tokens",
    "gka_backward_workspace_bytes",
    "gka_backward",
    "gka_backward_from_state",
    "gka_forward_sketched_workspace_bytes",
    "gka_forward_sketched",
    "gka_status_string",
    "gka_version",
)


class GkaParams(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("T", ctypes.c_int32),
        ("d_k", ctypes.c_int32), ("d_v", ctypes.c_int32), ("chunk", ctypes.c_int32),
        ("n_iter", ctypes.c_int32), ("io_dtype", ctypes.c_int32), ("compute", ctypes.c_int32),
        ("phase", ctypes.c_int32),
        ("stride_b", ctypes.c_int64), ("stride_t", ctypes.c_int64), ("stride_h", ctypes.c_int64),
        ("lambda_scale", ctypes.c_float), ("state_layout", ctypes.c_int32),
        ("beta", ctypes.c_void_p), ("alpha", ctypes.c_void_p), ("xhat_out", ctypes.c_void_p),
        ("slab_state_bytes", ctypes.c_int64), ("walk_chunks", ctypes.c_int32), ("path", ctypes.c_int32),
    ]


class GkaError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"libgka status {status}: {message}")
        self.status = status


_lib = None


def load_library():
    """Load libgka.so once; raise if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it first (python -m paper_2511_21016_amd.build)")
        # PyTorch ships its own HIP runtime (SONAME libamdhip64.so.7). Importing torch first makes libgka
        # bind to that same copy; loading libgka first would bring a second runtime into the process and
        # kernels launched on torch's streams would fail.
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        vp, fp = ctypes.c_void_p, ctypes.c_void_p
        lib.gka_forward_workspace_bytes.argtypes = [ctypes.POINTER(GkaParams)]
        lib.gka_forward_workspace_bytes.restype = ctypes.c_size_t
        lib.gka_forward.argtypes = [ctypes.POINTER(GkaParams), vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, vp,
                                    ctypes.c_size_t, vp]
        lib.gka_forward.restype = ctypes.c_int
        lib.gka_forward_static.argtypes = [ctypes.POINTER(GkaParams), vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, vp]
        lib.gka_forward_static.restype = ctypes.c_int
        lib.gka_forward_profile.argtypes = lib.gka_forward.argtypes + [ctypes.POINTER(ctypes.c_float),
                                                                       ctypes.POINTER(ctypes.c_float),
                                                                       ctypes.POINTER(ctypes.c_int32)]
        lib.gka_forward_profile.restype = ctypes.c_int
        lib.gka_decode_step.argtypes = [ctypes.POINTER(GkaParams), fp, fp, vp, vp, vp, fp, fp, vp, vp]
        lib.gka_decode_step.restype = ctypes.c_int
        lib.gka_decode_tokens.argtypes = lib.gka_decode_step.argtypes
        lib.gka_decode_tokens.restype = ctypes.c_int
        lib.gka_backward_workspace_bytes.argtypes = [ctypes.POINTER(GkaParams)]
        lib.gka_backward_workspace_bytes.restype = ctypes.c_size_t
        lib.gka_backward.argtypes = [ctypes.POINTER(GkaParams), vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp, fp, fp, vp,
                                     ctypes.c_size_t, vp]
        lib.gka_backward.restype = ctypes.c_int
        lib.gka_backward_from_state.argtypes = [ctypes.POINTER(GkaParams), vp, vp, vp, fp, fp, vp, fp, fp, fp, fp, fp,
                                                fp, fp, fp, fp, fp, fp, vp, ctypes.c_size_t, vp]
        lib.gka_backward_from_state.restype = ctypes.c_int
        lib.gka_forward_sketched_workspace_bytes.argtypes = [ctypes.POINTER(GkaParams), ctypes.c_int]
        lib.gka_forward_sketched_workspace_bytes.restype = ctypes.c_size_t
        lib.gka_forward_sketched.argtypes = [ctypes.POINTER(GkaParams), vp, vp, vp, fp, fp, fp, ctypes.c_int,
                                             ctypes.c_int, vp, vp, ctypes.c_size_t, vp]
        lib.gka_forward_sketched.restype = ctypes.c_int
        lib.gka_status_string.argtypes = [ctypes.c_int]
        lib.gka_status_string.restype = ctypes.c_char_p
        lib.gka_version.argtypes = []
        lib.gka_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status):
    return load_library().gka_status_string(int(status)).decode()


def version():
    return int(load_library().gka_version())


def make_params(B, H, T, d, n_iter, io_dtype, compute, chunk=64, d_v=None, strides=(0, 0, 0), phase=0,
                lambda_scale=0.0, beta=None, alpha=None, state_layout=0, xhat_out=None, slab_state_bytes=0,
                walk_chunks=0, path=0):
    """beta, alpha, xhat_out: device addresses (ints) of the optional per-token gates / solve output, or None."""
    return GkaParams(B=B, H=H, T=T, d_k=d, d_v=d if d_v is None else d_v, chunk=chunk, n_iter=n_iter,
                     io_dtype=io_dtype, compute=compute, phase=phase,
                     stride_b=strides[0], stride_t=strides[1], stride_h=strides[2],
                     lambda_scale=lambda_scale, state_layout=state_layout, beta=beta, alpha=alpha, xhat_out=xhat_out,
                     slab_state_bytes=slab_state_bytes, walk_chunks=walk_chunks, path=path)


def forward_workspace_bytes(params):
    return int(load_library().gka_forward_workspace_bytes(ctypes.byref(params)))


def forward_raw(params, q, k, v, gate, lam, o, H_init=None, U_init=None, H_final=None, U_final=None,
                fro_out=None, workspace=None, workspace_bytes=0, stream=None):
    """gka_forward on raw device addresses (ints or None). Returns the gka_status."""
    pp = None if params is None else ctypes.byref(params)
    return int(load_library().gka_forward(pp, q, k, v, gate, lam, o, H_init, U_init, H_final,
                                          U_final, fro_out, workspace, workspace_bytes, stream))


def forward_static_raw(params, q, k, v, gate, lam, o, H_init=None, U_init=None, H_final=None, U_final=None,
                       fro_out=None, stream=None):
    """gka_forward_static on raw device addresses (ints or None). Returns the gka_status."""
    pp = None if params is None else ctypes.byref(params)
    return int(load_library().gka_forward_static(pp, q, k, v, gate, lam, o, H_init, U_init, H_final, U_final,
                                                 fro_out, stream))


def forward_profile_raw(params, q, k, v, gate, lam, o, workspace, workspace_bytes, stream=None):
    """gka_forward_profile on raw device addresses. Returns (status, ms_states, ms_solve, n_solve_launches)."""
    a, b, n = ctypes.c_float(0), ctypes.c_float(0), ctypes.c_int32(0)
    st = int(load_library().gka_forward_profile(ctypes.byref(params), q, k, v, gate, lam, o, None, None, None, None,
                                                None, workspace, workspace_bytes, stream, ctypes.byref(a),
                                                ctypes.byref(b), ctypes.byref(n)))
    return st, a.value, b.value, n.value


def decode_step_raw(params, H_state, U_state, q, k, v, gate, lam, o, stream=None):
    pp = None if params is None else ctypes.byref(params)
    return int(load_library().gka_decode_step(pp, H_state, U_state, q, k, v, gate, lam, o, stream))


def decode_tokens_raw(params, H_state, U_state, q, k, v, gate, lam, o, stream=None):
    pp = None if params is None else ctypes.byref(params)
    return int(load_library().gka_decode_tokens(pp, H_state, U_state, q, k, v, gate, lam, o, stream))


def _check(status):
    if status != GKA_OK:
        raise GkaError(status, status_string(status))


def _io_dtype(t):
    import torch
    if t.dtype == torch.float32:
        return GKA_F32
    if t.dtype == torch.bfloat16:
        return GKA_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def _ptr(t):
    return None if t is None else t.data_ptr()


def gka_forward(q, k, v, gate, lam, n_iter, *, compute=None, chunk=64, H_init=None, U_init=None,
                return_state=False, return_fro=False, workspace=None, out=None, phase=GKA_PHASE_ALL,
                beta=None, alpha=None, lambda_scale=0.0, state_layout=GKA_STATE_FULL, return_xhat=False,
                slab_state_bytes=0, walk_chunks=0, path=GKA_PATH_AUTO):
    """gka_forward on torch CUDA tensors: q, k, v [B,T,H,d] (float32 or bfloat16, contiguous),
    gate, lam [B,T,H] float32 (lam None: lambda_t = lambda_scale * ||H_t||_F); beta, alpha: optional [B,T,H]
    float32 write gate and alpha-connection; return_xhat: also the solve's result [B,T,H,d] float32. Enqueues on torch's current stream and returns o (and a dict of
    the requested extras). Nothing here computes: it allocates outputs and passes pointers."""
    import torch
    if not (q.is_cuda and q.is_contiguous() and k.is_contiguous() and v.is_contiguous()):
        raise ValueError("q, k, v must be contiguous CUDA tensors")
    B, T, H, d = q.shape
    io = _io_dtype(q)
    if compute is None:
        compute = GKA_COMPUTE_BF16 if io == GKA_BF16 else GKA_COMPUTE_F32
    xhat = torch.empty((B, T, H, d), dtype=torch.float32, device=q.device) if return_xhat else None
    params = make_params(B, H, T, d, n_iter, io, compute, chunk=chunk, d_v=v.shape[-1], phase=phase,
                         lambda_scale=lambda_scale, beta=_ptr(beta), alpha=_ptr(alpha), state_layout=state_layout,
                         xhat_out=_ptr(xhat), slab_state_bytes=slab_state_bytes, walk_chunks=walk_chunks, path=path)
    nbytes = forward_workspace_bytes(params)
    if nbytes == 0:
        # let the library name the error
        _check(forward_raw(params, _ptr(q), _ptr(k), _ptr(v), _ptr(gate), _ptr(lam), _ptr(q)))
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
    o = torch.empty_like(v) if out is None else out
    extras = {}
    Hf = Uf = fro = None
    if return_state:
        Hf = torch.empty((B, H, d, d), dtype=torch.float32, device=q.device)
        Uf = torch.empty((B, H, d, d), dtype=torch.float32, device=q.device)
        extras["H_final"], extras["U_final"] = Hf, Uf
    if return_fro:
        fro = torch.empty((B, T, H), dtype=torch.float32, device=q.device)
        extras["fro"] = fro
    if return_xhat:
        extras["xhat"] = xhat
    stream = torch.cuda.current_stream(q.device).cuda_stream
    _check(forward_raw(params, _ptr(q), _ptr(k), _ptr(v), _ptr(gate), _ptr(lam), _ptr(o), _ptr(H_init),
                       _ptr(U_init), _ptr(Hf), _ptr(Uf), _ptr(fro), _ptr(workspace), workspace.numel(), stream))
    return (o, extras) if extras else o


def gka_decode_step(H_state, U_state, q, k, v, gate, lam, n_iter, *, out=None, beta=None, alpha=None,
                    lambda_scale=0.0, state_layout=GKA_STATE_FULL):
    """gka_decode_step on torch CUDA tensors: states [B,H,d,d] float32 (updated in place), q, k, v [B,H,d],
    gate, lam [B,H] float32 (lam None: lambda_scale * ||H||_F); beta, alpha: optional [B,H] float32."""
    import torch
    B, H, d = q.shape
    io = _io_dtype(q)
    params = make_params(B, H, 1, d, n_iter, io, GKA_COMPUTE_F32, lambda_scale=lambda_scale, beta=_ptr(beta),
                         alpha=_ptr(alpha), state_layout=state_layout)
    o = torch.empty_like(v) if out is None else out
    stream = torch.cuda.current_stream(q.device).cuda_stream
    _check(decode_step_raw(params, _ptr(H_state), _ptr(U_state), _ptr(q), _ptr(k), _ptr(v), _ptr(gate), _ptr(lam),
                           _ptr(o), stream))
    return o


def gka_decode_tokens(H_state, U_state, q, k, v, gate, lam, n_iter, *, out=None, beta=None, alpha=None,
                      lambda_scale=0.0, state_layout=GKA_STATE_FULL):
    """gka_decode_tokens on torch CUDA tensors: states [B,H,d,d] float32 (updated in place), q, k, v [B,T,H,d]
    contiguous, gate, lam [B,T,H] float32 (lam None: lambda_scale * ||H||_F); beta, alpha: optional [B,T,H]."""
    import torch
    B, T, H, d = q.shape
    for x in (q, k, v):
        if not x.is_contiguous():
            raise ValueError("gka_decode_tokens takes packed [B,T,H,d] tensors")
    io = _io_dtype(q)
    params = make_params(B, H, T, d, n_iter, io, GKA_COMPUTE_F32, lambda_scale=lambda_scale, beta=_ptr(beta),
                         alpha=_ptr(alpha), state_layout=state_layout)
    o = torch.empty_like(v) if out is None else out
    stream = torch.cuda.current_stream(q.device).cuda_stream
    _check(decode_tokens_raw(params, _ptr(H_state), _ptr(U_state), _ptr(q), _ptr(k), _ptr(v), _ptr(gate), _ptr(lam),
                             _ptr(o), stream))
    return o


def backward_workspace_bytes(params):
    return int(load_library().gka_backward_workspace_bytes(ctypes.byref(params)))


def backward_raw(params, q, k, v, gate, lam, dy, dq, dk, dv, dgate, dlam=None, dbeta=None, dalpha=None,
                 workspace=None, workspace_bytes=0, stream=None):
    pp = None if params is None else ctypes.byref(params)
    return int(load_library().gka_backward(pp, q, k, v, gate, lam, dy, dq, dk, dv, dgate, dlam, dbeta, dalpha,
                                           workspace, workspace_bytes, stream))


def backward_from_state_raw(params, q, k, v, gate, lam, dy, H_init, U_init, dq, dk, dv, dgate, dlam=None, dbeta=None,
                            dalpha=None, dH_init=None, dU_init=None, workspace=None, workspace_bytes=0, stream=None):
    pp = None if params is None else ctypes.byref(params)
    return int(load_library().gka_backward_from_state(pp, q, k, v, gate, lam, dy, H_init, U_init, dq, dk, dv, dgate,
                                                      dlam, dbeta, dalpha, dH_init, dU_init, workspace,
                                                      workspace_bytes, stream))


def gka_backward(q, k, v, gate, lam, dy, n_iter, *, compute=None, beta=None, alpha=None, lambda_scale=0.0,
                 workspace=None, H_init=None, U_init=None, return_state_grads=False, shape=None, strides=(0, 0, 0)):
    """gka_backward on torch CUDA tensors (packed [B,T,H,d] / [B,T,H]). lam None: the rule
    lambda_t = lambda_scale ||H_t||_F. Returns a dict of float32 gradients: dq, dk, dv, dgate, dlam (when lam is
    given) and, when given, dbeta, dalpha. H_init, U_init [B,H,d,d] float32: the sequence continues from these states
    (gka_backward_from_state); return_state_grads: also dH_init, dU_init. shape = (B, T, H, d) with strides = element
    strides (batch, token, head): q, k, v, dy are stored in another layout with a contiguous head dimension (the
    gradients come back packed [B,T,H,d])."""
    import torch
    if shape is None:
        B, T, H, d = q.shape
        for x in (q, k, v, dy):
            if not x.is_contiguous():
                raise ValueError("gka_backward takes packed tensors unless shape and strides are given")
    else:
        B, T, H, d = shape
    io = _io_dtype(q)
    if compute is None:
        compute = GKA_COMPUTE_BF16 if io == GKA_BF16 else GKA_COMPUTE_F32
    params = make_params(B, H, T, d, n_iter, io, compute, lambda_scale=lambda_scale, beta=_ptr(beta),
                         alpha=_ptr(alpha), strides=strides)
    nbytes = backward_workspace_bytes(params)
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=q.device)
    f32 = dict(dtype=torch.float32, device=q.device)
    out = {"dq": torch.empty((B, T, H, d), **f32), "dk": torch.empty((B, T, H, d), **f32),
           "dv": torch.empty((B, T, H, d), **f32), "dgate": torch.empty((B, T, H), **f32)}
    if lam is not None:
        out["dlam"] = torch.empty((B, T, H), **f32)
    if beta is not None:
        out["dbeta"] = torch.empty((B, T, H), **f32)
    if alpha is not None:
        out["dalpha"] = torch.empty((B, T, H), **f32)
    stream = torch.cuda.current_stream(q.device).cuda_stream
    if H_init is not None or return_state_grads:
        if return_state_grads:
            out["dH_init"] = torch.empty((B, H, d, d), **f32)
            out["dU_init"] = torch.empty((B, H, d, d), **f32)
        _check(backward_from_state_raw(params, _ptr(q), _ptr(k), _ptr(v), _ptr(gate), _ptr(lam), _ptr(dy),
                                       _ptr(H_init), _ptr(U_init), _ptr(out["dq"]), _ptr(out["dk"]), _ptr(out["dv"]),
                                       _ptr(out["dgate"]), _ptr(out.get("dlam")), _ptr(out.get("dbeta")),
                                       _ptr(out.get("dalpha")), _ptr(out.get("dH_init")), _ptr(out.get("dU_init")),
                                       _ptr(workspace), workspace.numel(), stream))
        return out
    _check(backward_raw(params, _ptr(q), _ptr(k), _ptr(v), _ptr(gate), _ptr(lam), _ptr(dy), _ptr(out["dq"]),
                        _ptr(out["dk"]), _ptr(out["dv"]), _ptr(out["dgate"]), _ptr(out.get("dlam")),
                        _ptr(out.get("dbeta")), _ptr(out.get("dalpha")), _ptr(workspace), workspace.numel(), stream))
    return out


def forward_sketched_workspace_bytes(params, d_s):
    return int(load_library().gka_forward_sketched_workspace_bytes(ctypes.byref(params), d_s))


def forward_sketched_raw(params, q, k, v, gate, lam, S, d_s, per_head, o, workspace=None, workspace_bytes=0,
                         stream=None):
    pp = None if params is None else ctypes.byref(params)
    return int(load_library().gka_forward_sketched(pp, q, k, v, gate, lam, S, d_s, per_head, o, workspace,
                                                   workspace_bytes, stream))


def gka_forward_sketched(q, k, v, gate, lam, S, n_iter, *, beta=None, lambda_scale=0.0, workspace=None, out=None):
    """gka_forward_sketched on torch CUDA tensors: bf16 q, k, v [B,T,H,d] (packed), S float32 [d_s,d] or [H,d_s,d]."""
    import torch
    B, T, H, d = q.shape
    for x in (q, k, v, S):
        if not x.is_contiguous():
            raise ValueError("gka_forward_sketched takes packed tensors")
    per_head = 1 if S.dim() == 3 else 0
    d_s = S.shape[-2]
    params = make_params(B, H, T, d, n_iter, _io_dtype(q), GKA_COMPUTE_BF16, lambda_scale=lambda_scale,
                         beta=_ptr(beta))
    nbytes = forward_sketched_workspace_bytes(params, d_s)
    if workspace is None:
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=q.device)
    o = torch.empty_like(v) if out is None else out
    stream = torch.cuda.current_stream(q.device).cuda_stream
    _check(forward_sketched_raw(params, _ptr(q), _ptr(k), _ptr(v), _ptr(gate), _ptr(lam), _ptr(S), d_s, per_head,
                                _ptr(o), _ptr(workspace), workspace.numel(), stream))
    return o
