"""Shared helpers of the GPU parity tests: upload/download and the error metric."""
import numpy as np

from paper_2511_21016_amd import synth


def to_device(x, dtype):
    """float32 numpy array (bf16-representable when dtype == 'bf16') -> torch CUDA tensor."""
    import torch
    if dtype == "bf16":
        bits = synth.bf16_bits(x)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def to_host(t):
    """torch tensor (float32 or bfloat16) -> float64 numpy array of the exact stored values."""
    import torch
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return synth.bf16_from_bits(bits).astype(np.float64)
    return t.detach().cpu().numpy().astype(np.float64)


def pair_rel_err(y, ref):
    """Gate metric: per (batch, head) pair, max |y - ref| over (t, i) divided by max |ref| over (t, i);
    returns the worst pair. y, ref: [B,T,H,d]."""
    num = np.abs(y - ref).max(axis=(1, 3))
    den = np.abs(ref).max(axis=(1, 3))
    return float((num / den).max())


def upload_inputs(x, dtype):
    return {
        "q": to_device(x["q"], dtype), "k": to_device(x["k"], dtype), "v": to_device(x["v"], dtype),
        "gate": to_device(x["gate"], "f32"), "lam": to_device(x["lam"], "f32"),
    }
