"""Helpers shared by the GPU parity tests (no arithmetic of the method here)."""
import numpy as np
import torch


def dev():
    return torch.device("cuda:0")


def to_np(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> numpy; bf16 comes back as uint16 bit patterns, int32 masks as uint32."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.int32:
        return t.numpy().view(np.uint32)
    return t.numpy()


def as_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def rel_l2(got: np.ndarray, want: np.ndarray) -> float:
    g, w = as_f64(got), as_f64(want)
    den = np.linalg.norm(w)
    return float(np.linalg.norm(g - w) / den) if den > 0 else float(np.linalg.norm(g))


TOL = {"f32": 1e-6, "bf16": 1e-2}


def pack_mask_np(received: np.ndarray) -> np.ndarray:
    r = np.asarray(received, bool)
    N, L = r.shape
    w = r.reshape(N, L // 32, 32).astype(np.uint64) << np.arange(32, dtype=np.uint64)
    return w.sum(axis=2).astype(np.uint32)


def masks_to_dev(m: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(m.view(np.int32).copy()).to(dev())
