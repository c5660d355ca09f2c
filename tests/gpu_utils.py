"""Helpers for the GPU parity tests: numpy workloads -> device tensors and back."""
import numpy as np
import torch

import paper_2502_01681_amd as dg4

TOL = {"f32": 1e-5, "bf16": 2e-2}       # max over nodes of ||gpu - ref||_2 / ||ref||_2


def tdtype(name):
    return torch.float32 if name == "f32" else torch.bfloat16


def to_dev(a: np.ndarray, dtype: str):
    """float32 numpy (values already representable in `dtype`) -> device tensor, exactly."""
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(tdtype(dtype)).contiguous()


def to_np(t) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> np.ndarray:
    num = np.linalg.norm(got.astype(np.float64) - ref, axis=1)
    den = np.linalg.norm(ref, axis=1)
    return num / np.maximum(den, 1e-30)


def elem_err(got: np.ndarray, ref: np.ndarray) -> np.ndarray:
    """Element-wise error |got - ref| / max(|ref|, RMS of the reference row): one badly wrong element of a
    row shows here even when the row's norm hides it."""
    rms = np.sqrt((ref * ref).mean(axis=1, keepdims=True))
    return np.abs(got.astype(np.float64) - ref) / np.maximum(np.maximum(np.abs(ref), rms), 1e-30)


def device_weights(w, dtype):
    return [(to_dev(w.wqkv[l], dtype), to_dev(w.wo[l], dtype), to_dev(w.rel_bias[l], "f32"))
            for l in range(len(w.wqkv))]


def cfg_of(c, **kw):
    base = dict(hidden=c.hidden, heads=c.heads, hops=c.hops, n_layers=c.n_layers, dtype=c.dtype)
    base.update(kw)
    return dg4.LayerConfig(**base)
