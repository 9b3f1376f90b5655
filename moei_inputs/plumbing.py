"""Host/device plumbing shared by the benchmark, the smoke run and the GPU tests: uploads,
pinned copies, weight views, the output error measure.  No arithmetic of the method and no
reference implementation is imported here."""
from __future__ import annotations

import numpy as np
import torch

EPS = 2.0 ** -20   # epsilon of Alg. 1's priority score in every configuration


def dev(a: np.ndarray) -> torch.Tensor:
    """Host array -> device tensor with the same bits (uint16 bf16 patterns travel as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def split_expert(cfg, w: np.ndarray):
    """Flat expert -> (W_gate [I][H], W_up [I][H], W_down [H][I]) views."""
    H, I = cfg.H, cfg.I
    return w[:I * H].reshape(I, H), w[I * H:2 * I * H].reshape(I, H), w[2 * I * H:].reshape(H, I)


def pack_bank(m, cfg, bank: np.ndarray) -> np.ndarray:
    """Experts drawn as plain matrices -> the library's slot layout (its own packer; data movement)."""
    desc = m.ModelDesc.from_config(cfg)
    out = np.empty_like(bank)
    for u in range(bank.shape[0]):
        m.expert_pack(desc, *split_expert(cfg, bank[u]), out=out[u])
    return out


def pinned(a: np.ndarray) -> torch.Tensor:
    """A pinned host copy (the library reads misses from it asynchronously)."""
    src = torch.from_numpy(np.ascontiguousarray(a).view(np.int16) if a.dtype == np.uint16 else np.ascontiguousarray(a))
    t = torch.empty(src.shape, dtype=src.dtype, pin_memory=True)
    t.copy_(src)
    return t


def rel_max_err(y: np.ndarray, ref: np.ndarray) -> float:
    """max |y - ref| / max |ref|  (the FFN tolerance is stated on this quantity)."""
    den = float(np.abs(ref).max())
    return float(np.abs(y.astype(np.float64) - ref).max()) / (den if den > 0 else 1.0)
