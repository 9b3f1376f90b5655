"""Shared plumbing of the GPU parity tests: uploads, weight views, tolerance checks."""
from __future__ import annotations

import numpy as np
import torch

import moei_inputs as mi
from oracle import moei_oracle as O

EPS = 2.0 ** -20


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


def logit_gaps(cfg, req, tokens: int) -> np.ndarray:
    """Smallest gap between the k-th and (k+1)-th oracle logit per token (over its layers)."""
    gaps = np.full(tokens, np.inf)
    for l in range(cfg.L):
        W = mi.router_weights(cfg, l)
        for t in range(tokens):
            z = np.sort(O.router_logits(W, req.x[t, l], req.bias[l]))[::-1]
            if cfg.k < cfg.E:
                gaps[t] = min(gaps[t], z[cfg.k - 1] - z[cfg.k])
            gaps[t] = min(gaps[t], np.min(-np.diff(z[:cfg.k])) if cfg.k > 1 else np.inf)
    return gaps


def pick_clear_tokens(cfg, req, want: int, min_gap: float = 1e-3) -> list:
    """Decode tokens whose routing cannot flip under fp32 summation-order noise: every
    logit gap that decides the pick set or its order is at least ``min_gap``."""
    gaps = logit_gaps(cfg, req, req.x.shape[0])
    keep = [t for t in range(req.x.shape[0]) if gaps[t] >= min_gap]
    assert len(keep) >= want, f"only {len(keep)} of {req.x.shape[0]} tokens have clear routing"
    return keep[:want]
