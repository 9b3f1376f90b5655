"""Shared helpers of the GPU parity tests: the plumbing (uploads, weight views, tolerance
measure) plus the token selection that needs the oracle's logits."""
from __future__ import annotations

import numpy as np

import moei_inputs as mi
from moei_inputs.plumbing import EPS, dev, pack_bank, pinned, rel_max_err, split_expert  # noqa: F401
from oracle import moei_oracle as O

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
