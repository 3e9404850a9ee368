"""Decode execution-time estimator and prefetch budget of the control plane (host code, no GPU).

The paper models the time of one decode iteration of a batch as  alpha * b + beta * L + delta  with
b = batch size and L = total prefix length of the batch, the three parameters coming from offline
profiling (Sec. 3.3.1, Eq. 2), and sizes the prefetch that can hide behind it as  B * T_hat  with B
the effective host-to-device bandwidth (Sec. 3.3.2, Eq. 6).  Here the parameters are fitted by least
squares to step times measured on the stage (bench.py --estimator).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class DecodeTimeModel:
    alpha: float      # seconds per request
    beta: float       # seconds per cached token
    delta: float      # seconds per step

    def predict(self, b, L):
        return self.alpha * np.asarray(b, dtype=np.float64) + self.beta * np.asarray(L, dtype=np.float64) + self.delta


def fit(b, L, t) -> DecodeTimeModel:
    """Least-squares fit of t ~ alpha*b + beta*L + delta."""
    b, L, t = (np.asarray(a, dtype=np.float64) for a in (b, L, t))
    A = np.stack([b, L, np.ones_like(b)], axis=1)
    (alpha, beta, delta), *_ = np.linalg.lstsq(A, t, rcond=None)
    return DecodeTimeModel(float(alpha), float(beta), float(delta))


def accuracy(model: DecodeTimeModel, b, L, t) -> dict:
    """actual / predicted statistics in the form the paper reports them (Sec. 4.3)."""
    r = np.asarray(t, dtype=np.float64) / model.predict(b, L)
    dev = np.abs(r - 1.0)
    return {"n": int(r.size), "within_5pct": float(np.mean(dev <= 0.05)), "worst_dev": float(dev.max()),
            "mean_ratio": float(r.mean())}


def prefetch_budget_bytes(t_hat: float, link_bytes_per_s: float) -> float:
    """Bytes that can be prefetched while a step of predicted duration t_hat runs (Eq. 6)."""
    return link_bytes_per_s * t_hat


def prefetch_budget_tokens(t_hat: float, link_bytes_per_s: float, kv_bytes_per_token: int) -> float:
    """The same budget in cached tokens of this stage (the unit Alg. 1 compares it in)."""
    return prefetch_budget_bytes(t_hat, link_bytes_per_s) / kv_bytes_per_token


def hidden_streamed_fraction(model: DecodeTimeModel, b: int, L: int, link_bytes_per_s: float,
                             kv_bytes_per_token: int) -> float:
    """sigma*: the fraction of a micro-batch's KV that can stream in behind one step of another."""
    t = float(model.predict(b, L))
    return min(1.0, prefetch_budget_tokens(t, link_bytes_per_s, kv_bytes_per_token) / max(L, 1))
