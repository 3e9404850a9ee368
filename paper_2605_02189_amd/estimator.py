"""Offline profiling step of the decode execution-time estimator (host code, no GPU).

The paper models the time of one decode iteration of a batch as  alpha * b + beta * L + delta  with
b = batch size and L = total prefix length of the batch, the three parameters coming from offline
profiling (Sec. 3.3.1, Eq. 2), and sizes the prefetch that can hide behind it as  B * T_hat  with B
the effective host-to-device bandwidth (Sec. 3.3.2, Eq. 6).  This module holds the fit only (least
squares on step times measured on the stage, see fit_estimator.py); evaluating the model and the
budget is the scheduler's job (pipemax_sched_predict, pipemax_sched_budget), and the accuracy check
below goes through it, so there is one implementation of Eq. 2 and Eq. 6 in the product.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class DecodeTimeModel:
    alpha: float      # seconds per request
    beta: float       # seconds per cached token
    delta: float      # seconds per step

    def scheduler(self, link_tokens_per_s: float = 1.0, n_batches: int = 1):
        """A scheduler object carrying these parameters (its predict / budget calls are Eq. 2 / Eq. 6)."""
        from . import binding as pm
        return pm.Scheduler(alpha_s=self.alpha, beta_s=self.beta, delta_s=self.delta,
                            link_tokens_per_s=link_tokens_per_s, n_batches=n_batches)


def fit(b, L, t) -> DecodeTimeModel:
    """Least-squares fit of t ~ alpha*b + beta*L + delta with alpha, beta, delta >= 0: each term of the model is a
    cost (per request, per cached token, per step), and on a profiling grid where the total length grows with the
    batch size an unconstrained fit can trade a slightly negative alpha against beta."""
    from scipy.optimize import nnls
    b, L, t = (np.asarray(a, dtype=np.float64) for a in (b, L, t))
    A = np.stack([b, L, np.ones_like(b)], axis=1)
    scale = np.maximum(np.abs(A).max(axis=0), 1e-300)        # columns of comparable size for the solver
    x, _ = nnls(A / scale, t)
    alpha, beta, delta = x / scale
    return DecodeTimeModel(float(alpha), float(beta), float(delta))


def accuracy(model: DecodeTimeModel, b, L, t) -> dict:
    """actual / predicted statistics in the form the paper reports them (Sec. 4.3); the prediction is the
    scheduler's (pipemax_sched_predict)."""
    sched = model.scheduler()
    pred = np.array([sched.predict(int(bi), int(Li)) for bi, Li in zip(np.atleast_1d(b), np.atleast_1d(L))])
    sched.destroy()
    r = np.asarray(t, dtype=np.float64) / pred
    dev = np.abs(r - 1.0)
    return {"n": int(r.size), "within_5pct": float(np.mean(dev <= 0.05)), "worst_dev": float(dev.max()),
            "mean_ratio": float(r.mean())}
