"""Context-aware latency model of the attention / KV path and can_schedule on top of it.

The paper models an iteration as (Sec. 4.2)

    Latency(P, C) = k1*P + k2*P*(P + C) + k3*P + k4*(P + C) + k5

with P the compute tokens and C the context tokens already in the KV cache.  This path
contributes the attention term k2, the memory-access term k4, a per-token term (the KV
append; k1 and k3 both multiply P and cannot be told apart from timings, so they are fitted
as one coefficient k_p) and the constant k5.  For a batch of several requests the features
are summed over the requests r (each request attends only its own context):

    f_P = sum_r P_r,   f_att = sum_r P_r*(P_r + C_r),   f_mem = sum_r (P_r + C_r).

`fit` is least squares on measured (batch, seconds) samples under the constraint that no
coefficient is negative (every term is a time: a negative one would make the predicted latency
fall as tokens are added, and `can_schedule`'s bisection relies on it rising); `can_schedule`
answers the scheduler's question: how many compute tokens of a request fit into the batch
without the predicted latency exceeding the time-between-tokens budget (0 = none).
"""
from dataclasses import dataclass
from typing import Iterable, List, Sequence, Tuple

import numpy as np

Request = Tuple[int, int]          # (P_r compute tokens, C_r context tokens)


def features(batch: Iterable[Request]) -> np.ndarray:
    f_p = f_att = f_mem = 0.0
    for p, c in batch:
        f_p += p
        f_att += p * (p + c)
        f_mem += p + c
    return np.array([f_p, f_att, f_mem, 1.0])


@dataclass
class LatencyModel:
    k_p: float      # seconds per compute token (k1 + k3 of the paper, as far as this path sees them)
    k2: float       # seconds per (query, key) pair
    k4: float       # seconds per cached token read
    k5: float       # seconds per call

    @property
    def coef(self) -> np.ndarray:
        return np.array([self.k_p, self.k2, self.k4, self.k5])

    def predict(self, batch: Iterable[Request]) -> float:
        return float(features(batch) @ self.coef)

    def can_schedule(self, batch: Sequence[Request], req_tokens: int, req_ctx: int, budget_s: float) -> int:
        """Largest n <= req_tokens such that the batch plus n compute tokens of the request
        (which already has req_ctx tokens cached) is predicted to finish within budget_s;
        0 if not even one token fits.  With non-negative coefficients the latency does not fall
        as n grows, so bisection is exact; a model with a negative coefficient is refused."""
        if min(self.k_p, self.k2, self.k4, self.k5) < 0:
            raise ValueError("latency model with a negative coefficient: the prediction is not monotone")
        base = list(batch)
        if req_tokens <= 0 or self.predict(base + [(1, req_ctx)]) > budget_s:
            return 0
        lo, hi = 1, req_tokens                      # invariant: lo fits
        while lo < hi:
            mid = (lo + hi + 1) // 2
            if self.predict(base + [(mid, req_ctx)]) <= budget_s:
                lo = mid
            else:
                hi = mid - 1
        return lo


def nonnegative_least_squares(A: np.ndarray, y: np.ndarray) -> np.ndarray:
    """argmin |A x - y| subject to x >= 0, for a handful of columns: the unconstrained solution on
    the best subset of columns whose solution is positive (all 2^n subsets are tried; n = 4 here,
    and the optimum of the constrained problem is always such a subset solution)."""
    n = A.shape[1]
    best, best_res = np.zeros(n), float(np.linalg.norm(y))
    for mask in range(1, 1 << n):
        cols = [j for j in range(n) if mask >> j & 1]
        x, *_ = np.linalg.lstsq(A[:, cols], y, rcond=None)
        if (x < 0).any():
            continue
        res = float(np.linalg.norm(A[:, cols] @ x - y))
        if res < best_res:
            best_res = res
            best = np.zeros(n)
            best[cols] = x
    return best


def fit(samples: Sequence[Tuple[Sequence[Request], float]]) -> Tuple[LatencyModel, np.ndarray]:
    """Least-squares fit with non-negative coefficients; returns the model and the relative error
    of every sample.  Rows are weighted by 1/y, so the fit minimises RELATIVE error (what the
    paper reports)."""
    A = np.stack([features(b) for b, _ in samples])
    y = np.array([t for _, t in samples], dtype=np.float64)
    w = 1.0 / y
    scale = np.abs(A * w[:, None]).max(axis=0)                  # columns span 12 orders of magnitude
    scale[scale == 0] = 1.0
    coef = nonnegative_least_squares(A * w[:, None] / scale, y * w) / scale
    m = LatencyModel(*[float(c) for c in coef])
    rel = np.abs(A @ coef - y) / y
    return m, rel
