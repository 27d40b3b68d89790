"""Test-side drivers that chain the oracle's routines into rounds of Alg. 1 (no arithmetic of their own)."""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import numpy as np

import oracle


def uniform_levels(S: int) -> np.ndarray:
    return (np.arange(S, dtype=np.float64) / (S - 1)).astype(np.float32)


class OracleQODA:
    """State of Alg. 1 kept by the checker: X_1, Y_t, the step-size accumulator and the previous messages."""

    def __init__(self, sizes, points, levels, K: int, x1: Sequence[np.ndarray], seed: int, q_hat: Optional[float] = None):
        self.q_hat = q_hat                                                          # None: eq. (general_stepsize); else eq. (Alt)
        self.lam, self.mu, self.gamma = 0.0, 0.0, np.float32(1.0)
        self.sizes = [int(s) for s in sizes]
        self.points = [int(s) for s in points]
        self.levels = [np.asarray(a, dtype=np.float32).copy() for a in levels]     # one table per layer
        self.K = K
        self.seed = seed
        self.x1 = [np.asarray(a, dtype=np.float32).copy() for a in x1]
        self.y = [np.zeros_like(a) for a in self.x1]                                # Y_1 = 0
        self.acc = 0.0                                                              # eta_1 = gamma_1 = 1
        self.eta = np.float32(1.0)
        self.prev: List[Optional[np.ndarray]] = [None] * K                          # Vhat_{k,1/2} = 0
        self.x_half = [a.copy() for a in self.x1]                                   # X_{3/2} = X_1
        self.x_next = [a.copy() for a in self.x1]
        self.round = 0

    def quantize_all(self, grads: Sequence[Sequence[np.ndarray]], round_: int):
        msgs, deltas, sumsqs = [], [], []
        for k in range(self.K):
            m, ss, dl, st = oracle.quantize(self.sizes, self.points, self.levels, grads[k], self.seed, round_, k,
                                            msg_prev=None if self.q_hat is not None else self.prev[k])
            assert st == 0
            msgs.append(m)
            deltas.append(dl)
            sumsqs.append(ss)
        return msgs, deltas, sumsqs

    def step(self, msgs, deltas):
        mean = oracle.dequant_aggregate(self.sizes, self.points, msgs)
        if self.q_hat is not None:
            eta_prev = self.eta
            self.eta, self.gamma = oracle.alt_step_size(self.lam, self.mu, self.q_hat)
            xn, xh, dx2 = oracle.oda_update_alt(self.sizes, mean, self.x1, self.y, eta_prev, self.eta, self.gamma)
            self.x_next, self.x_half = xn, xh
            self.lam, self.mu = oracle.alt_advance(deltas, dx2, self.lam, self.mu)
            self.last_dx2 = dx2
            self.prev = list(msgs)
            return mean
        self.acc, self.eta = oracle.step_size(deltas, self.acc)
        for l in range(len(self.sizes)):
            xn, xh = oracle.oda_update(mean[l], self.x1[l], self.y[l], self.eta, self.eta)
            self.x_next[l], self.x_half[l] = xn, xh
        self.prev = list(msgs)
        return mean

    def round_(self, grads, round_: int):
        msgs, deltas, _ = self.quantize_all(grads, round_)
        mean = self.step(msgs, deltas)
        self.round = round_
        return msgs, deltas, mean


def run_bilinear(K: int, rounds: int, points: int, seed: int, operator: Callable, x0, y0, quantize: bool = True,
                 q_hat: Optional[float] = None):
    """QODA on the two-block game; returns the list of query points X_{t+1/2} (concatenated) and the final state.
    ``quantize=False`` runs eq. (ODA) + eq. (general_stepsize) on the exact vectors in float64 (numpy, from the
    equations) as the unquantized comparison."""
    n = x0.size
    if quantize:
        st = OracleQODA([n, n], [points, points], [uniform_levels(points)] * 2, K, [x0, y0], seed, q_hat=q_hat)
        queries = []
        for t in range(1, rounds + 1):
            xq, yq = st.x_half
            queries.append(np.concatenate([xq, yq]).astype(np.float64))
            grads = [list(operator(xq, yq, k, t)) for k in range(K)]
            st.round_(grads, t)
        return queries, st
    x1 = np.concatenate([x0, y0]).astype(np.float64)
    y = np.zeros_like(x1)
    acc = lam = mu = 0.0
    prev = [np.zeros_like(x1) for _ in range(K)]
    xh = x1.copy()
    xt = x1.copy()
    queries = []
    for t in range(1, rounds + 1):
        queries.append(xh.copy())
        cur = [np.concatenate(operator(xh[:n].astype(np.float32), xh[n:].astype(np.float32), k, t)).astype(np.float64)
               for k in range(K)]
        mean = np.mean(cur, axis=0)
        if q_hat is None:
            acc += sum(float(np.sum((c - p) ** 2)) for c, p in zip(cur, prev)) / K ** 2
            eta = gamma = (1.0 + acc) ** -0.5
        else:                                        # eq. (Alt): sums up to round t-1 set the rates used after round t
            eta = (1.0 + lam + mu) ** -0.5
            gamma = (1.0 + lam) ** (q_hat - 0.5)
        y = y - mean
        xn = x1 + eta * y
        xh = xn - gamma * mean
        lam += sum(float(np.sum(c ** 2)) for c in cur) / K ** 2
        mu += float(np.sum((xt - xn) ** 2))
        xt = xn
        prev = cur
    return queries, None
