"""Oracle of Algorithm 2's outer-optimization schedule over many inner steps (TEST
INFRASTRUCTURE ONLY).

Written from the listing: after the inner update of step t, every fragment p with
(t - t_p) mod H == 0 (and t > t_p, Section 2.2) forms and compresses each replica's outer
gradient; tau steps later the averaged outer gradient is applied with the outer optimizer to
the previously synchronised parameters and mixed into the replica as it is then
(Section 2.3).  With a delay per worker (Section 3.3.2, slack between workers) the mean and
the outer update happen once, at the smallest delay, and worker m mixes at its own delay.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import (dequant_reduce_nesterov, fragment_outer_step, merge_overlap, quantize_outer_grad)
from .plan import RefPlan


class RefEngine:
    def __init__(self, plan: RefPlan, tau_m: Sequence[int], fmt: int, lr: float, mu: float, alpha: float,
                 g: np.ndarray, mom: np.ndarray, w: List[np.ndarray]):
        assert all(0 <= t < plan.H for t in tau_m)
        self.plan, self.tau, self.fmt, self.lr, self.mu, self.alpha = plan, list(tau_m), fmt, lr, mu, alpha
        self.g, self.mom, self.w = g, mom, w
        self.in_flight = {}          # p -> (send step, [per span (codes, scales)])

    def step(self, t: int):
        plan, M = self.plan, len(self.w)
        sent = received = 0
        for p in plan.sends(t):
            assert p not in self.in_flight
            if max(self.tau) == 0:
                for off, n, _ in plan.spans[p]:
                    sl = slice(off, off + n)
                    ws = [w[sl] for w in self.w]
                    fragment_outer_step(self.g[sl], self.mom[sl], ws, ws, self.fmt, self.lr, self.mu, self.alpha)
                sent += 1
                received += 1
                continue
            msgs = []
            for off, n, _ in plan.spans[p]:
                sl = slice(off, off + n)
                msgs.append(quantize_outer_grad(self.g[sl].copy(), [w[sl].copy() for w in self.w], self.fmt))
            self.in_flight[p] = (t, msgs)
            sent += 1
        for p in sorted(self.in_flight):
            ts, msgs = self.in_flight[p]
            if t == ts + min(self.tau):
                for (off, n, _), (codes, scales) in zip(plan.spans[p], msgs):
                    sl = slice(off, off + n)
                    dequant_reduce_nesterov(self.g[sl], self.mom[sl], codes, scales, self.fmt, self.lr, self.mu, n=n)
                received += 1
            for m in range(M):
                if t == ts + self.tau[m]:
                    for off, n, _ in plan.spans[p]:
                        sl = slice(off, off + n)
                        merge_overlap(self.g[sl], [self.w[m][sl]], self.alpha)
            if t >= ts + max(self.tau):
                del self.in_flight[p]
        return sent, received
