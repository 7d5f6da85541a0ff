"""Plain Python model of the coordinator's ScheduleWork handler of Adaptive Hogbatch
(Algorithm 2 of the paper, coordinator side; Section 6.3).  TEST INFRASTRUCTURE ONLY: like
the rest of this package it is imported by the tests alone and shares no code with the
library.

State, in the paper's notation: for every worker E the number of model updates u^E it has
reported and its current batch size b^E with the thresholds min_b^E <= b^E <= max_b^E; the
scaling factor alpha (default 2); the part of the training data not yet handed out in this
epoch, kept as a contiguous range [cursor, n).

One request (worker E asks for work and reports u^E):
  1. min_u / max_u = smallest / largest update count among all OTHER workers;
     if u^E < min_u the worker lags behind: b^E <- max(b^E / alpha, min_b^E);
     else if u^E > max_u it runs ahead:    b^E <- min(b^E * alpha, max_b^E).
     With no other worker nothing changes.
  2. if b^E <= |remaining|: hand out the next b^E examples, else hand out nothing (the
     worker is done for this epoch).
Readings: b^E / alpha is rounded to the nearest integer (halves away from zero) and never
below 1; batches are taken from the front of the remaining range, in order.
"""
from __future__ import annotations

import math


def _round_half_away(x: float) -> int:
    return int(math.floor(x + 0.5))


class AdaptiveSchedule:
    def __init__(self, n_examples, min_b, max_b, init_b, alpha=2.0):
        assert len(min_b) == len(max_b) == len(init_b) >= 1
        assert alpha > 1.0 and n_examples >= 0
        for lo, hi, b in zip(min_b, max_b, init_b):
            assert 1 <= lo <= b <= hi
        self.n = int(n_examples)
        self.min_b = [int(v) for v in min_b]
        self.max_b = [int(v) for v in max_b]
        self.b = [int(v) for v in init_b]
        self.u = [0.0] * len(self.b)
        self.alpha = float(alpha)
        self.cursor = 0

    def new_epoch(self):
        """The whole training set becomes available again; update counts and batch sizes stay."""
        self.cursor = 0

    def remaining(self):
        return self.n - self.cursor

    def request(self, worker, updates):
        """Returns (begin, count); count == 0 means no batch is sent."""
        self.u[worker] = float(updates)
        others = [self.u[w] for w in range(len(self.u)) if w != worker]
        if others:
            if self.u[worker] < min(others):
                self.b[worker] = max(max(_round_half_away(self.b[worker] / self.alpha), 1), self.min_b[worker])
            elif self.u[worker] > max(others):
                self.b[worker] = min(_round_half_away(self.b[worker] * self.alpha), self.max_b[worker])
        if self.b[worker] <= self.remaining():
            begin = self.cursor
            self.cursor += self.b[worker]
            return begin, self.b[worker]
        return self.cursor, 0
