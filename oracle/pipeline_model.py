"""Oracle for the chunk-pipeline timing model -- TEST INFRASTRUCTURE (plain Python/numpy, double).

Follows the paper's performance models and layer-0 timeline for ONE micro-batch slice on the
expert-group side:

  * every task time is linear in its workload, t = alpha + beta * x (Sec. 4.1, Eq. gm, Eq. a_r);
    with the token range of T tokens cut into r_2 = r chunks, a chunk carries m = T / r tokens
    (Sec. 4.2, "Determine r_2 and m_e": m_e = k' / r_2), so
        t_in(r)  = alpha_in  + beta_in  * T / r      (A2E stand-in)
        t_e(r)   = alpha_e   + beta_e   * T / r      (expert compute)
        t_out(r) = alpha_out + beta_out * T / r      (E2A stand-in)
  * three resources (inbound link, expert compute, outbound link) each run one task at a time, a
    chunk's compute starts after its inbound transfer, its outbound transfer after its compute
    (Sec. 3.2, Eq. limitation, rules 3-5 and 7-8);
  * the resulting finish time of the last outbound transfer is the layer-0 closed form of Sec. 4.2
    with i = 0:  t_in + t_e + t_out + (r - 1) * Y,  Y = max over the three resources
    (the paper assumes t_a2e = t_e2a, which gives its  2 t_a2e + t_e + (r_2 - 1) max(t_e, t_a2e)).

Extension for resources that are not independent (the paper's four "machines" are separate hardware,
Sec. 3.2; on one GPU a transfer in flight slows the compute beside it and the reverse): every task has a
second linear model, fitted from runs in which the other resources were active.  With one chunk nothing
overlaps, so r = 1 is priced with the first set; with r > 1 every task is priced with the second set
and the same timeline applies (makespan_overlap / simulate_overlap / best_r_overlap).  Equal sets give
the paper's model back.

Only tests, the smoke check and the benchmark's reporting may import this module.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Sequence, Tuple

import numpy as np


@dataclass(frozen=True)
class LinearModel:
    alpha: float
    beta: float

    def __call__(self, x: float) -> float:
        return self.alpha + self.beta * x


def fit_linear(x: Sequence[float], t: Sequence[float]) -> Tuple[float, float, float]:
    """Least-squares alpha, beta of t = alpha + beta x, and the coefficient of determination R^2."""
    x = np.asarray(x, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64)
    A = np.stack([np.ones_like(x), x], axis=1)
    (alpha, beta), *_ = np.linalg.lstsq(A, t, rcond=None)
    ss_res = float(np.sum((t - (alpha + beta * x)) ** 2))
    ss_tot = float(np.sum((t - t.mean()) ** 2))
    r2 = 1.0 if ss_tot == 0.0 else 1.0 - ss_res / ss_tot
    return float(alpha), float(beta), r2


def makespan(r: int, T: float, m_in: LinearModel, m_e: LinearModel, m_out: LinearModel) -> float:
    """Closed form (Sec. 4.2, layer 0, slice 0): finish time of the last outbound transfer."""
    m = T / r
    t_in, t_e, t_out = m_in(m), m_e(m), m_out(m)
    return t_in + t_e + t_out + (r - 1) * max(t_in, t_e, t_out)


def simulate(r: int, T: float, m_in: LinearModel, m_e: LinearModel, m_out: LinearModel) -> float:
    """Event-by-event schedule under Eq. limitation: each resource serial, chunk order kept,
    every task started as early as its rules allow.  Independent of the closed form."""
    m = T / r
    t_in, t_e, t_out = m_in(m), m_e(m), m_out(m)
    free_in = free_e = free_out = 0.0
    end = 0.0
    for _ in range(r):
        s_in = free_in
        free_in = s_in + t_in
        s_e = max(free_e, free_in)
        free_e = s_e + t_e
        s_out = max(free_out, free_e)
        free_out = s_out + t_out
        end = free_out
    return end


def best_r(T: float, m_in: LinearModel, m_e: LinearModel, m_out: LinearModel, r_max: int) -> int:
    """Brute force: the smallest r in 1..r_max with the smallest closed-form makespan."""
    best, best_t = 1, makespan(1, T, m_in, m_e, m_out)
    for r in range(2, r_max + 1):
        t = makespan(r, T, m_in, m_e, m_out)
        if t < best_t:
            best, best_t = r, t
    return best


def makespan_overlap(r: int, T: float, alone, beside) -> float:
    """Closed form with two sets of task models: `alone` = (m_in, m_e, m_out) for r = 1, where no two
    tasks run at once; `beside` = the same three for r > 1, fitted while the other resources ran."""
    return makespan(r, T, *(alone if r == 1 else beside))


def simulate_overlap(r: int, T: float, alone, beside) -> float:
    """The event-by-event schedule with each task's duration taken from the set that applies."""
    return simulate(r, T, *(alone if r == 1 else beside))


def best_r_overlap(T: float, alone, beside, r_max: int) -> int:
    """Brute force over r = 1..r_max; the smallest r with the smallest makespan."""
    best, best_t = 1, makespan_overlap(1, T, alone, beside)
    for r in range(2, r_max + 1):
        t = makespan_overlap(r, T, alone, beside)
        if t < best_t:
            best, best_t = r, t
    return best
