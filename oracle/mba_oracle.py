"""Oracle for the draft-length policy (Algorithm 1, "Marginal-Benefit-Aware Adaptive Speculation",
Section 3.4.2) and the throughput model it minimises (Section 3.4.1).

TEST INFRASTRUCTURE ONLY: plain Python, the steps in the paper's order and notation; nothing in
the product path imports it and it shares no code with the library's implementation.

Readings where the paper is silent:
  * beta[0] = 1 (the algorithm reads beta[gamma_l] with gamma_l = 0; position 0 is the token that is
    already accepted); beta is given for positions 1 .. n, and n >= gamma_max + 1 is required because
    the loop reads beta[gamma + 1] with gamma up to gamma_max - 1 ... gamma_max.
  * alpha = E(beta) is the mean of beta[1 .. gamma_max] (the positions a draft can occupy).
  * T_SD(B, gamma) is evaluated for gamma = 0 .. gamma_max from step_time[gamma] = D(B, gamma) +
    T(B, gamma), the measured time of one draft + verify step with gamma draft tokens at batch size
    B (gamma = 0: a plain decode step); ties in the arg-min go to the smaller gamma.
"""
from __future__ import annotations

from typing import Sequence, Tuple


def t_sd(alpha: float, step_time: float, gamma: int) -> float:
    """Expected time per generated token: (1 - alpha) (D + T) / (1 - alpha^(gamma + 1))."""
    if alpha >= 1.0:
        return step_time / (gamma + 1)          # limit alpha -> 1: every draft token is accepted
    return (1.0 - alpha) * step_time / (1.0 - alpha ** (gamma + 1))


def optimal_gamma(beta: Sequence[float], step_time: Sequence[float], gamma_max: int) -> int:
    alpha = sum(beta[:gamma_max]) / gamma_max if gamma_max > 0 else 0.0     # beta[i] is position i + 1
    best, best_t = 0, None
    for gamma in range(gamma_max + 1):
        t = t_sd(alpha, step_time[gamma], gamma)
        if best_t is None or t < best_t:
            best, best_t = gamma, t
    return best


def mba(B_h: int, B_l: int, beta: Sequence[float], gamma_max: int, lam: float,
        step_time: Sequence[float]) -> Tuple[int, int, int]:
    """(gamma_h, gamma_l, gamma_star).  beta[i] is the acceptance probability of draft position i + 1."""
    def b(k: int) -> float:                     # beta[k] in the paper's indexing, beta[0] = 1
        return 1.0 if k == 0 else beta[k - 1]

    B = B_h + B_l
    gamma_star = optimal_gamma(beta, step_time, gamma_max)
    budget = gamma_star * B
    if budget < B_h:
        return 0, 0, gamma_star
    gamma_h, gamma_l, remaining = 1, 0, budget - B_h
    while remaining > 0:
        benefit_h = B_h * (b(gamma_h) - b(gamma_h + 1))
        benefit_l = B_l * (b(gamma_l) - b(gamma_l + 1))
        if benefit_h > lam * benefit_l and gamma_h < gamma_max and remaining >= B_h:
            gamma_h += 1
            remaining -= B_h
        elif B_l > 0 and gamma_l < gamma_max and remaining >= B_l:
            gamma_l += 1
            remaining -= B_l
        else:
            break
    return gamma_h, gamma_l, gamma_star
