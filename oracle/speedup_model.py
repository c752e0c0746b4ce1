"""Closed-form speedup formulas of the paper and a tick-count model.  TEST INFRASTRUCTURE.

Eq. (3): speculative-decoding gain  rho = T_T(1) / (gamma T_D(1) + T_T(gamma)) * (E(gamma) + 1)
Eq. (4): expected accepted length   E(gamma) = sum_{h<gamma} h a^h (1-a) + gamma a^gamma
                                             = a (1 - a^gamma) / (1 - a)
Eq. (5): early-exit SD gain         rho = (1 - a^(gamma+1)) N / ((1 - a)(gamma E + N))
Eq. (6): overall acceptance         a_all(gamma) = E(gamma) / gamma
Eq. (7): pipeline gain              rho* = N / (a E + (1 - a) ceil(N/E) E)
Eq. (8): lambda = rho* / rho

Reading: Eq. (7)'s intermediate line mixes the draft and target times; the
final form is the one used (it reproduces the worked 1.31x of Sec. 5.3).  The
sentence after Eq. (8) giving lambda = gamma + N/E at a = 1 does not follow
from Eq. (8) (its limit is (gamma + N/E) / (gamma + 1)); lambda is computed
from Eq. (8) only.
"""
from __future__ import annotations

import math
from typing import Sequence


def expected_accept_len_sum(a: float, gamma: int) -> float:
    """Eq. (4), first line: the finite sum."""
    return sum(h * a ** h * (1 - a) for h in range(gamma)) + gamma * a ** gamma


def expected_accept_len(a: float, gamma: int) -> float:
    """Eq. (4), closed form (a < 1); at a = 1 every draft is accepted."""
    return float(gamma) if a == 1.0 else a * (1 - a ** gamma) / (1 - a)


def sd_gain(t_target_1: float, t_draft_1: float, t_target_gamma: float, a: float, gamma: int) -> float:
    """Eq. (3)."""
    return t_target_1 / (gamma * t_draft_1 + t_target_gamma) * (expected_accept_len(a, gamma) + 1)


def eesd_gain(a: float, gamma: int, E: int, N: int) -> float:
    """Eq. (5); the a -> 1 limit is (gamma + 1) N / (gamma E + N)."""
    if a == 1.0:
        return (gamma + 1) * N / (gamma * E + N)
    return (1 - a ** (gamma + 1)) * N / ((1 - a) * (gamma * E + N))


def overall_acceptance(a: float, gamma: int) -> float:
    """Eq. (6)."""
    return expected_accept_len(a, gamma) / gamma


def ppsd_gain(a: float, E: int, N: int) -> float:
    """Eq. (7), final form."""
    return N / (a * E + (1 - a) * math.ceil(N / E) * E)


def ppsd_over_eesd(a: float, gamma: int, E: int, N: int) -> float:
    """Eq. (8)."""
    return ppsd_gain(a, E, N) / eesd_gain(a, gamma, E, N)


def pipeline_ticks(accepts: Sequence[bool], E: int, N: int) -> int:
    """Stage-ticks to emit one token per entry of `accepts` on ceil(N/E) stages.

    An accepted draft costs one tick (the pipeline stays full); a rejected one
    costs a full pass of ceil(N/E) ticks (the pipeline drains and refills).
    Autoregressive decoding costs N/E ticks per token, so the simulated gain is
    len(accepts) * (N / E) / ticks, whose expectation is Eq. (7).
    """
    S = math.ceil(N / E)
    return sum(1 if ok else S for ok in accepts)
