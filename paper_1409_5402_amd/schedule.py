"""Host-side schedules of the SAME sampler: copies per token m_t and the minibatch weight rho_t.

The paper anneals by changing the number of copies per iteration (Section 3.1, last sentence)
and compares a constant m with three schedules whose average is m (Section 6.1.3); the
minibatch weight follows rho_t = (tau0 + t)^(-gamma) (Section 5.2).  The multinomial form of
the draw needs an integer number of copies, so schedule values are rounded half-to-even and
kept >= 1.
"""
from __future__ import annotations

import math


def _to_int(x: float) -> int:
    return max(1, int(round(x)))      # Python rounds half to even


def constant(m: float, t_max: int) -> list[int]:
    return [_to_int(m)] * t_max


def linear(m: float, t_max: int) -> list[int]:
    """m_t = 2 m t / (t_max + 1), t = 1..t_max (average m)."""
    return [_to_int(2.0 * m * t / (t_max + 1)) for t in range(1, t_max + 1)]


def logarithmic(m: float, t_max: int) -> list[int]:
    """m_t = m t_max log t / sum_s log s, t = 1..t_max."""
    z = sum(math.log(s) for s in range(1, t_max + 1))
    if z == 0.0:
        return constant(m, t_max)
    return [_to_int(m * t_max * math.log(t) / z) for t in range(1, t_max + 1)]


def invlinear(m: float, t_max: int) -> list[int]:
    """m_t = 2 m (t_max + 1 - t) / (t_max + 1), t = 1..t_max."""
    return [_to_int(2.0 * m * (t_max + 1 - t) / (t_max + 1)) for t in range(1, t_max + 1)]


def geometric(m_first: float, m_last: float, steps: int) -> list[int]:
    """m_first -> m_last in equal ratios over `steps` values (used for one streamed pass)."""
    if steps == 1:
        return [_to_int(m_last)]
    ratio = (m_last / m_first) ** (1.0 / (steps - 1))
    return [_to_int(m_first * ratio ** t) for t in range(steps)]


def rho(t: int, tau0: float = 1.0, gamma: float = 0.5) -> float:
    """Minibatch blending weight rho_t = (tau0 + t)^(-gamma), clipped to (0, 1]."""
    return min(1.0, (tau0 + t) ** (-gamma))
