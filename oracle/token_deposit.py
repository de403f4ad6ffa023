"""Oracle for the Token-Deposit release rule (Section 3.2; test infrastructure only).

Rule, restated: generated tokens enter a FIFO; while it is non-empty one token is delivered per
SLO interval; when it is empty the next token is delivered the moment it is generated; when the
request finishes the rest is delivered at once.  The paper prints no numbers for it, so the pins
are hand-worked cases of this rule (tests/test_token_deposit.py).
"""
from typing import List, Optional, Sequence, Tuple


def delivery_times(gen: Sequence[float], slo: float, finish: Optional[float] = None) -> List[float]:
    paced: List[float] = []
    for i, g in enumerate(gen):
        paced.append(g if i == 0 else max(g, paced[-1] + slo))
    if finish is None:
        return paced
    return [min(p, max(finish, g)) for p, g in zip(paced, gen)]


def violations(times: Sequence[float], slo: float) -> int:
    return sum(1 for a, b in zip(times, times[1:]) if b - a > slo * (1 + 1e-12))


def summary(gen: Sequence[float], slo: float, finish: Optional[float] = None) -> Tuple[int, int]:
    """(violations the user sees, violations of the generation itself)."""
    return violations(delivery_times(gen, slo, finish), slo), violations(gen, slo)
