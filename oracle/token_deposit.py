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


def replay(step_latency: Sequence[float], slo: float, finish_at_end: bool = False) -> dict:
    """SLO accounting of one request over a run of decode steps (Sections 2.1 and 3.2).

    Step k takes ``step_latency[k]`` and ends with one new token, so token k is generated at
    ``sum(step_latency[:k+1])``.  The clock starts at 0, the instant the request's previous token
    (the last one before the run) was delivered, with an empty deposit.  Written out from the
    metric definitions:

    * TBT of a token = time since the previous token; it is violated when it exceeds ``slo``.
      ``backend_violations`` counts this on generation times (what the engine does),
      ``visible_violations`` on delivery times (what the user sees behind the Token-Deposit).
    * TPOT = run time / tokens; ``tpot_violated`` compares it with the same target.
    * ``max_deposit`` = most tokens waiting at any generation instant, after delivering what is due then.
    """
    gen, t = [], 0.0
    for s in step_latency:
        t += float(s)
        gen.append(t)
    n = len(gen)
    if n == 0:
        return dict(tokens=0, backend_violations=0, visible_violations=0, tpot=0.0, tpot_violated=False,
                    max_deposit=0, max_visible_gap=0.0, delivery=[])
    deliv = []
    for i, g in enumerate(gen):                       # the previous delivery of token 0 is the clock's origin
        deliv.append(max(g, (deliv[-1] if i else 0.0) + slo))
    if finish_at_end:
        deliv = [min(d, max(gen[-1], g)) for d, g in zip(deliv, gen)]
    tol = slo * (1 + 1e-12)
    backend = sum(1 for a, b in zip([0.0] + gen, gen) if b - a > tol)
    gaps = [b - a for a, b in zip([0.0] + deliv, deliv)]
    visible = sum(1 for x in gaps if x > tol)
    waiting = [k + 1 - sum(1 for d in deliv if d <= g) for k, g in enumerate(gen)]
    tpot = gen[-1] / n
    return dict(tokens=n, backend_violations=backend, visible_violations=visible, tpot=tpot,
                tpot_violated=tpot > tol, max_deposit=max(waiting), max_visible_gap=max(gaps), delivery=deliv)
