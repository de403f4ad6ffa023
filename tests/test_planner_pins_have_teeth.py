"""Mutation check of the planner-model oracle's pins, on the CPU: one plausible misreading of the prefetch
rules (Section 3.3.1) at a time is planted in a COPY of oracle/latency_model.py, and the pin tests of
tests/test_planner.py (the paper's example totals, the hand-worked recurrences and closed forms - not the
comparisons with the library) are run against the copy.  Every mutant must be rejected by at least one pin;
the unmodified copy must pass them all."""
import os
import types

import pytest

import test_planner as tp

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "latency_model.py")

PINS = [tp.test_simulation_reproduces_the_stall_totals_of_the_papers_example,
        tp.test_single_request_matches_the_recurrence_worked_by_hand,
        tp.test_uniform_placement_equals_one_request_of_the_summed_size,
        tp.test_two_streams_share_the_link_and_the_share_is_redistributed,
        tp.test_a_busy_buffer_delays_the_next_fetch,
        tp.test_simulation_closed_forms]

SHARE = "(mark - served) * len(in_flight) / link"
MUTANTS = [
    ("control", None, None),
    ("every stream gets the whole link", SHARE, "(mark - served) * 1 / link"),
    ("the link is split by the number of requests, finished or not", SHARE, "(mark - served) * n_req / link"),
    ("a finished stream's share is not handed on during compute", "served += left * link / len(in_flight)",
     "served += left * link / n_req"),
    ("the buffer is free again as soon as its layer has landed",
     "            if holds[r] == 0:\n                holds[r] = next_offloaded(r, layer)",
     "            if holds[r] == 0 or (holds[r] <= layer and all(q != r for _, q in in_flight)):\n"
     "                holds[r] = next_offloaded(r, layer + 1 if holds[r] == layer else layer)"),
    ("the layer being entered is never fetched", "holds[r] = next_offloaded(r, layer)", "holds[r] = next_offloaded(r, layer + 1)"),
    ("transfers do not progress while a layer executes", "left = work[layer - 1]", "left = Fraction(0)"),
    ("the wait covers every transfer in flight, not only this layer's", "while any(holds[r] == layer for _, r in in_flight):",
     "while in_flight:"),
    ("stalls are not added to the batch latency", "total = sum(work, Fraction(0)) + sum(stalls, Fraction(0))",
     "total = sum(work, Fraction(0))"),
]


def _load(src):
    mod = types.ModuleType("latency_model_under_test")
    mod.__package__ = "oracle"
    exec(compile(src, SRC, "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planner_pins_reject_a_planted_misreading(monkeypatch, name, old, new):
    with open(SRC) as f:
        src = f.read()
    if old is not None:
        assert src.count(old) >= 1, "mutation site not found: " + name
        src = src.replace(old, new)
    monkeypatch.setattr(tp, "lm", _load(src))
    failed = []
    for pin in PINS:
        try:
            pin()
        except AssertionError:
            failed.append(pin.__name__)
    if old is None:
        assert not failed, failed
    else:
        assert failed, f"the pins accepted the mutant '{name}'"
