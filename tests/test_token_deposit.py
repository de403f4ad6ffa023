"""Token-Deposit: hand-worked cases of the release rule pin the oracle; the library's FIFO is then
compared with it on random traces and polling patterns.  Profile refresh helpers.  CPU only."""
import numpy as np
import pytest

import paper_2601_10729_amd as orbit
from oracle import token_deposit as td


def test_rule_hand_worked_cases():
    # generation faster than the SLO: the deposit fills and delivery is one token per interval
    assert td.delivery_times([0.0, 0.1, 0.2, 0.3], 1.0) == [0.0, 1.0, 2.0, 3.0]
    # generation slower than the SLO: the deposit stays empty, every token goes out on generation
    assert td.delivery_times([0.0, 2.0, 5.0], 1.0) == [0.0, 2.0, 5.0]
    assert td.summary([0.0, 2.0, 5.0], 1.0) == (2, 2)
    # early margin masks a later slow stretch: four quick tokens, then gaps of 2 intervals
    gen = [0.0, 0.1, 0.2, 0.3, 2.3, 4.3, 6.3]
    assert td.delivery_times(gen, 1.0) == [0.0, 1.0, 2.0, 3.0, 4.0, 5.0, 6.3]
    assert td.summary(gen, 1.0) == (1, 3)                # three backend violations, one seen
    # finish: what is still deposited leaves in one burst at the finish time
    assert td.delivery_times([0.0, 0.1, 0.2, 0.3], 1.0, finish=1.5) == [0.0, 1.0, 1.5, 1.5]


def test_replay_hand_worked_cases():
    """Step latencies through the deposit, worked by hand (clock origin = delivery of the previous token)."""
    # steps of 1 against a 2-unit target: generated at 1,2,3,4, paced out at 2,4,6,8; two tokens wait at t = 4
    r = td.replay([1, 1, 1, 1], 2.0)
    assert r["delivery"] == [2.0, 4.0, 6.0, 8.0] and (r["backend_violations"], r["visible_violations"]) == (0, 0)
    assert r["max_deposit"] == 2 and r["tpot"] == 1.0 and not r["tpot_violated"] and r["max_visible_gap"] == 2.0
    # the request finishes with the run: what is still deposited leaves at t = 4
    assert td.replay([1, 1, 1, 1], 2.0, finish_at_end=True)["delivery"] == [2.0, 4.0, 4.0, 4.0]
    # a spike of 5 after three quick steps: generated at 1,2,3,8,9; delivered 2,4,6,8,10 -> the spike is hidden
    r = td.replay([1, 1, 1, 5, 1], 2.0)
    assert r["delivery"] == [2.0, 4.0, 6.0, 8.0, 10.0]
    assert (r["backend_violations"], r["visible_violations"], r["max_deposit"]) == (1, 0, 2)
    # a spike of 6 is one unit too long for the two deposited tokens: delivered 2,4,6,9 -> seen once (gap 3)
    r = td.replay([1, 1, 1, 6], 2.0)
    assert r["delivery"] == [2.0, 4.0, 6.0, 9.0] and (r["backend_violations"], r["visible_violations"]) == (1, 1)
    assert r["max_visible_gap"] == 3.0
    # steps slower than the target: nothing is ever deposited, every violation shows, TPOT fails too
    r = td.replay([3, 3], 2.0)
    assert r["delivery"] == [3.0, 6.0] and (r["backend_violations"], r["visible_violations"]) == (2, 2)
    assert r["max_deposit"] == 0 and r["tpot"] == 3.0 and r["tpot_violated"]
    # TPOT can hold while TBT fails (Section 2.1): mean 1.75 <= 2 with one step of 4
    r = td.replay([1, 1, 4, 1], 2.0)
    assert not r["tpot_violated"] and r["backend_violations"] == 1
    assert td.replay([], 1.0)["tokens"] == 0


def test_replay_agrees_with_the_delivery_rule_on_random_runs():
    """replay() against delivery_times()/summary() fed the generation times it implies: the two are
    written separately and meet only here.  (The clock origin is modelled as a token generated and
    delivered at time 0.)"""
    rng = np.random.default_rng(5)
    for _ in range(100):
        n = int(rng.integers(1, 50))
        steps = rng.exponential(rng.uniform(0.3, 2.0), size=n)
        slo = float(rng.uniform(0.5, 2.0))
        gen = [0.0] + list(np.cumsum(steps))
        r = td.replay(steps, slo)
        assert np.allclose(r["delivery"], td.delivery_times(gen, slo)[1:], rtol=0, atol=1e-9)
        assert (r["visible_violations"], r["backend_violations"]) == td.summary(gen, slo)
        assert r["visible_violations"] <= r["backend_violations"]


def test_deposit_never_adds_violations_and_keeps_order():
    rng = np.random.default_rng(0)
    for _ in range(100):
        n = int(rng.integers(1, 60))
        gen = np.cumsum(rng.exponential(rng.uniform(0.2, 2.0), size=n))
        d = td.delivery_times(gen, 1.0)
        assert all(b >= a for a, b in zip(d, d[1:])) and all(x >= g for x, g in zip(d, gen))
        seen, backend = td.summary(gen, 1.0)
        assert seen <= backend


def test_library_fifo_matches_the_rule():
    rng = np.random.default_rng(1)
    for trial in range(60):
        n = int(rng.integers(1, 80))
        slo = float(rng.uniform(0.5, 2.0))
        gen = np.cumsum(rng.exponential(rng.uniform(0.2, 2.5), size=n))
        finish = float(gen[-1]) if trial % 2 else None
        dep = orbit.TokenDeposit(slo)
        polls = np.sort(rng.uniform(0, gen[-1] + n * slo + 1, size=int(rng.integers(1, 40))))
        got_tok, got_t, gi = [], [], 0
        events = sorted([(t, 0) for t in gen] + [(t, 1) for t in polls])
        for t, kind in events:
            if kind == 0:
                dep.push(1000 + gi, t)
                gi += 1
                if gi == n and finish is not None:
                    dep.finish(finish)
            else:
                a, b = dep.release(t)
                got_tok += a
                got_t += b
        a, b = dep.release(1e18)
        got_tok += a
        got_t += b
        want = td.delivery_times(list(gen), slo, finish)
        assert got_tok == [1000 + i for i in range(n)]
        np.testing.assert_allclose(got_t, want, rtol=0, atol=1e-9)
        st = dep.stats()
        assert st["waiting"] == 0 and st["delivered"] == n
        assert st["visible_violations"] == td.violations(want, slo)


def test_release_respects_time_and_capacity():
    dep = orbit.TokenDeposit(1.0)
    for i, t in enumerate([0.0, 0.1, 0.2]):
        dep.push(i, t)
    assert dep.release(0.5) == ([0], [0.0])
    assert dep.release(0.9) == ([], [])
    assert dep.release(2.5, cap=1) == ([1], [1.0])
    assert dep.stats()["waiting"] == 1 and dep.stats()["max_size"] == 3
    with pytest.raises(orbit.OrbitError):
        dep.push(9, 0.05)                                    # time runs backwards
    dep.finish(2.6)
    with pytest.raises(orbit.OrbitError):
        dep.push(9, 3.0)                                     # finished
    assert dep.release(2.6) == ([2], [2.0])


def test_profile_refresh_helpers():
    assert orbit.orbit_profile_mismatch(100.0, 131.0, 0.3) and not orbit.orbit_profile_mismatch(100.0, 129.0, 0.3)
    assert orbit.orbit_profile_mismatch(100.0, 60.0, 0.3)
    p = orbit.orbit_profile_ewma([1.0, 2.0, 4.0], [3.0, 2.0, 0.0], 0.25)
    np.testing.assert_allclose(p, [1.5, 2.0, 3.0])
    with pytest.raises(orbit.OrbitError):
        orbit.orbit_profile_ewma([1.0], [1.0], 1.5)
    # properties of a moving average that do not restate its update: n refreshes with a constant observation x
    # leave p0 + (x - p0)(1 - (1 - w)^n); a constant profile is a fixed point; weight 0 keeps, weight 1 replaces;
    # the refreshed value always lies between the old one and the observation
    p0, x, w = np.array([10.0, 0.5]), np.array([4.0, 2.5]), 0.2
    p = p0.copy()
    for n in range(1, 12):
        p = orbit.orbit_profile_ewma(p, x, w)
        np.testing.assert_allclose(p, p0 + (x - p0) * (1 - (1 - w) ** n), rtol=1e-12)
        assert np.all((p - x) * (p0 - x) >= 0) and np.all(np.abs(p - x) < np.abs(p0 - x))
    np.testing.assert_array_equal(orbit.orbit_profile_ewma(x, x, 0.37), x)
    np.testing.assert_array_equal(orbit.orbit_profile_ewma(p0, x, 0.0), p0)
    np.testing.assert_array_equal(orbit.orbit_profile_ewma(p0, x, 1.0), x)
    # the trigger is symmetric in the sign of the error and scale-free
    for pred, obs, frac in ((100.0, 131.0, 0.3), (100.0, 129.0, 0.3), (7.0, 7.0, 0.0), (5.0, 4.0, 0.25)):
        a = orbit.orbit_profile_mismatch(pred, obs, frac)
        assert a == orbit.orbit_profile_mismatch(pred, 2 * pred - obs, frac) == orbit.orbit_profile_mismatch(3 * pred, 3 * obs, frac)


def test_library_slo_replay_matches_the_oracle():
    rng = np.random.default_rng(6)
    keys = ("tokens", "backend_violations", "visible_violations", "max_deposit", "tpot_violated")
    for trial in range(150):
        n = int(rng.integers(0, 70))
        slo = float(rng.uniform(0.5, 2.0))
        if trial % 3 == 0:                                   # integer grid: exact ties between "due" and "generated"
            steps = rng.integers(0, 5, size=n).astype(np.float64)
            slo = float(rng.integers(1, 4))
        else:
            steps = rng.exponential(rng.uniform(0.3, 2.5), size=n)
        fin = bool(trial % 2)
        got, want = orbit.orbit_slo_replay(steps, slo, fin), td.replay(steps, slo, fin)
        assert all(got[k] == want[k] for k in keys), (trial, got, want)
        assert abs(got["tpot"] - want["tpot"]) <= 1e-12 * max(1.0, want["tpot"])
        assert abs(got["max_visible_gap"] - want["max_visible_gap"]) <= 1e-9
    assert orbit.orbit_slo_replay([1, 1, 1, 5, 1], 2.0)["visible_violations"] == 0      # the hand-worked spike
    with pytest.raises(orbit.OrbitError):
        orbit.orbit_slo_replay([1.0, -1.0], 1.0)
    with pytest.raises(orbit.OrbitError):
        orbit.orbit_slo_replay([1.0], 0.0)
