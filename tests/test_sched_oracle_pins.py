"""Pins of the scheduling-tick reference against what the paper states (Sec. 4.3), none of
which uses the reference to check itself: hand-worked cases and properties."""
import itertools
import math

import numpy as np
import pytest

from oracle import sched_oracle as so


def prog(i, c, phase="R", backend=0, status="active", t_act=0.0):
    return dict(id=i, context=c, backend=backend, phase=phase, status=status, t_act=t_act)


def test_no_pause_at_or_below_capacity_and_pause_above():
    ps = [prog(0, 400), prog(1, 600)]
    assert so.tick(ps, 1, 1000.0) == ([], [])                 # C_total < sum c is false at equality
    ps = [prog(0, 400), prog(1, 601)]
    paused, restored = so.tick(ps, 1, 1000.0)
    assert paused == [0] and restored == []                   # the shorter one goes: shortest first
    assert ps[0]["status"] == "paused" and ps[0]["backend"] == -1


def test_acting_programs_are_paused_before_any_reasoning_program():
    # the indicator dominates 1/c: a long acting program outranks a short reasoning one
    ps = [prog(0, 10, "R"), prog(1, 5000, "A", t_act=0.0), prog(2, 3000, "A", t_act=0.0), prog(3, 4000, "R")]
    paused, _ = so.tick(ps, 1, 7500.0, base=1.0)               # load 12010, must shed 4510
    assert paused == [2, 1]                                    # acting, shortest first; then enough
    assert so.s_pause(ps[1]) > so.s_pause(ps[0])


def test_decayed_weight_of_acting_programs():
    # hand-computed: c f(t) with f(t) = 2^-t
    assert so.weight(prog(0, 1024, "A", t_act=3.0), 2.0) == 128.0
    assert so.weight(prog(0, 1024, "R", t_act=3.0), 2.0) == 1024.0
    assert so.weight(prog(0, 1024, "A", t_act=3.0), 1.0) == 1024.0     # base 1: no decay
    # an idle acting program shrinks until a reasoning program fits beside it
    ps = [prog(0, 800, "A", t_act=0.0), prog(1, 600, "R", backend=-1, status="paused")]
    assert so.tick(ps, 1, 1000.0) == ([], [])                  # 800 + 600 > 1000: stays queued
    ps[0]["t_act"] = 1.0                                       # 400 + 600 <= 1000
    assert so.tick(ps, 1, 1000.0) == ([], [(1, 0)])
    # its decoding then raises the pressure: the idle cache is the first to go
    ps[1]["context"] = 900
    ps[0]["t_act"] = 1.0
    assert so.tick(ps, 1, 1000.0)[0] == [0]


def test_restore_prefers_reasoning_then_shortest_and_respects_the_watermarks():
    ps = [prog(0, 300, "A", -1, "paused", 0.0), prog(1, 500, "R", -1, "paused"), prog(2, 200, "R", -1, "paused"),
          prog(3, 100, "R", 0)]
    paused, restored = so.tick(ps, 1, 1000.0, base=1.0)
    assert paused == []
    assert [r[0] for r in restored] == [2, 1]                  # reasoning first, shortest first; 0 no longer fits
    # hysteresis: with lambda_min = 0.5 a backend at 60 % takes nobody, at 40 % it fills up to lambda_max
    ps = [prog(0, 600, "R", 0), prog(1, 100, "R", -1, "paused")]
    assert so.tick(ps, 1, 1000.0, lambda_max=0.9, lambda_min=0.5) == ([], [])
    ps = [prog(0, 400, "R", 0), prog(1, 100, "R", -1, "paused"), prog(2, 450, "R", -1, "paused")]
    paused, restored = so.tick(ps, 1, 1000.0, lambda_max=0.9, lambda_min=0.5)
    assert restored == [(1, 0)]                                # 400+100 = 500 is no longer below 0.5 C


def test_global_queue_restores_on_the_backend_with_most_room():
    ps = [prog(0, 700, "R", 0), prog(1, 200, "R", 1), prog(2, 500, "R", 2), prog(3, 250, "R", -1, "paused"),
          prog(4, 300, "R", -1, "paused")]
    _, restored = so.tick(ps, 3, 1000.0)
    assert restored == [(3, 1), (4, 1)]                        # rooms 300/800/500, then 300/550/500
    # a program paused on a full backend moves to an idle one within the same tick
    ps = [prog(0, 900, "R", 0), prog(1, 300, "R", 0), prog(2, 100, "R", 1)]
    paused, restored = so.tick(ps, 2, 1000.0)
    assert paused == [1] and restored == [(1, 1)]


def test_terminated_programs_count_for_nothing():
    ps = [prog(0, 900, "R", 0, "terminated"), prog(1, 900, "R", 0)]
    assert so.tick(ps, 1, 1000.0) == ([], [])


@pytest.mark.parametrize("seed", range(20))
def test_properties_on_random_tables(seed):
    rng = np.random.default_rng(seed)
    n, nb, cap = 40, 3, 20000.0
    ps = []
    for i in range(n):
        status = rng.choice(["active", "paused", "terminated"], p=[0.6, 0.3, 0.1])
        ps.append(prog(i, int(rng.integers(1, 6000)), rng.choice(["R", "A"]),
                       int(rng.integers(0, nb)) if status == "active" else -1, status,
                       float(rng.integers(0, 4))))
    before = {p["id"]: dict(p) for p in ps}
    paused, restored = so.tick(ps, nb, cap)
    after = {p["id"]: p for p in ps}
    # every backend ends at or below the limit, recomputed here from scratch
    for b in range(nb):
        load = sum((p["context"] if p["phase"] == "R" else p["context"] * 2.0 ** -p["t_act"])
                   for p in ps if p["status"] == "active" and p["backend"] == b)
        assert load <= cap + 1e-9
    # on each backend: an acting program that stayed means no reasoning program of that backend was
    # paused, and the paused ones of a class are the shortest of that class
    for b in range(nb):
        was = [p for p in before.values() if p["status"] == "active" and p["backend"] == b]
        gone = [p for p in was if p["id"] in paused]
        kept = [p for p in was if p["id"] not in paused]
        if any(p["phase"] == "A" for p in kept):
            assert all(p["phase"] == "A" for p in gone)
        for cls in "AR":
            g = [p["context"] for p in gone if p["phase"] == cls]
            k = [p["context"] for p in kept if p["phase"] == cls]
            if g and k:
                assert max(g) <= min(k)
    # nobody is both untouched-terminated and moved; restored programs were paused (before or in this tick)
    for pid, b in restored:
        assert before[pid]["status"] == "paused" or pid in paused
        assert after[pid]["status"] == "active" and after[pid]["backend"] == b
    for p in before.values():
        if p["status"] == "terminated":
            assert after[p["id"]] == p


def test_shortest_first_frees_the_demand_at_lower_quadratic_cost_than_longest_first():
    """The reason for shortest-first (recomputation cost grows with c^2): against the opposite
    greedy order, and against every subset of the same size, on small instances."""
    rng = np.random.default_rng(99)
    for _ in range(50):
        cs = sorted(int(x) for x in rng.integers(100, 4000, size=7))
        total = sum(cs)
        cap = float(total - int(rng.integers(1, total // 2)))
        ps = [prog(i, c) for i, c in enumerate(cs)]
        paused, _ = so.tick(ps, 1, cap, lambda_min=0.0)          # lambda_min 0: nothing comes back
        k = len(paused)
        chosen = [cs[i] for i in paused]
        assert chosen == cs[:k] and total - sum(chosen) <= cap   # a prefix of the sorted lengths, enough freed
        assert total - sum(chosen[:-1]) > cap                    # and not one more than needed
        cost = sum(c * c for c in chosen)
        longest, freed, j = 0, 0, len(cs)
        while total - freed > cap:
            j -= 1
            freed += cs[j]
            longest += cs[j] * cs[j]
        assert cost <= longest or k > len(cs) - j                # cheaper unless it needs more programs
        for other in itertools.combinations(cs, k):
            assert cost <= sum(c * c for c in other)             # the k shortest minimise sum c^2 among k-subsets
