"""CPU tests of the trace-driven policy simulator: the Python reference against hand-worked runs
and invariants, and the library's simulator against the reference, event by event."""
import os

import numpy as np
import pytest

from oracle import sim_oracle
from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
KINDS = {"EVICT": 1, "EVICT_FORCED": 2, "RESTORE": 3, "PREFILL": 4, "DECODE": 5, "RELEASE": 6}


def _golden(name):
    rows = []
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        rows.append((int(f[0]), dict(kind=KINDS[f[1]], program=int(f[2]), backend=int(f[3]), tokens=int(f[4]),
                                     context=int(f[5]), slots=[int(x) for x in f[6:]])))
    return rows


def _library_events(sim):
    events, slots = sim.tick()
    return [dict(kind=int(e["kind"]), program=int(e["program"]), backend=int(e["backend"]), tokens=int(e["tokens"]),
                 context=int(e["context"]),
                 slots=[int(x) for x in slots[int(e["first_slot"]): int(e["first_slot"]) + int(e["n_slots"])]])
            for e in events]


SCENARIOS = {
    "sim_two_programs.txt": dict(n_backends=1, pool_pages=4, steps_per_tick=2, max_context=64, time_per_tick=1.0,
                                 capacity=48.0, initial_context=[20, 30], turn_tokens=[[2, 1], [3, 1]],
                                 tool_ticks=[[1, 1], [2, 1]], tool_tokens=[[10, 5], [4, 4]], ticks=9),
    "sim_forced_eviction.txt": dict(n_backends=1, pool_pages=4, steps_per_tick=1, max_context=64, time_per_tick=1.0,
                                    capacity=60.0, initial_context=[30, 34], turn_tokens=[[1, 1], [2, 1]],
                                    tool_ticks=[[5, 1], [1, 1]], tool_tokens=[[3, 3], [2, 2]], ticks=8),
}


def _both(sc, lambda_max=1.0, lambda_min=1.0, base=2.0):
    args = (sc["n_backends"], sc["pool_pages"], sc["steps_per_tick"], sc["max_context"], sc["time_per_tick"],
            sc["capacity"], lambda_max, lambda_min, base, sc["initial_context"], sc["turn_tokens"], sc["tool_ticks"],
            sc["tool_tokens"])
    return sim_oracle.Simulator(*args), ta.Sim(*args)


@pytest.mark.parametrize("name", sorted(SCENARIOS))
def test_hand_worked_runs(name):
    """Both the reference and the library reproduce the runs worked out on paper: the order of the
    waiting queue, the decayed admission, the reclaiming of an idle cache, restores that cannot be
    carried out, page hand-out order, release at the end of the trace."""
    sc = SCENARIOS[name]
    want = _golden(name)
    ref, lib = _both(sc)
    got_ref, got_lib = [], []
    for tick in range(1, sc["ticks"] + 1):
        got_ref += [(tick, e) for e in ref.tick()]
        got_lib += [(tick, e) for e in _library_events(lib)]
    assert got_ref == want
    assert got_lib == want
    assert all(p["status"] == "terminated" for p in ref.programs)
    assert all(int(s) == ta.STATUS_TERMINATED for s in lib.programs()["status"])


def _random_scenario(seed, n_programs, n_backends, pool_pages, capacity, steps_per_tick, time_per_tick, max_context):
    tr = wl.agent_trace(seed, n_programs, n_turns=3, context_lo=100, context_hi=900, turn_lo=3, turn_hi=40,
                        tool_median_ticks=2.0, tool_sigma=1.0, out_lo=5, out_hi=200)
    return dict(n_backends=n_backends, pool_pages=pool_pages, steps_per_tick=steps_per_tick, max_context=max_context,
                time_per_tick=time_per_tick, capacity=capacity, initial_context=tr.initial_context.tolist(),
                turn_tokens=tr.turn_tokens.tolist(), tool_ticks=tr.tool_ticks.tolist(),
                tool_tokens=tr.tool_tokens.tolist())


CASES = [  # programs, backends, pool pages, capacity tokens, steps per tick, time per tick, max context, decay base
    (12, 1, 220, 3000.0, 4, 1.0, 2000, 2.0),
    (24, 2, 200, 2800.0, 6, 0.5, 1500, 2.0),
    (40, 4, 120, 1900.0, 3, 1.0, 1200, 2.0),    # tight pools: reclaiming and failed restores
    (16, 2, 300, 2500.0, 5, 1.0, 2000, 1.0),    # no decay
    (30, 3, 90, 1440.0, 8, 2.0, 1000, 4.0),     # fast decay, pool equal to the capacity
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_library_matches_reference_event_by_event_and_invariants_hold(case, seed):
    n, nb, pool, cap, steps, dt, max_ctx, base = case
    sc = _random_scenario(wl.SEED_BASE + 5000 + 17 * seed + n, n, nb, pool, cap, steps, dt, max_ctx)
    ref, lib = _both(sc, base=base)
    held = [dict() for _ in range(nb)]                 # page -> program, per backend
    context = list(sc["initial_context"])
    seen = {k: 0 for k in KINDS.values()}
    for tick in range(3000):
        want = ref.tick()
        got = _library_events(lib)
        assert got == want, f"tick {tick}"
        table = lib.programs()
        for e in want:
            seen[e["kind"]] += 1
            p, b = e["program"], e["backend"]
            if e["kind"] in (sim_oracle.EVICT, sim_oracle.EVICT_FORCED, sim_oracle.RELEASE):
                assert len(e["slots"]) == sim_oracle.pages_of(context[p])
                for s in e["slots"]:
                    assert held[b].pop(s) == p                      # it held exactly these pages
            else:
                for s in e["slots"]:
                    assert 0 <= s < pool and s not in held[b]       # a page is never handed out twice
                    held[b][s] = p
                if e["kind"] == sim_oracle.PREFILL:
                    context[p] += e["tokens"]
                elif e["kind"] == sim_oracle.DECODE:
                    context[p] += 1
                assert e["context"] == context[p] <= max_ctx
        for p in range(n):
            mine = lib.page_table(p)
            active = int(table["status"][p]) == ta.STATUS_ACTIVE
            assert len(mine) == (sim_oracle.pages_of(context[p]) if active else 0)
            if active:
                b = int(table["backend"][p])
                assert all(held[b][int(s)] == p for s in mine)
            assert int(table["context"][p]) == context[p] == ref.programs[p]["context"]
        if all(int(s) == ta.STATUS_TERMINATED for s in table["status"]):
            break
    else:
        pytest.fail("some program never finished its trace")
    assert all(not h for h in held), "every page is free again once all programs have ended"
    assert seen[sim_oracle.RESTORE] > 0 and seen[sim_oracle.DECODE] > 0 and seen[sim_oracle.PREFILL] > 0
    assert seen[sim_oracle.RELEASE] == n


def test_tight_pools_exercise_every_kind_of_event():
    totals = {k: 0 for k in KINDS.values()}
    for seed in (1, 2, 3):
        n, nb, pool, cap, steps, dt, max_ctx, base = CASES[2]
        sc = _random_scenario(wl.SEED_BASE + 5000 + 17 * seed + n, n, nb, pool, cap, steps, dt, max_ctx)
        ref, _ = _both(sc, base=base)
        for _ in range(400):
            for e in ref.tick():
                totals[e["kind"]] += 1
    assert all(v > 0 for v in totals.values()), totals


def test_invalid_configurations_are_refused():
    good = dict(SCENARIOS["sim_two_programs.txt"])
    good.pop("ticks")

    def make(**over):
        sc = dict(good, **over)
        return ta.Sim(sc["n_backends"], sc["pool_pages"], sc["steps_per_tick"], sc["max_context"], sc["time_per_tick"],
                      sc["capacity"], 1.0, 1.0, over.get("base", 2.0), sc["initial_context"], sc["turn_tokens"],
                      sc["tool_ticks"], sc["tool_tokens"])

    make().close()
    for bad in (dict(n_backends=0), dict(pool_pages=0), dict(max_context=10), dict(initial_context=[0, 30]),
                dict(turn_tokens=[[2, 0], [3, 1]]), dict(tool_ticks=[[0, 1], [2, 1]]), dict(base=0.5),
                dict(capacity=-1.0)):
        with pytest.raises(ta.TaError):
            make(**bad)
