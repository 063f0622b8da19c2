"""The library's scheduling tick against the plain reference (host code on both sides:
identical decisions are required, program by program, in order)."""
import numpy as np
import pytest

from oracle import sched_oracle as so
from paper_2602_13692_amd import binding as ta

PHASE = {ta.PHASE_REASONING: "R", ta.PHASE_ACTING: "A"}
STATUS = {ta.STATUS_ACTIVE: "active", ta.STATUS_PAUSED: "paused", ta.STATUS_TERMINATED: "terminated"}


def random_table(rng, n, n_backends, c_hi=8000):
    t = np.zeros(n, ta.PROGRAM_DTYPE)
    t["id"] = rng.permutation(n) + 100
    t["context"] = rng.integers(1, c_hi, size=n)
    t["phase"] = rng.integers(0, 2, size=n)
    t["status"] = rng.choice([0, 1, 2], size=n, p=[0.55, 0.35, 0.10])
    t["backend"] = np.where(t["status"] == ta.STATUS_ACTIVE, rng.integers(0, max(n_backends, 1), size=n), -1)
    t["acting_time"] = rng.integers(0, 24, size=n) * 0.25           # exact in float32
    return t


def as_dicts(t):
    return [dict(id=int(r["id"]), context=int(r["context"]), backend=int(r["backend"]), phase=PHASE[int(r["phase"])],
                 status=STATUS[int(r["status"])], t_act=float(r["acting_time"])) for r in t]


@pytest.mark.parametrize("seed", range(40))
def test_tick_matches_the_reference(seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(0, 200))
    nb = int(rng.integers(1, 9))
    cap = float(rng.integers(1000, 200000))
    lam_max = float(rng.choice([1.0, 0.9, 0.75]))
    lam_min = float(rng.choice([1.0, 0.9, 0.5, 0.0]))
    base = float(rng.choice([2.0, 1.0, 1.5, np.e]))
    t = random_table(rng, n, nb)
    ref = as_dicts(t)
    want_paused, want_restored = so.tick(ref, nb, cap, lam_max, lam_min, base)
    rc, paused, restored, backends = ta.ta_sched_tick(t, nb, cap, lam_max, lam_min, base)
    assert rc == ta.TA_OK
    assert list(paused) == want_paused
    assert list(zip(restored.tolist(), backends.tolist())) == want_restored
    got = as_dicts(t)
    assert got == ref                                               # the table after the tick, field by field


def test_repeated_ticks_reach_a_fixed_point():
    rng = np.random.default_rng(7)
    t = random_table(rng, 150, 4)
    for _ in range(3):
        ta.ta_sched_tick(t, 4, 60000.0)
    before = t.copy()
    rc, paused, restored, _ = ta.ta_sched_tick(t, 4, 60000.0)
    assert len(paused) == 0 and len(restored) == 0 and np.array_equal(before, t)


def test_bad_tables_are_rejected_untouched():
    t = np.zeros(3, ta.PROGRAM_DTYPE)
    t["context"] = [10, 0, 5]                                       # context < 1
    t["backend"] = 0
    keep = t.copy()
    assert ta.ta_sched_tick(t, 1, 100.0, check=False)[0] == ta.TA_ERR_INVALID_ARG
    assert np.array_equal(t, keep)
    t["context"] = [10, 20, 5]
    t["backend"] = [0, 3, 0]                                        # active on a backend that does not exist
    assert ta.ta_sched_tick(t, 2, 100.0, check=False)[0] == ta.TA_ERR_INVALID_ARG
    t["backend"] = 0
    assert ta.ta_sched_tick(t, 2, 100.0, decay_base=0.5, check=False)[0] == ta.TA_ERR_INVALID_ARG
    assert ta.ta_sched_tick(t, 2, float("nan"), check=False)[0] == ta.TA_ERR_INVALID_ARG
    assert ta.ta_sched_tick(t, 2, 100.0)[0] == ta.TA_OK
