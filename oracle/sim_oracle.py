"""Plain reference of the trace-driven policy simulator (test infrastructure only).

Follows the paper's middleware (Sec. 4.1, 4.3; workflows with tool calls as in Sec. 2.1 and
App. B): a table of programs that alternate reasoning turns and tool calls, the periodic
scheduling decision of sched_oracle.tick over several backends with one global waiting queue,
and a page allocator per backend, so that every decision becomes an event (evict, restore,
prefill, decode, release) naming the pool pages it concerns.  Pure Python; it shares no code
with the library's simulator and is compared with it event by event.

The trace (turn lengths, tool latencies in ticks, tool output sizes, initial contexts) is an
input; nothing here draws a random number.

Where the paper is silent the backend's own reclaiming of idle caches is modelled explicitly:
a grant that finds no free page takes the pages of the active program on that backend that is
waiting for a tool, has the highest S_pause and is not being served in this tick ("forced"
eviction); if there is none, the program asking leaves instead (a restore is not carried out).
"""
from __future__ import annotations

from typing import Dict, List

from . import sched_oracle

PAGE = 16
EVICT, EVICT_FORCED, RESTORE, PREFILL, DECODE, RELEASE = 1, 2, 3, 4, 5, 6


def pages_of(tokens: int) -> int:
    return (tokens + PAGE - 1) // PAGE


class Simulator:
    def __init__(self, n_backends: int, pool_pages: int, steps_per_tick: int, max_context: int,
                 time_per_tick: float, capacity: float, lambda_max: float, lambda_min: float, base: float,
                 initial_context, turn_tokens, tool_ticks, tool_tokens):
        self.nb, self.steps, self.max_context, self.dt = n_backends, steps_per_tick, max_context, time_per_tick
        self.policy = dict(capacity=capacity, lambda_max=lambda_max, lambda_min=lambda_min, base=base)
        self.turn_tokens, self.tool_ticks, self.tool_tokens = turn_tokens, tool_ticks, tool_tokens
        self.n_turns = len(turn_tokens[0])
        self.programs: List[Dict] = []
        for i, c in enumerate(initial_context):
            self.programs.append(dict(id=i, context=int(c), backend=-1, phase="R", status="paused", t_act=0.0,
                                      turn=0, tokens_left=int(turn_tokens[i][0]), tool_left=0, pending=0))
        self.pages: List[List[int]] = [[] for _ in initial_context]
        # each backend hands out page 0 first; freed pages are handed out again last-freed-first
        self.free: List[List[int]] = [list(range(pool_pages - 1, -1, -1)) for _ in range(n_backends)]
        self.events: List[Dict] = []

    # -- bookkeeping ---------------------------------------------------------------------------
    def _emit(self, kind, p, backend, tokens, slots):
        self.events.append(dict(kind=kind, program=p["id"], backend=backend, tokens=tokens,
                                context=p["context"], slots=list(slots)))

    def _give_up(self, kind, p, backend):
        mine = self.pages[p["id"]]
        self._emit(kind, p, backend, p["context"], mine)
        if backend >= 0:
            self.free[backend].extend(reversed(mine))
        self.pages[p["id"]] = []

    def _make_room(self, backend, need, served) -> bool:
        while len(self.free[backend]) < need:
            cands = [q for q in self.programs
                     if q["status"] == "active" and q["backend"] == backend and q["phase"] == "A"
                     and q["id"] not in served]
            if not cands:
                return False
            victim = max(cands, key=lambda q: (sched_oracle.s_pause(q), -q["id"]))
            self._give_up(EVICT_FORCED, victim, backend)
            victim["status"], victim["backend"] = "paused", -1
        return True

    def _take(self, p, backend, n):
        got = [self.free[backend].pop() for _ in range(n)]
        self.pages[p["id"]].extend(got)
        return got

    def _release(self, p):
        self._give_up(RELEASE, p, p["backend"])
        p["status"], p["backend"] = "terminated", -1

    def _grow(self, kind, p, new_context, tokens):
        b = p["backend"]
        need = pages_of(new_context) - len(self.pages[p["id"]])
        if need > 0 and not self._make_room(b, need, {p["id"]}):
            self._give_up(EVICT_FORCED, p, b)
            p["status"], p["backend"] = "paused", -1
            return
        got = self._take(p, b, max(need, 0))
        p["context"] = new_context
        self._emit(kind, p, b, tokens, got)

    # -- one tick --------------------------------------------------------------------------------
    def tick(self) -> List[Dict]:
        self.events = []
        # 1. tools
        for p in self.programs:
            if p["status"] == "terminated" or p["phase"] != "A":
                continue
            p["t_act"] = float(_f32(p["t_act"] + self.dt))
            p["tool_left"] -= 1
            if p["tool_left"] > 0:
                continue
            i = p["id"]
            p["pending"] = int(self.tool_tokens[i][p["turn"]])
            p["turn"] += 1
            p["tokens_left"] = int(self.turn_tokens[i][p["turn"]]) if p["turn"] < self.n_turns else 0
            p["phase"], p["t_act"] = "R", 0.0
        # 2. the policy
        before = [p["backend"] for p in self.programs]
        paused, restored = sched_oracle.tick(self.programs, self.nb, **self.policy)
        served = {i for i, _ in restored}
        for i in paused:
            self._give_up(EVICT, self.programs[i], before[i])
        for i, b in restored:
            p = self.programs[i]
            need = pages_of(p["context"])
            if not self._make_room(b, need, served):
                p["status"], p["backend"] = "paused", -1
                served.discard(i)
                continue
            self._take(p, b, need)
            self._emit(RESTORE, p, b, p["context"], self.pages[i])

        def running(p):
            return p["status"] == "active" and p["phase"] == "R"

        # 3. tool output waiting to be prefilled
        for p in self.programs:
            if not running(p) or p["pending"] == 0:
                continue
            if p["context"] + p["pending"] > self.max_context:
                self._release(p)
                continue
            self._grow(PREFILL, p, p["context"] + p["pending"], p["pending"])
            if p["status"] == "active":
                p["pending"] = 0
        # 4. decode steps
        for step in range(self.steps):
            for p in self.programs:
                if not running(p) or p["pending"] != 0 or p["tokens_left"] == 0:
                    continue
                if p["context"] + 1 > self.max_context:
                    self._release(p)
                    continue
                self._grow(DECODE, p, p["context"] + 1, step)
                if p["status"] == "active":
                    p["tokens_left"] -= 1
        # 5. finished turns
        for p in self.programs:
            if not running(p) or p["pending"] != 0 or p["tokens_left"] != 0:
                continue
            if p["turn"] >= self.n_turns:
                self._release(p)
                continue
            p["phase"], p["t_act"] = "A", 0.0
            p["tool_left"] = int(self.tool_ticks[p["id"]][p["turn"]])
        return self.events


def _f32(x: float) -> float:
    """The program table keeps the tool time in single precision."""
    import struct

    return struct.unpack("f", struct.pack("f", x))[0]
