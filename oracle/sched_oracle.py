"""Plain reference of the program-aware scheduling tick (test infrastructure only).

Follows the paper's scheduling policy (Sec. 4.3): the periodic capacity check with time
decay (the thrashing condition and its decayed form), Pause and Restore, the shortest-first
scores S_pause and S_restore, and the global waiting queue that restores a program on the
backend with the most available capacity.  Pure Python, float64, no code shared with the
library's implementation.

A program is a dict with the fields of the paper's tuple <ID, c, T, L, tau, s> that the
policy reads (the tool set T plays no part in it) plus the time its current tool call has
been running:
    id       int
    context  c, tokens (>= 1)
    backend  L: index of the backend it is bound to, or -1
    phase    tau: "R" (reasoning) or "A" (acting)
    status   s: "active", "paused" or "terminated"
    t_act    tool execution time so far in the current step (only read while acting)
"""
from __future__ import annotations

from typing import Dict, List, Tuple


def decay(t: float, base: float) -> float:
    """f(t) = base^(-t); the paper runs with base 2 (Sec. 5.1); base 1 is "no decay"."""
    return base ** (-t)


def weight(p: Dict, base: float) -> float:
    """Tokens a program counts for in the capacity check: c while reasoning, c f(t) while acting."""
    return float(p["context"]) if p["phase"] == "R" else float(p["context"]) * decay(p["t_act"], base)


def load_of(programs: List[Dict], backend: int, base: float) -> float:
    """Right-hand side of the decayed thrashing condition for one backend (program order)."""
    total = 0.0
    for p in programs:
        if p["status"] == "active" and p["backend"] == backend:
            total += weight(p, base)
    return total


def s_pause(p: Dict) -> float:
    return 1.0 / p["context"] + (1.0 if p["phase"] == "A" else 0.0)


def s_restore(p: Dict) -> float:
    return 1.0 / p["context"] + (1.0 if p["phase"] == "R" else 0.0)


def tick(programs: List[Dict], n_backends: int, capacity: float, lambda_max: float = 1.0,
         lambda_min: float = 1.0, base: float = 2.0) -> Tuple[List[int], List[Tuple[int, int]]]:
    """One periodic check over all backends.  Mutates `programs`; returns (paused ids in the
    order they were paused, (restored id, backend) in the order they were restored).

    Pause pass, backend by backend: while the decayed load exceeds lambda_max C_total, pause
    the active program on that backend with the highest S_pause (ties: lower id).
    Restore pass, over the global waiting queue in descending S_restore (ties: lower id): a
    paused program goes to the backend with the most room below lambda_max C_total among the
    backends whose load is below lambda_min C_total (ties: lower index), if its weight still
    fits below lambda_max C_total there; otherwise it stays in the queue.
    """
    hi, lo = lambda_max * capacity, lambda_min * capacity
    paused: List[int] = []
    for b in range(n_backends):
        while load_of(programs, b, base) > hi:
            cands = [p for p in programs if p["status"] == "active" and p["backend"] == b]
            if not cands:
                break
            victim = max(cands, key=lambda p: (s_pause(p), -p["id"]))
            victim["status"] = "paused"
            victim["backend"] = -1
            paused.append(victim["id"])
    restored: List[Tuple[int, int]] = []
    queue = sorted((p for p in programs if p["status"] == "paused"),
                   key=lambda p: (-s_restore(p), p["id"]))
    for p in queue:
        loads = [load_of(programs, b, base) for b in range(n_backends)]
        best, best_room = -1, 0.0
        for b in range(n_backends):
            room = hi - loads[b]
            if loads[b] < lo and (best < 0 or room > best_room):
                best, best_room = b, room
        if best >= 0 and loads[best] + weight(p, base) <= hi:
            p["status"] = "active"
            p["backend"] = best
            restored.append((p["id"], best))
    return paused, restored
