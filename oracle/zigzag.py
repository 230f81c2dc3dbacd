"""CPU oracle for live-scaling request scheduling.  TEST INFRASTRUCTURE ONLY.

Plain discrete-event simulations, in units of one layer's execution time, of the two policies the
paper describes for the period in which a new (target) instance is still loading layers while an
overloaded (source) instance holds the whole model (section 5.2):

  * best-effort: each request batch runs as many layers as are loaded (at most half of the model)
    on the target when it is dispatched there, the rest on the source, in arrival order;
  * ILP-free ZigZag: the target keeps every request in a queue ordered first-come-first-served,
    runs ONE layer of the first request whose next layer is already loaded, and leaves the request
    in the queue; the source, whenever it is idle, takes the first unfinished request and runs all
    of its remaining layers.

and a brute-force solver of the pipeline-configuration program (objective and constraints C1-C3
of section 5.2) for tiny instances.

Readings of points the text leaves open (the figure with the pseudocode is not available):
  - time 0 is the moment the first layer is resident on the target; layer k (0-based) is resident
    from k * load_time on;
  - every (request, layer) execution takes one unit on either instance; the activation hand-off
    takes no time (the paper calls it negligible);
  - the source is busy with earlier work until `source_free_at`; when it and the target become
    free at the same instant, the source chooses first;
  - the source never takes a request while the target is in the middle of one of its layers: it
    waits for that layer to end (it does not skip ahead in the queue: FCFS);
  - ZigZag puts no cap on the number of layers a request may run on the target.

Pins (tests/test_oracle_zigzag.py): the paper's worked example (7 layers, loading a layer takes 6
layer-times): request 1 gets configuration (1,6), requests 2 and 3 get (2,5), request 3 leaves the
source at time 17 = 12 + 5; invariants (every layer of every request executed exactly once and in
order, no layer executed on the target before it is resident, neither instance runs two things at
once, FCFS completion order on the source); limits (infinitely slow loading -> everything after
layer 0 on the source; instant loading and a busy source -> everything on the target); the
brute-force program against hand-enumerated tiny cases.  The paper's "32 -> 22" latency of
request 7 depends on details of a figure that is not available: parity unpinned for that number.
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass, field
from typing import List, Tuple


@dataclass
class Span:
    start: float
    end: float
    instance: str        # "target" or "source"
    request: int
    layer_a: int         # layers [layer_a, layer_b)
    layer_b: int


@dataclass
class Schedule:
    T: List[int]                 # layers each request ran on the target
    S: List[int]                 # layers each request ran on the source
    finish: List[float]          # time each request left the source (or the target if S == 0)
    spans: List[Span] = field(default_factory=list)

    @property
    def avg_latency(self) -> float:
        return sum(self.finish) / len(self.finish)


def _loaded(t: float, load_time: float, L: int) -> int:
    """Layers resident on the target at time t."""
    if load_time <= 0:
        return L
    return min(L, int(t // load_time) + 1)


def simulate_zigzag(L: int, n_requests: int, load_time: float, source_free_at: float = 0.0) -> Schedule:
    done = [0] * n_requests              # layers finished so far
    owner = [None] * n_requests          # "source" once the source has taken the request
    finish = [None] * n_requests
    T = [0] * n_requests
    spans: List[Span] = []
    t = 0.0
    target_free, source_free = 0.0, float(source_free_at)
    target_job = None                    # (request, end)
    guard = 0
    while any(f is None for f in finish):
        guard += 1
        assert guard < 100000, "simulation does not terminate"
        # retire the target's layer if it ends now
        if target_job is not None and target_job[1] <= t:
            r = target_job[0]
            done[r] += 1
            T[r] = done[r]
            if done[r] == L and finish[r] is None and owner[r] is None:
                finish[r] = target_job[1]
            target_job = None
        # source chooses first
        if source_free <= t:
            head = next((r for r in range(n_requests) if finish[r] is None and owner[r] is None), None)
            if head is not None and not (target_job is not None and target_job[0] == head):
                owner[head] = "source"
                remaining = L - done[head]
                if remaining > 0:
                    spans.append(Span(t, t + remaining, "source", head, done[head], L))
                source_free = t + remaining
                finish[head] = t + remaining
        # then the target: first request in FCFS order whose next layer is resident
        if target_job is None and target_free <= t:
            avail = _loaded(t, load_time, L)
            pick = next((r for r in range(n_requests)
                         if finish[r] is None and owner[r] is None and done[r] < avail), None)
            if pick is not None:
                spans.append(Span(t, t + 1, "target", pick, done[pick], done[pick] + 1))
                target_job = (pick, t + 1)
                target_free = t + 1
        # advance to the next event
        cand = []
        if target_job is not None:
            cand.append(target_job[1])
        if source_free > t:
            cand.append(source_free)
        if load_time > 0:
            nxt = (int(t // load_time) + 1) * load_time
            if nxt / load_time < L:
                cand.append(nxt)
        if source_free_at > t:
            cand.append(source_free_at)
        if not cand:
            break
        t = min(cand)
    S = [L - T[r] for r in range(n_requests)]
    return Schedule(T=T, S=S, finish=[float(f) for f in finish], spans=spans)


def simulate_best_effort(L: int, n_requests: int, load_time: float, source_free_at: float = 0.0) -> Schedule:
    half = max(1, L // 2)
    T, S, finish, spans = [], [], [], []
    t_target = 0.0
    t_source = float(source_free_at)
    for r in range(n_requests):
        k = max(1, min(_loaded(t_target, load_time, L), half))
        spans.append(Span(t_target, t_target + k, "target", r, 0, k))
        handed = t_target + k
        t_target = handed
        start = max(t_source, handed)
        spans.append(Span(start, start + (L - k), "source", r, k, L))
        t_source = start + (L - k)
        T.append(k)
        S.append(L - k)
        finish.append(t_source)
    return Schedule(T=T, S=S, finish=finish, spans=spans)


def program_constraints_hold(L: int, T: List[int], time_l: float) -> Tuple[bool, bool, bool]:
    """C1-C3 of the pipeline-configuration program for a configuration T (S = L - T), requests
    numbered from 1 as in the paper; sums with a missing lower limit start at j = 1."""
    n = len(T)
    S = [L - x for x in T]
    c1 = all(0 <= x <= L for x in T)
    c2 = all(sum(T[:i + 1]) <= sum(S[:i]) for i in range(1, n))
    c3 = all(time_l * T[i] <= sum(T[:i]) + (n - (i + 1) + 1) * (T[i] - 1) for i in range(1, n))
    return c1, c2, c3


def program_objective(L: int, T: List[int]) -> float:
    """Average over requests of the sum of S over the request and all earlier ones."""
    S = [L - x for x in T]
    n = len(T)
    return sum(sum(S[:r + 1]) for r in range(n)) / n


def solve_program_bruteforce(L: int, n_requests: int, time_l: float):
    """Enumerates every configuration; returns (best objective, best T) under C1-C3, or None."""
    best = None
    for T in itertools.product(range(0, L + 1), repeat=n_requests):
        c1, c2, c3 = program_constraints_hold(L, list(T), time_l)
        if c1 and c2 and c3:
            obj = program_objective(L, list(T))
            if best is None or obj < best[0] - 1e-12:
                best = (obj, list(T))
    return best
