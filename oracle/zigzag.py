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
  - ZigZag puts no cap on the number of layers a request may run on the target;
  - `layer_time` (section 5.4, the retrofit for LLMs): the time of a layer grows with the number of
    batched tokens, so every request batch gets a factor of its own, found by profiling; here
    layer_time[r] is the time ONE layer of request r takes on either instance (default 1 for all:
    the section 5.2 model).  Loading times stay in the same absolute unit.  The decision rules do
    not change; only the durations do.

Pins (tests/test_oracle_zigzag.py, values in tests/golden/zigzag_example.txt): the paper's worked
example (7 layers, loading a layer takes 6 layer-times) - request 1 gets (1,6), requests 2 and 3
get (2,5), requests 2-5 have each run two layers on the target when the third layer arrives, the
second-layer pass over requests 3-6 coincides with layers 3-6 of request 2 on the source, request 3
leaves the source at 17 = 12 + 5, and the late request's inference time (first layer started to
last layer finished) drops from 32 to 22; invariants (every layer of every request executed exactly
once and in order, no layer executed on the target before it is resident, neither instance runs
two things at once, FCFS completion order on the source); limits (infinitely slow loading ->
everything after layer 0 on the source; instant loading and a busy source -> everything on the
target); the program's constraints against hand-enumerated tiny cases and against the example's own
configurations; the ILP-free policy against the best of all fixed configurations on tiny cases;
per-request layer times against two timelines worked out by hand, against the unit-time schedule
when all factors are equal (times scale, configurations do not change) and against the invariants.

Parity unpinned (stated by the paper, not reproduced under these readings, reported by the tests):
  - "(2,5)" as the FINAL configuration of requests 4 and 5: the ILP-free rule gives (3,4) and (4,3);
    (2,5) holds for them only up to the arrival of the third layer;
  - "32 -> 22" for request 7: the pair is reproduced exactly by request 6 (the request the
    best-effort paragraph names as the one that misses its deadline); request 7 gives 36 -> 18.
  (Holding requests 2-5 at (2,5) would give the late request 27, not 22: the two go together.)
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
    first_start: List[float] = field(default_factory=list)   # when each request's first layer started, on either instance

    @property
    def avg_latency(self) -> float:
        return sum(self.finish) / len(self.finish)


def _loaded(t: float, load_time: float, L: int) -> int:
    """Layers resident on the target at time t: layer k is resident from k * load_time on.  The count is settled
    against the products k * load_time themselves (event times ARE such products; a quotient t / load_time may
    round to just below k when t is exactly k * load_time)."""
    if load_time <= 0:
        return L
    k = min(L, max(1, int(t // load_time) + 1))
    while k < L and k * load_time <= t:
        k += 1
    while k > 1 and (k - 1) * load_time > t:
        k -= 1
    return k


def _next_arrival(t: float, load_time: float, L: int):
    """Time at which the next layer becomes resident after t, or None (all resident, or loading is instant)."""
    if load_time <= 0:
        return None
    k = _loaded(t, load_time, L)          # layers 0 .. k-1 are resident, so layer k is the next to arrive
    return k * load_time if k < L else None


def _first_starts(spans: List[Span], n: int) -> List[float]:
    return [min(sp.start for sp in spans if sp.request == r) for r in range(n)]


def _layer_times(n_requests: int, layer_time) -> List[float]:
    if layer_time is None:
        return [1.0] * n_requests
    w = [float(x) for x in layer_time]
    assert len(w) == n_requests and all(x > 0 for x in w)
    return w


def simulate_zigzag(L: int, n_requests: int, load_time: float, source_free_at: float = 0.0,
                    layer_time=None) -> Schedule:
    w = _layer_times(n_requests, layer_time)
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
                    spans.append(Span(t, t + remaining * w[head], "source", head, done[head], L))
                source_free = t + remaining * w[head]
                finish[head] = t + remaining * w[head]
        # then the target: first request in FCFS order whose next layer is resident
        if target_job is None and target_free <= t:
            avail = _loaded(t, load_time, L)
            pick = next((r for r in range(n_requests)
                         if finish[r] is None and owner[r] is None and done[r] < avail), None)
            if pick is not None:
                spans.append(Span(t, t + w[pick], "target", pick, done[pick], done[pick] + 1))
                target_job = (pick, t + w[pick])
                target_free = t + w[pick]
        # advance to the next event
        cand = []
        if target_job is not None:
            cand.append(target_job[1])
        if source_free > t:
            cand.append(source_free)
        nxt = _next_arrival(t, load_time, L)
        if nxt is not None:
            cand.append(nxt)
        if source_free_at > t:
            cand.append(source_free_at)
        if not cand:
            break
        t = min(cand)
    S = [L - T[r] for r in range(n_requests)]
    return Schedule(T=T, S=S, finish=[float(f) for f in finish], spans=spans,
                    first_start=_first_starts(spans, n_requests))


def simulate_best_effort(L: int, n_requests: int, load_time: float, source_free_at: float = 0.0,
                         layer_time=None) -> Schedule:
    w = _layer_times(n_requests, layer_time)
    half = max(1, L // 2)
    T, S, finish, spans = [], [], [], []
    t_target = 0.0
    t_source = float(source_free_at)
    for r in range(n_requests):
        k = max(1, min(_loaded(t_target, load_time, L), half))
        spans.append(Span(t_target, t_target + k * w[r], "target", r, 0, k))
        handed = t_target + k * w[r]
        t_target = handed
        T.append(k)
        S.append(L - k)
        if k == L:                               # a one-layer model: nothing is left for the source
            finish.append(handed)
            continue
        start = max(t_source, handed)
        spans.append(Span(start, start + (L - k) * w[r], "source", r, k, L))
        t_source = start + (L - k) * w[r]
        finish.append(t_source)
    return Schedule(T=T, S=S, finish=finish, spans=spans, first_start=_first_starts(spans, n_requests))


def simulate_configuration(L: int, T: List[int], load_time: float, source_free_at: float = 0.0) -> Schedule:
    """Timeline of a FIXED pipeline configuration T (request r runs layers [0, T[r]) on the target,
    the rest on the source): the target serves its queue in the ZigZag order (first request, in
    arrival order, that still owes target layers and whose next layer is resident; one layer at a
    time), the source serves requests first-come-first-served and starts request r only when the
    target has finished all T[r] of its layers.  Used to give the solutions of the
    pipeline-configuration program real latencies, waiting included (the program's own objective
    models neither the wait for a layer to arrive nor an idle source)."""
    n = len(T)
    assert all(0 <= x <= L for x in T)
    done = [0] * n
    ready_at = [0.0 if T[r] == 0 else None for r in range(n)]     # when the target finished its share
    finish: List[float] = [None] * n
    first_start: List[float] = [None] * n
    spans: List[Span] = []
    t_target = 0.0
    # target side: event loop over "free at t_target"
    guard = 0
    while any(done[r] < T[r] for r in range(n)):
        guard += 1
        assert guard < 100000
        avail = _loaded(t_target, load_time, L)
        pick = next((r for r in range(n) if done[r] < T[r] and done[r] < avail), None)
        if pick is None:                       # wait for the next layer to arrive
            t_target = _next_arrival(t_target, load_time, L)
            continue
        spans.append(Span(t_target, t_target + 1, "target", pick, done[pick], done[pick] + 1))
        if first_start[pick] is None:
            first_start[pick] = t_target
        done[pick] += 1
        t_target += 1
        if done[pick] == T[pick]:
            ready_at[pick] = t_target
    t_source = float(source_free_at)
    for r in range(n):
        if T[r] == L:                          # nothing left for the source
            finish[r] = ready_at[r]
            continue
        start = max(t_source, ready_at[r])
        if first_start[r] is None:
            first_start[r] = start
        spans.append(Span(start, start + (L - T[r]), "source", r, T[r], L))
        t_source = start + (L - T[r])
        finish[r] = t_source
    return Schedule(T=list(T), S=[L - x for x in T], finish=[float(f) for f in finish], spans=spans,
                    first_start=[float(f) for f in first_start])


def program_constraints_hold(L: int, T: List[int], time_l: float, c3_reading: str = "first_layer_origin",
                             c3_for_first: bool = True) -> Tuple[bool, bool, bool]:
    """C1-C3 of the pipeline-configuration program (section 5.2) for a configuration T (S = L - T),
    requests numbered from 1 as in the paper; sums with a missing lower limit start at j = 1.

    C3 (load limit) has two readings here:
      "printed"             time_l * T_i       <= sum_{j<i} T_j + (N - i + 1) * (T_i - 1), for i > 1,
                            exactly as typeset.  With the paper's own example (7 layers, time_l = 6,
                            7 requests) it rejects the configurations the example uses: request 2
                            with T = 2 needs 12 <= 1 + 6.
      "first_layer_origin"  time_l * (T_i - 1) <= the same right-hand side.  The right-hand side
                            counts execution time, and execution starts when the FIRST layer is
                            resident (caption of the ZigZag figure), by which time one load time
                            has already passed; T_i layers are then resident after (T_i - 1) more
                            load times.  This reading accepts the example's (1,6), (2,5), (2,5), ...
                            and is the default.  Requests with T_i = 0 need no layer and pass.
    c3_for_first: also apply C3 to request 1 (empty sum = 0); as printed the first request has no
    load limit, and the optimum then puts layers on the target that cannot be there yet."""
    n = len(T)
    S = [L - x for x in T]
    c1 = all(0 <= x <= L for x in T)
    c2 = all(sum(T[:i + 1]) <= sum(S[:i]) for i in range(1, n))
    assert c3_reading in ("printed", "first_layer_origin")
    c3 = True
    for i in range(0 if c3_for_first else 1, n):
        if T[i] == 0:
            continue
        lhs = time_l * T[i] if c3_reading == "printed" else time_l * (T[i] - 1)
        if lhs > sum(T[:i]) + (n - (i + 1) + 1) * (T[i] - 1) + 1e-12:
            c3 = False
    return c1, c2, c3


def program_objective(L: int, T: List[int]) -> float:
    """Average over requests of the sum of S over the request and all earlier ones."""
    S = [L - x for x in T]
    n = len(T)
    return sum(sum(S[:r + 1]) for r in range(n)) / n


def solve_program_bruteforce(L: int, n_requests: int, time_l: float, c3_reading: str = "first_layer_origin",
                             c3_for_first: bool = True):
    """Enumerates every configuration; returns (best objective, best T) under C1-C3, or None.
    Ties go to the configuration that comes first in lexicographic order."""
    best = None
    for T in itertools.product(range(0, L + 1), repeat=n_requests):
        c1, c2, c3 = program_constraints_hold(L, list(T), time_l, c3_reading, c3_for_first)
        if c1 and c2 and c3:
            obj = program_objective(L, list(T))
            if best is None or obj < best[0] - 1e-12:
                best = (obj, list(T))
    return best


def best_fixed_configuration(L: int, n_requests: int, load_time: float, source_free_at: float = 0.0):
    """True optimum among fixed configurations: every T executed by simulate_configuration, the one
    with the smallest average finish time returned as (average, T).  (L + 1) ** n_requests runs."""
    best = None
    for T in itertools.product(range(0, L + 1), repeat=n_requests):
        s = simulate_configuration(L, list(T), load_time, source_free_at)
        if best is None or s.avg_latency < best[0] - 1e-12:
            best = (s.avg_latency, list(T))
    return best
