"""Pins for the scheduling oracle (oracle/zigzag.py): the paper's worked example, structural
invariants of every schedule, limiting cases with closed forms, and the brute-force program."""
import os

import pytest

from oracle import zigzag as Z


def _golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "zigzag_example.txt")
    out = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            out[k] = [int(x) for x in v]
    return out


def test_paper_worked_example():
    g = _golden()
    L, load = g["layers"][0], g["load_time"][0]
    s = Z.simulate_zigzag(L, 7, load, source_free_at=1)       # the source picks request 1 after its first layer
    assert [s.T[0], s.S[0]] == g["request1_config"]
    assert [s.T[1], s.S[1]] == g["request2_config"]
    assert [s.T[2], s.S[2]] == g["request3_config"]
    assert s.finish[1] == g["requests_1_2_done_at"][0]
    assert s.finish[2] == g["request3_latency"][0]
    # best-effort keeps (1,6) for every batch dispatched before the second layer arrives
    b = Z.simulate_best_effort(L, 7, load, source_free_at=1)
    assert b.T[:6] == [1] * 6 and b.S[:6] == [6] * 6
    # the point of the example: the late request is served sooner under ZigZag
    assert s.finish[6] < b.finish[6] and s.avg_latency < b.avg_latency


def _check_schedule(s, L, n, load_time):
    per_req = {r: [] for r in range(n)}
    for sp in s.spans:
        assert sp.end > sp.start
        per_req[sp.request].append(sp)
        if sp.instance == "target":
            # no layer runs on the target before it is resident
            for k in range(sp.layer_a, sp.layer_b):
                t_k = sp.start + (k - sp.layer_a)
                assert load_time <= 0 or t_k >= k * load_time - 1e-9, (sp, k)
    for r, spans in per_req.items():
        spans.sort(key=lambda x: x.start)
        nxt, t = 0, 0.0
        for sp in spans:                         # every layer exactly once, in order, no overlap in time
            assert sp.layer_a == nxt and sp.start >= t - 1e-9
            nxt, t = sp.layer_b, sp.end
        assert nxt == L
        assert s.T[r] + s.S[r] == L              # constraint C1
        assert abs(s.finish[r] - t) < 1e-9
    for inst in ("target", "source"):            # an instance does one thing at a time
        spans = sorted([sp for sp in s.spans if sp.instance == inst], key=lambda x: x.start)
        for a, b in zip(spans, spans[1:]):
            assert b.start >= a.end - 1e-9
    src = sorted([sp for sp in s.spans if sp.instance == "source"], key=lambda x: x.start)
    assert [sp.request for sp in src] == sorted(sp.request for sp in src)     # FCFS on the source


@pytest.mark.parametrize("L,n,load,free", [(7, 7, 6, 1), (4, 3, 2, 0), (8, 10, 3, 5), (5, 6, 0.5, 2), (6, 4, 10, 0),
                                          (3, 8, 1, 1), (12, 5, 7, 30),
                                          # the source becomes free in the middle of a layer of the target
                                          (7, 5, 2, 1.5), (6, 6, 1, 0.25), (5, 4, 2.5, 3.75)])
def test_invariants(L, n, load, free):
    _check_schedule(Z.simulate_zigzag(L, n, load, free), L, n, load)
    _check_schedule(Z.simulate_best_effort(L, n, load, free), L, n, load)


def test_limits_with_closed_forms():
    # loading never progresses beyond layer 0 within the horizon and the source is free from time 1:
    # request r is taken by the source at 1 + r*(L-1) after exactly one layer on the target
    L, n = 5, 4
    s = Z.simulate_zigzag(L, n, 10 ** 6, source_free_at=1)
    assert s.T == [1] * n and s.finish == [1 + (r + 1) * (L - 1) for r in range(n)]
    # everything resident at once and the source busy for a long time: the target runs all layers of
    # request 0 first (FCFS), then request 1, ...; each request leaves at (r+1)*L
    s = Z.simulate_zigzag(L, n, 0, source_free_at=10 ** 6)
    assert s.T == [L] * n and s.S == [0] * n and s.finish == [(r + 1) * L for r in range(n)]
    # an idle source at time 0 takes the first request whole (nothing has run on the target yet)
    s = Z.simulate_zigzag(L, 2, 3, source_free_at=0)
    assert (s.T[0], s.S[0], s.finish[0]) == (0, L, L)
    # a source that becomes free while the target is inside layer 0 of the first request waits for that layer
    # to end (it may not run it a second time): it takes the request at time 1 with L - 1 layers left
    s = Z.simulate_zigzag(L, 1, 10 ** 6, source_free_at=0.5)
    assert (s.T[0], s.S[0], s.finish[0]) == (1, L - 1, L)
    # best-effort never puts more than half of the layers on the target
    b = Z.simulate_best_effort(8, 6, 0, source_free_at=0)
    assert b.T == [4] * 6


def test_program_objective_and_constraints_on_hand_cases():
    # L = 3, two requests, T = (1, 1): S = (2, 2); latencies 2 and 4 -> average 3
    assert Z.program_objective(3, [1, 1]) == 3.0
    # C2 for request 2: T1 + T2 <= S1  ->  2 <= 2 holds; with T = (1, 2): 3 <= 2 fails
    assert Z.program_constraints_hold(3, [1, 1], 0.0)[1] is True
    assert Z.program_constraints_hold(3, [1, 2], 0.0)[1] is False
    # C3 for request 2 with N = 2: time_l * T2 <= T1 + (N - 2 + 1) * (T2 - 1)
    assert Z.program_constraints_hold(3, [1, 1], 1.0)[2] is True       # 1 <= 1 + 0
    assert Z.program_constraints_hold(3, [1, 1], 1.5)[2] is False      # 1.5 <= 1 fails
    # brute force on a case small enough to enumerate by hand: L = 2, N = 2, time_l = 0.5.
    # C2 (request 2): 2*T1 + T2 <= 2;  C3 (request 2): 0.5*T2 <= T1 + (T2 - 1).
    #   (0,0): C3 0 <= -1 fails      (0,1): C3 0.5 <= 0 fails     (0,2): both hold, S = (2,0), latencies 2, 2 -> 2.0
    #   (1,0): both hold, S = (1,2), latencies 1, 3 -> 2.0        every other T breaks C2
    feasible = {(0, 2), (1, 0)}
    for t1 in range(3):
        for t2 in range(3):
            assert all(Z.program_constraints_hold(2, [t1, t2], 0.5)) == ((t1, t2) in feasible), (t1, t2)
    assert Z.program_objective(2, [0, 2]) == 2.0 and Z.program_objective(2, [1, 0]) == 2.0
    best = Z.solve_program_bruteforce(2, 2, 0.5)
    assert best is not None and best[0] == 2.0 and tuple(best[1]) in feasible
    # with time_l = 0, C3 becomes 0 <= T1 + T2 - 1 and (0,1) joins the feasible set
    best0 = Z.solve_program_bruteforce(2, 2, 0.0)
    # feasible now: (0,1) [S=(2,1): 2, 3 -> 2.5], (0,2) [2.0], (1,0) [2.0]; minimum still 2.0
    assert best0[0] == 2.0
