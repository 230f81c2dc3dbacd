"""Pins for the scale-plan oracle (section 5.1): what the prose and the figure captions state, closed
forms of the layer-pipelined chain, and brute force over all plans on tiny topologies."""
import itertools

import pytest

from oracle import multicast_plan as P

GB = 1e9


def _node(i, role, *, gpus=1, bw=25 * GB, leaf=0, busy=False):
    return P.Node(id=i, n_gpus=gpus, gpu_bw=bw, leaf=leaf, role=role, out_busy=busy)


def test_chain_length_costs_one_layer_per_hop_not_one_model():
    # figure "chain is friendly to broadcast", part (a): with equal links the transfer time is
    # |M|/B plus one layer per extra hop, whatever the number of instances
    L, layer, B = 32, 0.4 * GB, 25 * GB
    for n in (1, 2, 5, 9):
        ready = P.chain_ready_times([B] * n, L, layer)
        for k, t in enumerate(ready):
            assert t == pytest.approx((L + k) * layer / B, rel=1e-12)
        assert ready[-1] - L * layer / B == pytest.approx((n - 1) * layer / B, rel=1e-9)


def test_slowest_hop_bounds_the_chain():
    L, layer = 16, 1.0 * GB
    ready = P.chain_ready_times([50 * GB, 10 * GB, 50 * GB], L, layer)
    # after the slow hop every layer arrives at the slow rate; the fast hop behind it adds one layer
    assert ready[1] == pytest.approx(layer / (50 * GB) + L * layer / (10 * GB), rel=1e-12)
    assert ready[2] == pytest.approx(ready[1] + layer / (50 * GB), rel=1e-12)


def test_faster_target_first_halves_its_waiting_time():
    # part (b) of the same figure: S reaches T2 twice as fast as T1
    S = _node(0, P.SOURCE, bw=50 * GB)
    T1 = _node(1, P.SPARE, bw=25 * GB)
    T2 = _node(2, P.SPARE, bw=50 * GB)
    plan = P.generate([S, T1, T2], 2)
    assert plan.chains == [[0, 2, 1]]
    L, layer = 40, 0.5 * GB
    ready = P.plan_ready_times(plan, L, layer)
    by = {n.id: n for n in (S, T1, T2)}
    other = P.chain_ready_times([P.link_bw(S, T1, 1.0), P.link_bw(T1, T2, 1.0)], L, layer)   # S -> T1 -> T2
    assert ready[2] == pytest.approx(L * layer / (50 * GB))
    assert ready[2] == pytest.approx(other[1] / 2, rel=0.03)          # half, up to one layer of pipeline fill
    # brute force over both orders: the greedy order has the smaller total waiting time
    totals = {}
    for order in itertools.permutations([1, 2]):
        chain = [0, *order]
        hops = [P.link_bw(by[chain[k]], by[chain[k + 1]], 1.0) for k in range(2)]
        totals[order] = sum(P.chain_ready_times(hops, L, layer))
    assert min(totals, key=totals.get) == (2, 1)


def test_sharded_transfer_between_four_gpu_nodes_takes_a_quarter():
    L, layer = 32, 0.4 * GB
    one = P.generate([_node(0, P.SOURCE), _node(1, P.SPARE)], 1)
    four = P.generate([_node(0, P.SOURCE, gpus=4), _node(1, P.SPARE, gpus=4)], 1)
    t1 = P.plan_ready_times(one, L, layer)[1]
    t4 = P.plan_ready_times(four, L, layer)[1]
    assert t4 == pytest.approx(t1 / 4, rel=1e-12)
    # the narrower side decides
    mixed = P.generate([_node(0, P.SOURCE, gpus=2), _node(1, P.SPARE, gpus=4)], 1)
    assert P.plan_ready_times(mixed, L, layer)[1] == pytest.approx(t1 / 2, rel=1e-12)


def test_two_sources_give_two_chains_and_two_live_candidates():
    # figure "multiple chains": with one source only the tail can scale live; with two both can
    one = P.generate([_node(0, P.SOURCE), _node(2, P.SPARE), _node(3, P.SPARE)], 2)
    two = P.generate([_node(0, P.SOURCE), _node(1, P.SOURCE), _node(2, P.SPARE), _node(3, P.SPARE)], 2)
    assert len(one.chains) == 1 and len(one.tails) == 1
    assert sorted(map(len, two.chains)) == [2, 2] and sorted(two.tails) == [2, 3]


def test_source_with_busy_outgoing_link_is_pruned():
    # figure "pd-scale": the prefill instance streams KV cache out, the decode instance only receives
    prefill = _node(0, P.SOURCE, busy=True)
    decode = _node(1, P.SOURCE)
    plan = P.generate([prefill, decode, _node(2, P.SPARE), _node(3, P.SPARE)], 2)
    assert [c[0] for c in plan.chains] == [1] and not plan.interferes
    # nothing else to load from: the plan still exists but says that it interferes
    forced = P.generate([prefill, _node(2, P.SPARE)], 1)
    assert forced.chains == [[0, 2]] and forced.interferes


def test_leaves_with_their_own_source_get_no_inter_leaf_hop():
    nodes = [_node(0, P.SOURCE, leaf=0), _node(1, P.SOURCE, leaf=1),
             _node(2, P.SPARE, leaf=0), _node(3, P.SPARE, leaf=1), _node(4, P.SPARE, leaf=0),
             _node(5, P.SPARE, leaf=2)]
    plan = P.generate(nodes, 3, oversub=4.0)
    leaf = {n.id: n.leaf for n in nodes}
    for chain in plan.chains:
        assert all(leaf[i] == leaf[chain[0]] for i in chain[1:])
    assert sorted(i for c in plan.chains for i in c[1:]) == [2, 3, 4]      # the leaf-2 node is chosen last
    # when it has to be used it hangs off some source across the spine at 1/oversub of the link
    plan4 = P.generate(nodes, 4, oversub=4.0)
    hop = {c[k + 1]: b for c, hops in zip(plan4.chains, plan4.hop_bw) for k, b in enumerate(hops)}
    assert hop[5] == pytest.approx(25 * GB / 4)


def test_every_chosen_target_appears_once_and_hops_match_the_model():
    nodes = [_node(0, P.SOURCE, gpus=8, leaf=0), _node(1, P.SOURCE, gpus=4, leaf=1, busy=True),
             _node(2, P.OTHER, leaf=0)] + [_node(3 + i, P.SPARE, gpus=1 + i % 4, bw=(10 + 5 * (i % 3)) * GB, leaf=i % 3)
                                            for i in range(9)]
    by = {n.id: n for n in nodes}
    for n in range(1, 10):
        plan = P.generate(nodes, n, oversub=2.0)
        seen = [i for c in plan.chains for i in c[1:]]
        assert len(seen) == n == len(set(seen))
        for chain, hops in zip(plan.chains, plan.hop_bw):
            assert by[chain[0]].role == P.SOURCE and not by[chain[0]].out_busy
            assert hops == [P.link_bw(by[chain[k]], by[chain[k + 1]], 2.0) for k in range(len(chain) - 1)]
            speeds = [P.link_bw(by[chain[0]], by[i], 2.0) for i in chain[1:]]
            assert speeds == sorted(speeds, reverse=True)
    with pytest.raises(ValueError):
        P.generate(nodes, 10)
    with pytest.raises(ValueError):
        P.generate([n for n in nodes if n.role != P.SOURCE], 1)


def _all_plans(roots, targets):
    """Every way to hang the targets, in some order, under the roots."""
    for assign in itertools.product(range(len(roots)), repeat=len(targets)):
        groups = [[t for t, a in zip(targets, assign) if a == r] for r in range(len(roots))]
        for orders in itertools.product(*[list(itertools.permutations(g)) for g in groups]):
            yield [[roots[r], *orders[r]] for r in range(len(roots)) if orders[r]]


@pytest.mark.parametrize("n_src,n_tgt", [(1, 1), (1, 3), (2, 2), (2, 3), (2, 4), (3, 4)])
def test_no_plan_finishes_earlier_on_uniform_topologies(n_src, n_tgt):
    L, layer = 8, 1.0 * GB
    nodes = [_node(i, P.SOURCE) for i in range(n_src)] + [_node(10 + i, P.SPARE) for i in range(n_tgt)]
    by = {n.id: n for n in nodes}
    plan = P.generate(nodes, n_tgt)
    greedy = max(P.plan_ready_times(plan, L, layer).values())
    best = min(
        max(max(P.chain_ready_times([P.link_bw(by[c[k]], by[c[k + 1]], 1.0) for k in range(len(c) - 1)], L, layer))
            for c in chains)
        for chains in _all_plans(list(range(n_src)), [10 + i for i in range(n_tgt)]))
    assert greedy == pytest.approx(best, rel=1e-12)


def _finish(by, chains, L, layer, oversub):
    return max(max(P.chain_ready_times([P.link_bw(by[c[k]], by[c[k + 1]], oversub) for k in range(len(c) - 1)], L, layer))
               for c in chains)


def test_spare_with_the_faster_link_is_chosen_when_fewer_targets_than_spares():
    # two spares under the source's leaf, one target wanted: of the two single-hop plans the one to the
    # spare with the faster link is ready first, and that is the plan generated
    L, layer = 16, 0.5 * GB
    nodes = [_node(0, P.SOURCE, gpus=4), _node(1, P.SPARE, gpus=1), _node(2, P.SPARE, gpus=4), _node(3, P.SPARE, gpus=2)]
    by = {n.id: n for n in nodes}
    times = {t: _finish(by, [[0, t]], L, layer, 1.0) for t in (1, 2, 3)}
    plan = P.generate(nodes, 1)
    assert plan.chains == [[0, min(times, key=times.get)]] == [[0, 2]]
    # with two wanted, the slowest spare stays out
    assert sorted(P.generate(nodes, 2).chains[0][1:]) == [2, 3]


def test_target_on_a_leaf_without_sources_hangs_off_the_root_that_reaches_it_fastest():
    # sources on leaves 0 and 1 (one GPU and four GPUs), a four-GPU target on leaf 2: across the spine the
    # four-GPU source reaches it four times as fast, and brute force over both roots agrees
    L, layer, over = 16, 0.5 * GB, 2.0
    nodes = [_node(0, P.SOURCE, gpus=1, leaf=0), _node(1, P.SOURCE, gpus=4, leaf=1), _node(2, P.SPARE, gpus=4, leaf=2)]
    by = {n.id: n for n in nodes}
    times = {r: _finish(by, [[r, 2]], L, layer, over) for r in (0, 1)}
    assert times[1] == pytest.approx(times[0] / 4)
    plan = P.generate(nodes, 1, oversub=over)
    assert plan.chains == [[1, 2]]
    assert plan.hop_bw == [[4 * 25 * GB / over]]


def test_equal_roots_share_remote_targets_instead_of_stacking_them_on_one_chain():
    # two equal sources, two equal targets on leaves of their own: one target per root finishes one layer
    # time earlier than both on one chain, and gives two tails (two live-scaling candidates)
    L, layer, over = 8, 1.0 * GB, 2.0
    nodes = [_node(0, P.SOURCE, leaf=0), _node(1, P.SOURCE, leaf=1), _node(2, P.SPARE, leaf=2), _node(3, P.SPARE, leaf=3)]
    by = {n.id: n for n in nodes}
    plan = P.generate(nodes, 2, oversub=over)
    assert plan.chains == [[0, 2], [1, 3]] and plan.tails == [2, 3]
    best = min(_finish(by, chains, L, layer, over) for chains in _all_plans([0, 1], [2, 3]))
    stacked = _finish(by, [[0, 2, 3]], L, layer, over)
    mine = max(P.plan_ready_times(plan, L, layer).values())
    assert mine == pytest.approx(best, rel=1e-12)
    assert stacked - mine == pytest.approx(layer / (25 * GB / over), rel=1e-9)
