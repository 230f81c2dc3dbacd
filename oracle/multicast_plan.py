"""CPU oracle for the scale-plan generator.  TEST INFRASTRUCTURE ONLY.

Section 5.1 of the paper: when a model has to be scaled onto new machines, a planner picks sources
that hold the parameters and spare targets, and emits serial forwarding chains
S -> T1 -> T2 -> ... along which the layers are pushed one after the other, every node forwarding
layer k while it receives layer k+1.  The paper's listing of the algorithm is a figure that is not
available; what the prose fixes is

  (a) the network model: machines joined by a scale-up fabric form one node whose internal transfers
      are free; a node's GPUs each have a link of some bandwidth to a leaf switch; two nodes under
      the same leaf talk at the smaller of their aggregated bandwidths, two nodes under different
      leaves at most at that, here divided by an oversubscription factor >= 1;
  (b) three greedy steps: prune sources whose outgoing direction already carries serving traffic;
      treat scale-up groups as units; form several chains, one per leaf that has both a source and
      targets so that no hop crosses leaves needlessly, ordered by decreasing link speed;
  (c) a source and a target that both hold k GPUs move 1/k of the bytes per GPU pair, so the hop
      runs at the aggregated bandwidth (the "parallel sharded transfer");
  (d) the tail of a chain (slowest link, forwards to nobody) is the natural live-scaling candidate.

Readings where the prose is silent (the exact listing cannot be checked: parity unpinned for
them; the pins below only cover what (a)-(d) and the figures' captions state):
  P1  if pruning removes every source, all sources are kept and the plan is marked `interferes`;
  P2  targets are chosen among spare nodes by (leaf has a usable source first, larger aggregated
      bandwidth first, lower id first);
  P3  inside a leaf that has usable sources and chosen targets, every usable source of the leaf
      roots a chain (more chains = more tails = more live-scaling candidates), strongest source
      first; the leaf's targets, strongest first, are dealt to those chains in turn;
  P4  a chosen target whose leaf has no usable source joins the chain rooted at the source that
      reaches it fastest (ties: fewer nodes in the chain so far, then lower root id); sources not
      yet rooting a chain count as empty chains;
  P5  inside a chain the targets are ordered by decreasing link speed from the root (ties: id);
  P6  time model: store-and-forward per layer,
        ready(k, l) = max(ready(k-1, l), ready(k, l-1)) + layer_bytes / bw(hop k),
      the root holding every layer at time 0.

Pins (tests/test_oracle_multicast_plan.py): equal links -> the last node of an n-node chain is
ready at |M|/B + (n-1)*layer/B, i.e. chain length costs one layer per hop, not one model (figure
"chain is friendly to broadcast", part a); a target reached twice as fast placed first halves its
own waiting time and a brute force over both orders confirms the greedy order (part b); four GPUs
on both ends cut the hop time to a quarter (figure "sharded parameter transfer"); two sources and
two targets give two chains and two tails where one chain gives one (figure "multiple chains");
a prefill-instance source whose outgoing link carries KV traffic is never a root while a
decode-instance source is (figure "pd-scale", part d); leaves that have their own source get no
inter-leaf hop; on tiny uniform topologies no assignment of the same targets to chains (brute force)
finishes earlier than the greedy plan.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence

SOURCE, SPARE, OTHER = 0, 1, 2


@dataclass(frozen=True)
class Node:
    id: int
    n_gpus: int
    gpu_bw: float          # bytes/s per GPU, each direction
    leaf: int
    role: int              # SOURCE, SPARE or OTHER
    out_busy: bool = False # its outgoing direction already carries serving traffic

    @property
    def agg_bw(self) -> float:
        return self.n_gpus * self.gpu_bw


@dataclass
class Plan:
    chains: List[List[int]]                 # node ids, root first
    hop_bw: List[List[float]]               # hop_bw[c][k]: bandwidth into chains[c][k+1]
    interferes: bool
    tails: List[int] = field(default_factory=list)


def link_bw(a: Node, b: Node, oversub: float) -> float:
    bw = min(a.agg_bw, b.agg_bw)
    return bw if a.leaf == b.leaf else bw / oversub


def generate(nodes: Sequence[Node], n_targets: int, oversub: float = 1.0) -> Plan:
    by_id: Dict[int, Node] = {n.id: n for n in nodes}
    sources = [n for n in nodes if n.role == SOURCE]
    if not sources:
        raise ValueError("no source holds the parameters")
    usable = [s for s in sources if not s.out_busy]
    interferes = False
    if not usable:
        usable, interferes = list(sources), True
    src_leaves = {s.leaf for s in usable}
    spare = sorted((n for n in nodes if n.role == SPARE),
                   key=lambda n: (0 if n.leaf in src_leaves else 1, -n.agg_bw, n.id))
    if n_targets < 1 or n_targets > len(spare):
        raise ValueError("not enough spare nodes")
    chosen = spare[:n_targets]

    members: Dict[int, List[int]] = {}      # root id -> target ids (unordered until the end)
    # leaves with their own sources: one chain per source of the leaf, targets dealt in turn
    for leaf in sorted(src_leaves):
        roots = sorted((s for s in usable if s.leaf == leaf), key=lambda n: (-n.agg_bw, n.id))
        local = sorted((t for t in chosen if t.leaf == leaf), key=lambda n: (-n.agg_bw, n.id))
        for i, t in enumerate(local):
            members.setdefault(roots[i % len(roots)].id, []).append(t.id)
    # the rest: fastest reachable root; fewer nodes; lower id
    rest = sorted((t for t in chosen if t.leaf not in src_leaves), key=lambda n: (-n.agg_bw, n.id))
    for t in rest:
        best = min(usable, key=lambda s: (-link_bw(s, t, oversub), len(members.get(s.id, [])), s.id))
        members.setdefault(best.id, []).append(t.id)

    chains, hops = [], []
    for root_id in sorted(members):
        root = by_id[root_id]
        order = sorted(members[root_id], key=lambda i: (-link_bw(root, by_id[i], oversub), i))
        chain = [root_id] + order
        chains.append(chain)
        hops.append([link_bw(by_id[chain[k]], by_id[chain[k + 1]], oversub) for k in range(len(chain) - 1)])
    return Plan(chains=chains, hop_bw=hops, interferes=interferes, tails=[c[-1] for c in chains])


def chain_ready_times(hop_bw: Sequence[float], n_layers: int, layer_bytes: float) -> List[float]:
    """Time at which each node after the root holds the whole model (reading P6)."""
    prev = [0.0] * n_layers                  # the root holds everything at time 0
    out = []
    for bw in hop_bw:
        cur, t = [], 0.0
        for l in range(n_layers):
            t = max(prev[l], t) + layer_bytes / bw
            cur.append(t)
        out.append(cur[-1])
        prev = cur
    return out


def plan_ready_times(plan: Plan, n_layers: int, layer_bytes: float) -> Dict[int, float]:
    out: Dict[int, float] = {}
    for chain, hops in zip(plan.chains, plan.hop_bw):
        for node, t in zip(chain[1:], chain_ready_times(hops, n_layers, layer_bytes)):
            out[node] = t
    return out
