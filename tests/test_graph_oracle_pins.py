"""Pins for the graph-frontend oracle (Sec. IV: Eq. 1, topological stage, affix set, Cluster; Sec. V:
Split / Join): hand-worked small graphs, the definitions checked by brute force on seeded random DAGs,
and limiting cases with a known answer."""
import math
import random

import pytest

from oracle import ago_graph_oracle as G


def _random_dag(seed, n, p):
    r = random.Random(seed)
    order = list(range(n))
    r.shuffle(order)                       # ids are not in topological order
    edges = [(order[i], order[j]) for i in range(n) for j in range(i + 1, n) if r.random() < p]
    weight = [round(r.uniform(0.5, 4.0), 3) for _ in range(n)]
    cplx = [r.random() < 0.35 for _ in range(n)]
    return edges, weight, cplx


def _quotient_is_dag(n, edges, part):
    q = {(part[u], part[v]) for u, v in edges if part[u] != part[v]}
    k = max(part) + 1
    reach = G.reachable(sorted(q), k)
    return all(i not in reach[i] for i in range(k))


def _connected(ids, edges):
    ids = set(ids)
    seen, todo = set(), [min(ids)]
    while todo:
        v = todo.pop()
        if v in seen:
            continue
        seen.add(v)
        todo += [b for a, b in edges if a == v and b in ids] + [a for a, b in edges if b == v and a in ids]
    return seen == ids


def test_op_weight_eq1():
    # seven loops of a 2-d convolution, N=1 I=32 O=64 H=W=28 R=C=3: the batch loop has log(1) = 0
    assert G.op_weight([1, 32, 64, 28, 28, 3, 3], 2.0, 5.0) == 5.0
    ext = [32, 64, 28, 28, 3, 3]
    want = 2.0 * math.log(32) * math.log(64) * math.log(28) ** 2 * math.log(3) ** 2 + 5.0
    assert abs(G.op_weight(ext, 2.0, 5.0) - want) < 1e-12 * want
    assert abs(G.op_weight([math.e] * 4, 3.0, 1.5) - 4.5) < 1e-12        # every log is 1
    assert G.op_weight([], 3.0, 1.5) == 1.5
    assert G.op_weight([8, 8], 1.0, 0.0) < G.op_weight([8, 16], 1.0, 0.0)


def test_topological_stage_and_affix_set():
    # diamond with a shortcut: a->b, a->c, b->d, c->d, a->d
    edges = [(0, 1), (0, 2), (1, 3), (2, 3), (0, 3)]
    ts = G.topological_stage(range(4), edges)
    assert ts == {0: 1, 1: 2, 2: 2, 3: 3}                       # longest path, not shortest
    assert G.affix_set(0, range(4), edges, ts) == {1, 2}          # d is adjacent but two stages away
    assert G.affix_set(3, range(4), edges, ts) == {1, 2}
    assert G.affix_set(1, range(4), edges, ts) == {0, 3}          # c has the same stage: never affix
    ts = G.topological_stage(range(5), [(i, i + 1) for i in range(4)])
    assert [ts[i] for i in range(5)] == [1, 2, 3, 4, 5]
    # every edge goes up in stage
    edges, _, _ = _random_dag(3, 14, 0.25)
    ts = G.topological_stage(range(14), edges)
    assert all(ts[u] < ts[v] for u, v in edges)


def test_cluster_cyclic_dependency_example():
    """The situation of the paper's cyclic-dependency figure: conv1 -> conv2 -> conv3 and conv1 -> conv3.
    conv1 and conv3 alone may never form a subgraph (conv2 would depend on it and feed it)."""
    edges = [(0, 1), (1, 2), (0, 2)]
    assert G.is_acyclic_partition(3, edges, [0, 1, 0]) is False    # the forbidden grouping
    assert G.is_acyclic_partition(3, edges, [0, 0, 1]) and G.is_acyclic_partition(3, edges, [0, 1, 1])
    assert G.cluster(3, [3.0, 1.0, 3.0], edges, 100.0) == [0, 0, 0]
    # threshold admits one pair only: conv1 (heaviest, lowest id) takes its only affix node conv2
    assert G.cluster(3, [3.0, 1.0, 3.0], edges, 4.5) == [0, 0, 1]
    # nothing fits
    assert G.cluster(3, [3.0, 1.0, 3.0], edges, 4.0) == [0, 1, 2]


def test_cluster_chain_by_hand():
    # six unit weights in a chain, Td = 2.5: pairs (0,1) (2,3) (4,5), worked by hand from the greedy rule
    edges = [(i, i + 1) for i in range(5)]
    assert G.cluster(6, [1.0] * 6, edges, 2.5) == [0, 0, 1, 1, 2, 2]
    # heaviest first: node 3 (weight 2) takes its lightest affix node, 4 (0.2), then 2 (0.3); 1 (0.9) no longer fits
    assert G.cluster(6, [1.0, 0.9, 0.3, 2.0, 0.2, 1.0], edges, 3.0) == [0, 0, 1, 1, 1, 2]
    # strict inequality w_v + w_u < Td
    assert G.cluster(2, [1.0, 1.0], [(0, 1)], 2.0) == [0, 1]
    assert G.cluster(2, [1.0, 1.0], [(0, 1)], 2.0001) == [0, 0]


@pytest.mark.parametrize("seed", range(12))
def test_cluster_properties_on_random_dags(seed):
    n = 10 + seed
    edges, weight, _ = _random_dag(100 + seed, n, 0.22)
    for td in (3.0, 6.0, 12.0):
        part = G.cluster(n, weight, edges, td)
        assert sorted(set(part)) == list(range(max(part) + 1))
        assert G.is_acyclic_partition(n, edges, part)
        assert _quotient_is_dag(n, edges, part)
        for sid in set(part):
            ids = [v for v in range(n) if part[v] == sid]
            assert len(ids) == 1 or sum(weight[v] for v in ids) < td
            assert _connected(ids, edges)
    # no threshold: one subgraph per connected component
    part = G.cluster(n, weight, edges, float("inf"))
    for sid in set(part):
        ids = {v for v in range(n) if part[v] == sid}
        assert _connected(ids, edges)
        assert not any((a in ids) != (b in ids) for a, b in edges)
    # threshold below every pair: nothing merges
    assert G.cluster(n, weight, edges, 1.0) == list(range(n))


@pytest.mark.parametrize("seed", range(6))
def test_split_and_join(seed):
    n = 16
    edges, weight, cplx = _random_dag(200 + seed, n, 0.25)
    part = G.cluster(n, weight, edges, 15.0)
    mini, parent = G.split(n, weight, edges, part, cplx, 6.0)
    assert G.join(mini, parent) == part                          # Join undoes Split
    for m in set(mini):
        ids = [v for v in range(n) if mini[v] == m]
        assert sum(cplx[v] for v in ids) <= 1                    # at most one complex operator
        assert len({part[v] for v in ids}) == 1                  # a mini-subgraph stays inside its subgraph
    assert G.is_acyclic_partition(n, edges, mini)
