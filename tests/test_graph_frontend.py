"""The library's graph frontend (host only, through the C ABI) against the plain-Python oracle:
bit-exact partitions on seeded random DAGs and on an operator graph shaped like the networks the
kernels come from, plus argument validation."""
import math
import random

import pytest

from oracle import ago_graph_oracle as G
from paper_2212_01005_amd import binding as ago


def _random_dag(seed, n, p):
    r = random.Random(seed)
    order = list(range(n))
    r.shuffle(order)
    edges = [(order[i], order[j]) for i in range(n) for j in range(i + 1, n) if r.random() < p]
    weight = [round(r.uniform(0.5, 4.0), 3) for _ in range(n)]
    # equal weights on purpose now and then: the tie rules must agree too
    for i in range(0, n, 3):
        weight[i] = 2.0
    cplx = [r.random() < 0.35 for _ in range(n)]
    return edges, weight, cplx


def test_op_weight_matches_eq1():
    for ext in ([1, 32, 64, 28, 28, 3, 3], [32, 64, 28, 28, 3, 3], [7], [2048, 768, 3072], []):
        assert ago.graph_op_weight(ext, 1.7, 0.4) == pytest.approx(G.op_weight(ext, 1.7, 0.4), rel=1e-15, abs=0)
    assert math.isnan(ago.graph_op_weight([4, 0], 1.0, 0.0))


@pytest.mark.parametrize("seed", range(20))
def test_cluster_split_join_match_the_oracle(seed):
    n = 6 + 2 * seed
    edges, weight, cplx = _random_dag(300 + seed, n, 0.2)
    ts = G.topological_stage(range(n), edges)
    assert ago.graph_topological_stage(n, edges) == [ts[v] for v in range(n)]
    for td in (2.0, 4.5, 9.0, 30.0, float("inf")):
        part = ago.graph_cluster(n, weight, edges, td)
        assert part == G.cluster(n, weight, edges, td)
        assert G.is_acyclic_partition(n, edges, part)
        capped = ago.graph_cluster(n, weight, edges, td, cplx, 2)
        assert capped == G.cluster(n, weight, edges, td, cplx, 2)
        mini, parent = ago.graph_split(n, weight, edges, part, cplx, td / 2)
        assert (mini, parent) == G.split(n, weight, edges, part, cplx, td / 2)
        assert ago.graph_join(mini, parent) == part


def _mobile_block_graph(blocks):
    """Operator graph of `blocks` inverted-residual blocks in a row: pw, bias, relu6, dw, bias, relu6, pw,
    bias, (add with the block input).  Returns (n, edges, loop extents per node, is_complex)."""
    edges, loops, cplx = [], [], []

    def node(ext, complex_):
        loops.append(ext)
        cplx.append(complex_)
        return len(loops) - 1

    prev = node([1, 32, 14, 14], False)                      # the input tensor's producer (a simple op)
    for _ in range(blocks):
        src = prev
        chain = [node([1, 192, 14, 14, 32], True), node([1, 192, 14, 14], False), node([1, 192, 14, 14], False),
                 node([1, 192, 14, 14, 3, 3], True), node([1, 192, 14, 14], False), node([1, 192, 14, 14], False),
                 node([1, 32, 14, 14, 192], True), node([1, 32, 14, 14], False)]
        for a, b in zip([src] + chain[:-1], chain):
            edges.append((a, b))
        add = node([1, 32, 14, 14], False)
        edges += [(chain[-1], add), (src, add)]
        prev = add
    return len(loops), edges, loops, cplx


def test_partition_of_a_mobile_network_prefix():
    """With Eq. 1 weights the partitioner groups operators of the inverted-residual chain into subgraphs
    that hold several complex operators (what the fused block kernel runs), stays acyclic in the presence
    of the residual edges, and Split leaves at most one complex operator per mini-subgraph."""
    n, edges, loops, cplx = _mobile_block_graph(3)
    c, b = 0.01, 1.0
    weight = [ago.graph_op_weight(ext, c, b) for ext in loops]
    assert weight == [pytest.approx(G.op_weight(ext, c, b), rel=1e-15) for ext in loops]
    block_weight = sum(weight[1:10])
    part = ago.graph_cluster(n, weight, edges, 1.2 * block_weight)
    assert part == G.cluster(n, weight, edges, 1.2 * block_weight)
    assert G.is_acyclic_partition(n, edges, part)
    per_sub = {}
    for v in range(n):
        per_sub[part[v]] = per_sub.get(part[v], 0) + int(cplx[v])
    assert max(per_sub.values()) >= 2                          # intensive fusion candidates exist
    mini, parent = ago.graph_split(n, weight, edges, part, cplx, 0.6 * block_weight)
    for m in set(mini):
        assert sum(cplx[v] for v in range(n) if mini[v] == m) <= 1
    assert ago.graph_join(mini, parent) == part


def test_graph_calls_validate_their_arguments():
    with pytest.raises(ago.AgoError):
        ago.graph_cluster(3, [1.0, 1.0, 1.0], [(0, 1), (1, 2), (2, 0)], 10.0)      # cyclic edges
    with pytest.raises(ago.AgoError):
        ago.graph_cluster(3, [1.0, 1.0, 1.0], [(0, 3)], 10.0)                      # node id out of range
    with pytest.raises(ago.AgoError):
        ago.graph_cluster(2, [1.0, -1.0], [(0, 1)], 10.0)                          # negative weight
    with pytest.raises(ago.AgoError):
        ago.graph_cluster(2, [1.0, float("nan")], [(0, 1)], 10.0)
    with pytest.raises(ago.AgoError):
        ago.graph_topological_stage(2, [(1, 1)])                                   # self-loop
    with pytest.raises(ago.AgoError):
        ago.graph_join([0, 5], [0])                                                # mini id out of range
    assert ago.graph_cluster(1, [1.0], [], 10.0) == [0]
    assert ago.graph_cluster(4, [1.0] * 4, [], 10.0) == [0, 1, 2, 3]               # no edges: nothing to merge
