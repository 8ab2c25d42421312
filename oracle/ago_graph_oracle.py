"""Plain-Python oracle of the graph frontend (TEST INFRASTRUCTURE, not product code).

Operator weight (Sec. IV-A, Eq. 1), topological stage and affix set (Sec. IV-B, the three
definitions before the theorem) and the greedy acyclic partition (Sec. IV-B, Algorithm "Graph
Partition", function Cluster), with the Split / Join steps of the reformer layer (Sec. V).  Written as
small set / dict manipulations over node ids; every step recomputes what it needs from scratch (no
incremental bookkeeping), so that it can be read against the paper.  Only tests may import this module.

Readings taken where the paper leaves a choice (the same ones the library documents):
  * log in Eq. 1 is the natural logarithm; an operator with no loops has weight b.
  * UC_v, "the nodes v can connect to in the underlying undirected graph", is read as v's neighbours
    (predecessors and successors), so a subgraph is always connected.
  * ties: the heaviest candidate with the lowest id is chosen; among affix nodes that satisfy the
    threshold the lightest with the lowest id is taken.  A hyper node's id is the smallest id it contains.
  * a node that was removed from the candidate set can still be absorbed by a later candidate.
  * "Update E, TopStage": the graph is contracted (parallel edges merged, the edge inside the pair
    dropped) and every topological stage is recomputed as a longest path on the contracted graph.
  * Split = Cluster on the sub-graph induced by one subgraph with the extra rule that a hyper node holds
    at most one complex operator; Join returns the parent subgraph of every mini-subgraph.
"""

import math


def op_weight(loop_extents, c, b):
    """Eq. 1: w_v = c * prod_{l in L_v} log(s_l) + b."""
    prod = 1.0
    for s in loop_extents:
        prod *= math.log(s)
    return c * prod + b if len(loop_extents) else b


def topological_stage(nodes, edges):
    """Definition "topological stage": length (in nodes) of the longest path from a root to v; roots are 1."""
    preds = {v: set() for v in nodes}
    for u, v in edges:
        preds[v].add(u)
    ts = {}

    def longest(v):
        if v not in ts:
            ts[v] = 1 + max((longest(u) for u in preds[v]), default=0)
        return ts[v]

    for v in nodes:
        longest(v)
    return ts


def affix_set(v, nodes, edges, ts):
    """Definition "affix set": neighbours of v whose stage differs from v's by exactly one."""
    nb = {b_ for a, b_ in edges if a == v} | {a for a, b_ in edges if b_ == v}
    return {u for u in nb if abs(ts[u] - ts[v]) == 1}


def cluster(n_nodes, weight, edges, td, is_complex=None, max_complex=0):
    """Function Cluster.  Returns subgraph_of[node] with subgraphs numbered by their smallest member."""
    members = {v: {v} for v in range(n_nodes)}          # hyper node id -> original nodes
    w = {v: float(weight[v]) for v in range(n_nodes)}
    ncomplex = {v: int(bool(is_complex[v])) if is_complex is not None else 0 for v in range(n_nodes)}
    E = {(u, v) for u, v in edges}
    cand = set(range(n_nodes))
    while cand:
        ts = topological_stage(list(members), E)
        v = min(cand, key=lambda x: (-w[x], x))
        ok = [u for u in affix_set(v, members, E, ts)
              if w[v] + w[u] < td and (max_complex <= 0 or ncomplex[v] + ncomplex[u] <= max_complex)]
        if not ok:
            cand.discard(v)
            continue
        u = min(ok, key=lambda x: (w[x], x))
        keep, gone = min(u, v), max(u, v)
        members[keep] |= members.pop(gone)
        w[keep] = w[u] + w[v]
        ncomplex[keep] = ncomplex[u] + ncomplex[v]
        del w[gone], ncomplex[gone]
        E = {(keep if a == gone else a, keep if b_ == gone else b_) for a, b_ in E}
        E = {(a, b_) for a, b_ in E if a != b_}
        cand.discard(u)
        cand.discard(v)
        cand.add(keep)
    out = [0] * n_nodes
    for sid, root in enumerate(sorted(members)):
        for m in members[root]:
            out[m] = sid
    return out


def split(n_nodes, weight, edges, subgraph_of, is_complex, td_mini):
    """Split every subgraph into mini-subgraphs with at most one complex operator each.  Returns
    (mini_of[node], parent_of_mini[mini])."""
    mini_of = [0] * n_nodes
    parent = []
    for sid in sorted(set(subgraph_of)):
        ids = [v for v in range(n_nodes) if subgraph_of[v] == sid]
        local = {v: i for i, v in enumerate(ids)}
        sub_edges = [(local[a], local[b_]) for a, b_ in edges if a in local and b_ in local]
        part = cluster(len(ids), [weight[v] for v in ids], sub_edges, td_mini,
                       [is_complex[v] for v in ids], 1)
        base = len(parent)
        for v in ids:
            mini_of[v] = base + part[local[v]]
        parent += [sid] * (max(part) + 1)
    return mini_of, parent


def join(mini_of, parent_of_mini):
    """Join: the subgraph every node returns to."""
    return [parent_of_mini[m] for m in mini_of]


# ---- checks used by the pins (definitions written out, exponential-time where simplest) -------------

def reachable(edges, n):
    """reach[u] = set of nodes with a directed path (length >= 1) from u; plain transitive closure."""
    reach = [set() for _ in range(n)]
    for u, v in edges:
        reach[u].add(v)
    changed = True
    while changed:
        changed = False
        for u in range(n):
            new = set()
            for v in reach[u]:
                new |= reach[v]
            if not new <= reach[u]:
                reach[u] |= new
                changed = True
    return reach


def is_acyclic_partition(n_nodes, edges, part):
    """Definition "n-way acyclic partition": no two parts i != j with a path from a node of i to a node of
    j and a path from a node of j to a node of i."""
    reach = reachable(edges, n_nodes)
    for u in range(n_nodes):
        for v in reach[u]:
            if part[u] == part[v]:
                continue
            for v2 in range(n_nodes):
                if part[v2] != part[v]:
                    continue
                if any(part[u2] == part[u] for u2 in reach[v2]):
                    return False
    return True
