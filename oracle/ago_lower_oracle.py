"""Plain-Python oracle of the lowering step (TEST INFRASTRUCTURE, not product code).

Which operators of a partitioned graph run as one fused launch: the structures that intensive fusion covers
(Sec. III-B, Sec. VI: pw -> dw -> pw, its two pairs, a general convolution under a general convolution,
matmul -> simple operators -> matmul) and sibling products that share an input (Sec. III).  The rule is this
build's own (the paper's tuner searches instead); it is written here a second time, independently of the
library: operator kinds become one-letter tokens, the structures are regular expressions over them, the side
conditions are spelled out per structure.  Only tests may import this module.

Graph form: parallel lists over the nodes in topological order -- ``ops`` (names), ``inputs`` (producer ids,
first operand first), ``attrs`` (a dict per node with what the rule looks at):
    dwconv   stride            conv3x3  channels          scale  alpha
    gemm     w_shape (K, N), rows (of its input)          bmm_nt head_dim
    to_heads heads, head_major
"""

import re

_TOKEN = {"conv1x1": "P", "dwconv": "D", "conv3x3": "C", "gemm": "G", "bmm_nt": "T", "bmm_nn": "N",
          "bias": "b", "relu": "r", "relu6": "6", "gelu_tanh": "g", "add": "+", "scale": "s", "softmax": "x",
          "input": "i", "to_heads": "h"}

# longest first; matched from the first operator of a chain
_STRUCTURES = [
    ("invres", re.compile(r"Pb?6Db?6Pb?\+?")),
    ("conv_chain", re.compile(r"Cb?rCb?\+?r")),
    ("ffn", re.compile(r"Gb?[gr6]Gb?")),
    ("attn", re.compile(r"TsxN")),
    ("pw_dw", re.compile(r"Pb?6Db?6")),
    ("dw_pw", re.compile(r"Db?6Pb?")),
]


def consumers(inputs):
    out = [[] for _ in inputs]
    for i, inp in enumerate(inputs):
        for src in inp:
            out[src].append(i)
    return out


def _side_conditions(ops, inputs, attrs, dtype, kind, ids):
    first_in = inputs[ids[0]][0]
    for k in ids:
        if ops[k] == "add":
            outside = [s for s in inputs[k] if s not in ids]
            if len(outside) != 1 or outside[0] != first_in:        # the residual is the block's own input
                return False
    if kind == "invres":
        has_add = any(ops[k] == "add" for k in ids)
        stride = [attrs[k].get("stride", 1) for k in ids if ops[k] == "dwconv"][0]
        return not has_add or stride == 1
    if kind == "conv_chain":
        return dtype == "bf16" and attrs[ids[0]]["channels"] == 64
    if kind == "ffn":
        return dtype == "bf16"
    if kind == "attn":
        t, sc, sm, nn = ids
        return (dtype == "bf16" and inputs[nn][0] == sm and inputs[sm][0] == sc and inputs[sc][0] == t
                and float(attrs[sc].get("alpha", 0.0)) > 0.0 and attrs[t]["head_dim"] in (64, 128))
    return True


def _sibling_projections(ops, inputs, attrs, dtype, cons, subgraph_of, done, i):
    if ops[i] != "gemm" or dtype != "bf16":
        return None
    src = inputs[i][0]
    sibs = [j for j in cons[src] if ops[j] == "gemm" and not done[j] and subgraph_of[j] == subgraph_of[i]]
    if len(sibs) != 3 or sibs[0] != i or len(cons[src]) != 3:
        return None
    chains = []
    for j in sibs:
        chain = [j]
        while len(cons[chain[-1]]) == 1:
            nx = cons[chain[-1]][0]
            if ops[nx] not in ("bias", "to_heads") or subgraph_of[nx] != subgraph_of[i]:
                break
            chain.append(nx)
            if ops[nx] == "to_heads":
                break
        chains.append(chain)
    forms = ["".join(_TOKEN[ops[k]] for k in c) for c in chains]
    if forms[0] not in ("Gh", "Gbh") or forms.count(forms[0]) != 3:
        return None
    w = [tuple(attrs[c[0]]["w_shape"]) for c in chains]
    views = [(attrs[c[-1]]["heads"], bool(attrs[c[-1]].get("head_major", True))) for c in chains]
    if w.count(w[0]) != 3 or views.count(views[0]) != 3:
        return None
    return sorted(k for c in chains for k in c)


def lower(ops, inputs, attrs, dtype, subgraph_of, ffn_pays=None):
    """[(kind, node ids)] in execution order.  ``ffn_pays(M, K, F, K2)``, when given, decides between the fused
    matmul chain ("ffn", True) and two products with fused epilogues ("ffn_epilogue", anything else)."""
    cons = consumers(inputs)
    n = len(ops)
    done = [False] * n
    plan = []
    for i in range(n):
        if done[i]:
            continue
        if ops[i] == "input":
            done[i] = True
            continue
        sib = _sibling_projections(ops, inputs, attrs, dtype, cons, subgraph_of, done, i)
        if sib is not None:
            plan.append(("qkv", sib))
            for k in sib:
                done[k] = True
            continue
        chain = [i]
        while True:
            last = chain[-1]
            if len(cons[last]) != 1:
                break
            j = cons[last][0]
            if done[j] or subgraph_of[j] != subgraph_of[i] or ops[j] == "input":
                break
            others = [s for s in inputs[j] if s != last]
            foreign = [o for o in others if o >= chain[0] and o not in chain]    # computed after the chain's start, not on it
            if ops[j] == "add":
                if len(others) != 1 or foreign:
                    break
            elif ops[j] in ("bmm_nt", "bmm_nn"):
                if foreign:
                    break
            elif others:
                break
            chain.append(j)
        tokens = "".join(_TOKEN[ops[k]] for k in chain)
        chosen = ("op", [i])
        for kind, pat in _STRUCTURES:
            m = pat.match(tokens)
            if m and "+" in m.group(0) and not _side_conditions(ops, inputs, attrs, dtype, kind, chain[:m.end()]):
                m = pat.match(tokens[:tokens.index("+")])              # the same structure without its residual
            if m and _side_conditions(ops, inputs, attrs, dtype, kind, chain[:m.end()]):
                ids = chain[:m.end()]
                if kind == "ffn" and ffn_pays is not None:
                    gemms = [k for k in ids if ops[k] == "gemm"]
                    (k_in, f_hid), (_, k_out) = attrs[gemms[0]]["w_shape"], attrs[gemms[1]]["w_shape"]
                    if ffn_pays(attrs[gemms[0]]["rows"], k_in, f_hid, k_out) is not True:
                        kind = "ffn_epilogue"
                chosen = (kind, ids)
                break
        plan.append(chosen)
        for k in chosen[1]:
            done[k] = True
    return plan
