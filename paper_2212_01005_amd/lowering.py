"""From an operator graph to fused-kernel launches (AGO Sec. IV -> Sec. III-B).

The graph frontend of the library decides which operators form one subgraph (``ago_graph_cluster``: Eq. 1
weights, acyclic Cluster) and which operator chains inside each subgraph become one fused launch
(``ago_graph_lower``: the structures of Sec. III-B and VI: pw -> dw -> pw, the pw / dw pairs, 3x3 -> 3x3,
matmul -> activation -> matmul, matmul -> scale -> softmax -> matmul, sibling projections); whatever is left runs
operator by operator on the un-fused kernels.  This module holds the graph form, marshals it for those two calls
and executes the resulting plan: only host-side bookkeeping, every decision and every tensor operation is a call
into the library.

Graph form: ``Graph.nodes`` is a list in topological order; node i is ``Node(op, inputs, attrs)`` with
``inputs`` = ids of producer nodes.  Operators and their attributes:

    input                      a tensor supplied at run time (attrs: name, shape)
    conv1x1  (w)               x:[N,H,W,Cin]  w:[Cin,Cout]
    dwconv   (w, stride)       w:[k,k,C], k = 3 or 5, zero padding (k-1)/2
    conv3x3  (w)               w:[3,3,C,C]
    gemm     (w)               x:[M,K]  w:[K,N]
    bmm_nt / bmm_nn            two inputs, batched over the leading dimensions
    bias (b) relu relu6 gelu_tanh add(two inputs) scale (alpha) softmax
    to_heads (batch, heads, head_major)   [B*S, Hh*D] viewed as [B,S,Hh,D], transposed to [B,Hh,S,D] if head_major

Weights / biases are named entries of ``Graph.params``.
"""

from dataclasses import dataclass, field

COMPLEX = {"conv1x1", "dwconv", "conv3x3", "gemm", "bmm_nt", "bmm_nn"}


@dataclass
class Node:
    op: str
    inputs: list
    attrs: dict = field(default_factory=dict)


@dataclass
class Graph:
    nodes: list
    params: dict
    dtype: str = "bf16"

    def add(self, op, inputs=(), **attrs):
        self.nodes.append(Node(op, list(inputs), attrs))
        return len(self.nodes) - 1

    def edges(self):
        return [(src, i) for i, n in enumerate(self.nodes) for src in n.inputs]

    def consumers(self):
        out = [[] for _ in self.nodes]
        for i, n in enumerate(self.nodes):
            for src in n.inputs:
                out[src].append(i)
        return out


def infer_shapes(g):
    """Output shape of every node (NHWC / row-major conventions of the library)."""
    shapes = []
    for n in g.nodes:
        s_in = [shapes[i] for i in n.inputs]
        if n.op == "input":
            s = tuple(n.attrs["shape"])
        elif n.op == "conv1x1":
            s = s_in[0][:-1] + (g.params[n.attrs["w"]].shape[1],)
        elif n.op == "dwconv":
            st = n.attrs.get("stride", 1)
            nb, h, w, c = s_in[0]
            s = (nb, (h - 1) // st + 1, (w - 1) // st + 1, c)
        elif n.op == "gemm":
            s = s_in[0][:-1] + (g.params[n.attrs["w"]].shape[1],)
        elif n.op == "to_heads":            # [B*S, Hh*D] -> [B, Hh, S, D] (head_major) or [B, S, Hh, D]
            rows, cols = s_in[0]
            b_, hh = n.attrs["batch"], n.attrs["heads"]
            s = (b_, hh, rows // b_, cols // hh) if n.attrs.get("head_major", True) else (b_, rows // b_, hh, cols // hh)
        elif n.op == "bmm_nt":
            s = s_in[0][:-1] + (s_in[1][-2],)
        elif n.op == "bmm_nn":
            s = s_in[0][:-1] + (s_in[1][-1],)
        else:                       # conv3x3 (C -> C, stride 1) and the simple operators keep the shape
            s = s_in[0]
        shapes.append(tuple(int(v) for v in s))
    return shapes


def loop_extents(g, shapes, i):
    """Extents of the loop nest of operator i (Sec. IV-A: the weight follows the loop nest)."""
    n, out = g.nodes[i], shapes[i]
    if n.op == "conv1x1" or n.op == "gemm":
        return list(out) + [g.params[n.attrs["w"]].shape[0]]
    if n.op == "dwconv":
        k = g.params[n.attrs["w"]].shape[0]
        return list(out) + [k, k]
    if n.op == "conv3x3":
        return list(out) + [out[-1], 3, 3]
    if n.op == "bmm_nt" or n.op == "bmm_nn":
        return list(out) + [shapes[n.inputs[0]][-1]]
    return list(out)


def partition(g, binding, c=0.01, b=1.0, td=float("inf")):
    """Eq. 1 weights and Cluster through the library; returns (subgraph_of, weights)."""
    shapes = infer_shapes(g)
    weight = [binding.graph_op_weight(loop_extents(g, shapes, i), c, b) for i in range(len(g.nodes))]
    return binding.graph_cluster(len(g.nodes), weight, g.edges(), td), weight


def node_attributes(g, shapes):
    """What the library's lowering needs to know about every node beyond its kind (``ago_graph_lower``)."""
    attr, attr_f = [], []
    for n in g.nodes:
        a, f = [0, 0, 0, 0], 0.0
        if n.op == "dwconv":
            a[0] = int(n.attrs.get("stride", 1))
        elif n.op == "conv3x3":
            a[0] = int(g.params[n.attrs["w"]].shape[2])
        elif n.op == "gemm":
            rows = 1
            for d in shapes[n.inputs[0]][:-1]:
                rows *= int(d)
            a[0], a[1], a[2] = int(g.params[n.attrs["w"]].shape[0]), int(g.params[n.attrs["w"]].shape[1]), rows
        elif n.op == "bmm_nt":
            a[0] = int(shapes[n.inputs[0]][-1])
        elif n.op == "to_heads":
            a[0], a[1] = int(n.attrs["heads"]), 1 if n.attrs.get("head_major", True) else 0
        elif n.op == "scale":
            f = float(n.attrs.get("alpha", 0.0))
        attr.append(a)
        attr_f.append(f)
    return attr, attr_f


def lower(g, subgraph_of, binding=None):
    """Launch plan: a list of (kind, node ids) in execution order, made by the library (``ago_graph_lower``:
    the structures, the chain rule and the admissibility checks are documented with its declaration).  kind is
    one of the fused structures ("invres", "conv_chain", "ffn", "attn", "pw_dw", "dw_pw", "qkv"), "ffn_epilogue"
    (the matmul -> activation -> matmul chain as two products with fused epilogues: what the chain becomes when
    the library's fuse-or-not decision says the fused kernel would lose at this row count; asked for only when
    ``binding`` is given, otherwise the chain is always fused) or "op" (one operator on its un-fused kernel);
    "input" nodes launch nothing.  This function only marshals the graph."""
    from . import binding as _ago
    shapes = infer_shapes(g)
    attr, attr_f = node_attributes(g, shapes)
    return _ago.graph_lower([n.op for n in g.nodes], [n.inputs for n in g.nodes], attr, attr_f, subgraph_of,
                            _ago.BF16 if g.dtype == "bf16" else _ago.F32, binding is not None)


# ---- execution (GPU) ---------------------------------------------------------------------------------

_ACT_OF = {"relu": "ACT_RELU", "relu6": "ACT_RELU6", "gelu_tanh": "ACT_GELU_TANH"}


class Executor:
    """Runs a launch plan with the library's kernels.  ``params`` are device tensors (weights in the graph's
    storage dtype, biases fp32); ``run(inputs)`` returns the tensor of every node that has no consumer."""

    def __init__(self, g, plan, binding, torch, device="cuda:0", pack_weights=False):
        """pack_weights: the weights of a graph are constants, so the matrix products that have a kernel for it
        get their weights re-laid out once (``ago_pack_weight``, on the first ``run``) into matrix-instruction
        fragments and run on the packed kernels from then on: the data-layout choice the paper's tuner makes at
        compile time (Sec. III), here with one fixed alternative layout."""
        self.g, self.plan, self.ago, self.torch, self.device = g, plan, binding, torch, device
        self.shapes = infer_shapes(g)
        self.td = torch.bfloat16 if g.dtype == "bf16" else torch.float32
        self.launches = 0
        self.pack_weights = bool(pack_weights) and g.dtype == "bf16"
        self.packed = {}                   # parameter name -> packed copy

    def _packed(self, name):
        """The packed copy of weight `name`, made on first use."""
        if name not in self.packed:
            w = self.g.params[name]
            wp = self.torch.empty(self.ago.packed_weight_shape(w.shape[0], w.shape[1]), dtype=w.dtype, device=self.device)
            self.ago.ago_pack_weight(w, wp)
            self.packed[name] = wp
        return self.packed[name]

    def _new(self, i):
        return self.torch.empty(self.shapes[i], dtype=self.td, device=self.device)

    def _workspace(self, op, dims, dt):
        """Scratch the library asks for (cross-workgroup partial results), or None."""
        nbytes = self.ago.workspace_bytes(op, [int(d) for d in dims], dt)
        return self.torch.empty(max(nbytes, 16), dtype=self.torch.uint8, device=self.device) if nbytes else None

    def _bias_of(self, nodes, after):
        """The bias that directly follows position `after` in a matched chain, or None."""
        if after + 1 < len(nodes) and nodes[after + 1].op == "bias":
            return self.g.params[nodes[after + 1].attrs["b"]]
        return None

    def run(self, inputs):
        g, ago, P, val = self.g, self.ago, self.g.params, {}
        for i, n in enumerate(g.nodes):
            if n.op == "input":
                val[i] = inputs[n.attrs["name"]]
        for kind, ids in self.plan:
            nodes = [g.nodes[k] for k in ids]
            x = val[nodes[0].inputs[0]]
            self.launches += 1
            if kind == "qkv":
                ends = [k for k in ids if g.nodes[k].op == "to_heads"]
                gemms = [k for k in ids if g.nodes[k].op == "gemm"]
                biases = [next((P[g.nodes[b_].attrs["b"]] for b_ in ids if g.nodes[b_].op == "bias" and g.nodes[b_].inputs[0] == gm), None)
                          for gm in gemms]
                outs = [self._new(e) for e in ends]
                ago.ago_fused_qkv(x, *(P[g.nodes[gm].attrs["w"]] for gm in gemms), *biases, *outs,
                                  head_major=g.nodes[ends[0]].attrs.get("head_major", True))
                for e, o in zip(ends, outs):
                    val[e] = o
                continue
            out = self._new(ids[-1])
            if kind == "invres":
                pos = [k for k, n in enumerate(nodes) if n.op in COMPLEX]
                w1, wd, w2 = (P[nodes[p].attrs["w"]] for p in pos)
                residual = any(n.op == "add" for n in nodes)
                stride = nodes[pos[1]].attrs.get("stride", 1)
                fn = ago.ago_fused_invres if wd.shape[0] == 3 else ago.ago_fused_invres_k
                dt = ago.BF16 if x.dtype == self.torch.bfloat16 else ago.F32
                ws = self._workspace(ago.OP_FUSED_INVRES, list(x.shape) + [w1.shape[1], w2.shape[1], stride, wd.shape[0]], dt)
                fn(x, w1, self._bias_of(nodes, pos[0]), wd, self._bias_of(nodes, pos[1]), w2,
                   self._bias_of(nodes, pos[2]), out, stride, residual, ws)
            elif kind == "pw_dw":
                pos = [k for k, n in enumerate(nodes) if n.op in COMPLEX]
                wd = P[nodes[pos[1]].attrs["w"]]
                fn = ago.ago_fused_pw_dw if wd.shape[0] == 3 else ago.ago_fused_pw_dw_k
                fn(x, P[nodes[pos[0]].attrs["w"]], self._bias_of(nodes, pos[0]), wd, self._bias_of(nodes, pos[1]), out,
                   nodes[pos[1]].attrs.get("stride", 1))
            elif kind == "dw_pw":
                pos = [k for k, n in enumerate(nodes) if n.op in COMPLEX]
                dt = ago.BF16 if x.dtype == self.torch.bfloat16 else ago.F32
                w2 = P[nodes[pos[1]].attrs["w"]]
                wd = P[nodes[pos[0]].attrs["w"]]
                ws = self._workspace(ago.OP_FUSED_DW_PW,
                                     list(x.shape) + [w2.shape[1], nodes[pos[0]].attrs.get("stride", 1), wd.shape[0]], dt)
                fn = ago.ago_fused_dw_pw if wd.shape[0] == 3 else ago.ago_fused_dw_pw_k
                fn(x, wd, self._bias_of(nodes, pos[0]), w2, self._bias_of(nodes, pos[1]), out,
                   nodes[pos[0]].attrs.get("stride", 1), ws)
            elif kind == "conv_chain":
                pos = [k for k, n in enumerate(nodes) if n.op in COMPLEX]
                ago.ago_fused_conv_chain(x, P[nodes[pos[0]].attrs["w"]], self._bias_of(nodes, pos[0]),
                                         P[nodes[pos[1]].attrs["w"]], self._bias_of(nodes, pos[1]), out,
                                         any(n.op == "add" for n in nodes))
            elif kind in ("ffn", "ffn_epilogue"):
                pos = [k for k, n in enumerate(nodes) if n.op in COMPLEX]
                act = next(n.op for n in nodes if n.op in _ACT_OF)
                w1, w2 = P[nodes[pos[0]].attrs["w"]], P[nodes[pos[1]].attrs["w"]]
                dims = [x.shape[0], x.shape[1], w1.shape[1], w2.shape[1]]
                n1, n2 = nodes[pos[0]].attrs["w"], nodes[pos[1]].attrs["w"]
                if kind == "ffn":
                    if self.pack_weights and ago.fused_ffn_packed_supported(*dims):
                        ws = self._workspace(ago.OP_FUSED_FFN_PACKED, dims, ago.BF16)
                        ago.ago_fused_ffn_packed(x, self._packed(n1), self._bias_of(nodes, pos[0]), self._packed(n2),
                                                 self._bias_of(nodes, pos[1]), out, getattr(ago, _ACT_OF[act]), ws)
                    else:
                        ws = self._workspace(ago.OP_FUSED_FFN, dims, ago.BF16)
                        ago.ago_fused_ffn(x, w1, self._bias_of(nodes, pos[0]), w2, self._bias_of(nodes, pos[1]), out,
                                          getattr(ago, _ACT_OF[act]), ws)
                else:                                  # two products with fused epilogues (two launches)
                    self.launches += 1
                    ws = self._workspace(ago.OP_UNFUSED_FFN, dims, ago.BF16)
                    if (self.pack_weights and ago.gemm_packed_supported(dims[0], dims[1], dims[2])
                            and ago.gemm_packed_supported(dims[0], dims[2], dims[3])):
                        ago.ago_unfused_ffn_packed(x, self._packed(n1), self._bias_of(nodes, pos[0]), self._packed(n2),
                                                   self._bias_of(nodes, pos[1]), out, getattr(ago, _ACT_OF[act]), ws)
                    else:
                        ago.ago_unfused_ffn(x, w1, self._bias_of(nodes, pos[0]), w2, self._bias_of(nodes, pos[1]), out,
                                            getattr(ago, _ACT_OF[act]), True, ws)
            elif kind == "attn":
                k_t = val[nodes[0].inputs[1]]
                v_t = val[[s for s in nodes[3].inputs if s not in ids][0]]
                ago.ago_fused_attn(x, k_t, v_t, out, float(nodes[1].attrs["alpha"]))
            else:
                self._single(nodes[0], ids[0], val, out)
            val[ids[-1]] = out
        cons = g.consumers()
        return {i: val[i] for i in range(len(g.nodes)) if not cons[i] and g.nodes[i].op != "input"}

    def capture(self, example_inputs):
        """Record one pass of the plan into a HIP graph: a plan of small kernels (a network at batch 1 is a
        few microseconds per launch) is bound by launch overhead, and a replay issues all of them with one call.
        Returns (replay, inputs, outputs): copy new data into ``inputs[name]`` (static buffers), call
        ``replay()``, read ``outputs`` (the same dict ``run`` returns, static buffers as well).  One eager
        pass runs first so that one-time set-up (function attributes) stays out of the capture."""
        torch = self.torch
        static_in = {k: v.clone() for k, v in example_inputs.items()}
        self.run(static_in)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            static_out = self.run(static_in)
        self._graph = graph                # keeps the graph (and its memory pool) alive with the executor
        return graph.replay, static_in, static_out

    def _single(self, n, i, val, out):
        ago, P = self.ago, self.g.params
        a = val[n.inputs[0]]
        if n.op == "conv1x1":
            ago.ago_conv1x1(a, P[n.attrs["w"]], None, None, out)
        elif n.op == "gemm":
            w = P[n.attrs["w"]]
            if self.pack_weights and ago.gemm_packed_supported(a.shape[0], w.shape[0], w.shape[1]):
                ago.ago_gemm_packed(a, self._packed(n.attrs["w"]), None, out)
            else:
                ago.ago_gemm(a, w, None, None, out)
        elif n.op == "dwconv":
            if P[n.attrs["w"]].shape[0] != 3:
                raise NotImplementedError("un-fused depthwise kernels other than 3x3")
            ago.ago_dwconv3x3(a, P[n.attrs["w"]], None, out, n.attrs.get("stride", 1))
        elif n.op == "conv3x3":
            ago.ago_conv3x3(a, P[n.attrs["w"]], None, None, out)
        elif n.op == "bias":
            ago.ago_bias_act(a, P[n.attrs["b"]], out)
        elif n.op in _ACT_OF:
            ago.ago_bias_act(a, None, out, getattr(ago, _ACT_OF[n.op]))
        elif n.op == "add":
            ago.ago_add_act(a, val[n.inputs[1]], out)
        elif n.op == "scale":
            ago.ago_scale(a, out, float(n.attrs["alpha"]))
        elif n.op == "softmax":
            ago.ago_softmax_rows(a, out)
        elif n.op == "to_heads":
            b_, hh = n.attrs["batch"], n.attrs["heads"]
            v4 = a.view(b_, a.shape[0] // b_, hh, a.shape[1] // hh)
            out.copy_(v4.permute(0, 2, 1, 3) if n.attrs.get("head_major", True) else v4)   # a device copy, no arithmetic
        elif n.op == "bmm_nt":
            ago.ago_bmm_nt(a, val[n.inputs[1]], out)
        elif n.op == "bmm_nn":
            ago.ago_bmm_nn(a, val[n.inputs[1]], out)
        else:
            raise ValueError(n.op)
