"""Plumbing shared by the tests and the benchmark: put a workload's tensors on the GPU,
allocate outputs / workspaces with torch, and call the library through the binding.
Nothing here computes any part of a subgraph.
"""

import numpy as np
import torch

from . import binding as ago


def _torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_device(case, device="cuda:0"):
    """numpy fp64 tensors of a workloads.*Case -> dict of device tensors in storage dtype."""
    td = _torch_dtype(case.dtype)
    out = {}
    for name, arr in case.tensors().items():
        if arr is None:
            out[name] = None
        elif name.startswith("b") and arr.ndim == 1:      # biases are always fp32
            out[name] = torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(device)
        else:
            # values are already exactly representable in the storage dtype
            out[name] = torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(device).to(td).contiguous()
    return out


def _dims(case):
    k = type(case).__name__
    if k == "InvresCase":
        return [case.N, case.H, case.W, case.Cin, case.Cexp, case.Cout, case.stride, case.ksize]
    if k == "ChainCase":
        return [case.N, case.H, case.W, case.C]
    if k == "FfnCase":
        return [case.M, case.K, case.F, case.K2]
    return [case.B, case.Hh, case.S, case.D]


_FUSED_OP = {"InvresCase": ago.OP_FUSED_INVRES, "ChainCase": ago.OP_FUSED_CONV_CHAIN,
             "FfnCase": ago.OP_FUSED_FFN, "AttnCase": ago.OP_FUSED_ATTN}


def alloc_output(case, device="cuda:0"):
    td = _torch_dtype(case.dtype)
    k = type(case).__name__
    if k == "PairCase":
        return torch.empty(case.out_shape(), dtype=td, device=device)
    if k == "QkvCase":          # q, k, v stacked
        inner = (case.B, case.Hh, case.S, case.D) if case.head_major else (case.B, case.S, case.Hh, case.D)
        return torch.empty((3,) + inner, dtype=td, device=device)
    if k == "InvresCase":
        shape = (case.N, case.OH, case.OW, case.Cout)
    elif k == "ChainCase":
        shape = (case.N, case.H, case.W, case.C)
    elif k == "FfnCase":
        shape = (case.M, case.K2)
    else:
        shape = (case.B, case.Hh, case.S, case.D)
    return torch.empty(shape, dtype=td, device=device)


def alloc_workspace(case, fused=True, device="cuda:0"):
    if type(case).__name__ == "QkvCase":
        return None
    if type(case).__name__ == "PairCase":
        if not fused or case.kind not in ("pw_pw", "dw_pw"):
            return None
        if case.kind == "dw_pw":
            n = ago.workspace_bytes(ago.OP_FUSED_DW_PW, [case.N, case.H, case.W, case.C1, case.C2, case.stride, case.ksize],
                                    ago.BF16 if case.dtype == "bf16" else ago.F32)
        else:
            n = ago.workspace_bytes(ago.OP_FUSED_PW_PW, [case.N, case.H, case.W, case.C1, case.C2, case.C3], ago.BF16)
        return torch.empty(max(n, 16), dtype=torch.uint8, device=device) if n > 0 else None
    op = _FUSED_OP[type(case).__name__] + (0 if fused else 4)
    n = ago.workspace_bytes(op, _dims(case), ago.BF16 if case.dtype == "bf16" else ago.F32)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device) if n > 0 else None


_ACT = {"none": ago.ACT_NONE, "relu": ago.ACT_RELU, "relu6": ago.ACT_RELU6, "gelu_tanh": ago.ACT_GELU_TANH}


def _fused_call(case, t, y, ws):
    k = type(case).__name__
    if k == "PairCase":
        if case.kind == "pw_dw":
            fn = ago.ago_fused_pw_dw if case.ksize == 3 else ago.ago_fused_pw_dw_k
            return fn, (t["x"], t["w1"], t["b1"], t["wd"], t["bd"], y, case.stride, ws)
        if case.kind == "dw_pw":
            fn = ago.ago_fused_dw_pw if case.ksize == 3 else ago.ago_fused_dw_pw_k
            return fn, (t["x"], t["wd"], t["bd"], t["w2"], t["b2"], y, case.stride, ws)
        if case.kind == "dw_dw":
            return ago.ago_fused_dw_dw, (t["x"], t["wd"], t["bd"], t["wd2"], t["bd2"], y, case.stride, ws)
        return ago.ago_fused_pw_pw, (t["x"], t["w1"], t["b1"], t["w2"], t["b2"], y, _ACT[case.act], ws)
    if k == "QkvCase":
        return ago.ago_fused_qkv, (t["x"], t["wq"], t["wk"], t["wv"], t["bq"], t["bk"], t["bv"], y[0], y[1], y[2],
                                   case.head_major, ws)
    if k == "InvresCase" and case.ksize != 3:
        return ago.ago_fused_invres_k, (t["x"], t["w1"], t["b1"], t["wd"], t["bd"], t["w2"], t["b2"], y,
                                        case.stride, case.residual, ws)
    if k == "InvresCase":
        return ago.ago_fused_invres, (t["x"], t["w1"], t["b1"], t["wd"], t["bd"], t["w2"], t["b2"], y,
                                      case.stride, case.residual, ws)
    if k == "ChainCase":
        return ago.ago_fused_conv_chain, (t["x"], t["wa"], t["ba"], t["wb"], t["bb"], y, case.residual, ws)
    if k == "FfnCase":
        return ago.ago_fused_ffn, (t["x"], t["w1"], t["b1"], t["w2"], t["b2"], y, ago.ACT_GELU_TANH, ws)
    if case.bias != "none":
        return ago.ago_fused_attn_bias, (t["q"], t["k"], t["v"], t["bias"], y, case.scale, ws)
    return ago.ago_fused_attn, (t["q"], t["k"], t["v"], y, case.scale, ws)


def run_fused(case, t, y, ws=None):
    fn, args = _fused_call(case, t, y, ws)
    fn(*args)
    return y


def prepare_fused(case, t, y, ws=None):
    """Zero-argument launcher of the fused subgraph on these buffers (arguments marshalled once)."""
    fn, args = _fused_call(case, t, y, ws)
    return ago.prepare(fn, *args)


def _unfused_call(case, t, y, ws, epilogue_fused):
    k = type(case).__name__
    if k == "InvresCase":
        return ago.ago_unfused_invres, (t["x"], t["w1"], t["b1"], t["wd"], t["bd"], t["w2"], t["b2"], y,
                                        case.stride, case.residual, epilogue_fused, ws)
    if k == "ChainCase":
        return ago.ago_unfused_conv_chain, (t["x"], t["wa"], t["ba"], t["wb"], t["bb"], y, case.residual,
                                            epilogue_fused, ws)
    if k == "FfnCase":
        return ago.ago_unfused_ffn, (t["x"], t["w1"], t["b1"], t["w2"], t["b2"], y, ago.ACT_GELU_TANH,
                                     epilogue_fused, ws)
    return ago.ago_unfused_attn, (t["q"], t["k"], t["v"], y, case.scale, epilogue_fused, ws)


def run_unfused(case, t, y, ws, epilogue_fused):
    fn, args = _unfused_call(case, t, y, ws, epilogue_fused)
    fn(*args)
    return y


def prepare_unfused(case, t, y, ws, epilogue_fused):
    fn, args = _unfused_call(case, t, y, ws, epilogue_fused)
    return ago.prepare(fn, *args)


def _pair_unfused_calls(case, t, y, scratch):
    if case.kind == "pw_dw":
        return [(ago.ago_conv1x1, (t["x"], t["w1"], t["b1"], None, scratch, ago.ACT_RELU6)),
                (ago.ago_dwconv3x3, (scratch, t["wd"], t["bd"], y, case.stride, ago.ACT_RELU6))]
    if case.kind == "dw_pw":
        return [(ago.ago_dwconv3x3, (t["x"], t["wd"], t["bd"], scratch, case.stride, ago.ACT_RELU6)),
                (ago.ago_conv1x1, (scratch, t["w2"], t["b2"], None, y, ago.ACT_NONE))]
    if case.kind == "dw_dw":
        return [(ago.ago_dwconv3x3, (t["x"], t["wd"], t["bd"], scratch, case.stride, ago.ACT_RELU6)),
                (ago.ago_dwconv3x3, (scratch, t["wd2"], t["bd2"], y, 1, ago.ACT_RELU6))]
    return [(ago.ago_conv1x1, (t["x"], t["w1"], t["b1"], None, scratch, _ACT[case.act])),
            (ago.ago_conv1x1, (scratch, t["w2"], t["b2"], None, y, ago.ACT_NONE))]


def run_pair_unfused(case, t, y, scratch):
    """The pair operator by operator with epilogue-fused kernels (the conventional-fusion baseline);
    `scratch` holds the intermediate tensor."""
    for fn, args in _pair_unfused_calls(case, t, y, scratch):
        fn(*args)
    return y


def prepare_pair_unfused(case, t, y, scratch):
    launches = [ago.prepare(fn, *args) for fn, args in _pair_unfused_calls(case, t, y, scratch)]

    def run():
        for launch in launches:
            launch()
    return run


def alloc_pair_scratch(case, device="cuda:0"):
    td = _torch_dtype(case.dtype)
    if case.kind == "pw_dw":
        shape = (case.N, case.H, case.W, case.C2)
    elif case.kind in ("dw_pw", "dw_dw"):
        shape = (case.N, case.OH, case.OW, case.C1)
    else:
        shape = (case.N, case.H, case.W, case.C2)
    return torch.empty(shape, dtype=td, device=device)


def to_numpy64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)
