"""Shapes, distributions and seeds of the five benchmark subgraphs, plus small
variants of each that a slow CPU oracle finishes in seconds.

Every tensor is returned as float64 holding *exactly* the value that is stored
for the GPU (fp32 or bfloat16 storage), so both sides start from the same numbers.
Seeds: ``22120100 + 16 * config_index + tensor_index``.
"""

from dataclasses import dataclass, field
import numpy as np

from . import rng

_SEED0 = 22120100


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return rng.round_to_bf16(x)
    return np.asarray(x, dtype=np.float32).astype(np.float64)


def _f32(x):
    return np.asarray(x, dtype=np.float32).astype(np.float64)


@dataclass
class InvresCase:
    """1x1 expand (+b1, ReLU6) -> depthwise ksize x ksize, pad (ksize-1)/2 (+bd, ReLU6) -> 1x1 project (+b2) [+x]."""
    N: int; H: int; W: int; Cin: int; Cexp: int; Cout: int
    stride: int = 1
    residual: bool = False
    bias: bool = True
    dtype: str = "f32"
    seed: int = _SEED0
    x_scale: float = 1.0
    name: str = "invres"
    ksize: int = 3

    @property
    def OH(self): return (self.H + 2 - 3) // self.stride + 1
    @property
    def OW(self): return (self.W + 2 - 3) // self.stride + 1

    def flops(self):
        pe = self.N * self.H * self.W
        po = self.N * self.OH * self.OW
        return (2 * pe * self.Cin * self.Cexp + 2 * self.ksize ** 2 * po * self.Cexp
                + 2 * po * self.Cexp * self.Cout)

    def alg_bytes(self):
        e = 2 if self.dtype == "bf16" else 4
        nb = 4 * (2 * self.Cexp + self.Cout) if self.bias else 0
        return e * (self.N * self.H * self.W * self.Cin + self.Cin * self.Cexp + self.ksize ** 2 * self.Cexp
                    + self.Cexp * self.Cout + self.N * self.OH * self.OW * self.Cout) + nb

    def tensors(self):
        s, d = self.seed, self.dtype
        t = {
            "x": _store(self.x_scale * rng.uniform(s + 0, (self.N, self.H, self.W, self.Cin), -1.0, 1.0), d),
            "w1": _store(rng.normal(s + 1, (self.Cin, self.Cexp), (1.0 / self.Cin) ** 0.5), d),
            "wd": _store(rng.normal(s + 2, (self.ksize, self.ksize, self.Cexp), 1.0 / self.ksize), d),
            "w2": _store(rng.normal(s + 3, (self.Cexp, self.Cout), (1.0 / self.Cexp) ** 0.5), d),
        }
        if self.bias:
            t["b1"] = _f32(rng.uniform(s + 4, (self.Cexp,), -0.1, 0.1))
            t["bd"] = _f32(rng.uniform(s + 5, (self.Cexp,), -0.1, 0.1))
            t["b2"] = _f32(rng.uniform(s + 6, (self.Cout,), -0.1, 0.1))
        else:
            t["b1"] = t["bd"] = t["b2"] = None
        return t


@dataclass
class ChainCase:
    """conv3x3 pad 1 (+ba, ReLU) -> conv3x3 pad 1 (+bb) [+x] -> ReLU, C -> C channels."""
    N: int; H: int; W: int; C: int
    residual: bool = True
    dtype: str = "bf16"
    seed: int = _SEED0 + 32
    name: str = "conv_chain"

    def flops(self):
        return 2 * 2 * 9 * self.N * self.H * self.W * self.C * self.C

    def alg_bytes(self):
        e = 2 if self.dtype == "bf16" else 4
        return e * (2 * self.N * self.H * self.W * self.C + 2 * 9 * self.C * self.C) + 4 * 2 * self.C

    def tensors(self):
        s, d = self.seed, self.dtype
        std = (2.0 / (9 * self.C)) ** 0.5
        return {
            "x": _store(rng.normal(s + 0, (self.N, self.H, self.W, self.C), 1.0), d),
            "wa": _store(rng.normal(s + 1, (3, 3, self.C, self.C), std), d),
            "wb": _store(rng.normal(s + 2, (3, 3, self.C, self.C), std), d),
            "ba": _f32(rng.uniform(s + 3, (self.C,), -0.1, 0.1)),
            "bb": _f32(rng.uniform(s + 4, (self.C,), -0.1, 0.1)),
        }


@dataclass
class FfnCase:
    """y = gelu_tanh(x w1 + b1) w2 + b2, x:[M,K] w1:[K,F] w2:[F,K2]."""
    M: int; K: int; F: int; K2: int
    dtype: str = "bf16"
    seed: int = _SEED0 + 48
    name: str = "ffn"

    def flops(self):
        return 2 * self.M * self.K * self.F + 2 * self.M * self.F * self.K2

    def alg_bytes(self):
        e = 2 if self.dtype == "bf16" else 4
        return e * (self.M * self.K + self.K * self.F + self.F * self.K2 + self.M * self.K2) \
            + 4 * (self.F + self.K2)

    def tensors(self):
        s, d = self.seed, self.dtype
        return {
            "x": _store(rng.normal(s + 0, (self.M, self.K), 1.0), d),
            "w1": _store(rng.normal(s + 1, (self.K, self.F), 0.02), d),
            "w2": _store(rng.normal(s + 2, (self.F, self.K2), 0.02), d),
            "b1": _f32(rng.uniform(s + 3, (self.F,), -0.1, 0.1)),
            "b2": _f32(rng.uniform(s + 4, (self.K2,), -0.1, 0.1)),
        }


@dataclass
class AttnCase:
    """o = softmax_rows(scale * q k^T [+ bias]) v per (batch, head); q,k,v,o:[B,Hh,S,D].

    bias: "none"; "full" = [B,Hh,S,S] random; "head" = [1,Hh,S,S] random (a relative-position table
    shared by the batch); "batch" = [B,1,S,S] key-padding mask (0 for the first len_b keys of batch b,
    -10000 for the rest, len_b seeded in [S/2, S])."""
    B: int; Hh: int; S: int; D: int
    scale: float = 0.125
    dtype: str = "bf16"
    seed: int = _SEED0 + 64
    name: str = "attn"
    bias: str = "none"

    def flops(self):
        return 2 * 2 * self.B * self.Hh * self.S * self.S * self.D

    def alg_bytes(self):
        e = 2 if self.dtype == "bf16" else 4
        return e * 4 * self.B * self.Hh * self.S * self.D

    def tensors(self):
        s, d = self.seed, self.dtype
        shp = (self.B, self.Hh, self.S, self.D)
        t = {
            "q": _store(rng.normal(s + 0, shp, 1.0), d),
            "k": _store(rng.normal(s + 1, shp, 1.0), d),
            "v": _store(rng.normal(s + 2, shp, 1.0), d),
        }
        if self.bias == "full":
            t["bias"] = _store(rng.normal(s + 3, (self.B, self.Hh, self.S, self.S), 1.0), d)
        elif self.bias == "head":
            t["bias"] = _store(rng.normal(s + 3, (1, self.Hh, self.S, self.S), 1.0), d)
        elif self.bias == "batch":
            lens = self.S // 2 + (rng.uniform(s + 3, (self.B,), 0.0, 1.0) * (self.S - self.S // 2 + 1)).astype(np.int64)
            lens = np.minimum(lens, self.S)
            keys = np.arange(self.S)[None, None, None, :]
            m = np.where(keys < lens[:, None, None, None], 0.0, -10000.0)
            t["bias"] = _store(np.broadcast_to(m, (self.B, 1, self.S, self.S)).copy(), d)
        elif self.bias != "none":
            raise ValueError(self.bias)
        return t


BASELINE_NAMES = ["invres_14x14x32_f32", "invres_56x56x24_s2_bf16", "chain_8x56x56x64_bf16",
                  "ffn_2048x768x3072_bf16", "attn_8x12x384x64_bf16"]


def baseline_case(i: int):
    """The i-th benchmark configuration at its full size."""
    if i == 0:
        return InvresCase(1, 14, 14, 32, 192, 32, stride=1, residual=True, bias=True,
                          dtype="f32", seed=_SEED0, name=BASELINE_NAMES[0])
    if i == 1:
        return InvresCase(1, 56, 56, 24, 144, 32, stride=2, residual=False, bias=False,
                          dtype="bf16", seed=_SEED0 + 16, name=BASELINE_NAMES[1])
    if i == 2:
        return ChainCase(8, 56, 56, 64, residual=True, dtype="bf16", seed=_SEED0 + 32,
                         name=BASELINE_NAMES[2])
    if i == 3:
        return FfnCase(2048, 768, 3072, 768, dtype="bf16", seed=_SEED0 + 48, name=BASELINE_NAMES[3])
    if i == 4:
        return AttnCase(8, 12, 384, 64, scale=0.125, dtype="bf16", seed=_SEED0 + 64,
                        name=BASELINE_NAMES[4])
    raise IndexError(i)


@dataclass
class QkvCase:
    """Sibling projections q, k, v = x wq + bq, x wk + bk, x wv + bv; x:[B*S, K], w:[K, Hh*D];
    outputs [B, Hh, S, D] (head_major) or [B, S, Hh, D]."""
    B: int; S: int; K: int; Hh: int; D: int
    head_major: bool = True
    bias: bool = True
    dtype: str = "bf16"
    seed: int = _SEED0 + 3000
    name: str = "qkv"

    def flops(self):
        return 3 * 2 * self.B * self.S * self.K * self.Hh * self.D

    def alg_bytes(self):
        n = self.Hh * self.D
        return 2 * (self.B * self.S * self.K + 3 * self.K * n + 3 * self.B * self.S * n) + (12 * n if self.bias else 0)

    def tensors(self):
        s, d, n = self.seed, self.dtype, self.Hh * self.D
        t = {"x": _store(rng.normal(s + 0, (self.B * self.S, self.K), 1.0), d)}
        for i, nm in enumerate("qkv"):
            t["w" + nm] = _store(rng.normal(s + 1 + i, (self.K, n), (1.0 / self.K) ** 0.5), d)
            t["b" + nm] = _f32(rng.uniform(s + 4 + i, (n,), -0.1, 0.1)) if self.bias else None
        return t


@dataclass
class PairCase:
    """Two-operator pairs of the inverted residual block (the paper's Fig. 13 micro-benchmarks).
    kind "pw_dw": 1x1 C1 -> C2 (+b1, ReLU6) -> depthwise 3x3 (+bd, ReLU6)
    kind "dw_pw": depthwise 3x3 on C1 channels (+bd, ReLU6) -> 1x1 C1 -> C2 (+b2)
    kind "dw_dw": depthwise 3x3 (stride) on C1 channels (+bd, ReLU6) -> depthwise 3x3 (+bd2, ReLU6); C2 = C1
    kind "pw_pw": 1x1 C1 -> C2 (+b1, act) -> 1x1 C2 -> C3 (+b2)"""
    kind: str
    N: int; H: int; W: int; C1: int; C2: int
    C3: int = 0
    stride: int = 1
    bias: bool = True
    act: str = "relu"
    dtype: str = "bf16"
    seed: int = _SEED0 + 2000
    name: str = "pair"
    ksize: int = 3            # depthwise size of pw_dw / dw_pw (3 or 5)

    @property
    def OH(self): return (self.H - 1) // self.stride + 1 if self.kind != "pw_pw" else self.H
    @property
    def OW(self): return (self.W - 1) // self.stride + 1 if self.kind != "pw_pw" else self.W

    def out_shape(self):
        c = {"pw_dw": self.C2, "dw_pw": self.C2, "dw_dw": self.C1, "pw_pw": self.C3}[self.kind]
        return (self.N, self.OH, self.OW, c)

    def flops(self):
        pe, po = self.N * self.H * self.W, self.N * self.OH * self.OW
        if self.kind == "pw_dw":
            return 2 * pe * self.C1 * self.C2 + 2 * self.ksize ** 2 * po * self.C2
        if self.kind == "dw_pw":
            return 2 * self.ksize ** 2 * po * self.C1 + 2 * po * self.C1 * self.C2
        if self.kind == "dw_dw":
            return 2 * 2 * 9 * po * self.C1
        return 2 * pe * self.C2 * (self.C1 + self.C3)

    def alg_bytes(self):
        e = 2 if self.dtype == "bf16" else 4
        t = self.tensors()
        n_in = sum(v.size * (4 if k.startswith("b") else e) for k, v in t.items() if v is not None)
        n_out = 1
        for d in self.out_shape():
            n_out *= d
        return n_in + n_out * e

    def tensors(self):
        s, d = self.seed, self.dtype
        b = (lambda k, n: _f32(rng.uniform(s + k, (n,), -0.1, 0.1))) if self.bias else (lambda k, n: None)
        if self.kind == "pw_dw":
            return {"x": _store(rng.uniform(s, (self.N, self.H, self.W, self.C1), -1.0, 1.0), d),
                    "w1": _store(rng.normal(s + 1, (self.C1, self.C2), (1.0 / self.C1) ** 0.5), d),
                    "wd": _store(rng.normal(s + 2, (self.ksize, self.ksize, self.C2), (1.0 / self.ksize ** 2) ** 0.5), d),
                    "b1": b(4, self.C2), "bd": b(5, self.C2)}
        if self.kind == "dw_pw":
            return {"x": _store(rng.uniform(s, (self.N, self.H, self.W, self.C1), -1.0, 1.0), d),
                    "wd": _store(rng.normal(s + 2, (self.ksize, self.ksize, self.C1), (1.0 / self.ksize ** 2) ** 0.5), d),
                    "w2": _store(rng.normal(s + 3, (self.C1, self.C2), (1.0 / self.C1) ** 0.5), d),
                    "bd": b(5, self.C1), "b2": b(6, self.C2)}
        if self.kind == "dw_dw":
            return {"x": _store(rng.uniform(s, (self.N, self.H, self.W, self.C1), -1.0, 1.0), d),
                    "wd": _store(rng.normal(s + 2, (3, 3, self.C1), (1.0 / 9.0) ** 0.5), d),
                    "wd2": _store(rng.normal(s + 7, (3, 3, self.C1), (1.0 / 9.0) ** 0.5), d),
                    "bd": b(5, self.C1), "bd2": b(8, self.C1)}
        return {"x": _store(rng.uniform(s, (self.N, self.H, self.W, self.C1), -1.0, 1.0), d),
                "w1": _store(rng.normal(s + 1, (self.C1, self.C2), (1.0 / self.C1) ** 0.5), d),
                "w2": _store(rng.normal(s + 3, (self.C2, self.C3), (1.0 / self.C2) ** 0.5), d),
                "b1": b(4, self.C2), "b2": b(6, self.C3)}


def pair_cases():
    """The two-operator pairs at the block shapes of configurations 0 and 1 plus ragged variants."""
    s = _SEED0 + 2000
    return [
        PairCase("pw_dw", 1, 14, 14, 32, 192, stride=1, dtype="f32", seed=s, name="pw_dw_14x14x32_f32"),
        PairCase("pw_dw", 1, 56, 56, 24, 144, stride=2, bias=False, dtype="bf16", seed=s + 16, name="pw_dw_56x56x24_s2_bf16"),
        PairCase("pw_dw", 2, 9, 11, 16, 96, stride=2, dtype="bf16", seed=s + 32, name="pw_dw_ragged_bf16"),
        PairCase("dw_pw", 1, 14, 14, 192, 32, stride=1, dtype="f32", seed=s + 48, name="dw_pw_14x14x192_f32"),
        PairCase("dw_pw", 1, 56, 56, 144, 32, stride=2, bias=False, dtype="bf16", seed=s + 64, name="dw_pw_56x56x144_s2_bf16"),
        PairCase("dw_pw", 2, 13, 10, 96, 24, stride=1, dtype="bf16", seed=s + 80, name="dw_pw_ragged_bf16"),
        PairCase("dw_dw", 1, 14, 14, 192, 192, stride=1, dtype="f32", seed=s + 128, name="dw_dw_14x14x192_f32"),
        PairCase("dw_dw", 1, 56, 56, 144, 144, stride=2, bias=False, dtype="bf16", seed=s + 144, name="dw_dw_56x56x144_s2_bf16"),
        PairCase("dw_dw", 2, 11, 9, 40, 40, stride=2, dtype="bf16", seed=s + 160, name="dw_dw_ragged_bf16"),
        PairCase("dw_dw", 3, 7, 19, 72, 72, stride=1, dtype="f32", seed=s + 176, name="dw_dw_ragged_f32"),
        PairCase("pw_pw", 2, 14, 14, 64, 384, 384, act="relu", dtype="bf16", seed=s + 96, name="pw_pw_2x14x14x64_bf16"),
        PairCase("pw_pw", 1, 10, 13, 64, 128, 128, act="relu6", dtype="bf16", seed=s + 112, name="pw_pw_ragged_bf16"),
    ]


def network_block_cases(batch=1, dtype="bf16"):
    """Inverted-residual blocks with the layer shapes of a MobileNetV2-style network (expansion 6, 224 x 224
    input; the paper's Sec. VI evaluates whole networks of this family): one block per distinct
    (resolution, channels, stride), from the 112 x 112 x 16 stage down to the 7 x 7 x 960-wide blocks."""
    s = _SEED0 + 3000
    shapes = [(112, 16, 96, 24, 2), (56, 24, 144, 24, 1), (56, 24, 144, 32, 2), (28, 32, 192, 32, 1),
              (28, 32, 192, 64, 2), (14, 64, 384, 64, 1), (14, 64, 384, 96, 1), (14, 96, 576, 96, 1),
              (14, 96, 576, 160, 2), (7, 160, 960, 160, 1), (7, 160, 960, 320, 1)]
    return [InvresCase(batch, hw, hw, ci, ce, co, st, st == 1 and ci == co, True, dtype, s + 16 * i,
                       name="block_%dx%dx%d_%d_%d_s%d" % (hw, hw, ci, ce, co, st))
            for i, (hw, ci, ce, co, st) in enumerate(shapes)]


def small_cases():
    """Reduced-size variants: several tiles plus a ragged tail, seconds for the oracle."""
    s = _SEED0 + 1000
    return [
        InvresCase(1, 14, 14, 32, 192, 32, 1, True, True, "f32", s + 0, name="invres_f32_s1"),
        InvresCase(2, 9, 11, 16, 96, 24, 2, False, True, "f32", s + 16, name="invres_f32_s2_ragged"),
        InvresCase(1, 14, 14, 32, 192, 32, 1, True, True, "f32", s + 32, x_scale=16.0,
                   name="invres_f32_clamp"),
        InvresCase(1, 20, 20, 24, 144, 32, 2, False, False, "bf16", s + 48, name="invres_bf16_s2"),
        InvresCase(2, 13, 10, 32, 192, 32, 1, True, True, "bf16", s + 64, name="invres_bf16_s1_res"),
        ChainCase(1, 20, 17, 64, True, "bf16", s + 80, name="chain_ragged"),
        ChainCase(2, 14, 14, 64, False, "bf16", s + 96, name="chain_nores"),
        FfnCase(200, 768, 3072, 768, "bf16", s + 112, name="ffn_ragged_rows"),
        FfnCase(96, 256, 512, 128, "bf16", s + 128, name="ffn_small"),
        FfnCase(70, 192, 384, 384, "bf16", s + 176, name="ffn_single_slice_ragged"),
        FfnCase(130, 64, 768, 768, "bf16", s + 192, name="ffn_two_k_tiles"),
        AttnCase(1, 2, 384, 64, 0.125, "bf16", s + 144, name="attn_s384"),
        AttnCase(2, 3, 100, 64, 0.125, "bf16", s + 160, name="attn_ragged_s100"),
        AttnCase(1, 3, 600, 64, 0.125, "bf16", s + 208, name="attn_long_s600"),
    ]
