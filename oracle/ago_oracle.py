"""ctypes loader for the fp64 CPU oracle (TEST INFRASTRUCTURE, not product code).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It builds ``libago_oracle.so`` from ``ago_oracle.c`` with gcc on
first use (plain C, OpenMP over outer loops) and wraps each function so that it
takes and returns float64 numpy arrays.  Nothing here touches the GPU library.
"""

import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ago_oracle.c")
_LIB = os.path.join(_HERE, "libago_oracle.so")
_lib = None

_D = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(_D)


def _c(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def num_threads() -> int:
    """Threads the OpenMP loops will use."""
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_get_max_threads.restype = ctypes.c_int
    lib()
    return int(omp.omp_get_max_threads())


# ---- single operators -----------------------------------------------------

def conv1x1(x, w):
    x, w = _c(x), _c(w)
    cin, cout = w.shape
    y = np.empty(x.shape[:-1] + (cout,), dtype=np.float64)
    lib().ago_oracle_conv1x1(_p(x), _p(w), _p(y), ctypes.c_long(x.size // cin), cin, cout)
    return y


def gemm(a, b):
    a, b = _c(a), _c(b)
    m, k = a.shape
    n = b.shape[1]
    c = np.empty((m, n), dtype=np.float64)
    lib().ago_oracle_gemm(_p(a), _p(b), _p(c), m, k, n)
    return c


def dwconv3x3(x, w, stride=1):
    x, w = _c(x), _c(w)
    n, h, wd, c = x.shape
    oh, ow = (h - 1) // stride + 1, (wd - 1) // stride + 1
    y = np.empty((n, oh, ow, c), dtype=np.float64)
    lib().ago_oracle_dwconv3x3(_p(x), _p(w), _p(y), n, h, wd, c, stride)
    return y


def dwconv(x, w, stride=1):
    """Depthwise R x R, odd R = w.shape[0], zero pad (R - 1) / 2."""
    x, w = _c(x), _c(w)
    n, h, wd, c = x.shape
    r = w.shape[0]
    assert r % 2 == 1 and w.shape == (r, r, c)
    oh, ow = (h - 1) // stride + 1, (wd - 1) // stride + 1
    y = np.empty((n, oh, ow, c), dtype=np.float64)
    lib().ago_oracle_dwconv(_p(x), _p(w), _p(y), n, h, wd, c, stride, r)
    return y


def conv3x3(x, w):
    x, w = _c(x), _c(w)
    n, h, wd, cin = x.shape
    cout = w.shape[3]
    y = np.empty((n, h, wd, cout), dtype=np.float64)
    lib().ago_oracle_conv3x3(_p(x), _p(w), _p(y), n, h, wd, cin, cout)
    return y


def bmm_nt(a, k):
    a, k = _c(a), _c(k)
    s, d = a.shape[-2:]
    s2 = k.shape[-2]
    batch = a.size // (s * d)
    out = np.empty(a.shape[:-2] + (s, s2), dtype=np.float64)
    lib().ago_oracle_bmm_nt(_p(a), _p(k), _p(out), ctypes.c_long(batch), s, s2, d)
    return out


def bmm_nn(p, v):
    p, v = _c(p), _c(v)
    s, s2 = p.shape[-2:]
    d = v.shape[-1]
    batch = p.size // (s * s2)
    out = np.empty(p.shape[:-2] + (s, d), dtype=np.float64)
    lib().ago_oracle_bmm_nn(_p(p), _p(v), _p(out), ctypes.c_long(batch), s, s2, d)
    return out


def bias(y, b):
    y, b = _c(y).copy(), _c(b)
    c = b.shape[0]
    lib().ago_oracle_bias(_p(y), _p(b), ctypes.c_long(y.size // c), c)
    return y


def _unary(name):
    def f(y):
        y = _c(y).copy()
        getattr(lib(), name)(_p(y), ctypes.c_long(y.size))
        return y
    return f


relu = _unary("ago_oracle_relu")
relu6 = _unary("ago_oracle_relu6")
gelu_tanh = _unary("ago_oracle_gelu_tanh")


def add(y, x):
    y, x = _c(y).copy(), _c(x)
    assert y.shape == x.shape
    lib().ago_oracle_add(_p(y), _p(x), ctypes.c_long(y.size))
    return y


def scale(y, a):
    y = _c(y).copy()
    lib().ago_oracle_scale(_p(y), ctypes.c_double(a), ctypes.c_long(y.size))
    return y


def softmax_rows(s):
    s = _c(s).copy()
    cols = s.shape[-1]
    lib().ago_oracle_softmax_rows(_p(s), ctypes.c_long(s.size // cols), cols)
    return s


# ---- subgraphs --------------------------------------------------------------

def invres(x, w1, b1, wd, bd, w2, b2, stride=1, residual=False):
    x, w1, wd, w2 = _c(x), _c(w1), _c(wd), _c(w2)
    b1, bd, b2 = _c(b1), _c(bd), _c(b2)
    n, h, w, cin = x.shape
    cexp, cout = w2.shape
    oh, ow = (h - 1) // stride + 1, (w - 1) // stride + 1
    if residual:
        assert stride == 1 and cin == cout
    y = np.empty((n, oh, ow, cout), dtype=np.float64)
    rc = lib().ago_oracle_invres(_p(x), _p(w1), _p(b1), _p(wd), _p(bd), _p(w2), _p(b2), _p(y),
                                 n, h, w, cin, cexp, cout, stride, int(bool(residual)))
    assert rc == 0
    return y


def invres_k(x, w1, b1, wd, bd, w2, b2, stride=1, residual=False):
    """The block with an R x R depthwise (R = wd.shape[0]): the operators called one after another."""
    e = conv1x1(x, w1)
    if b1 is not None:
        e = bias(e, b1)
    d = dwconv(relu6(e), wd, stride)
    if bd is not None:
        d = bias(d, bd)
    y = conv1x1(relu6(d), w2)
    if b2 is not None:
        y = bias(y, b2)
    return add(y, x) if residual else y


def conv_chain(x, wa, ba, wb, bb, residual=True):
    x, wa, wb, ba, bb = _c(x), _c(wa), _c(wb), _c(ba), _c(bb)
    n, h, w, c = x.shape
    y = np.empty_like(x)
    rc = lib().ago_oracle_conv_chain(_p(x), _p(wa), _p(ba), _p(wb), _p(bb), _p(y),
                                     n, h, w, c, int(bool(residual)))
    assert rc == 0
    return y


ACT = {"none": 0, "relu": 1, "relu6": 2, "gelu_tanh": 3}


def ffn(x, w1, b1, w2, b2, act="gelu_tanh"):
    x, w1, w2, b1, b2 = _c(x), _c(w1), _c(w2), _c(b1), _c(b2)
    m, k = x.shape
    f, k2 = w2.shape
    y = np.empty((m, k2), dtype=np.float64)
    rc = lib().ago_oracle_ffn(_p(x), _p(w1), _p(b1), _p(w2), _p(b2), _p(y), m, k, f, k2, ACT[act])
    assert rc == 0
    return y


def attn(q, k, v, scale_=0.125):
    q, k, v = _c(q), _c(k), _c(v)
    b, hh, s, d = q.shape
    o = np.empty_like(q)
    rc = lib().ago_oracle_attn(_p(q), _p(k), _p(v), _p(o), b, hh, s, d, ctypes.c_double(scale_))
    assert rc == 0
    return o


def attn_bias(q, k, v, b, scale_=0.125):
    """softmax_rows(scale * q k^T + b) v: the attention chain of Sec. VI-C with one more simple operator
    (an elementwise add of a bias / mask) between the two products.  b broadcasts over the batch and
    head dimensions: b:[Bb,Hb,S,S] with Bb in {1, B}, Hb in {1, Hh}."""
    q, k, v, b = _c(q), _c(k), _c(v), _c(b)
    bq, hh, s, _ = q.shape
    assert b.shape[0] in (1, bq) and b.shape[1] in (1, hh) and b.shape[2:] == (s, s)
    sc = scale(bmm_nt(q, k), scale_)
    sc = add(sc, np.ascontiguousarray(np.broadcast_to(b, sc.shape)))
    return bmm_nn(softmax_rows(sc), v)


def qkv(x, wq, wk, wv, bq, bk, bv, batch, heads, head_major=True):
    """Three sibling products that share their input (sibling fusion, Sec. III): x:[B*S, K] times
    wq / wk / wv:[K, Hh*D], plus biases; each result viewed as [B, S, Hh, D] and, when head_major,
    transposed to [B, Hh, S, D] (the transpose that follows the projections in an attention layer)."""
    outs = []
    for w, b in ((wq, bq), (wk, bk), (wv, bv)):
        y = gemm(x, w)
        if b is not None:
            y = bias(y, b)
        m, n = y.shape
        y = y.reshape(batch, m // batch, heads, n // heads)
        outs.append(np.ascontiguousarray(y.transpose(0, 2, 1, 3)) if head_major else y)
    return tuple(outs)


# ---- two-operator pairs (Sec. VI, Fig. 13): the operators above called one after another --------

def _dw(x, wd, stride):
    """The depthwise of a pair: 3 x 3, or R x R read off the weight's shape (the MNasNet-style 5 x 5)."""
    return dwconv3x3(x, wd, stride) if wd.shape[0] == 3 else dwconv(x, wd, stride)


def pw_dw(x, w1, b1, wd, bd, stride=1):
    """relu6(dw(relu6(x * w1 + b1)) + bd); the padding of the depthwise pads the activated tensor."""
    e = conv1x1(x, w1)
    if b1 is not None:
        e = bias(e, b1)
    e = relu6(e)
    d = _dw(e, wd, stride)
    if bd is not None:
        d = bias(d, bd)
    return relu6(d)


def dw_pw(x, wd, bd, w2, b2, stride=1):
    """relu6(dw(x) + bd) * w2 + b2."""
    d = _dw(x, wd, stride)
    if bd is not None:
        d = bias(d, bd)
    y = conv1x1(relu6(d), w2)
    if b2 is not None:
        y = bias(y, b2)
    return y


def dw_dw(x, wa, ba, wb, bb, stride=1):
    """relu6(dw3x3(relu6(dw3x3(x, wa, stride) + ba), wb, 1) + bb)."""
    t = dwconv3x3(x, wa, stride)
    if ba is not None:
        t = bias(t, ba)
    y = dwconv3x3(relu6(t), wb, 1)
    if bb is not None:
        y = bias(y, bb)
    return relu6(y)


def pw_pw(x, w1, b1, w2, b2, act="relu"):
    """act(x * w1 + b1) * w2 + b2 on an NHWC tensor."""
    h = conv1x1(x, w1)
    if b1 is not None:
        h = bias(h, b1)
    h = {"none": lambda v: v, "relu": relu, "relu6": relu6, "gelu_tanh": gelu_tanh}[act](h)
    y = conv1x1(h, w2)
    if b2 is not None:
        y = bias(y, b2)
    return y


def run_case(case):
    """Evaluate a workloads.*Case on the oracle; returns the fp64 output."""
    t = case.tensors()
    kind = type(case).__name__
    if kind == "PairCase":
        if case.kind == "pw_dw":
            return pw_dw(t["x"], t["w1"], t["b1"], t["wd"], t["bd"], case.stride)
        if case.kind == "dw_pw":
            return dw_pw(t["x"], t["wd"], t["bd"], t["w2"], t["b2"], case.stride)
        if case.kind == "dw_dw":
            return dw_dw(t["x"], t["wd"], t["bd"], t["wd2"], t["bd2"], case.stride)
        return pw_pw(t["x"], t["w1"], t["b1"], t["w2"], t["b2"], case.act)
    if kind == "InvresCase" and case.ksize != 3:
        return invres_k(t["x"], t["w1"], t["b1"], t["wd"], t["bd"], t["w2"], t["b2"],
                        case.stride, case.residual)
    if kind == "InvresCase":
        return invres(t["x"], t["w1"], t["b1"], t["wd"], t["bd"], t["w2"], t["b2"],
                      case.stride, case.residual)
    if kind == "ChainCase":
        return conv_chain(t["x"], t["wa"], t["ba"], t["wb"], t["bb"], case.residual)
    if kind == "FfnCase":
        return ffn(t["x"], t["w1"], t["b1"], t["w2"], t["b2"])
    if kind == "QkvCase":
        return np.stack(qkv(t["x"], t["wq"], t["wk"], t["wv"], t["bq"], t["bk"], t["bv"], case.B, case.Hh,
                            case.head_major))
    if kind == "AttnCase" and case.bias != "none":
        return attn_bias(t["q"], t["k"], t["v"], t["bias"], case.scale)
    if kind == "AttnCase":
        return attn(t["q"], t["k"], t["v"], case.scale)
    raise TypeError(kind)
