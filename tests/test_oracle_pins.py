"""Pins for the CPU oracle: things the paper and the mathematics fix, none of
which is the oracle's own code.

 * brute force: the un-fused loop nest of Sec. III-A (Fig. 3), written here in
   pure Python in the paper's own NCHW / OIHW index form on an explicitly
   zero-padded input, for every operator and every subgraph, strides 1 and 2;
 * delta / identity weights (pin the shift direction = no kernel flip, and the
   zero padding of the *intermediate* tensor);
 * all-ones closed forms (pin output size and which side is padded);
 * linearity; pointwise == matrix product (Sec. III-B) against numpy;
 * GELU and softmax identities;
 * fused == un-fused (Figs. 3-5 compute the same tensor).
"""

import math
import numpy as np
import pytest

import workloads as wl
from workloads import rng


# --------------------------------------------------------------------------
# brute force in the paper's index form (Sec. III-A, Fig. 3): NCHW input, OIHW weight, the window walks
# the input forwards from the output position (cross-correlation)
# --------------------------------------------------------------------------

def _pad_nchw(inp, pad):
    n, c, h, w = len(inp), len(inp[0]), len(inp[0][0]), len(inp[0][0][0])
    out = [[[[0.0] * (w + 2 * pad) for _ in range(h + 2 * pad)] for _ in range(c)] for _ in range(n)]
    for a in range(n):
        for b in range(c):
            for i in range(h):
                for j in range(w):
                    out[a][b][i + pad][j + pad] = inp[a][b][i][j]
    return out


def brute_conv_nchw(inp, weight, pad, stride, groups_depthwise=False):
    """inp [N][I][H][W] lists, weight [O][I or 1][R][C] lists -> [N][O][OH][OW]."""
    N, I = len(inp), len(inp[0])
    H, W = len(inp[0][0]), len(inp[0][0][0])
    O, R, C = len(weight), len(weight[0][0]), len(weight[0][0][0])
    xp = _pad_nchw(inp, pad)
    OH = (H + 2 * pad - R) // stride + 1
    OW = (W + 2 * pad - C) // stride + 1
    out = [[[[0.0] * OW for _ in range(OH)] for _ in range(O)] for _ in range(N)]
    for n in range(N):
        for o in range(O):
            for h in range(OH):
                for w in range(OW):
                    acc = 0.0
                    chans = [o] if groups_depthwise else range(I)
                    for ri in chans:
                        for rr in range(R):
                            for rc in range(C):
                                wv = weight[o][0 if groups_depthwise else ri][rr][rc]
                                acc += xp[n][ri][h * stride + rr][w * stride + rc] * wv
                    out[n][o][h][w] = acc
    return out


def nhwc_to_lists(x):       # numpy NHWC -> nested lists NCHW
    return np.transpose(x, (0, 3, 1, 2)).tolist()


def lists_to_nhwc(lst):
    return np.transpose(np.array(lst, dtype=np.float64), (0, 2, 3, 1))


def w1x1_to_oihw(w):        # [Cin][Cout] -> [O][I][1][1]
    return np.transpose(w, (1, 0))[:, :, None, None].tolist()


def w3x3_to_oihw(w):        # [3][3][Cin][Cout] -> [O][I][3][3]
    return np.transpose(w, (3, 2, 0, 1)).tolist()


def wdw_to_oihw(w):         # [3][3][C] -> [C][1][3][3]
    return np.transpose(w, (2, 0, 1))[:, None, :, :].tolist()


def brute_bias_act(t, b, act):
    """t NCHW lists; separate passes for bias and activation as in Fig. 3."""
    out = []
    for n in range(len(t)):
        on = []
        for o in range(len(t[n])):
            oo = []
            for row in t[n][o]:
                r = []
                for v in row:
                    s = v + (b[o] if b is not None else 0.0)
                    if act == "relu":
                        s = max(s, 0.0)
                    elif act == "relu6":
                        s = min(max(s, 0.0), 6.0)
                    r.append(s)
                oo.append(r)
            on.append(oo)
        out.append(on)
    return out


def _tiny(seed, shape, lo=-1.0, hi=1.0):
    return rng.uniform(seed, shape, lo, hi)


@pytest.mark.parametrize("shape", [(1, 5, 5, 3, 4), (2, 4, 6, 2, 5)])
def test_conv1x1_brute(oracle, shape):
    n, h, w, ci, co = shape
    x, wt = _tiny(1, (n, h, w, ci)), _tiny(2, (ci, co))
    ref = lists_to_nhwc(brute_conv_nchw(nhwc_to_lists(x), w1x1_to_oihw(wt), 0, 1))
    np.testing.assert_allclose(oracle.conv1x1(x, wt), ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("hw", [(5, 5), (6, 7), (4, 3)])
def test_dwconv_brute(oracle, stride, hw):
    h, w = hw
    x, wt = _tiny(3, (2, h, w, 3)), _tiny(4, (3, 3, 3))
    ref = lists_to_nhwc(brute_conv_nchw(nhwc_to_lists(x), wdw_to_oihw(wt), 1, stride, True))
    got = oracle.dwconv3x3(x, wt, stride)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("hw,r", [((6, 7), 5), ((3, 4), 5), ((5, 5), 3), ((9, 8), 7), ((4, 4), 1)])
def test_dwconv_general_brute(oracle, stride, hw, r):
    """Odd depthwise sizes against the padded brute force, and the embedding identities that tie the
    general routine to the 3x3 one."""
    h, w = hw
    x, wt = _tiny(13, (2, h, w, 3)), _tiny(14, (r, r, 3))
    ref = lists_to_nhwc(brute_conv_nchw(nhwc_to_lists(x), wdw_to_oihw(wt), (r - 1) // 2, stride, True))
    got = oracle.dwconv(x, wt, stride)
    assert got.shape == ref.shape == (2, (h - 1) // stride + 1, (w - 1) // stride + 1, 3)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-13)
    if r == 3:
        np.testing.assert_array_equal(got, oracle.dwconv3x3(x, wt, stride))
    if r == 5:
        # a 3x3 kernel embedded in the centre of a zero 5x5 kernel is the 3x3 depthwise
        w3 = _tiny(15, (3, 3, 3))
        w5 = np.zeros((5, 5, 3))
        w5[1:4, 1:4] = w3
        np.testing.assert_allclose(oracle.dwconv(x, w5, stride), oracle.dwconv3x3(x, w3, stride), rtol=0, atol=1e-14)
        # a single off-centre tap shifts the image: tap (r0, s0) reads x[oh*st + r0 - 2, ow*st + s0 - 2]
        tap = np.zeros((5, 5, 3))
        tap[0, 3] = 1.0
        xp = np.pad(x, ((0, 0), (2, 2), (2, 2), (0, 0)))
        np.testing.assert_array_equal(oracle.dwconv(x, tap, stride), xp[:, 0:h:stride, 3:3 + w:stride][:, :got.shape[1], :got.shape[2]])


def test_invres_k_composition(oracle):
    """The block with a general depthwise equals the monolithic 3x3 block when the kernel is 3x3, and with a
    5x5 kernel whose ring is zero."""
    x, w1, w2 = _tiny(20, (2, 6, 5, 4)), _tiny(21, (4, 8)), _tiny(22, (8, 4))
    b1, bd, b2 = _tiny(23, (8,)), _tiny(24, (8,)), _tiny(25, (4,))
    wd3 = _tiny(26, (3, 3, 8))
    wd5 = np.zeros((5, 5, 8))
    wd5[1:4, 1:4] = wd3
    for stride, res in ((1, True), (2, False)):
        ref = oracle.invres(x, w1, b1, wd3, bd, w2, b2, stride, res)
        np.testing.assert_allclose(oracle.invres_k(x, w1, b1, wd3, bd, w2, b2, stride, res), ref, rtol=0, atol=1e-13)
        np.testing.assert_allclose(oracle.invres_k(x, w1, b1, wd5, bd, w2, b2, stride, res), ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("hw", [(5, 5), (3, 6)])
def test_conv3x3_brute(oracle, hw):
    h, w = hw
    x, wt = _tiny(5, (2, h, w, 3)), _tiny(6, (3, 3, 3, 4))
    ref = lists_to_nhwc(brute_conv_nchw(nhwc_to_lists(x), w3x3_to_oihw(wt), 1, 1))
    np.testing.assert_allclose(oracle.conv3x3(x, wt), ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("stride,residual", [(1, True), (2, False), (1, False)])
def test_invres_brute(oracle, stride, residual):
    n, h, w, ci, ce = 1, 5, 6, 3, 5
    co = ci if residual else 4
    # weights scaled up so both ReLU6 clamps are hit
    x = _tiny(10, (n, h, w, ci), -2, 2)
    w1, wd, w2 = 3 * _tiny(11, (ci, ce)), 2 * _tiny(12, (3, 3, ce)), _tiny(13, (ce, co))
    b1, bd, b2 = _tiny(14, (ce,)), _tiny(15, (ce,)), _tiny(16, (co,))
    e = brute_bias_act(brute_conv_nchw(nhwc_to_lists(x), w1x1_to_oihw(w1), 0, 1), b1.tolist(), "relu6")
    assert np.max(e) == 6.0 and np.min(e) == 0.0
    d = brute_bias_act(brute_conv_nchw(e, wdw_to_oihw(wd), 1, stride, True), bd.tolist(), "relu6")
    yl = brute_bias_act(brute_conv_nchw(d, w1x1_to_oihw(w2), 0, 1), b2.tolist(), None)
    ref = lists_to_nhwc(yl)
    if residual:
        ref = ref + x
    got = oracle.invres(x, w1, b1, wd, bd, w2, b2, stride, residual)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("residual", [True, False])
def test_conv_chain_brute(oracle, residual):
    n, h, w, c = 1, 4, 5, 3
    x = _tiny(20, (n, h, w, c))
    wa, wb = _tiny(21, (3, 3, c, c)), _tiny(22, (3, 3, c, c))
    ba, bb = _tiny(23, (c,)), _tiny(24, (c,))
    t = brute_bias_act(brute_conv_nchw(nhwc_to_lists(x), w3x3_to_oihw(wa), 1, 1), ba.tolist(), "relu")
    y = lists_to_nhwc(brute_bias_act(brute_conv_nchw(t, w3x3_to_oihw(wb), 1, 1), bb.tolist(), None))
    if residual:
        y = y + x
    ref = np.maximum(y, 0.0)
    np.testing.assert_allclose(oracle.conv_chain(x, wa, ba, wb, bb, residual), ref, rtol=0, atol=1e-12)


def test_ffn_brute(oracle):
    m, k, f, k2 = 3, 4, 5, 2
    x, w1, w2 = _tiny(30, (m, k), -2, 2), _tiny(31, (k, f)), _tiny(32, (f, k2))
    b1, b2 = _tiny(33, (f,)), _tiny(34, (k2,))
    ref = np.zeros((m, k2))
    for i in range(m):
        hrow = []
        for j in range(f):
            s = sum(x[i, a] * w1[a, j] for a in range(k)) + b1[j]
            hrow.append(0.5 * s * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (s + 0.044715 * s ** 3))))
        for o in range(k2):
            ref[i, o] = sum(hrow[j] * w2[j, o] for j in range(f)) + b2[o]
    np.testing.assert_allclose(oracle.ffn(x, w1, b1, w2, b2), ref, rtol=0, atol=1e-13)


def test_attn_brute(oracle):
    b, hh, s, d = 1, 2, 5, 3
    q, k, v = _tiny(40, (b, hh, s, d), -2, 2), _tiny(41, (b, hh, s, d), -2, 2), _tiny(42, (b, hh, s, d))
    ref = np.zeros((b, hh, s, d))
    for bi in range(b):
        for h in range(hh):
            for i in range(s):
                sc = [0.5 * sum(q[bi, h, i, t] * k[bi, h, j, t] for t in range(d)) for j in range(s)]
                mx = max(sc)
                ex = [math.exp(z - mx) for z in sc]
                den = sum(ex)
                for t in range(d):
                    ref[bi, h, i, t] = sum(ex[j] / den * v[bi, h, j, t] for j in range(s))
    np.testing.assert_allclose(oracle.attn(q, k, v, 0.5), ref, rtol=0, atol=1e-13)


def test_qkv_brute_and_layouts(oracle):
    """Sibling projections against plain loops; the two output layouts are transposes of each other; the
    siblings do not see each other's weights."""
    b, s_, k, hh, d = 2, 3, 4, 2, 3
    x = _tiny(50, (b * s_, k))
    w = [_tiny(51 + i, (k, hh * d)) for i in range(3)]
    bs = [_tiny(54 + i, (hh * d,)) for i in range(3)]
    got = oracle.qkv(x, w[0], w[1], w[2], bs[0], bs[1], bs[2], b, hh, head_major=True)
    for i in range(3):
        ref = np.zeros((b, hh, s_, d))
        for bi in range(b):
            for si in range(s_):
                for h in range(hh):
                    for di in range(d):
                        ref[bi, h, si, di] = sum(x[bi * s_ + si, kk] * w[i][kk, h * d + di] for kk in range(k)) \
                            + bs[i][h * d + di]
        np.testing.assert_allclose(got[i], ref, rtol=0, atol=1e-13)
    flat = oracle.qkv(x, w[0], w[1], w[2], bs[0], bs[1], bs[2], b, hh, head_major=False)
    for i in range(3):
        assert flat[i].shape == (b, s_, hh, d)
        np.testing.assert_array_equal(flat[i].transpose(0, 2, 1, 3), got[i])
    other = oracle.qkv(x, w[0], 2 * w[1], w[2], bs[0], bs[1], None, b, hh, head_major=True)
    np.testing.assert_array_equal(other[0], got[0])
    np.testing.assert_allclose(other[1], 2 * (got[1] - bs[1].reshape(hh, 1, d)) + bs[1].reshape(hh, 1, d), rtol=0, atol=1e-13)
    np.testing.assert_allclose(other[2], got[2] - bs[2].reshape(hh, 1, d), rtol=0, atol=1e-13)


def test_attn_bias_brute(oracle):
    # bias [1, Hh, S, S] broadcast over the batch, added after the scale and before the softmax
    b, hh, s, d = 2, 2, 5, 3
    q, k, v = _tiny(43, (b, hh, s, d), -2, 2), _tiny(44, (b, hh, s, d), -2, 2), _tiny(45, (b, hh, s, d))
    bs = _tiny(46, (1, hh, s, s), -3, 3)
    ref = np.zeros((b, hh, s, d))
    for bi in range(b):
        for h in range(hh):
            for i in range(s):
                sc = [0.5 * sum(q[bi, h, i, t] * k[bi, h, j, t] for t in range(d)) + bs[0, h, i, j] for j in range(s)]
                den = sum(math.exp(z) for z in sc)
                for t in range(d):
                    ref[bi, h, i, t] = sum(math.exp(sc[j]) / den * v[bi, h, j, t] for j in range(s))
    np.testing.assert_allclose(oracle.attn_bias(q, k, v, bs, 0.5), ref, rtol=0, atol=1e-13)


def test_attn_bias_properties(oracle):
    def attn_kv(q_, k_, v_, c):       # the chain with a key count that differs from the query count
        return oracle.bmm_nn(oracle.softmax_rows(oracle.scale(oracle.bmm_nt(q_, k_), c)), v_)

    b, hh, s, d = 2, 2, 7, 4
    q, k, v = _tiny(94, (b, hh, s, d), -2, 2), _tiny(95, (b, hh, s, d), -2, 2), _tiny(96, (b, hh, s, d))
    o = oracle.attn(q, k, v, 0.5)
    # a zero bias, and a bias that is constant along every row (softmax is shift invariant), change nothing
    np.testing.assert_allclose(oracle.attn_bias(q, k, v, np.zeros((1, 1, s, s)), 0.5), o, rtol=0, atol=1e-14)
    rows = np.broadcast_to(_tiny(97, (b, hh, s, 1), -4, 4), (b, hh, s, s))
    np.testing.assert_allclose(oracle.attn_bias(q, k, v, rows, 0.5), o, rtol=0, atol=1e-13)
    # a large negative bias on some keys removes them: the result is attention over the remaining keys
    keep = np.array([0, 2, 3, 6])
    mask = np.full((1, 1, s, s), -1e4)
    mask[..., keep] = 0.0
    np.testing.assert_allclose(oracle.attn_bias(q, k, v, mask, 0.5),
                               attn_kv(q, k[:, :, keep], v[:, :, keep], 0.5), rtol=0, atol=1e-13)
    # a bias of +log(2) on one key weighs it twice: the same as listing that key (and its value) twice
    dup = np.zeros((1, 1, s, s))
    dup[..., 4] = math.log(2.0)
    k2, v2 = np.concatenate([k, k[:, :, 4:5]], 2), np.concatenate([v, v[:, :, 4:5]], 2)
    np.testing.assert_allclose(oracle.attn_bias(q, k, v, dup, 0.5), attn_kv(q, k2, v2, 0.5), rtol=0, atol=1e-13)
    # the bias is not scaled: doubling the scale and halving q leaves the result alone only because
    # the bias stays outside the product
    bs = _tiny(98, (b, 1, s, s), -2, 2)
    np.testing.assert_allclose(oracle.attn_bias(0.5 * q, k, v, bs, 1.0), oracle.attn_bias(q, k, v, bs, 0.5),
                               rtol=0, atol=1e-13)
    # per-batch bias [B, 1, S, S]: batch 1's bias must not leak into batch 0
    bs2 = bs.copy()
    bs2[1] += _tiny(99, (1, s, s), -1, 1)
    np.testing.assert_allclose(oracle.attn_bias(q, k, v, bs2, 0.5)[0], oracle.attn_bias(q, k, v, bs, 0.5)[0],
                               rtol=0, atol=0)


# --------------------------------------------------------------------------
# delta / identity weights
# --------------------------------------------------------------------------

def test_dw_centre_delta_is_copy(oracle):
    x = _tiny(50, (1, 6, 7, 4))
    wd = np.zeros((3, 3, 4)); wd[1, 1, :] = 1.0
    np.testing.assert_array_equal(oracle.dwconv3x3(x, wd, 1), x)
    np.testing.assert_array_equal(oracle.dwconv3x3(x, wd, 2), x[:, ::2, ::2, :])


def test_dw_corner_delta_shifts_without_flip(oracle):
    """w[0][0]=1 reads the pixel up-left: y[h][w] = x[h-1][w-1], first row/col zero."""
    x = _tiny(51, (1, 5, 6, 2))
    wd = np.zeros((3, 3, 2)); wd[0, 0, :] = 1.0
    y = oracle.dwconv3x3(x, wd, 1)
    assert np.all(y[:, 0, :, :] == 0) and np.all(y[:, :, 0, :] == 0)
    np.testing.assert_array_equal(y[:, 1:, 1:, :], x[:, :-1, :-1, :])
    wd = np.zeros((3, 3, 2)); wd[2, 1, :] = 1.0      # reads the pixel below
    y = oracle.dwconv3x3(x, wd, 1)
    assert np.all(y[:, -1, :, :] == 0)
    np.testing.assert_array_equal(y[:, :-1, :, :], x[:, 1:, :, :])


def test_conv3x3_delta_identity(oracle):
    x = _tiny(52, (2, 4, 5, 3))
    w = np.zeros((3, 3, 3, 3)); w[1, 1] = np.eye(3)
    np.testing.assert_array_equal(oracle.conv3x3(x, w), x)
    w = np.zeros((3, 3, 3, 3)); w[1, 2] = np.eye(3)   # reads the pixel to the right
    y = oracle.conv3x3(x, w)
    assert np.all(y[:, :, -1, :] == 0)
    np.testing.assert_array_equal(y[:, :, :-1, :], x[:, :, 1:, :])


def test_invres_padding_pads_the_intermediate(oracle):
    """With identity pointwise weights and a corner-delta depthwise kernel the block is a
    shifted copy of relu6(x + b1); the border that reads padding must be exactly bd's
    activation of 0 (the *intermediate* is padded with 0), not relu6(b1) shifted in."""
    c = 3
    x = rng.uniform(53, (1, 5, 5, c), 0.5, 1.5)
    eye = np.eye(c)
    b1 = np.full(c, 0.25); bd = np.zeros(c); b2 = np.zeros(c)
    wd = np.zeros((3, 3, c)); wd[0, 0, :] = 1.0
    y = oracle.invres(x, eye, b1, wd, bd, eye, b2, 1, False)
    assert np.all(y[:, 0, :, :] == 0.0) and np.all(y[:, :, 0, :] == 0.0)
    np.testing.assert_allclose(y[:, 1:, 1:, :], x[:, :-1, :-1, :] + 0.25, rtol=0, atol=1e-15)


def test_chain_padding_pads_the_intermediate(oracle):
    c = 2
    x = rng.uniform(54, (1, 4, 4, c), 0.5, 1.5)
    wa = np.zeros((3, 3, c, c)); wa[1, 1] = np.eye(c)
    wb = np.zeros((3, 3, c, c)); wb[0, 1] = np.eye(c)          # reads the pixel above
    ba = np.full(c, 0.5); bb = np.zeros(c)
    y = oracle.conv_chain(x, wa, ba, wb, bb, residual=False)
    assert np.all(y[:, 0, :, :] == 0.0)          # not relu(ba) = 0.5
    np.testing.assert_allclose(y[:, 1:, :, :], x[:, :-1, :, :] + 0.5, rtol=0, atol=1e-15)


# --------------------------------------------------------------------------
# all-ones closed forms: window counts
# --------------------------------------------------------------------------

def test_all_ones_counts_stride1(oracle):
    x = np.ones((1, 6, 7, 1)); w = np.ones((3, 3, 1))
    y = oracle.dwconv3x3(x, w, 1)[0, :, :, 0]
    assert y[0, 0] == 4 and y[0, -1] == 4 and y[-1, 0] == 4 and y[-1, -1] == 4
    assert np.all(y[0, 1:-1] == 6) and np.all(y[1:-1, 0] == 6)
    assert np.all(y[1:-1, 1:-1] == 9)
    y3 = oracle.conv3x3(np.ones((1, 6, 7, 2)), np.ones((3, 3, 2, 1)))[0, :, :, 0]
    np.testing.assert_array_equal(y3, 2 * y)


def test_all_ones_counts_stride2_56(oracle):
    """56 -> 28 with stride 2, pad 1: the first output row/col touches padding, the last
    reads rows 53..55 and does not."""
    y = oracle.dwconv3x3(np.ones((1, 56, 56, 1)), np.ones((3, 3, 1)), 2)[0, :, :, 0]
    assert y.shape == (28, 28)
    assert y[0, 0] == 4 and np.all(y[0, 1:] == 6) and np.all(y[1:, 0] == 6)
    assert np.all(y[1:, 1:] == 9)


def test_output_size_odd_input(oracle):
    assert oracle.dwconv3x3(np.ones((1, 9, 11, 1)), np.ones((3, 3, 1)), 2).shape == (1, 5, 6, 1)


# --------------------------------------------------------------------------
# linearity, library special cases
# --------------------------------------------------------------------------

def test_linearity_of_complex_ops(oracle):
    x1, x2 = _tiny(60, (1, 5, 6, 3)), _tiny(61, (1, 5, 6, 3))
    a, b = 0.7, -1.3
    w1, wd, w3 = _tiny(62, (3, 4)), _tiny(63, (3, 3, 3)), _tiny(64, (3, 3, 3, 2))
    for f in (lambda t: oracle.conv1x1(t, w1), lambda t: oracle.dwconv3x3(t, wd, 2),
              lambda t: oracle.conv3x3(t, w3)):
        np.testing.assert_allclose(f(a * x1 + b * x2), a * f(x1) + b * f(x2), rtol=0, atol=1e-13)


def test_invres_is_affine_inside_the_clamps(oracle):
    """Positive weights and inputs keep every pre-activation in (0, 6): the block is linear."""
    c = wl.InvresCase(1, 6, 6, 4, 8, 4, 1, False, False, "f32", 70)
    t = c.tensors()
    w1, wd, w2 = np.abs(t["w1"]) * 0.2, np.abs(t["wd"]) * 0.2, t["w2"]
    x1, x2 = rng.uniform(71, (1, 6, 6, 4), 0.1, 1), rng.uniform(72, (1, 6, 6, 4), 0.1, 1)
    f = lambda x: oracle.invres(x, w1, None, wd, None, w2, None, 1, False)
    np.testing.assert_allclose(f(0.3 * x1 + 0.6 * x2), 0.3 * f(x1) + 0.6 * f(x2), rtol=0, atol=1e-13)


def test_pointwise_is_matmul(oracle):
    x, w = _tiny(80, (2, 7, 5, 6)), _tiny(81, (6, 9))
    np.testing.assert_allclose(oracle.conv1x1(x, w), (x.reshape(-1, 6) @ w).reshape(2, 7, 5, 9),
                               rtol=0, atol=1e-13)
    a, b = _tiny(82, (17, 33)), _tiny(83, (33, 8))
    np.testing.assert_allclose(oracle.gemm(a, b), a @ b, rtol=0, atol=1e-13)
    q, k = _tiny(84, (3, 5, 4)), _tiny(85, (3, 6, 4))
    np.testing.assert_allclose(oracle.bmm_nt(q, k), np.einsum("bid,bjd->bij", q, k), rtol=0, atol=1e-13)
    p, v = _tiny(86, (3, 5, 6)), _tiny(87, (3, 6, 4))
    np.testing.assert_allclose(oracle.bmm_nn(p, v), np.einsum("bij,bjd->bid", p, v), rtol=0, atol=1e-13)


def test_conv3x3_one_by_one_image_is_centre_tap_matmul(oracle):
    x, w = _tiny(88, (3, 1, 1, 4)), _tiny(89, (3, 3, 4, 5))
    np.testing.assert_allclose(oracle.conv3x3(x, w).reshape(3, 5), x.reshape(3, 4) @ w[1, 1],
                               rtol=0, atol=1e-14)


# --------------------------------------------------------------------------
# simple operators
# --------------------------------------------------------------------------

def test_gelu_identities(oracle):
    x = np.linspace(-12, 12, 4801)
    g = oracle.gelu_tanh(x)
    assert oracle.gelu_tanh(np.zeros(1))[0] == 0.0
    np.testing.assert_allclose(g - g[::-1], x, rtol=0, atol=1e-14)       # gelu(x) - gelu(-x) = x
    big = x >= 10
    np.testing.assert_allclose(g[big], x[big], rtol=0, atol=1e-12)
    assert np.all(np.abs(g[x <= -10]) < 1e-12)
    pos = g[x > 0]
    assert np.all(np.diff(pos) > 0)
    # one value computed by hand from the definition: x = 1
    u = math.sqrt(2 / math.pi) * (1 + 0.044715)
    assert abs(oracle.gelu_tanh(np.ones(1))[0] - 0.5 * (1 + math.tanh(u))) < 1e-15
    # the tanh form stays within 5e-4 of the erf form it approximates
    erf_form = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in x])
    assert np.max(np.abs(g - erf_form)) < 5e-4


def test_relu_relu6_bias_add(oracle):
    x = np.array([-3.0, -0.0, 0.0, 2.5, 6.0, 7.5])
    np.testing.assert_array_equal(oracle.relu(x), [0, 0, 0, 2.5, 6.0, 7.5])
    np.testing.assert_array_equal(oracle.relu6(x), [0, 0, 0, 2.5, 6.0, 6.0])
    y = oracle.bias(np.zeros((2, 3, 4)), np.array([1.0, 2.0, 3.0, 4.0]))
    assert np.all(y == np.array([1.0, 2.0, 3.0, 4.0]))
    np.testing.assert_array_equal(oracle.add(x, x), 2 * x)


def test_softmax_properties(oracle):
    s = _tiny(90, (7, 13), -5, 5)
    p = oracle.softmax_rows(s)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=0, atol=1e-14)
    np.testing.assert_allclose(oracle.softmax_rows(s + 100.0), p, rtol=0, atol=1e-13)
    np.testing.assert_allclose(oracle.softmax_rows(np.zeros((2, 8))), 1 / 8, rtol=0, atol=0)
    two = oracle.softmax_rows(np.array([[0.0, math.log(3.0)]]))
    np.testing.assert_allclose(two, [[0.25, 0.75]], rtol=0, atol=1e-15)
    assert np.all(np.isfinite(oracle.softmax_rows(np.array([[1e4, -1e4, 0.0]]))))


def test_attention_properties(oracle):
    b, hh, s, d = 1, 2, 9, 4
    q, k, v = _tiny(91, (b, hh, s, d), -2, 2), _tiny(92, (b, hh, s, d), -2, 2), _tiny(93, (b, hh, s, d))
    o = oracle.attn(q, k, v, 0.5)
    # q = 0 -> uniform weights -> column mean of v
    o0 = oracle.attn(np.zeros_like(q), k, v, 0.5)
    np.testing.assert_allclose(o0, np.broadcast_to(v.mean(2, keepdims=True), v.shape), rtol=0, atol=1e-14)
    # permuting keys and values together changes nothing
    perm = np.array([3, 1, 8, 0, 2, 7, 6, 5, 4])
    np.testing.assert_allclose(oracle.attn(q, k[:, :, perm], v[:, :, perm], 0.5), o, rtol=0, atol=1e-13)
    # sequence length 1 -> o = v
    np.testing.assert_allclose(oracle.attn(q[:, :, :1], k[:, :, :1], v[:, :, :1], 0.5), v[:, :, :1],
                               rtol=0, atol=0)
    # scale enters before the softmax: doubling q equals doubling the scale
    np.testing.assert_allclose(oracle.attn(2 * q, k, v, 0.25), o, rtol=0, atol=1e-13)
    # outputs are convex combinations of the value rows
    assert np.all(o <= v.max(2, keepdims=True) + 1e-14) and np.all(o >= v.min(2, keepdims=True) - 1e-14)


# --------------------------------------------------------------------------
# fused == un-fused: the subgraph functions against the operators called one by one
# --------------------------------------------------------------------------

def test_subgraphs_equal_op_by_op(oracle):
    for case in wl.small_cases():
        t = case.tensors()
        kind = type(case).__name__
        if kind == "InvresCase":
            e = oracle.conv1x1(t["x"], t["w1"])
            if t["b1"] is not None: e = oracle.bias(e, t["b1"])
            e = oracle.relu6(e)
            d = oracle.dwconv3x3(e, t["wd"], case.stride)
            if t["bd"] is not None: d = oracle.bias(d, t["bd"])
            d = oracle.relu6(d)
            y = oracle.conv1x1(d, t["w2"])
            if t["b2"] is not None: y = oracle.bias(y, t["b2"])
            if case.residual: y = oracle.add(y, t["x"])
        elif kind == "ChainCase":
            a = oracle.relu(oracle.bias(oracle.conv3x3(t["x"], t["wa"]), t["ba"]))
            y = oracle.bias(oracle.conv3x3(a, t["wb"]), t["bb"])
            if case.residual: y = oracle.add(y, t["x"])
            y = oracle.relu(y)
        elif kind == "FfnCase":
            if case.M > 100: continue
            h = oracle.gelu_tanh(oracle.bias(oracle.gemm(t["x"], t["w1"]), t["b1"]))
            y = oracle.bias(oracle.gemm(h, t["w2"]), t["b2"])
        else:
            if case.S > 128: continue
            p = oracle.softmax_rows(oracle.scale(oracle.bmm_nt(t["q"], t["k"]), case.scale))
            y = oracle.bmm_nn(p, t["v"])
        np.testing.assert_array_equal(oracle.run_case(case), y)


# --------------------------------------------------------------------------
# input generator sanity (not part of the method, but both sides rely on it)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("stride", [1, 2])
def test_pair_pw_dw_brute(oracle, stride):
    """pw -> dw pair against the paper's loop nest: pointwise, bias, ReLU6, then a depthwise pass
    over the zero-padded activated tensor."""
    x = _tiny(901, (1, 5, 6, 3)); w1 = _tiny(902, (3, 4)); wd = _tiny(903, (3, 3, 4))
    b1 = _tiny(904, (4,), -0.3, 0.3); bd = _tiny(905, (4,), -0.3, 0.3)
    e = brute_bias_act(brute_conv_nchw(nhwc_to_lists(x), w1x1_to_oihw(w1), 0, 1), b1.tolist(), "relu6")
    d = brute_bias_act(brute_conv_nchw(e, wdw_to_oihw(wd), 1, stride, groups_depthwise=True), bd.tolist(), "relu6")
    np.testing.assert_allclose(oracle.pw_dw(x, w1, b1, wd, bd, stride), lists_to_nhwc(d), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("stride", [1, 2])
def test_pair_dw_pw_brute(oracle, stride):
    x = _tiny(911, (2, 4, 5, 3)); wd = _tiny(912, (3, 3, 3)); w2 = _tiny(913, (3, 5))
    bd = _tiny(914, (3,), -0.3, 0.3); b2 = _tiny(915, (5,), -0.3, 0.3)
    d = brute_bias_act(brute_conv_nchw(nhwc_to_lists(x), wdw_to_oihw(wd), 1, stride, groups_depthwise=True), bd.tolist(), "relu6")
    y = brute_bias_act(brute_conv_nchw(d, w1x1_to_oihw(w2), 0, 1), b2.tolist(), "none")
    np.testing.assert_allclose(oracle.dw_pw(x, wd, bd, w2, b2, stride), lists_to_nhwc(y), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("stride", [1, 2])
def test_pair_dw_dw_brute(oracle, stride):
    x = _tiny(931, (1, 6, 5, 3)); wa = _tiny(932, (3, 3, 3)); wb = _tiny(933, (3, 3, 3))
    ba = _tiny(934, (3,), -0.3, 0.3); bb = _tiny(935, (3,), -0.3, 0.3)
    t = brute_bias_act(brute_conv_nchw(nhwc_to_lists(x), wdw_to_oihw(wa), 1, stride, groups_depthwise=True), ba.tolist(), "relu6")
    y = brute_bias_act(brute_conv_nchw(t, wdw_to_oihw(wb), 1, 1, groups_depthwise=True), bb.tolist(), "relu6")
    np.testing.assert_allclose(oracle.dw_dw(x, wa, ba, wb, bb, stride), lists_to_nhwc(y), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("stride", [1, 2])
def test_pairs_with_a_5x5_depthwise_brute(oracle, stride):
    """The two pairs with a 5 x 5 depthwise (zero padding 2) against the loop nest, and the closed form
    of an all-ones kernel on an all-ones image: 25 taps inside, 15 on an edge, 9 in a corner."""
    x = _tiny(941, (1, 6, 7, 3)); w1 = _tiny(942, (3, 4)); wd = _tiny(943, (5, 5, 4))
    b1 = _tiny(944, (4,), -0.3, 0.3); bd = _tiny(945, (4,), -0.3, 0.3)
    e = brute_bias_act(brute_conv_nchw(nhwc_to_lists(x), w1x1_to_oihw(w1), 0, 1), b1.tolist(), "relu6")
    d = brute_bias_act(brute_conv_nchw(e, wdw_to_oihw(wd), 2, stride, groups_depthwise=True), bd.tolist(), "relu6")
    np.testing.assert_allclose(oracle.pw_dw(x, w1, b1, wd, bd, stride), lists_to_nhwc(d), rtol=1e-12, atol=1e-12)
    x2 = _tiny(946, (2, 5, 6, 4)); w2 = _tiny(947, (4, 3)); b2 = _tiny(948, (3,), -0.3, 0.3)
    d2 = brute_bias_act(brute_conv_nchw(nhwc_to_lists(x2), wdw_to_oihw(wd), 2, stride, groups_depthwise=True), bd.tolist(), "relu6")
    y2 = brute_bias_act(brute_conv_nchw(d2, w1x1_to_oihw(w2), 0, 1), b2.tolist(), "none")
    np.testing.assert_allclose(oracle.dw_pw(x2, wd, bd, w2, b2, stride), lists_to_nhwc(y2), rtol=1e-12, atol=1e-12)
    if stride == 1:
        ones = oracle.pw_dw(np.ones((1, 7, 7, 2)), np.eye(2), None, np.full((5, 5, 2), 0.2), None, 1)[0, :, :, 0]
        assert ones[3, 3] == pytest.approx(5.0) and ones[0, 3] == pytest.approx(3.0) and ones[0, 0] == pytest.approx(1.8)
        assert ones[1, 1] == pytest.approx(16 * 0.2) and ones[6, 6] == pytest.approx(1.8)


def test_pairs_compose_to_the_block_and_to_the_ffn(oracle):
    """pw_dw followed by the projection, and the expansion followed by dw_pw, both give the
    inverted residual; pw_pw on an NHWC tensor is the FFN chain on its rows."""
    x = _tiny(921, (1, 6, 7, 4)); w1 = _tiny(922, (4, 8)); wd = _tiny(923, (3, 3, 8)); w2 = _tiny(924, (8, 4))
    b1 = _tiny(925, (8,), -0.2, 0.2); bd = _tiny(926, (8,), -0.2, 0.2); b2 = _tiny(927, (4,), -0.2, 0.2)
    full = oracle.invres(x, w1, b1, wd, bd, w2, b2, 2, False)
    via_pw_dw = oracle.bias(oracle.conv1x1(oracle.pw_dw(x, w1, b1, wd, bd, 2), w2), b2)
    via_dw_pw = oracle.dw_pw(oracle.relu6(oracle.bias(oracle.conv1x1(x, w1), b1)), wd, bd, w2, b2, 2)
    np.testing.assert_allclose(via_pw_dw, full, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(via_dw_pw, full, rtol=1e-13, atol=1e-13)
    h = oracle.pw_pw(x, w1, b1, w2, b2, "gelu_tanh")
    f = oracle.ffn(x.reshape(-1, 4), w1, b1, w2, b2)
    np.testing.assert_allclose(h.reshape(-1, 4), f, rtol=1e-13, atol=1e-13)


def test_generator_is_counter_based_and_calibrated():
    a = rng.uniform(123, (1000,), -1, 1)
    b = rng.uniform(123, (4000,), -1, 1)
    np.testing.assert_array_equal(a, b[:1000])            # element i depends on (seed, i) only
    assert abs(b.mean()) < 0.05 and abs(b.var() - 1 / 3) < 0.02
    z = rng.normal(7, (200000,), 2.0)
    assert abs(z.mean()) < 0.02 and abs(z.std() - 2.0) < 0.02
    assert abs(np.mean(z ** 4) / z.var() ** 2 - 3.0) < 0.1
    assert not np.array_equal(rng.uniform(124, (10,)), rng.uniform(123, (10,)))


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -2.5, 0.0, 3.140625])
    r = rng.round_to_bf16(x)
    np.testing.assert_array_equal(r, [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7, -2.5, 0.0, 3.140625])
    bits = rng.bf16_bits(np.array([1.0, -2.0]))
    assert bits.tolist() == [0x3F80, 0xC000]
    np.testing.assert_array_equal(rng.bf16_from_bits(bits), [1.0, -2.0])


def test_baseline_shapes_and_work_counts():
    c = [wl.baseline_case(i) for i in range(5)]
    assert [k.flops() for k in c] == [5494272, 30933504, 3699376128, 19327352832, 3623878656]
    assert [k.alg_bytes() for k in c] == [107904, 219424, 6570496, 15744000, 18874368]
