"""Host-side checks that need no GPU: the shared library loads, exports every symbol the header
declares, rejects bad arguments before touching HIP, sizes workspaces, and its recompute model
reproduces the closed forms of the paper's redundancy analysis (Sec. III-B)."""

import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ago.h")
LIB = os.path.join(ROOT, "paper_2212_01005_amd", "libago.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2212_01005_amd import build
        build.build()
    return ctypes.CDLL(LIB)


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ago_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for must in ("ago_fused_invres", "ago_fused_ffn", "ago_fused_conv_chain", "ago_fused_attn",
                 "ago_gemm", "ago_conv1x1", "ago_dwconv3x3", "ago_conv3x3", "ago_bias_act",
                 "ago_add_act", "ago_softmax_rows", "ago_bmm_nt", "ago_bmm_nn",
                 "ago_unfused_invres", "ago_unfused_ffn", "ago_workspace_bytes", "ago_status_string"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), "libago.so does not export " + name


def test_binding_covers_every_declared_symbol(lib):
    from paper_2212_01005_amd import binding
    assert set(declared_functions()) == set(binding.EXPORTED)


def _fake(addr=0x1000):
    return ctypes.c_void_p(addr)


def test_pair_entry_points_validate_before_any_gpu_call(lib):
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    p = _fake()
    lib.ago_fused_pw_dw.argtypes = [vp] * 6 + [ci] * 7 + [vp, sz, vp]
    pwdw = lambda N, H, W, Cin, Cexp, st, dt=1, x=p: lib.ago_fused_pw_dw(
        x, p, None, p, None, p, N, H, W, Cin, Cexp, st, dt, None, 0, None)
    assert pwdw(1, 8, 8, 16, 96, 1, x=None) == 1
    assert pwdw(1, 8, 8, 16, 96, 3) == 2                                  # stride
    assert pwdw(1, 0, 8, 16, 96, 1) == 2
    assert pwdw(1, 8, 8, 16, 96, 1, dt=5) == 3
    assert pwdw(1, 8, 8, 16, 96, 1, x=_fake(0x1008)) == 4
    assert pwdw(1, 8, 8, 12, 96, 1) == 5                                  # Cin % 8
    assert pwdw(1, 8, 8, 16, 100, 1) == 5                                 # Cexp % 16
    lib.ago_fused_dw_pw.argtypes = [vp] * 6 + [ci] * 7 + [vp, sz, vp]
    dwpw = lambda N, H, W, C, Cout, st, dt=1, y=p: lib.ago_fused_dw_pw(
        p, p, None, p, None, y, N, H, W, C, Cout, st, dt, None, 0, None)
    assert dwpw(1, 8, 8, 96, 24, 1, y=None) == 1
    assert dwpw(1, 8, 8, 96, 24, 0) == 2
    assert dwpw(1, 8, 8, 90, 24, 1) == 5                                  # C % 16
    assert dwpw(1, 8, 8, 96, 20, 1) == 5                                  # Cout % 8
    lib.ago_fused_pw_pw.argtypes = [vp] * 6 + [ci] * 8 + [vp, sz, vp]
    pwpw = lambda N, H, W, C1, C2, C3, act=1, dt=1, ws=None, wsz=0: lib.ago_fused_pw_pw(
        p, p, None, p, None, p, N, H, W, C1, C2, C3, act, dt, ws, wsz, None)
    assert pwpw(0, 8, 8, 64, 128, 128) == 2
    assert pwpw(1, 8, 8, 64, 128, 128, act=11) == 3
    assert pwpw(1, 8, 8, 60, 128, 128) == 5                               # same divisibility rules as the FFN chain
    assert pwpw(1, 8, 8, 64, 768, 128) == 6                               # several hidden slices need a workspace
    ll = ctypes.c_longlong
    lib.ago_fused_attn_strided.argtypes = [vp] * 4 + [ci] * 4 + [ll] * 3 + [ctypes.c_float, ci, vp, sz, vp]
    att = lambda sb, sh, ss, D=64: lib.ago_fused_attn_strided(p, p, p, p, 2, 4, 100, D, sb, sh, ss, 0.125, 1, None, 0, None)
    assert att(0, 64, 256) == 2                                           # strides must be positive
    assert att(25600, 64, 32) == 2                                        # rows would overlap
    assert att(25600, 60, 256) == 4                                       # row starts must stay 16-byte aligned
    assert att(25600, 64, 256, D=32) == 5                                 # head dimension other than 64 / 128
    lib.ago_fused_invres_k.argtypes = [vp] * 8 + [ci] * 10 + [vp, sz, vp]
    irk = lambda ks, st=1, res=0, Cexp=96: lib.ago_fused_invres_k(p, p, None, p, None, p, None, p, 1, 8, 8, 16, Cexp, 16,
                                                              st, ks, res, 1, None, 0, None)
    assert irk(4) == 5 and irk(7) == 5 and irk(1) == 5                    # depthwise sizes 3 and 5 only
    assert irk(5, st=3) == 2
    assert irk(5, st=2, res=1) == 2                                       # a residual needs stride 1
    assert irk(5, Cexp=100) == 5
    lib.ago_fused_qkv.argtypes = [vp] * 10 + [ci] * 7 + [vp, sz, vp]
    qkv = lambda B=2, S=10, K=64, Hh=2, D=32, dt=1, x=p, v=p: lib.ago_fused_qkv(
        x, p, p, p, None, None, None, p, p, v, B, S, K, Hh, D, 1, dt, None, 0, None)
    assert qkv(x=None) == 1 and qkv(v=None) == 1
    assert qkv(S=0) == 2
    assert qkv(dt=9) == 3
    assert qkv(x=_fake(0x1008)) == 4
    assert qkv(dt=0) == 5                                                 # bf16 only
    assert qkv(K=60) == 5 and qkv(Hh=3, D=4) == 5                         # K % 8, (Hh D) % 8
    lib.ago_fused_attn_bias.argtypes = [vp] * 5 + [ci] * 4 + [ll] * 2 + [ctypes.c_float, ci, vp, sz, vp]
    atb = lambda sb, sh, bias=p, S=100: lib.ago_fused_attn_bias(p, p, p, bias, p, 2, 4, S, 64, sb, sh, 0.125, 1, None, 0, None)
    assert atb(0, 0, bias=None) == 1                                      # the bias is not optional here
    assert atb(0, 9999) == 2                                              # head stride below one [S][S] plane
    assert atb(30000, 10000) == 2                                         # batch stride below Hh planes
    assert atb(9999, 0) == 2                                              # batch stride below one plane
    assert atb(0, 0, bias=_fake(0x1001)) == 4                             # bf16 elements are 2-byte aligned
    assert atb(0, 0, S=0) == 2
    from paper_2212_01005_amd import binding as ago
    # the pair's workspace is the FFN chain's on N*H*W rows
    assert ago.workspace_bytes(ago.OP_FUSED_PW_PW, [1, 8, 8, 64, 768, 128], ago.BF16) == \
        ago.workspace_bytes(ago.OP_FUSED_FFN, [64, 64, 768, 128], ago.BF16) > 0


def test_noalloc_entry_point_refuses_what_its_buffer_cannot_hold(lib):
    """ago_fused_invres_noalloc validates like ago_fused_invres_k and returns AGO_ERR_WORKSPACE (6), before any GPU
    call, when the partial sums of the preferred plan exceed the library's own scratch buffer."""
    vp, ci = ctypes.c_void_p, ctypes.c_int
    p = _fake()
    lib.ago_fused_invres_noalloc.argtypes = [vp] * 8 + [ci] * 10 + [vp]
    call = lambda N, H, W, Cin, Cexp, Cout, st=1, ks=3, res=0, dt=1, x=p: lib.ago_fused_invres_noalloc(
        x, p, None, p, None, p, None, p, N, H, W, Cin, Cexp, Cout, st, ks, res, dt, None)
    assert call(1, 7, 7, 160, 960, 160, x=None) == 1
    assert call(1, 7, 7, 160, 960, 160, st=3) == 2
    assert call(1, 7, 7, 160, 960, 160, ks=4) == 5
    assert call(1, 7, 7, 160, 960, 160, x=_fake(0x1004)) == 4
    assert call(32, 7, 7, 160, 960, 160) == 6            # 8 slices x 32 x 7 x 7 x 160 x 4 bytes > 4 MiB


def test_validation_runs_before_any_gpu_call(lib):
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.ago_fused_ffn.argtypes = [vp] * 6 + [ci] * 6 + [vp, sz, vp]
    p = _fake()
    ffn = lambda x, w1, w2, y, M, K, F, K2, act=3, dt=1, ws=None, wsz=0: lib.ago_fused_ffn(
        x, w1, None, w2, None, y, M, K, F, K2, act, dt, ws, wsz, None)
    assert ffn(None, p, p, p, 128, 64, 64, 64) == 1                       # NULL
    assert ffn(p, p, p, p, 128, 64, 64, 64, dt=7) == 3                    # dtype
    assert ffn(p, p, p, p, 128, 64, 64, 64, act=9) == 3                   # activation
    assert ffn(p, p, p, p, 0, 64, 64, 64) == 2                            # shape
    assert ffn(_fake(0x1004), p, p, p, 128, 64, 64, 64) == 4              # alignment
    assert ffn(p, p, p, p, 128, 64, 64, 64, dt=0) == 5                    # fp32 FFN unsupported
    assert ffn(p, p, p, p, 128, 64, 76, 64) == 5                          # F not a multiple of 8
    assert ffn(p, p, p, p, 128, 64, 72, 60) == 5                          # K2 not a multiple of 8
    assert ffn(p, p, p, p, 128, 96, 72, 64) == 5                          # K not a multiple of 64
    assert ffn(p, p, p, p, 128, 64, 3072, 768) == 6                       # workspace missing
    assert ffn(p, p, p, p, 128, 64, 3072, 768, ws=_fake(), wsz=16) == 6   # workspace too small

    lib.ago_fused_invres.argtypes = [vp] * 8 + [ci] * 9 + [vp, sz, vp]
    inv = lambda N, H, W, Cin, Cexp, Cout, st, res, dt=0, x=p: lib.ago_fused_invres(
        x, p, None, p, None, p, None, p, N, H, W, Cin, Cexp, Cout, st, res, dt, None, 0, None)
    assert inv(1, 14, 14, 32, 192, 32, 1, 1, x=None) == 1
    assert inv(1, 14, 14, 32, 192, 32, 3, 0) == 2                         # stride
    assert inv(1, 14, 14, 32, 192, 24, 1, 1) == 2                         # residual needs Cin == Cout
    assert inv(1, 14, 14, 32, 192, 32, 2, 1) == 2                         # residual needs stride 1
    assert inv(1, 14, 14, 30, 192, 32, 1, 0) == 5                         # Cin % 8

    lib.ago_fused_conv_chain.argtypes = [vp] * 6 + [ci] * 6 + [vp, sz, vp]
    assert lib.ago_fused_conv_chain(p, p, None, p, None, p, 1, 8, 8, 32, 0, 1, None, 0, None) == 5
    assert lib.ago_fused_conv_chain(p, p, None, p, None, p, 1, 8, 8, 64, 0, 0, None, 0, None) == 5
    assert lib.ago_fused_conv_chain(p, p, None, p, None, p, 1, -8, 8, 64, 0, 1, None, 0, None) == 2

    lib.ago_fused_attn.argtypes = [vp] * 4 + [ci] * 4 + [ctypes.c_float, ci, vp, sz, vp]
    assert lib.ago_fused_attn(p, p, p, None, 1, 1, 8, 64, 0.125, 1, None, 0, None) == 1
    assert lib.ago_fused_attn(p, p, p, p, 1, 1, 8, 32, 0.125, 1, None, 0, None) == 5
    assert lib.ago_fused_attn(p, p, p, p, 1, 1, 8, 64, -1.0, 1, None, 0, None) == 5

    lib.ago_gemm.argtypes = [vp] * 5 + [ci] * 5 + [vp]
    assert lib.ago_gemm(p, p, None, None, None, 8, 8, 8, 0, 1, None) == 1
    assert lib.ago_gemm(p, p, None, None, p, 8, 12, 8, 0, 1, None) == 5


def test_packed_weight_entry_points_validate_on_the_host(lib):
    """Weight pre-packing and the kernels that consume packed weights: sizes, divisibility rules and the
    workspace check all run before any GPU call."""
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.ago_packed_weight_bytes.argtypes = [ci, ci]
    lib.ago_packed_weight_bytes.restype = sz
    assert lib.ago_packed_weight_bytes(768, 3072) == 768 * 3072 * 2
    assert lib.ago_packed_weight_bytes(32, 16) == 1024                 # one fragment
    assert lib.ago_packed_weight_bytes(48, 16) == 0                    # K % 32
    assert lib.ago_packed_weight_bytes(32, 24) == 0                    # N % 16
    assert lib.ago_packed_weight_bytes(0, 16) == 0
    p = _fake()
    lib.ago_pack_weight.argtypes = [vp, vp, ci, ci, ci, vp]
    assert lib.ago_pack_weight(None, p, 32, 16, 1, None) == 1
    assert lib.ago_pack_weight(p, p, 32, 16, 0, None) == 5             # fp32
    assert lib.ago_pack_weight(p, p, 40, 16, 1, None) == 5
    assert lib.ago_pack_weight(p, _fake(0x1008), 32, 16, 1, None) == 4
    assert lib.ago_pack_weight(p, p, -32, 16, 1, None) == 2

    lib.ago_workspace_bytes.restype = sz
    lib.ago_workspace_bytes.argtypes = [ci, ctypes.POINTER(ci), ci, ci]
    dims = (ci * 4)(2000, 768, 3072, 768)
    need = lib.ago_workspace_bytes(12, dims, 4, 1)
    assert need == 8 * 2048 * 768 * 4                                  # 8 slices, rows padded to 64, fp32
    dims1 = (ci * 4)(64, 128, 384, 384)
    assert lib.ago_workspace_bytes(12, dims1, 4, 1) == 64 * 384 * 4    # one slice still goes through the workspace
    lib.ago_fused_ffn_packed.argtypes = [vp] * 6 + [ci] * 6 + [vp, sz, vp]
    ffn = lambda x, w1, w2, y, M, K, F, K2, act=3, dt=1, ws=None, wsz=0: lib.ago_fused_ffn_packed(
        x, w1, None, w2, None, y, M, K, F, K2, act, dt, ws, wsz, None)
    assert ffn(None, p, p, p, 128, 64, 64, 64) == 1
    assert ffn(p, p, p, p, 128, 64, 64, 64, dt=0) == 5
    assert ffn(p, p, p, p, 128, 96, 64, 64) == 5                       # K % 64
    assert ffn(p, p, p, p, 128, 64, 96, 64) == 5                       # F % 64
    assert ffn(p, p, p, p, 128, 64, 64, 72) == 5                       # K2 % 16
    assert ffn(p, p, p, p, 128, 1280, 64, 64) == 5                     # a row block of x no longer fits LDS
    assert ffn(p, p, p, p, 2000, 768, 3072, 768) == 6                  # workspace missing
    assert ffn(p, p, p, p, 2000, 768, 3072, 768, ws=p, wsz=need - 1) == 6

    lib.ago_gemm_packed.argtypes = [vp] * 4 + [ci] * 5 + [vp]
    assert lib.ago_gemm_packed(p, p, None, None, 128, 128, 192, 0, 1, None) == 1
    assert lib.ago_gemm_packed(p, p, None, p, 128, 128, 200, 0, 1, None) == 5      # N fits neither tiling
    assert lib.ago_gemm_packed(p, p, None, p, 128, 64, 192, 0, 1, None) == 5       # K % 128
    assert lib.ago_gemm_packed(p, p, None, p, 128, 256, 96, 0, 1, None) == 5       # narrow tiling needs K % 512
    lib.ago_unfused_ffn_packed.argtypes = [vp] * 6 + [ci] * 6 + [vp, sz, vp]
    assert lib.ago_unfused_ffn_packed(p, p, None, p, None, p, 128, 128, 192, 100, 3, 1, p, 1 << 20, None) == 5
    assert lib.ago_unfused_ffn_packed(p, p, None, p, None, p, 128, 128, 192, 192, 3, 1, None, 0, None) == 6


def test_tensors_of_two_to_the_31_elements_are_refused(lib):
    """Sizes whose element counts do not fit 32-bit offsets return UNSUPPORTED on the host (no GPU call)."""
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    p = _fake()
    lib.ago_fused_invres.argtypes = [vp] * 8 + [ci] * 9 + [vp, sz, vp]
    inv = lambda N, H, W, Cin, Cexp, Cout: lib.ago_fused_invres(
        p, p, None, p, None, p, None, p, N, H, W, Cin, Cexp, Cout, 1, 0, 1, None, 0, None)
    assert inv(4096, 1024, 1024, 8, 16, 8) == 5
    assert inv(64, 1024, 1024, 8, 48, 8) == 5                              # the expanded tensor counts too
    lib.ago_fused_conv_chain.argtypes = [vp] * 6 + [ci] * 6 + [vp, sz, vp]
    assert lib.ago_fused_conv_chain(p, p, None, p, None, p, 2048, 128, 128, 64, 0, 1, None, 0, None) == 5
    lib.ago_fused_attn.argtypes = [vp] * 4 + [ci] * 4 + [ctypes.c_float, ci, vp, sz, vp]
    assert lib.ago_fused_attn(p, p, p, p, 64, 64, 8192, 64, 0.125, 1, None, 0, None) == 5
    lib.ago_fused_ffn.argtypes = [vp] * 6 + [ci] * 6 + [vp, sz, vp]
    assert lib.ago_fused_ffn(p, p, None, p, None, p, 1 << 20, 4096, 64, 64, 3, 1, None, 0, None) == 5
    lib.ago_gemm.argtypes = [vp] * 5 + [ci] * 5 + [vp]
    assert lib.ago_gemm(p, p, None, None, p, 1 << 20, 4096, 8, 0, 1, None) == 5


def test_status_strings(lib):
    lib.ago_status_string.restype = ctypes.c_char_p
    lib.ago_status_string.argtypes = [ctypes.c_int]
    seen = set()
    for code in range(8):
        s = lib.ago_status_string(code).decode()
        assert s.startswith("AGO_") and s not in seen
        seen.add(s)
    assert lib.ago_status_string(99).decode().startswith("unknown")


def test_workspace_sizes(lib):
    from paper_2212_01005_amd import binding as ago
    # FFN 2048x768x3072x768 with the built-in 384-wide hidden slices: 8 fp32 partial matrices
    assert ago.workspace_bytes(ago.OP_FUSED_FFN, [2048, 768, 3072, 768], ago.BF16) == 8 * 2048 * 768 * 4
    assert ago.workspace_bytes(ago.OP_FUSED_FFN, [64, 64, 64, 64], ago.BF16) == 0       # single slice
    assert ago.workspace_bytes(ago.OP_FUSED_ATTN, [8, 12, 384, 64], ago.BF16) == 0
    assert ago.workspace_bytes(ago.OP_UNFUSED_FFN, [2048, 768, 3072, 768], ago.BF16) == 2048 * 3072 * 2
    assert ago.workspace_bytes(ago.OP_UNFUSED_ATTN, [8, 12, 384, 64], ago.BF16) == 96 * 384 * 384 * (4 + 2)
    assert ago.workspace_bytes(ago.OP_UNFUSED_INVRES, [1, 56, 56, 24, 144, 32, 2], ago.BF16) == \
        (56 * 56 + 28 * 28) * 144 * 2
    assert ago.workspace_bytes(ago.OP_UNFUSED_CONV_CHAIN, [8, 56, 56, 64], ago.BF16) == 8 * 56 * 56 * 64 * 2
    assert ago.workspace_bytes(ago.OP_FUSED_FFN, [0, 768, 3072, 768], ago.BF16) == 0


def test_tile_config_hook(lib):
    from paper_2212_01005_amd import binding as ago
    for op in (ago.OP_FUSED_INVRES, ago.OP_FUSED_CONV_CHAIN, ago.OP_FUSED_FFN, ago.OP_FUSED_ATTN):
        n = ago.num_tile_configs(op)
        assert n >= 1
        assert ago.set_tile_config(op, n) == -1
        assert ago.set_tile_config(op, n - 1) == 0
        assert ago.set_tile_config(op, -1) == 0
    assert ago.num_tile_configs(42) == 0 and ago.set_tile_config(42, 0) == -1
    # the FFN workspace follows the selected slice width
    ago.set_tile_config(ago.OP_FUSED_FFN, 1)      # 128-wide slices -> 24 partials
    try:
        assert ago.workspace_bytes(ago.OP_FUSED_FFN, [2048, 768, 3072, 768], ago.BF16) == 24 * 2048 * 768 * 4
    finally:
        ago.set_tile_config(ago.OP_FUSED_FFN, -1)


# ---- the redundancy model of Sec. III-B -------------------------------------------------

def _golden():
    rows = []
    with open(os.path.join(ROOT, "tests", "golden", "recompute_counts.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append([int(v) for v in line.split()])
    return rows


def test_recompute_model_matches_the_papers_closed_forms(lib):
    from paper_2212_01005_amd import binding as ago
    for (N, O1, O2, H2, W2, R2, C2, to2, th2, tw2, fused, unfused) in _golden():
        got = ago.fused_upstream_iterations(N, O1, O2, H2, W2, R2, C2, to2, th2, tw2)
        assert got == (fused, unfused)


def test_recompute_model_symbolic_forms(lib):
    from paper_2212_01005_amd import binding as ago
    import itertools
    for N, O1, O2, H2, W2, R2, C2 in itertools.product((1, 2), (3, 8), (4, 16), (6, 32), (16, 48), (1, 3), (1, 3)):
        # the 1 x 1 x 16 downstream tile of Fig. 5
        fused, unf = ago.fused_upstream_iterations(N, O1, O2, H2, W2, R2, C2, 1, 1, 16)
        assert fused == N * O2 * H2 * (W2 // 16) * O1 * R2 * (15 + C2)
        assert unf == N * O1 * (H2 + R2 - 1) * (W2 + C2 - 1)
        # Fig. 7b: pointwise downstream (R2 = C2 = 1) with all output channels in the tile -> no redundancy
        f2, u2 = ago.fused_upstream_iterations(N, O1, O2, H2, W2, 1, 1, O2, 1, 16)
        assert f2 == u2
        # untiled downstream -> no redundancy for any window
        f3, u3 = ago.fused_upstream_iterations(N, O1, O2, H2, W2, R2, C2, O2, H2, W2)
        assert f3 == u3
        # spatial tiling of a 3x3 downstream costs ((th+2)(tw+2))/(th tw) on the tile grid
        if R2 == 3 and C2 == 3 and H2 % 2 == 0:
            f4, _ = ago.fused_upstream_iterations(N, O1, O2, H2, W2, 3, 3, O2, 2, 16)
            assert f4 == N * O1 * (H2 // 2) * (W2 // 16) * 4 * 18
    assert ago.fused_upstream_iterations(1, 8, 8, 7, 16, 3, 3, 1, 2, 16)[0] == -1   # tile must divide


def test_planned_tilings_follow_the_papers_redundancy_algebra(lib):
    """The planners' recompute term is upstream work = |GS2/TS2 x (GS1/TS1 - GS2/TS2)| |TS1| (Sec. III-B): the
    executed / algorithmic ratio of the planned tiling equals the closed form: (TH+2)(TW+2) tiles / (N H W) for the
    3x3 chain (|TS2| < |TS1|), exactly 1 for the two "downstream pointwise" tilings (Fig. 7b)."""
    from paper_2212_01005_amd import binding as ago
    p = ago.fused_conv_chain_plan(8, 56, 56, 64)                # the benchmark shape: 7 x 14 tiles, one per compute unit
    assert (p["config"], p["tile_h"], p["tile_w"], p["workgroups"], p["rounds"]) == (0, 7, 14, 256, 1)
    assert abs(p["recompute"] - (9 * 16) / (7 * 14)) < 1e-12 and abs(p["recompute"] - 1.469) < 1e-3
    # the same number from the closed form below Fig. 5 (no padding there: its un-fused count is over the
    # (H2 + 2) x (W2 + 2) upstream image, the padded chain's over H x W)
    fused, _ = ago.fused_upstream_iterations(8, 64, 64, 56, 56, 3, 3, 64, 7, 14)
    assert fused == 8 * 8 * 4 * 64 * 9 * 16
    assert abs(p["recompute"] - fused / (8 * 64 * 56 * 56)) < 1e-12
    q = ago.fused_conv_chain_plan(1, 56, 56, 64)                # few tiles: smaller tiles, more re-computation
    assert (q["tile_h"], q["tile_w"], q["workgroups"]) == (7, 7, 64) and abs(q["recompute"] - 81 / 49) < 1e-12
    r = ago.fused_conv_chain_plan(2, 60, 60, 64)                # ragged: tiles x window / image
    tiles = 2 * -(-60 // r["tile_h"]) * -(-60 // r["tile_w"])
    assert r["workgroups"] == tiles
    assert abs(r["recompute"] - tiles * (r["tile_h"] + 2) * (r["tile_w"] + 2) / (2 * 60 * 60)) < 1e-12
    for dims in ((8, 12, 384, 64), (2, 12, 4096, 64), (3, 5, 100, 64), (8, 12, 384, 128)):
        a = ago.fused_attn_plan(*dims)
        assert abs(a["recompute"] - 1.0) < 1e-12
        assert a["workgroups"] == dims[0] * dims[1] * -(-dims[2] // a["queries"])
    for dims in ((2048, 768, 3072, 768), (100, 128, 392, 256), (8192, 1024, 4096, 1024)):
        f = ago.fused_ffn_plan(*dims)
        assert abs(f["recompute"] - 1.0) < 1e-12
    # the choices the measurements back: 96-query workgroups two to a compute unit for the benchmark shape
    # (within 1 % of the 192-query ones), 128-query workgroups for long sequences
    assert ago.fused_attn_plan(8, 12, 384, 64)["queries"] in (96, 192)
    assert ago.fused_attn_plan(2, 12, 4096, 64)["queries"] == 128
    # pinned candidate
    ago.set_tile_config(ago.OP_FUSED_CONV_CHAIN, 2)
    try:
        assert ago.fused_conv_chain_plan(8, 56, 56, 64)["tile_h"] == 8
    finally:
        ago.set_tile_config(ago.OP_FUSED_CONV_CHAIN, -1)
    with pytest.raises(ago.AgoError):
        ago.fused_conv_chain_plan(8, 56, 56, 32)
    with pytest.raises(ago.AgoError):
        ago.fused_attn_plan(8, 12, 384, 80)


def test_invres_plan_is_a_host_query(lib):
    """The tiling query runs without a GPU: plans fit LDS, large channel counts are chunked, more images cost
    more predicted time, and an explicit tile configuration is honoured."""
    from paper_2212_01005_amd import binding as ago
    small = ago.fused_invres_plan(1, 14, 14, 32, 192, 32, 1, 3, ago.F32)
    assert small["chunks"] == 1 and small["chunk_channels"] == 192 and 0 < small["lds_bytes"] <= 160 * 1024
    big = ago.fused_invres_plan(32, 7, 7, 160, 960, 160, 1, 3, ago.BF16)
    assert big["chunks"] > 1 and big["chunk_channels"] % 32 == 0 and big["lds_bytes"] <= 160 * 1024
    assert big["chunks"] * big["chunk_channels"] >= 960 > (big["chunks"] - 1) * big["chunk_channels"]
    t = [ago.fused_invres_plan(n, 28, 28, 40, 240, 40, 1, 3, ago.BF16)["predicted_us"] for n in (1, 8, 64, 512)]
    assert t[0] <= t[1] < t[2] < t[3]
    # with many images the planner moves to tiles with less halo per output pixel than the 2x2 of one image
    one = ago.fused_invres_plan(1, 28, 28, 40, 240, 40, 1, 3, ago.BF16)
    many = ago.fused_invres_plan(64, 28, 28, 40, 240, 40, 1, 3, ago.BF16)
    assert many["tile_h"] * many["tile_w"] > one["tile_h"] * one["tile_w"]
    k5 = ago.fused_invres_plan(8, 28, 28, 40, 240, 40, 1, 5, ago.BF16)
    assert k5["predicted_us"] > ago.fused_invres_plan(8, 28, 28, 40, 240, 40, 1, 3, ago.BF16)["predicted_us"]
    try:
        assert ago.set_tile_config(ago.OP_FUSED_INVRES, 5) == 0
        forced = ago.fused_invres_plan(8, 28, 28, 40, 240, 40, 1, 3, ago.BF16)
        assert (forced["config"], forced["tile_h"], forced["tile_w"]) == (5, 7, 7)
    finally:
        ago.set_tile_config(ago.OP_FUSED_INVRES, -1)
    # channel split: a wide block on one image asks for a workspace and, given it, spreads its chunks over
    # workgroups (one chunk each); with less workspace than that it keeps the one-workgroup-per-tile plan
    dims = [1, 7, 7, 160, 960, 160, 1, 3]
    need = ago.workspace_bytes(ago.OP_FUSED_INVRES, dims, ago.BF16)
    split = ago.fused_invres_plan(*dims, ago.BF16, need)
    assert split["split"] > 1 and split["chunks"] == 1 and need == split["split"] * 49 * 160 * 4
    assert split["split"] * split["chunk_channels"] >= 960 and split["chunk_channels"] % 32 == 0
    whole = ago.fused_invres_plan(*dims, ago.BF16, need - 1)
    assert whole["split"] < split["split"] and whole["predicted_us"] >= split["predicted_us"]
    assert ago.fused_invres_plan(*dims, ago.BF16, 0)["split"] == 1
    assert ago.workspace_bytes(ago.OP_FUSED_INVRES, [1, 14, 14, 32, 192, 32, 1], ago.F32) == 0      # narrow: no split
    assert ago.workspace_bytes(ago.OP_FUSED_INVRES, [512, 7, 7, 160, 960, 160, 1], ago.BF16) == 0   # chip already full
    assert ago.workspace_bytes(ago.OP_FUSED_DW_PW, [1, 7, 7, 960, 160, 1], ago.BF16) > 0
    try:                                                                  # explicit: tile 13 (1x1) + 16 * option 2 (64 wide)
        assert ago.set_tile_config(ago.OP_FUSED_INVRES, 16 * 2 + 13) == 0
        forced = ago.fused_invres_plan(*dims, ago.BF16, 1 << 30)
        assert (forced["tile_h"], forced["tile_w"], forced["chunk_channels"], forced["split"]) == (1, 1, 64, 15)
        with pytest.raises(ago.AgoError):
            ago.fused_invres_plan(*dims, ago.BF16, 0)                     # that configuration needs the workspace
    finally:
        ago.set_tile_config(ago.OP_FUSED_INVRES, -1)
    with pytest.raises(ago.AgoError):
        ago.fused_invres_plan(1, 14, 14, 32, 192, 32, 1, 4, ago.F32)       # depthwise size
    with pytest.raises(ago.AgoError):
        ago.fused_invres_plan(1, 14, 14, 30, 192, 32, 1, 3, ago.F32)       # Cin % 8


def test_binding_refuses_tensors_that_do_not_match_the_sizes_it_passes(lib):
    """The marshalling step checks device, layout, shape and element type of every tensor before the C
    call: a mismatch would be an out-of-bounds access on the GPU.  Checked here with CPU tensors (refused
    as such) and through the checker itself."""
    import torch
    from paper_2212_01005_amd import binding as ago
    x = torch.zeros(4, 8)
    with pytest.raises(ValueError, match="device"):
        ago.ago_fused_ffn.marshal(x, x, None, x, None, x)
    with pytest.raises(ValueError, match="required"):
        ago._want("x", None, (1,))
    ago._want("b", None, (1,), optional=True)

    class Fake:                     # stands in for a device tensor: only the attributes the check reads
        def __init__(self, shape, dtype=torch.bfloat16, contiguous=True):
            self.shape, self.dtype, self.is_cuda, self._c = torch.Size(shape), dtype, True, contiguous
        def is_contiguous(self):
            return self._c
    ago._want("w", Fake((8, 16)), (8, 16), torch.bfloat16)
    with pytest.raises(ValueError, match="shape"):
        ago._want("w", Fake((8, 16)), (16, 8), torch.bfloat16)
    with pytest.raises(ValueError, match="dtype"):
        ago._want("w", Fake((8, 16), torch.float32), (8, 16), torch.bfloat16)
    with pytest.raises(ValueError, match="contiguous"):
        ago._want("w", Fake((8, 16), contiguous=False), (8, 16))
    with pytest.raises(ValueError, match="dtype"):
        ago._want_bias("b1", Fake((16,), torch.bfloat16), 16)


def test_ffn_fuse_or_not_is_a_host_decision(lib):
    """Fuse or not comes from the planner's two time models (fused: workgroups x weight tiles + the fp32 partial sums
    of the hidden slices; un-fused: two products with fused epilogues).  Measured on an MI355X (fused / un-fused us):
    768 x 3072: M = 128: 28 / 74, 2048: 42 / 42, 4096: 78 / 80, 8192: 153 / 126, 16384: 358 / 254;
    1024 x 4096, M = 2048: 107 / 114; 512 x 2048: M = 2048: 39 / 68, 8192: 108 / 114."""
    from paper_2212_01005_amd import binding as ago
    assert ago.fused_ffn_pays(128, 768, 3072, 768)
    assert ago.fused_ffn_pays(2048, 768, 3072, 768)             # the benchmark shape: a tie, which goes to the fused kernel
    assert ago.fused_ffn_pays(4096, 768, 3072, 768)
    assert not ago.fused_ffn_pays(8192, 768, 3072, 768)
    assert not ago.fused_ffn_pays(16384, 768, 3072, 768) and not ago.fused_ffn_pays(32768, 768, 3072, 768)
    assert ago.fused_ffn_pays(2048, 1024, 4096, 1024)
    assert ago.fused_ffn_pays(2048, 512, 2048, 512) and ago.fused_ffn_pays(8192, 512, 2048, 512)
    assert ago.fused_ffn_pays(1, 64, 8, 8)
    plan = ago.fused_ffn_plan(2048, 768, 3072, 768)
    assert (plan["rows"], plan["slice"], plan["slices"], plan["workgroups"], plan["rounds"]) == (64, 384, 8, 256, 1)
    assert abs(plan["predicted_us"] - 42.2) < 5 and abs(plan["predicted_unfused_us"] - 41.7) < 5
    assert ago.fused_ffn_plan(8192, 768, 3072, 768)["fuse"] == 0
    with pytest.raises(ValueError):
        ago.fused_ffn_pays(0, 768, 3072, 768)
