"""GPU parity: every HIP entry point against the fp64 CPU oracle, element by element, on the
same seeded inputs, through the C ABI (ctypes binding).

Tolerance (spec bar): max relative error 1e-4 for fp32 storage, 2e-2 for bf16 storage with
fp32 accumulation.  "Relative" is taken per element against max(|oracle_i|, rms(oracle)) so that
exact zeros after a ReLU and sign changes do not make the ratio meaningless.
"""

import warnings

import numpy as np
import pytest

import workloads as wl
from workloads import rng

pytestmark = pytest.mark.gpu

RTOL = {"f32": 1e-4, "bf16": 2e-2}


def assert_close(got, ref, dtype, what="", scale=1.0):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in " + what
    rms = float(np.sqrt(np.mean(ref ** 2)))
    denom = np.maximum(np.abs(ref), rms if rms > 0 else 1.0)
    err = np.abs(got - ref) / denom
    worst = float(err.max())
    assert worst <= scale * RTOL[dtype], "%s: max rel err %.3e > %.1e at %s" % (
        what, worst, scale * RTOL[dtype], np.unravel_index(int(err.argmax()), err.shape))
    return worst


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2212_01005_amd import binding, runner
    return torch, binding, runner


def _cases():
    return wl.small_cases()


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c.name)
def test_fused_matches_oracle(gpu, oracle, case):
    torch, ago, runner = gpu
    t = runner.to_device(case)
    y = runner.alloc_output(case)
    ws = runner.alloc_workspace(case, fused=True)
    runner.run_fused(case, t, y, ws)
    torch.cuda.synchronize()
    assert_close(runner.to_numpy64(y), oracle.run_case(case), case.dtype, case.name)


@pytest.mark.parametrize("epilogue_fused", [0, 1])
@pytest.mark.parametrize("case", _cases(), ids=lambda c: c.name)
def test_unfused_matches_oracle(gpu, oracle, case, epilogue_fused):
    torch, ago, runner = gpu
    t = runner.to_device(case)
    y = runner.alloc_output(case)
    ws = runner.alloc_workspace(case, fused=False)
    runner.run_unfused(case, t, y, ws, epilogue_fused)
    torch.cuda.synchronize()
    assert_close(runner.to_numpy64(y), oracle.run_case(case), case.dtype, case.name)


@pytest.mark.parametrize("idx", range(5))
def test_fused_full_size_baseline(gpu, oracle, idx):
    """The five benchmark configurations at full size, in the launch configuration bench.py times."""
    torch, ago, runner = gpu
    case = wl.baseline_case(idx)
    t = runner.to_device(case)
    y = runner.alloc_output(case)
    ws = runner.alloc_workspace(case, fused=True)
    runner.run_fused(case, t, y, ws)
    torch.cuda.synchronize()
    ref = oracle.run_case(case)
    assert_close(runner.to_numpy64(y), ref, case.dtype, case.name)
    # determinism: a second run gives identical bits (no atomics in any reduction)
    y2 = runner.alloc_output(case)
    runner.run_fused(case, t, y2, ws)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)


@pytest.mark.parametrize("idx", range(5))
@pytest.mark.parametrize("epilogue_fused", [0, 1])
def test_unfused_full_size_baseline(gpu, oracle, idx, epilogue_fused):
    torch, ago, runner = gpu
    case = wl.baseline_case(idx)
    t = runner.to_device(case)
    y = runner.alloc_output(case)
    ws = runner.alloc_workspace(case, fused=False)
    runner.run_unfused(case, t, y, ws, epilogue_fused)
    torch.cuda.synchronize()
    assert_close(runner.to_numpy64(y), oracle.run_case(case), case.dtype, case.name)


def test_every_tile_config_gives_the_same_answer(gpu, oracle):
    """All selectable tile configurations of each fused kernel agree with the oracle
    (different tilings = different LDS hand-offs; a missing barrier would show here)."""
    torch, ago, runner = gpu
    picks = {"InvresCase": [c for c in _cases() if c.name in ("invres_f32_s1", "invres_bf16_s2")],
             "ChainCase": [c for c in _cases() if c.name == "chain_ragged"],
             "FfnCase": [c for c in _cases() if c.name == "ffn_ragged_rows"],
             "AttnCase": [c for c in _cases() if c.name in ("attn_s384", "attn_ragged_s100", "attn_long_s600")]}
    ops = {"InvresCase": ago.OP_FUSED_INVRES, "ChainCase": ago.OP_FUSED_CONV_CHAIN, "FfnCase": ago.OP_FUSED_FFN,
           "AttnCase": ago.OP_FUSED_ATTN}
    try:
        for kind, cases in picks.items():
            for case in cases:
                ref = oracle.run_case(case)
                t = runner.to_device(case)
                for cfg in range(ago.num_tile_configs(ops[kind])):
                    assert ago.set_tile_config(ops[kind], cfg) == 0
                    y = runner.alloc_output(case)
                    y.zero_()
                    try:
                        ws = runner.alloc_workspace(case, fused=True)
                        runner.run_fused(case, t, y, ws)
                    except ago.AgoError as e:
                        assert e.status == 5, e      # UNSUPPORTED for this shape is fine
                        continue
                    torch.cuda.synchronize()
                    assert_close(runner.to_numpy64(y), ref, case.dtype, "%s cfg %d" % (case.name, cfg))
    finally:
        for op in ops.values():
            ago.set_tile_config(op, -1)


def test_attention_strided_layout(gpu, oracle):
    """[B][S][Hh][D] tensors through the strided entry point give the [B][Hh][S][D] answer."""
    torch, ago, runner = gpu
    for case in (wl.AttnCase(2, 3, 200, 64, 0.125, "bf16", 6100, name="attn_bshd_s200"),
                 wl.AttnCase(1, 12, 384, 64, 0.125, "bf16", 6101, name="attn_bshd_s384")):
        ref = oracle.run_case(case)                                    # [B, Hh, S, D]
        t = runner.to_device(case)
        q, k, v = (t[n].permute(0, 2, 1, 3).contiguous() for n in ("q", "k", "v"))   # [B, S, Hh, D]
        o = torch.zeros_like(q)
        ago.ago_fused_attn_bshd(q, k, v, o, case.scale)
        torch.cuda.synchronize()
        assert_close(runner.to_numpy64(o.permute(0, 2, 1, 3)), ref, "bf16", case.name)


def test_attention_reference_moves_only_when_it_must(gpu, oracle):
    """The kernel keeps its softmax reference until some row's maximum grows by more than 2^8.  Scores whose
    scale rises along the keys (later blocks dominate: the reference has to move, and the accumulators are
    rescaled, in every block) and scores whose scale falls (it never moves again) both match the oracle, in
    every tile configuration, with ragged and long sequences."""
    torch, ago, runner = gpu
    for seed, S, ramp in ((6150, 384, 8.0), (6151, 384, 1.0 / 8.0), (6152, 600, 6.0), (6153, 100, 5.0), (6154, 1100, 3.0)):
        case = wl.AttnCase(1, 2, S, 64, 0.125, "bf16", seed, name="attn_ramp")
        t = case.tensors()
        gain = ramp ** (np.arange(S) / float(S - 1))                      # 1 at the first key, `ramp` at the last
        k = wl.round_to_bf16(t["k"] * gain[None, None, :, None])
        ref = oracle.attn(t["q"], k, t["v"], case.scale)
        dev = {n: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0").to(torch.bfloat16)
               for n, a in (("q", t["q"]), ("k", k), ("v", t["v"]))}
        try:
            for cfg in [-1] + list(range(ago.num_tile_configs(ago.OP_FUSED_ATTN))):
                ago.set_tile_config(ago.OP_FUSED_ATTN, cfg)
                o = torch.zeros_like(dev["q"])
                ago.ago_fused_attn(dev["q"], dev["k"], dev["v"], o, case.scale)
                torch.cuda.synchronize()
                assert_close(runner.to_numpy64(o), ref, "bf16", "attn ramp %g S %d cfg %d" % (ramp, S, cfg))
        finally:
            ago.set_tile_config(ago.OP_FUSED_ATTN, -1)


def test_attention_long_sequences(gpu, oracle):
    """Two dozen key blocks and more through the LDS ring (buffers re-used many times, the softmax reference
    carried across all of them): a ragged S = 3000 at head dimension 64 and S = 2048 at 128, both layouts."""
    torch, ago, runner = gpu
    for case in (wl.AttnCase(1, 2, 3000, 64, 0.125, "bf16", 6160, name="attn_s3000"),
                 wl.AttnCase(1, 2, 2048, 128, 0.0884, "bf16", 6161, name="attn_s2048_d128")):
        ref = oracle.run_case(case)
        t = runner.to_device(case)
        o = runner.alloc_output(case)
        o.zero_()
        runner.run_fused(case, t, o)
        torch.cuda.synchronize()
        assert_close(runner.to_numpy64(o), ref, "bf16", case.name)
        if case.D == 64:
            q, k, v = (t[n].permute(0, 2, 1, 3).contiguous() for n in ("q", "k", "v"))
            ob = torch.zeros_like(q)
            ago.ago_fused_attn_bshd(q, k, v, ob, case.scale)
            torch.cuda.synchronize()
            assert_close(runner.to_numpy64(ob.permute(0, 2, 1, 3)), ref, "bf16", case.name + " bshd")


def test_invres_5x5_depthwise(gpu, oracle):
    """The block with a 5x5 depthwise (2-pixel halo): both dtypes and strides, residual, ragged images,
    images smaller than the kernel, the built-in tile choice and explicit tile configurations."""
    torch, ago, runner = gpu
    cases = [wl.InvresCase(1, 14, 14, 40, 240, 40, 1, True, True, "f32", 6300, name="invres5_f32_s1_res", ksize=5),
             wl.InvresCase(1, 28, 28, 24, 144, 40, 2, False, False, "bf16", 6301, name="invres5_bf16_s2", ksize=5),
             wl.InvresCase(2, 9, 11, 16, 96, 24, 2, False, True, "f32", 6302, name="invres5_f32_s2_ragged", ksize=5),
             wl.InvresCase(2, 13, 10, 32, 192, 32, 1, True, True, "bf16", 6303, name="invres5_bf16_s1_res", ksize=5),
             wl.InvresCase(3, 1, 2, 8, 16, 8, 1, True, True, "f32", 6304, name="invres5_tiny", ksize=5),
             wl.InvresCase(1, 3, 3, 8, 48, 16, 2, False, True, "bf16", 6305, name="invres5_3x3_image", ksize=5)]
    for case in cases:
        ref = oracle.run_case(case)
        t = runner.to_device(case)
        try:
            ran = 0
            for cfg in (-1, 1, 3, 9, 13):
                ago.set_tile_config(ago.OP_FUSED_INVRES, cfg)
                y = runner.alloc_output(case)
                try:
                    runner.run_fused(case, t, y)
                except ago.AgoError as e:
                    assert cfg >= 0 and e.status == 5, e      # an explicit tile that does not fit LDS
                    continue
                ran += 1
                torch.cuda.synchronize()
                assert_close(runner.to_numpy64(y), ref, case.dtype, "%s cfg %d" % (case.name, cfg))
            assert ran >= 2, case.name
        finally:
            ago.set_tile_config(ago.OP_FUSED_INVRES, -1)


def test_invres_expanded_channels_in_chunks(gpu, oracle):
    """Blocks whose weights and expanded tensor exceed LDS (the 576-, 672- and 960-channel blocks of the
    mobile networks): the kernel walks the expanded channels in chunks and carries the projection's
    accumulators across them.  Full block in both dtypes, 5x5 depthwise, and both pairs."""
    torch, ago, runner = gpu
    cases = [wl.InvresCase(2, 7, 7, 160, 960, 160, 1, True, True, "bf16", 6400, name="invres_960_bf16"),
             wl.InvresCase(1, 14, 14, 96, 576, 96, 1, True, True, "f32", 6401, name="invres_576_f32"),
             wl.InvresCase(1, 14, 14, 112, 672, 160, 2, False, True, "bf16", 6402, name="invres5_672_s2_bf16", ksize=5),
             wl.InvresCase(1, 9, 7, 160, 944, 320, 1, False, False, "bf16", 6403, name="invres_944_ragged_chunk"),
             wl.PairCase("pw_dw", 1, 7, 7, 160, 960, stride=1, dtype="bf16", seed=6404, name="pw_dw_960"),
             wl.PairCase("dw_pw", 1, 7, 7, 960, 160, stride=1, dtype="bf16", seed=6405, name="dw_pw_960"),
             wl.PairCase("pw_dw", 1, 9, 9, 96, 576, stride=2, dtype="f32", seed=6406, name="pw_dw_576_f32_s2"),
             wl.PairCase("dw_pw", 1, 9, 9, 576, 96, stride=2, dtype="f32", seed=6407, name="dw_pw_576_f32_s2")]
    for case in cases:
        ref = oracle.run_case(case)
        t = runner.to_device(case)
        try:
            ran = 0
            for cfg in (-1, 1, 3, 5, 10):
                ago.set_tile_config(ago.OP_FUSED_INVRES, cfg)
                y = runner.alloc_output(case)
                y.zero_()
                try:
                    runner.run_fused(case, t, y)
                except ago.AgoError as e:
                    assert cfg >= 0 and e.status == 5, e      # an explicit tile that cannot run
                    continue
                ran += 1
                torch.cuda.synchronize()
                assert_close(runner.to_numpy64(y), ref, case.dtype, "%s cfg %d" % (case.name, cfg))
            assert ran >= 2, case.name
        finally:
            ago.set_tile_config(ago.OP_FUSED_INVRES, -1)


def test_invres_channel_split(gpu, oracle):
    """Wide blocks on few pixels with a workspace: the chunks of expanded channels go to different
    workgroups, fp32 partials are summed by a second kernel (with b2 and the residual).  The built-in
    plan (which must split these shapes), explicit split configurations, and the same call without
    workspace (one workgroup walks the chunks) all agree with the oracle."""
    torch, ago, runner = gpu
    cases = [wl.InvresCase(1, 7, 7, 160, 960, 160, 1, True, True, "bf16", 6600, name="split_960_bf16_res"),
             wl.InvresCase(1, 7, 7, 160, 960, 320, 1, False, True, "bf16", 6601, name="split_960_320"),
             wl.InvresCase(2, 14, 14, 96, 576, 96, 1, True, True, "f32", 6602, name="split_576_f32_res"),
             wl.InvresCase(1, 14, 14, 112, 672, 160, 2, False, True, "bf16", 6603, name="split5_672_s2", ksize=5),
             wl.InvresCase(1, 9, 7, 160, 944, 320, 1, False, False, "bf16", 6604, name="split_944_ragged_chunk"),
             wl.InvresCase(1, 5, 3, 64, 400, 64, 1, True, True, "f32", 6605, name="split_400_f32_ragged"),
             wl.PairCase("dw_pw", 1, 7, 7, 960, 160, stride=1, dtype="bf16", seed=6606, name="split_dw_pw_960"),
             wl.PairCase("dw_pw", 1, 9, 9, 576, 96, stride=2, dtype="f32", seed=6607, name="split_dw_pw_576_f32_s2")]
    for case in cases:
        ref = oracle.run_case(case)
        t = runner.to_device(case)
        ws = runner.alloc_workspace(case, fused=True)
        assert ws is not None, "%s: the built-in plan should ask for a workspace" % case.name
        big = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0")      # enough for any explicit split
        try:
            ran = 0
            for cfg, w in ((-1, ws), (-1, None), (16 * 1 + 13, big), (16 * 2 + 3, big), (16 * 4 + 5, big), (16 * 6 + 1, big)):
                ago.set_tile_config(ago.OP_FUSED_INVRES, cfg)
                y = runner.alloc_output(case)
                y.fill_(7.0)
                try:
                    runner.run_fused(case, t, y, w)
                except ago.AgoError as e:
                    assert cfg >= 0 and e.status == 5, e      # an explicit configuration that cannot run
                    continue
                ran += 1
                torch.cuda.synchronize()
                assert_close(runner.to_numpy64(y), ref, case.dtype, "%s cfg %d ws %s" % (case.name, cfg, w is not None))
            assert ran >= 3, case.name
        finally:
            ago.set_tile_config(ago.OP_FUSED_INVRES, -1)
    # the plan query reports the split, and falls back when the workspace is too small
    if True:
        full = ago.fused_invres_plan(1, 7, 7, 160, 960, 160, 1, 3, ago.BF16, 1 << 30)
        none = ago.fused_invres_plan(1, 7, 7, 160, 960, 160, 1, 3, ago.BF16, 0)
        assert full["split"] > 1 and full["chunks"] == 1 and none["split"] == 1 and none["chunks"] > 1
        need = ago.workspace_bytes(ago.OP_FUSED_INVRES, [1, 7, 7, 160, 960, 160, 1, 3], ago.BF16)
        assert need == full["split"] * 7 * 7 * 160 * 4
        assert ago.fused_invres_plan(1, 7, 7, 160, 960, 160, 1, 3, ago.BF16, need - 4)["split"] != full["split"]


def test_invres_planner_choice_is_near_the_best_candidate(gpu):
    """Report only (a warning, never a failure).  The built-in tile choice (cost model) is timed against every selectable tile on three shapes the
    model was not tuned for one by one: a latency-bound single image, a batch that fills the chip several
    times over, a chunked wide block, and a wide block on one image (channel split, with workspace)."""
    torch, ago, runner = gpu

    def us(fn, n=40):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n * 1e3

    for case in (wl.InvresCase(1, 28, 28, 24, 144, 24, 1, True, True, "bf16", 6500, name="plan_single"),
                 wl.InvresCase(16, 28, 28, 32, 192, 48, 1, False, True, "bf16", 6501, name="plan_batch16"),
                 wl.InvresCase(8, 14, 14, 80, 480, 112, 1, False, True, "bf16", 6502, name="plan_wide"),
                 wl.InvresCase(1, 7, 7, 160, 960, 160, 1, True, True, "bf16", 6503, name="plan_split")):
        t = runner.to_device(case)
        y = runner.alloc_output(case)
        ws = torch.empty(32 << 20, dtype=torch.uint8, device="cuda:0")
        times = {}
        try:
            for cfg in [-1] + list(range(ago.num_tile_configs(ago.OP_FUSED_INVRES))):
                ago.set_tile_config(ago.OP_FUSED_INVRES, cfg)
                try:
                    fn = runner.prepare_fused(case, t, y, ws)
                    fn()
                except ago.AgoError:
                    continue
                times[cfg] = us(fn)
        finally:
            ago.set_tile_config(ago.OP_FUSED_INVRES, -1)
        best = min(v for k, v in times.items() if k >= 0)
        print("%s built-in %.2f us, best candidate %.2f us" % (case.name, times[-1], best))
        # a timing is not a correctness result: a slow choice is reported, it does not fail the parity run
        if times[-1] > 1.25 * best + 1.0:
            warnings.warn("planner choice for %s: %.2f us against %.2f us for the best candidate" % (case.name, times[-1], best))


def test_planner_choices_of_the_chain_ffn_and_attention_kernels(gpu):
    """Report only (a warning, never a failure): the candidate the analytic planners pick is timed against every
    selectable candidate on shapes away from the benchmark's; a choice more than 10 % slower than the best
    candidate is reported."""
    torch, ago, runner = gpu

    def us(fn, n=30):
        for _ in range(4):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n * 1e3

    cases = [(wl.ChainCase(1, 56, 56, 64, True, "bf16", 6510, name="plan_chain_1x56"), ago.OP_FUSED_CONV_CHAIN),
             (wl.ChainCase(16, 28, 28, 64, True, "bf16", 6511, name="plan_chain_16x28"), ago.OP_FUSED_CONV_CHAIN),
             (wl.ChainCase(6, 80, 80, 64, True, "bf16", 6512, name="plan_chain_6x80"), ago.OP_FUSED_CONV_CHAIN),
             (wl.AttnCase(4, 12, 1536, 64, 0.125, "bf16", 6513, name="plan_attn_s1536"), ago.OP_FUSED_ATTN),
             (wl.AttnCase(24, 8, 256, 64, 0.125, "bf16", 6514, name="plan_attn_s256"), ago.OP_FUSED_ATTN),
             (wl.AttnCase(2, 6, 200, 64, 0.125, "bf16", 6515, name="plan_attn_s200"), ago.OP_FUSED_ATTN),
             (wl.FfnCase(1024, 768, 3072, 768, "bf16", 6516, name="plan_ffn_1024"), ago.OP_FUSED_FFN),
             (wl.FfnCase(3072, 512, 2048, 512, "bf16", 6517, name="plan_ffn_3072"), ago.OP_FUSED_FFN)]
    for case, op in cases:
        t = runner.to_device(case)
        y = runner.alloc_output(case)
        times = {}
        try:
            for cfg in [-1] + list(range(ago.num_tile_configs(op))):
                ago.set_tile_config(op, cfg)
                try:
                    fn = runner.prepare_fused(case, t, y, runner.alloc_workspace(case, fused=True))
                    fn()
                except ago.AgoError:
                    continue
                times[cfg] = us(fn)
        finally:
            ago.set_tile_config(op, -1)
        best = min(v for k, v in times.items() if k >= 0)
        print("%s built-in %.2f us, best candidate %.2f us" % (case.name, times[-1], best))
        if times[-1] > 1.10 * best:
            warnings.warn("planner choice for %s: %.2f us against %.2f us for the best candidate" % (case.name, times[-1], best))


def test_ffn_ragged_hidden_slices_and_column_blocks(gpu, oracle):
    """F and K2 that are not multiples of the streaming kernel's 384-wide hidden slices / column blocks
    (BERT-large's 1024 -> 4096 -> 1024 among them): the last slice / block is clamped and masked."""
    torch, ago, runner = gpu
    cases = [wl.FfnCase(100, 128, 520, 264, "bf16", 6700, name="ffn_f520_k264"),
             wl.FfnCase(70, 64, 8, 8, "bf16", 6701, name="ffn_f8_k8"),
             wl.FfnCase(130, 192, 392, 768, "bf16", 6702, name="ffn_f392"),
             wl.FfnCase(64, 256, 768, 1000, "bf16", 6703, name="ffn_k1000"),
             wl.FfnCase(512, 1024, 4096, 1024, "bf16", 6704, name="ffn_bert_large_512")]
    for case in cases:
        ref = oracle.run_case(case)
        t = runner.to_device(case)
        try:
            for cfg in (-1, 3, 4):
                ago.set_tile_config(ago.OP_FUSED_FFN, cfg)
                y = runner.alloc_output(case)
                y.zero_()
                runner.run_fused(case, t, y, runner.alloc_workspace(case, fused=True))
                torch.cuda.synchronize()
                assert_close(runner.to_numpy64(y), ref, "bf16", "%s cfg %d" % (case.name, cfg))
        finally:
            ago.set_tile_config(ago.OP_FUSED_FFN, -1)


def test_specialised_instantiations_match_the_general_kernel(gpu, oracle):
    """The shape-specialised instantiations of the inverted-residual kernel (compile-time geometry) against the
    general instantiation forced through the tile-configuration switch: the same arithmetic in the same order,
    so the outputs are bit-identical; and both match the oracle."""
    torch, ago, runner = gpu
    cases = [wl.baseline_case(0), wl.baseline_case(1)] + [c for c in wl.network_block_cases(1)
                                                           if c.name in ("block_112x112x16_96_24_s2", "block_28x28x32_192_64_s2",
                                                                         "block_14x14x64_384_96_s1", "block_7x7x160_960_160_s1")]
    for case in cases:
        dt = ago.BF16 if case.dtype == "bf16" else ago.F32
        t = runner.to_device(case)
        ws = runner.alloc_workspace(case, fused=True)
        plan = ago.fused_invres_plan(case.N, case.H, case.W, case.Cin, case.Cexp, case.Cout, case.stride, case.ksize, dt,
                                     ws.numel() if ws is not None else 0)
        y_spec = runner.alloc_output(case)
        y_spec.zero_()
        runner.run_fused(case, t, y_spec, ws)
        torch.cuda.synchronize()
        y_gen = runner.alloc_output(case)
        y_gen.zero_()
        try:
            ago.set_tile_config(ago.OP_FUSED_INVRES, plan["config"])      # the same tile, general instantiation
            runner.run_fused(case, t, y_gen, ws)
            torch.cuda.synchronize()
        finally:
            ago.set_tile_config(ago.OP_FUSED_INVRES, -1)
        assert torch.equal(y_spec, y_gen), case.name
        assert_close(runner.to_numpy64(y_spec), oracle.run_case(case), case.dtype, case.name)


def _packed_reference(w):
    """The packed layout written out from its definition: fragment (ks, nt), lane l, element e holds
    w[32 ks + 8 (l // 16) + e][16 nt + l % 16]."""
    K, N = w.shape
    ks, nt, l, e = np.meshgrid(np.arange(K // 32), np.arange(N // 16), np.arange(64), np.arange(8), indexing="ij")
    return w[32 * ks + 8 * (l // 16) + e, 16 * nt + l % 16]


def test_weight_packing_is_the_documented_permutation(gpu):
    torch, ago, runner = gpu
    for K, N in ((32, 16), (64, 48), (768, 3072), (3072, 768), (96, 400)):
        w = torch.arange(K * N, device="cuda", dtype=torch.float32).remainder_(251.0).reshape(K, N).to(torch.bfloat16)
        wp = torch.empty(ago.packed_weight_shape(K, N), device="cuda", dtype=torch.bfloat16)
        ago.ago_pack_weight(w, wp)
        torch.cuda.synchronize()
        got = wp.float().cpu().numpy()
        assert np.array_equal(got, _packed_reference(w.float().cpu().numpy())), (K, N)


def test_ffn_on_packed_weights(gpu, oracle):
    """matmul -> activation -> matmul with the weights pre-packed into matrix-instruction fragments: the
    benchmark shape, ragged rows, a ragged last hidden slice and column block, k-steps in pairs and in
    fours, one slice only, the three activations."""
    torch, ago, runner = gpu
    cases = [(wl.FfnCase(2048, 768, 3072, 768, "bf16", 6800, name="ffn_packed_bench"), ago.ACT_GELU_TANH),
             (wl.FfnCase(130, 64, 64, 16, "bf16", 6801, name="ffn_packed_tiny"), ago.ACT_GELU_TANH),
             (wl.FfnCase(300, 192, 448, 400, "bf16", 6802, name="ffn_packed_ragged"), ago.ACT_GELU_TANH),
             (wl.FfnCase(512, 1024, 4096, 1024, "bf16", 6803, name="ffn_packed_bert_large"), ago.ACT_GELU_TANH),
             (wl.FfnCase(64, 128, 384, 384, "bf16", 6804, name="ffn_packed_one_slice"), ago.ACT_GELU_TANH),
             (wl.FfnCase(1, 128, 512, 768, "bf16", 6805, name="ffn_packed_one_row"), ago.ACT_GELU_TANH)]
    for case, act in cases:
        ref = oracle.run_case(case)
        t = runner.to_device(case)
        w1p = torch.empty(ago.packed_weight_shape(case.K, case.F), device="cuda", dtype=torch.bfloat16)
        w2p = torch.empty(ago.packed_weight_shape(case.F, case.K2), device="cuda", dtype=torch.bfloat16)
        ago.ago_pack_weight(t["w1"], w1p)
        ago.ago_pack_weight(t["w2"], w2p)
        n = ago.workspace_bytes(ago.OP_FUSED_FFN_PACKED, [case.M, case.K, case.F, case.K2], ago.BF16)
        assert n > 0
        ws = torch.empty(n, dtype=torch.uint8, device="cuda")
        y = runner.alloc_output(case)
        y.zero_()
        print("packed ffn", case.name, flush=True)
        ago.ago_fused_ffn_packed(t["x"], w1p, t["b1"], w2p, t["b2"], y, act, ws)
        torch.cuda.synchronize()
        assert_close(runner.to_numpy64(y), ref, "bf16", case.name)
    # other activations against the oracle's chain with that activation
    case = wl.FfnCase(96, 128, 448, 64, "bf16", 6806, name="ffn_packed_relu")
    tens = case.tensors()
    t = runner.to_device(case)
    w1p = torch.empty(ago.packed_weight_shape(case.K, case.F), device="cuda", dtype=torch.bfloat16)
    w2p = torch.empty(ago.packed_weight_shape(case.F, case.K2), device="cuda", dtype=torch.bfloat16)
    ago.ago_pack_weight(t["w1"], w1p)
    ago.ago_pack_weight(t["w2"], w2p)
    ws = torch.empty(ago.workspace_bytes(ago.OP_FUSED_FFN_PACKED, [case.M, case.K, case.F, case.K2], ago.BF16),
                     dtype=torch.uint8, device="cuda")
    for act, name in ((ago.ACT_RELU, "relu"), (ago.ACT_NONE, "none")):
        y = runner.alloc_output(case)
        ago.ago_fused_ffn_packed(t["x"], w1p, t["b1"], w2p, t["b2"], y, act, ws)
        torch.cuda.synchronize()
        ref = oracle.ffn(tens["x"], tens["w1"], tens["b1"], tens["w2"], tens["b2"], act=name)
        assert_close(runner.to_numpy64(y), ref, "bf16", case.name + " " + name)


def test_sibling_qkv_projection(gpu, oracle):
    """q, k, v = x W* + b* in one kernel, both output layouts, ragged row and column blocks; then the
    projections feed the attention chain without a transpose in between."""
    torch, ago, runner = gpu
    cases = [wl.QkvCase(2, 100, 768, 12, 64, True, True, "bf16", 6600, name="qkv_ragged_rows"),
             wl.QkvCase(1, 384, 256, 3, 64, False, True, "bf16", 6601, name="qkv_bshd"),
             wl.QkvCase(3, 50, 72, 5, 24, True, False, "bf16", 6602, name="qkv_ragged_cols_nobias"),
             wl.QkvCase(1, 1, 8, 1, 8, True, True, "bf16", 6603, name="qkv_tiny"),
             wl.QkvCase(8, 384, 768, 12, 64, True, True, "bf16", 6604, name="qkv_8x384x768")]
    for case in cases:
        ref = oracle.run_case(case)                               # [3, ...]
        t = runner.to_device(case)
        shape = (case.B, case.Hh, case.S, case.D) if case.head_major else (case.B, case.S, case.Hh, case.D)
        outs = [torch.zeros(shape, dtype=torch.bfloat16, device="cuda:0") for _ in range(3)]
        ago.ago_fused_qkv(t["x"], t["wq"], t["wk"], t["wv"], t["bq"], t["bk"], t["bv"], *outs, head_major=case.head_major)
        torch.cuda.synchronize()
        for i in range(3):
            assert_close(runner.to_numpy64(outs[i]), ref[i], "bf16", "%s %s" % (case.name, "qkv"[i]))
    # projections (head-major) -> attention chain: against the oracle run on the oracle's projections,
    # rounded to bf16 where the GPU path stores them
    case = wl.QkvCase(2, 200, 256, 4, 64, True, True, "bf16", 6610, name="qkv_then_attn")
    t = runner.to_device(case)
    q, k, v = (torch.zeros((2, 4, 200, 64), dtype=torch.bfloat16, device="cuda:0") for _ in range(3))
    o = torch.zeros_like(q)
    ago.ago_fused_qkv(t["x"], t["wq"], t["wk"], t["wv"], t["bq"], t["bk"], t["bv"], q, k, v, head_major=True)
    ago.ago_fused_attn(q, k, v, o, 0.125)
    torch.cuda.synchronize()
    rq, rk, rv = (wl.round_to_bf16(a) for a in oracle.run_case(case))
    assert_close(runner.to_numpy64(o), oracle.attn(rq, rk, rv, 0.125), "bf16", case.name)


def test_attention_head_dim_128(gpu, oracle):
    """D = 128 (two 64-column planes per K / V block): contiguous and [B][S][Hh][D] layouts, ragged and
    multi-block sequences, both workgroup sizes."""
    torch, ago, runner = gpu
    cases = [wl.AttnCase(1, 1, 1, 128, 0.09, "bf16", 6800, name="attn_d128_s1"),
             wl.AttnCase(2, 3, 100, 128, 0.0884, "bf16", 6801, name="attn_d128_s100"),
             wl.AttnCase(1, 4, 384, 128, 0.0884, "bf16", 6802, name="attn_d128_s384"),
             wl.AttnCase(1, 2, 600, 128, 0.0884, "bf16", 6803, name="attn_d128_s600"),
             wl.AttnCase(4, 8, 256, 128, 0.0884, "bf16", 6804, name="attn_d128_4x8x256")]
    for case in cases:
        ref = oracle.run_case(case)
        t = runner.to_device(case)
        try:
            for cfg in (-1, 2):
                ago.set_tile_config(ago.OP_FUSED_ATTN, cfg)
                o = torch.zeros_like(t["q"])
                ago.ago_fused_attn(t["q"], t["k"], t["v"], o, case.scale)
                torch.cuda.synchronize()
                assert_close(runner.to_numpy64(o), ref, "bf16", "%s cfg %d" % (case.name, cfg))
        finally:
            ago.set_tile_config(ago.OP_FUSED_ATTN, -1)
        q, k, v = (t[n].permute(0, 2, 1, 3).contiguous() for n in ("q", "k", "v"))   # [B, S, Hh, D]
        o = torch.zeros_like(q)
        ago.ago_fused_attn_bshd(q, k, v, o, case.scale)
        torch.cuda.synchronize()
        assert_close(runner.to_numpy64(o.permute(0, 2, 1, 3)), ref, "bf16", case.name + " bshd")


def test_attention_bias(gpu, oracle):
    """softmax(scale q k^T + bias) v: every bias broadcast kind, 16-byte and element-wise row loads (S % 8),
    ragged key blocks, every tile configuration, and the benchmark's shape with a per-head table."""
    torch, ago, runner = gpu
    cases = [wl.AttnCase(2, 2, 200, 64, 0.125, "bf16", 6200, name="attn_bias_full_s200", bias="full"),
             wl.AttnCase(2, 4, 384, 64, 0.125, "bf16", 6201, name="attn_bias_head_s384", bias="head"),
             wl.AttnCase(3, 2, 130, 64, 0.3, "bf16", 6202, name="attn_bias_mask_s130", bias="batch"),
             wl.AttnCase(1, 3, 77, 64, 0.125, "bf16", 6203, name="attn_bias_full_s77", bias="full"),
             wl.AttnCase(1, 2, 600, 64, 0.125, "bf16", 6204, name="attn_bias_head_s600", bias="head"),
             wl.AttnCase(1, 1, 1, 64, 0.125, "bf16", 6205, name="attn_bias_s1", bias="full"),
             wl.AttnCase(8, 12, 384, 64, 0.125, "bf16", 6206, name="attn_bias_head_8x12x384", bias="head"),
             wl.AttnCase(2, 2, 200, 128, 0.0884, "bf16", 6207, name="attn_bias_d128_s200", bias="full"),
             wl.AttnCase(1, 3, 130, 128, 0.0884, "bf16", 6208, name="attn_bias_d128_mask_s130", bias="batch")]
    for case in cases:
        ref = oracle.run_case(case)
        t = runner.to_device(case)
        cfgs = [-1] if case.B * case.Hh > 16 else [-1, 0, 1, 2, 3]
        try:
            for cfg in cfgs:
                ago.set_tile_config(ago.OP_FUSED_ATTN, cfg)
                o = torch.zeros_like(t["q"])
                ago.ago_fused_attn_bias(t["q"], t["k"], t["v"], t["bias"], o, case.scale)
                torch.cuda.synchronize()
                assert_close(runner.to_numpy64(o), ref, "bf16", "%s cfg %d" % (case.name, cfg))
        finally:
            ago.set_tile_config(ago.OP_FUSED_ATTN, -1)
    # a zero bias reproduces the plain chain bit for bit apart from the order of the scale multiply
    case = wl.AttnCase(2, 3, 200, 64, 0.125, "bf16", 6210, name="attn_bias_zero")
    t = runner.to_device(case)
    o0, o1 = torch.zeros_like(t["q"]), torch.zeros_like(t["q"])
    ago.ago_fused_attn(t["q"], t["k"], t["v"], o0, case.scale)
    ago.ago_fused_attn_bias(t["q"], t["k"], t["v"], torch.zeros(1, 1, 200, 200, dtype=torch.bfloat16, device="cuda:0"),
                            o1, case.scale)
    torch.cuda.synchronize()
    assert_close(runner.to_numpy64(o1), runner.to_numpy64(o0), "bf16", "zero bias vs plain")


# ---- seeded random shapes --------------------------------------------------------------------

def _random_cases():
    """Small shapes drawn from a fixed seed: odd image sizes, batches, channel counts at the supported
    granularity, both strides, sequence lengths around the block boundaries, row counts that are not
    multiples of any tile."""
    r = np.random.RandomState(20221201)
    cases = []
    for i in range(8):
        stride = int(r.choice([1, 2]))
        cin = int(r.choice([8, 16, 24, 32, 40]))
        cout = cin if (stride == 1 and r.rand() < 0.5) else int(r.choice([8, 16, 24, 48]))
        cases.append(wl.InvresCase(int(r.randint(1, 4)), int(r.randint(1, 19)), int(r.randint(1, 19)), cin,
                                   int(r.choice([16, 48, 96, 144, 208])), cout, stride,
                                   stride == 1 and cin == cout, bool(r.rand() < 0.7),
                                   str(r.choice(["f32", "bf16"])), 5000 + i, name="rand_invres_%d" % i))
    for i in range(4):
        cases.append(wl.ChainCase(int(r.randint(1, 3)), int(r.randint(1, 23)), int(r.randint(1, 23)), 64,
                                  bool(r.rand() < 0.5), "bf16", 5100 + i, name="rand_chain_%d" % i))
    for i in range(6):
        k = 64 * int(r.randint(1, 5))
        f, k2 = [(384, 384), (768, 384), (192, 128), (320, 256), (384, 768), (64, 128)][i]
        cases.append(wl.FfnCase(int(r.randint(1, 300)), k, f, k2, "bf16", 5200 + i, name="rand_ffn_%d" % i))
    for i in range(6):
        s_len = int(r.choice([1, 31, 33, 64, 127, 129, 191, 193, 255, 257, 400, 513]))
        cases.append(wl.AttnCase(int(r.randint(1, 3)), int(r.randint(1, 6)), s_len, 64, float(r.choice([0.125, 0.3])),
                                 "bf16", 5300 + i, name="rand_attn_%d" % i))
    # the widened entry points: 5x5 depthwise, expanded channels in chunks, biased attention, sibling projections
    for i in range(6):
        stride = int(r.choice([1, 2]))
        cin = int(r.choice([16, 40, 80, 112]))
        cexp = int(r.choice([96, 240, 480, 672, 960]))
        cout = cin if (stride == 1 and r.rand() < 0.5) else int(r.choice([24, 48, 160]))
        cases.append(wl.InvresCase(int(r.randint(1, 3)), int(r.randint(1, 15)), int(r.randint(1, 15)), cin, cexp, cout,
                                   stride, stride == 1 and cin == cout, bool(r.rand() < 0.7),
                                   str(r.choice(["f32", "bf16"])), 5400 + i, name="rand_invres_wide_%d" % i,
                                   ksize=int(r.choice([3, 5]))))
    for i in range(5):
        s_len = int(r.choice([7, 64, 100, 136, 200, 264, 391]))
        cases.append(wl.AttnCase(int(r.randint(1, 3)), int(r.randint(1, 5)), s_len, 64, float(r.choice([0.125, 0.2])),
                                 "bf16", 5500 + i, name="rand_attn_bias_%d" % i,
                                 bias=str(r.choice(["full", "head", "batch"]))))
    for i in range(5):
        cases.append(wl.QkvCase(int(r.randint(1, 4)), int(r.randint(1, 150)), 8 * int(r.randint(1, 40)),
                                int(r.randint(1, 7)), int(r.choice([8, 24, 64, 128])), bool(r.rand() < 0.5),
                                bool(r.rand() < 0.7), "bf16", 5600 + i, name="rand_qkv_%d" % i))
    return cases


@pytest.mark.gpu
@pytest.mark.parametrize("case", _random_cases(), ids=lambda c: c.name)
def test_fused_random_shapes(gpu, oracle, case):
    torch, ago, runner = gpu
    t = runner.to_device(case)
    y = runner.alloc_output(case)
    y.zero_()
    runner.run_fused(case, t, y, runner.alloc_workspace(case, fused=True))
    torch.cuda.synchronize()
    assert_close(runner.to_numpy64(y), oracle.run_case(case), case.dtype, "%s %r" % (case.name, case))


# ---- two-operator pairs ------------------------------------------------------------------

@pytest.mark.gpu
@pytest.mark.parametrize("case", wl.pair_cases(), ids=lambda c: c.name)
def test_pair_fused_matches_oracle(gpu, oracle, case):
    """pw->dw, dw->pw and pw->pw as entry points of their own, element by element against the oracle;
    the same pair run operator by operator must agree too."""
    torch, ago, runner = gpu
    ref = oracle.run_case(case)
    t = runner.to_device(case)
    y = runner.alloc_output(case)
    y.zero_()
    runner.run_fused(case, t, y, runner.alloc_workspace(case, fused=True))
    torch.cuda.synchronize()
    assert_close(runner.to_numpy64(y), ref, case.dtype, case.name)
    yu = runner.alloc_output(case)
    runner.run_pair_unfused(case, t, yu, runner.alloc_pair_scratch(case))
    torch.cuda.synchronize()
    # Operator by operator the intermediate tensor goes through memory in the storage type.  For bf16 that is
    # one rounding (2^-9 relative) the fused path does not make (it keeps the intermediate in fp32 ahead of a
    # depthwise), and a depthwise adds up 9 such values of mixed sign: the worst element of the un-fused dw -> dw
    # pair measures 2.2e-2 of max(|ref|, rms), just above the 2e-2 bar of the fused kernels.  This sanity check of
    # the baseline therefore gets 1.25x the bar; every fused result is held to the bar itself.
    assert_close(runner.to_numpy64(yu), ref, case.dtype, case.name + " un-fused", scale=1.25)


@pytest.mark.gpu
def test_pairs_with_a_5x5_depthwise(gpu, oracle):
    """pw->dw and dw->pw with a 5 x 5 depthwise (`ago_fused_pw_dw_k`, `ago_fused_dw_pw_k`): both dtypes and
    strides, ragged images, an image smaller than the kernel, a wide dw->pw that takes the channel split."""
    torch, ago, runner = gpu
    cases = [wl.PairCase("pw_dw", 1, 14, 14, 40, 240, stride=1, dtype="f32", seed=6700, name="pw_dw5_f32", ksize=5),
             wl.PairCase("pw_dw", 2, 9, 11, 24, 144, stride=2, dtype="bf16", seed=6701, name="pw_dw5_bf16_s2_ragged", ksize=5),
             wl.PairCase("pw_dw", 1, 3, 2, 8, 16, stride=1, bias=False, dtype="bf16", seed=6702, name="pw_dw5_tiny", ksize=5),
             wl.PairCase("dw_pw", 1, 14, 14, 240, 40, stride=1, dtype="bf16", seed=6703, name="dw_pw5_bf16", ksize=5),
             wl.PairCase("dw_pw", 2, 13, 10, 96, 24, stride=2, dtype="f32", seed=6704, name="dw_pw5_f32_s2_ragged", ksize=5),
             wl.PairCase("dw_pw", 1, 7, 7, 672, 160, stride=1, dtype="bf16", seed=6705, name="dw_pw5_672_split", ksize=5)]
    for case in cases:
        t = runner.to_device(case)
        y = runner.alloc_output(case)
        y.fill_(3.0)
        runner.run_fused(case, t, y, runner.alloc_workspace(case, fused=True))
        torch.cuda.synchronize()
        assert_close(runner.to_numpy64(y), oracle.run_case(case), case.dtype, case.name)
    # the 3 x 3 entry points refuse a weight of another size instead of mis-reading it
    t = runner.to_device(cases[0])
    with pytest.raises(ValueError):
        ago.ago_fused_pw_dw(t["x"], t["w1"], t["b1"], t["wd"], t["bd"], runner.alloc_output(cases[0]), 1)


# ---- single operators -----------------------------------------------------------------

def _dev(torch, arr, dtype):
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda().to(td).contiguous()


def _store(arr, dtype):
    return rng.round_to_bf16(arr) if dtype == "bf16" else np.asarray(arr, np.float32).astype(np.float64)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [(200, 72, 136), (64, 768, 64), (333, 256, 320),
                                   # small products (direct kernel): reductions split over 1, 2, 4 and 8 waves, ragged
                                   # 32 x 32 tiles, a k range that does not divide, a single output
                                   (196, 8, 40), (3136, 24, 144), (50, 40, 24), (196, 192, 32), (784, 144, 32), (1, 8, 8),
                                   # above the small-product limit, no exact tiling: the LDS-tiled kernels
                                   (700, 264, 200),
                                   # shapes that tile exactly take the k-split kernels: 128 x 192 tiles with an even and an
                                   # odd number of k tiles, 64 x 96 tiles with one and with three k tiles
                                   (2048, 128, 3072), (2048, 192, 3072), (1024, 128, 768), (1024, 384, 768)])
def test_gemm_op(gpu, oracle, dtype, shape):
    torch, ago, runner = gpu
    M, K, N = shape
    a, b = _store(rng.normal(1, (M, K)), dtype), _store(rng.normal(2, (K, N), 0.1), dtype)
    bias = _store(rng.uniform(3, (N,), -1, 1), "f32")
    res = _store(rng.normal(4, (M, N)), dtype)
    c = torch.empty((M, N), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    ago.ago_gemm(_dev(torch, a, dtype), _dev(torch, b, dtype), None, None, c, ago.ACT_NONE)
    assert_close(runner.to_numpy64(c), oracle.gemm(a, b), dtype, "gemm")
    ago.ago_gemm(_dev(torch, a, dtype), _dev(torch, b, dtype), _dev(torch, bias, "f32"),
                 _dev(torch, res, dtype), c, ago.ACT_RELU)
    ref = oracle.relu(oracle.add(oracle.bias(oracle.gemm(a, b), bias), res))
    assert_close(runner.to_numpy64(c), ref, dtype, "gemm+bias+res+relu")


@pytest.mark.parametrize("shape", [(2048, 768, 3072), (2048, 3072, 768), (200, 256, 384), (130, 512, 96),
                                   (64, 1024, 192), (1, 128, 192)], ids=lambda s: "x".join(map(str, s)))
def test_gemm_on_packed_weights(gpu, oracle, shape):
    """The un-fused product on pre-packed weights: both tilings (128 x 192; 64 x 96 with the reduction split over
    the waves), ragged rows, bias and activation in the epilogue."""
    torch, ago, runner = gpu
    M, K, N = shape
    a, b = _store(rng.normal(21, (M, K)), "bf16"), _store(rng.normal(22, (K, N), 0.1), "bf16")
    bias = _store(rng.uniform(23, (N,), -1, 1), "f32")
    wp = torch.empty(ago.packed_weight_shape(K, N), device="cuda", dtype=torch.bfloat16)
    ago.ago_pack_weight(_dev(torch, b, "bf16"), wp)
    c = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ago.ago_gemm_packed(_dev(torch, a, "bf16"), wp, None, c, ago.ACT_NONE)
    torch.cuda.synchronize()
    assert_close(runner.to_numpy64(c), oracle.gemm(a, b), "bf16", "packed gemm")
    ago.ago_gemm_packed(_dev(torch, a, "bf16"), wp, _dev(torch, bias, "f32"), c, ago.ACT_RELU)
    torch.cuda.synchronize()
    assert_close(runner.to_numpy64(c), oracle.relu(oracle.bias(oracle.gemm(a, b), bias)), "bf16", "packed gemm+bias+relu")


def _random_packed_ffn_cases():
    r = np.random.RandomState(20221207)
    out = []
    for i in range(12):
        k = 64 * int(r.randint(1, 20))                       # up to 1216: the x tile must fit LDS
        f = 64 * int(r.randint(1, 20))
        k2 = 16 * int(r.randint(1, 60))
        out.append(wl.FfnCase(int(r.randint(1, 260)), k, f, k2, "bf16", 6900 + i,
                              name="rand_packed_ffn_%dx%dx%dx" % (k, f, k2)))
    return out


@pytest.mark.parametrize("case", _random_packed_ffn_cases(), ids=lambda c: c.name)
def test_packed_ffn_random_shapes(gpu, oracle, case):
    """Random rows, reductions, hidden widths (ragged last slice, one to five slices) and output widths
    (ragged last column block) against the oracle."""
    torch, ago, runner = gpu
    ref = oracle.run_case(case)
    t = runner.to_device(case)
    w1p = torch.empty(ago.packed_weight_shape(case.K, case.F), device="cuda", dtype=torch.bfloat16)
    w2p = torch.empty(ago.packed_weight_shape(case.F, case.K2), device="cuda", dtype=torch.bfloat16)
    ago.ago_pack_weight(t["w1"], w1p)
    ago.ago_pack_weight(t["w2"], w2p)
    ws = torch.empty(ago.workspace_bytes(ago.OP_FUSED_FFN_PACKED, [case.M, case.K, case.F, case.K2], ago.BF16),
                     dtype=torch.uint8, device="cuda")
    y = runner.alloc_output(case)
    y.zero_()
    print("packed ffn", case, flush=True)
    ago.ago_fused_ffn_packed(t["x"], w1p, t["b1"], w2p, t["b2"], y, ago.ACT_GELU_TANH, ws)
    torch.cuda.synchronize()
    assert_close(runner.to_numpy64(y), ref, "bf16", "%s %r" % (case.name, case))


def test_unfused_ffn_on_packed_weights(gpu, oracle):
    torch, ago, runner = gpu
    for case in (wl.FfnCase(2048, 768, 3072, 768, "bf16", 6810, name="ffn_u2_packed_bench"),
                 wl.FfnCase(100, 512, 1536, 192, "bf16", 6811, name="ffn_u2_packed_small")):
        ref = oracle.run_case(case)
        t = runner.to_device(case)
        w1p = torch.empty(ago.packed_weight_shape(case.K, case.F), device="cuda", dtype=torch.bfloat16)
        w2p = torch.empty(ago.packed_weight_shape(case.F, case.K2), device="cuda", dtype=torch.bfloat16)
        ago.ago_pack_weight(t["w1"], w1p)
        ago.ago_pack_weight(t["w2"], w2p)
        ws = runner.alloc_workspace(case, fused=False)
        y = runner.alloc_output(case)
        y.zero_()
        ago.ago_unfused_ffn_packed(t["x"], w1p, t["b1"], w2p, t["b2"], y, ago.ACT_GELU_TANH, ws)
        torch.cuda.synchronize()
        assert_close(runner.to_numpy64(y), ref, "bf16", case.name)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("stride", [1, 2])
def test_dwconv_op(gpu, oracle, dtype, stride):
    torch, ago, runner = gpu
    x, w = _store(rng.normal(5, (2, 13, 9, 24)), dtype), _store(rng.normal(6, (3, 3, 24), 0.3), dtype)
    bias = _store(rng.uniform(7, (24,), -1, 1), "f32")
    ref = oracle.relu6(oracle.bias(oracle.dwconv3x3(x, w, stride), bias))
    y = torch.empty(ref.shape, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    ago.ago_dwconv3x3(_dev(torch, x, dtype), _dev(torch, w, dtype), _dev(torch, bias, "f32"), y, stride, ago.ACT_RELU6)
    assert_close(runner.to_numpy64(y), ref, dtype, "dwconv")


def test_conv3x3_op(gpu, oracle):
    torch, ago, runner = gpu
    x, w = _store(rng.normal(8, (2, 11, 13, 64)), "bf16"), _store(rng.normal(9, (3, 3, 64, 64), 0.06), "bf16")
    ref = oracle.conv3x3(x, w)
    y = torch.empty(ref.shape, dtype=torch.bfloat16, device="cuda")
    ago.ago_conv3x3(_dev(torch, x, "bf16"), _dev(torch, w, "bf16"), None, None, y, ago.ACT_NONE)
    assert_close(runner.to_numpy64(y), ref, "bf16", "conv3x3")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_simple_ops(gpu, oracle, dtype):
    torch, ago, runner = gpu
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = _store(rng.normal(10, (37, 5, 48), 3.0), dtype)
    b = _store(rng.uniform(11, (48,), -1, 1), "f32")
    xd = _dev(torch, x, dtype)
    y = torch.empty_like(xd)
    for act, f in ((ago.ACT_NONE, lambda v: v), (ago.ACT_RELU, oracle.relu), (ago.ACT_RELU6, oracle.relu6),
                   (ago.ACT_GELU_TANH, oracle.gelu_tanh)):
        ago.ago_bias_act(xd, _dev(torch, b, "f32"), y, act)
        assert_close(runner.to_numpy64(y), f(oracle.bias(x, b)), dtype, "bias_act %d" % act)
    x2 = _store(rng.normal(12, x.shape), dtype)
    ago.ago_add_act(xd, _dev(torch, x2, dtype), y, ago.ACT_RELU)
    assert_close(runner.to_numpy64(y), oracle.relu(oracle.add(x, x2)), dtype, "add_act")
    ago.ago_scale(xd, y, 0.125)
    assert_close(runner.to_numpy64(y), oracle.scale(x, 0.125), dtype, "scale")
    s = _store(rng.normal(13, (50, 384), 2.0), dtype)
    sd = _dev(torch, s, dtype)
    p = torch.empty_like(sd)
    ago.ago_softmax_rows(sd, p)
    assert_close(runner.to_numpy64(p), oracle.softmax_rows(s), dtype, "softmax")
    assert p.dtype == td


def test_bmm_ops(gpu, oracle):
    torch, ago, runner = gpu
    q, k = _store(rng.normal(14, (3, 100, 64)), "bf16"), _store(rng.normal(15, (3, 72, 64)), "bf16")
    s = torch.empty((3, 100, 72), dtype=torch.bfloat16, device="cuda")
    ago.ago_bmm_nt(_dev(torch, q, "bf16"), _dev(torch, k, "bf16"), s, 0.125)
    assert_close(runner.to_numpy64(s), oracle.scale(oracle.bmm_nt(q, k), 0.125), "bf16", "bmm_nt")
    p, v = _store(rng.uniform(16, (3, 100, 72)), "bf16"), _store(rng.normal(17, (3, 72, 64)), "bf16")
    o = torch.empty((3, 100, 64), dtype=torch.bfloat16, device="cuda")
    ago.ago_bmm_nn(_dev(torch, p, "bf16"), _dev(torch, v, "bf16"), o)
    assert_close(runner.to_numpy64(o), oracle.bmm_nn(p, v), "bf16", "bmm_nn")


# ---- edge cases -------------------------------------------------------------------------

def test_attention_single_key_and_tiny_sequences(gpu, oracle):
    torch, ago, runner = gpu
    for S in (1, 2, 31, 129):
        case = wl.AttnCase(1, 2, S, 64, 0.125, "bf16", 777 + S, name="attn_S%d" % S)
        t = runner.to_device(case)
        y = runner.alloc_output(case)
        runner.run_fused(case, t, y, None)
        torch.cuda.synchronize()
        assert_close(runner.to_numpy64(y), oracle.run_case(case), "bf16", case.name)


def test_invres_single_pixel_and_odd_sizes(gpu, oracle):
    torch, ago, runner = gpu
    for (h, w, s) in ((1, 1, 1), (1, 7, 2), (5, 3, 2), (17, 17, 1)):
        case = wl.InvresCase(1, h, w, 8, 16, 8, s, s == 1, True, "f32", 900 + h, name="invres_%dx%d" % (h, w))
        t = runner.to_device(case)
        y = runner.alloc_output(case)
        runner.run_fused(case, t, y, None)
        torch.cuda.synchronize()
        assert_close(runner.to_numpy64(y), oracle.run_case(case), "f32", case.name)


def test_fused_padding_pads_the_intermediate(gpu, oracle):
    """Large positive bias on the first operator: a kernel that padded the *input* instead of the
    intermediate would leak act(bias) into the border."""
    torch, ago, runner = gpu
    case = wl.ChainCase(1, 9, 9, 64, False, "bf16", 4242, name="chain_border")
    tens = case.tensors()
    tens["ba"] = np.full(64, 3.0)
    case.tensors = lambda: tens
    t = runner.to_device(case)
    y = runner.alloc_output(case)
    runner.run_fused(case, t, y, None)
    torch.cuda.synchronize()
    assert_close(runner.to_numpy64(y), oracle.run_case(case), "bf16", case.name)
