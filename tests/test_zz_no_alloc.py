"""The allocation-free entry point (`ago_fused_invres_noalloc`) against the entry point it is a variant of
(`ago_fused_invres_k` with a caller workspace): same kernels, the partial sums in the library's own buffer.
Two calls in a row, the second on a smaller input (the buffer keeps the first call's contents)."""

import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def test_noalloc_entry_point_matches_the_workspace_entry_point(oracle):
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2212_01005_amd import binding as ago, runner
    # both shapes take the channel split (their projection is cut over several workgroups, partial sums in scratch)
    cases = [wl.InvresCase(1, 14, 14, 96, 576, 96, 1, True, True, "bf16", 7100, name="noalloc_14x14x96"),
             wl.InvresCase(1, 7, 7, 160, 960, 160, 1, True, True, "bf16", 7101, name="noalloc_7x7x160"),
             wl.InvresCase(1, 7, 7, 64, 384, 64, 1, True, True, "f32", 7102, name="noalloc_7x7x64_f32", ksize=5)]
    for case in cases:
        dt = ago.BF16 if case.dtype == "bf16" else ago.F32
        dims = [case.N, case.H, case.W, case.Cin, case.Cexp, case.Cout, case.stride, case.ksize]
        need = ago.workspace_bytes(ago.OP_FUSED_INVRES, dims, dt)
        assert 0 < need <= ago.NOALLOC_SCRATCH_BYTES
        plan = ago.fused_invres_plan(*dims, dt, need)
        assert plan["split"] > 1, "the case is meant to use the scratch buffer"
        t = runner.to_device(case)
        y_ws, y_na = runner.alloc_output(case), runner.alloc_output(case)
        y_ws.zero_(); y_na.zero_()
        ws = torch.empty(need, dtype=torch.uint8, device="cuda:0")
        args = (t["x"], t["w1"], t["b1"], t["wd"], t["bd"], t["w2"], t["b2"])
        ago.ago_fused_invres_k(*args, y_ws, case.stride, case.residual, ws)
        ago.ago_fused_invres_noalloc(*args, y_na, case.stride, case.residual)
        torch.cuda.synchronize()
        a, b = runner.to_numpy64(y_ws), runner.to_numpy64(y_na)
        assert np.array_equal(a, b), case.name             # same kernels, same order of additions
        ref = oracle.run_case(case)
        rms = float(np.sqrt(np.mean(ref ** 2)))
        err = np.abs(b - ref) / np.maximum(np.abs(ref), rms)
        assert float(err.max()) <= (2e-2 if case.dtype == "bf16" else 1e-4), case.name
    # a shape whose partial sums exceed the buffer is refused before any GPU work
    big = wl.InvresCase(32, 7, 7, 160, 960, 160, 1, True, True, "bf16", 7103, name="noalloc_too_big")
    dims = [big.N, big.H, big.W, big.Cin, big.Cexp, big.Cout, big.stride, big.ksize]
    assert ago.workspace_bytes(ago.OP_FUSED_INVRES, dims, ago.BF16) > ago.NOALLOC_SCRATCH_BYTES
    t = runner.to_device(big)
    with pytest.raises(ago.AgoError):
        ago.ago_fused_invres_noalloc(t["x"], t["w1"], t["b1"], t["wd"], t["bd"], t["w2"], t["b2"],
                                     runner.alloc_output(big), big.stride, big.residual)
