"""Calibration data of the tile planners: time every tile candidate, compare with what the library predicts.

The paper's tuner searches tile sizes by running candidates (Sec. III-B: re-computation against
parallelism); this library instead ships analytic / fitted time models (`ago_fused_*_plan`).  This
module is how their constants were obtained and how they can be checked on another machine:

    python -m paper_2212_01005_amd.calibrate sweep  --out sweep.json     # needs the GPU
    python -m paper_2212_01005_amd.calibrate report sweep.json           # host only, prints markdown

`sweep` times, per shape, every tile candidate of the four fused kernels with event-timed loops of
back-to-back launches (and, for the FFN, the two products with fused epilogues).  `report` asks the
library for the predicted time of each candidate (`ago_set_tile_config` + the plan call, no GPU work)
and lists prediction error and the time lost by the planner's pick against the best candidate.
"""

import argparse
import json
import sys

INVRES_SHAPES = [
    (1, 14, 14, 32, 192, 32, 1, "f32", 3), (1, 56, 56, 24, 144, 32, 2, "bf16", 3), (8, 28, 28, 40, 240, 40, 1, "bf16", 3),
    (8, 28, 28, 40, 240, 40, 1, "bf16", 5), (16, 14, 14, 64, 384, 64, 1, "bf16", 3), (4, 56, 56, 24, 144, 24, 1, "bf16", 3),
    (8, 56, 56, 24, 144, 32, 2, "bf16", 3), (32, 7, 7, 160, 960, 160, 1, "bf16", 3), (8, 14, 14, 96, 576, 96, 1, "f32", 3),
    (1, 112, 112, 16, 96, 24, 2, "bf16", 3), (8, 28, 28, 40, 240, 80, 2, "bf16", 5), (16, 14, 14, 112, 672, 112, 1, "bf16", 5),
    (32, 56, 56, 24, 144, 24, 1, "bf16", 3), (32, 28, 28, 32, 192, 32, 1, "f32", 3), (64, 14, 14, 64, 384, 96, 1, "bf16", 3),
    (2, 56, 56, 24, 144, 24, 1, "f32", 3), (4, 28, 28, 32, 192, 64, 2, "bf16", 3), (64, 7, 7, 160, 960, 320, 1, "bf16", 3),
    (1, 28, 28, 32, 192, 32, 1, "bf16", 3), (2, 14, 14, 96, 576, 96, 1, "bf16", 3), (1, 7, 7, 160, 960, 160, 1, "bf16", 3)]
CHAIN_SHAPES = [(1, 56, 56), (8, 56, 56), (32, 56, 56), (8, 28, 28), (32, 28, 28), (32, 14, 14), (1, 28, 28), (4, 112, 112),
                (128, 14, 14), (2, 60, 60)]
FFN_SHAPES = [(128, 768, 3072, 768), (512, 768, 3072, 768), (2048, 768, 3072, 768), (4096, 768, 3072, 768),
              (8192, 768, 3072, 768), (2048, 1024, 4096, 1024), (512, 512, 2048, 512), (2048, 512, 2048, 512),
              (8192, 512, 2048, 512), (1024, 256, 1024, 256), (16384, 768, 3072, 768)]
ATTN_SHAPES = [(8, 12, 384, 64), (8, 12, 128, 64), (32, 12, 384, 64), (2, 12, 4096, 64), (1, 12, 384, 64), (8, 12, 1024, 64),
               (1, 4, 96, 64), (16, 16, 256, 64), (4, 8, 2048, 64)]


def _sweep(out_path, iters):
    import torch
    import workloads as wl
    from . import binding as ago, runner

    def us(fn):
        for _ in range(4):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return round(a.elapsed_time(b) / iters * 1e3, 2)

    def candidates(case, op, workspace, unfused):
        t = runner.to_device(case)
        y = runner.alloc_output(case)
        row = {}
        for cfg in [-1] + list(range(ago.num_tile_configs(op))):
            ago.set_tile_config(op, cfg)
            try:
                ws = runner.alloc_workspace(case, fused=True) if workspace else None
                fn = runner.prepare_fused(case, t, y, ws)
                fn()
                row[str(cfg)] = us(fn)
            except ago.AgoError:
                pass                                     # candidate not legal for this shape
        ago.set_tile_config(op, -1)
        if unfused:
            fn = runner.prepare_unfused(case, t, y, runner.alloc_workspace(case, fused=False), 1)
            fn()
            row["u2"] = us(fn)
        return row

    res = {"invres": [], "chain": [], "ffn": [], "attn": []}
    for s in INVRES_SHAPES:
        n, h, w, ci, ce, co, st, dt, ks = s
        case = wl.InvresCase(n, h, w, ci, ce, co, st, st == 1 and ci == co, True, dt, 1, ksize=ks)
        res["invres"].append({"shape": list(s), "us": candidates(case, ago.OP_FUSED_INVRES, False, False)})
        print("invres", s, res["invres"][-1]["us"], flush=True)
    for s in CHAIN_SHAPES:
        case = wl.ChainCase(s[0], s[1], s[2], 64, True, "bf16", 9000)
        res["chain"].append({"shape": list(s), "us": candidates(case, ago.OP_FUSED_CONV_CHAIN, True, True)})
        print("chain", s, res["chain"][-1]["us"], flush=True)
    for s in FFN_SHAPES:
        case = wl.FfnCase(s[0], s[1], s[2], s[3], "bf16", 9001)
        res["ffn"].append({"shape": list(s), "us": candidates(case, ago.OP_FUSED_FFN, True, True)})
        print("ffn", s, res["ffn"][-1]["us"], flush=True)
    for s in ATTN_SHAPES:
        case = wl.AttnCase(s[0], s[1], s[2], s[3], s[3] ** -0.5, "bf16", 9002)
        res["attn"].append({"shape": list(s), "us": candidates(case, ago.OP_FUSED_ATTN, True, True)})
        print("attn", s, res["attn"][-1]["us"], flush=True)
    with open(out_path, "w") as f:
        json.dump(res, f, indent=1)


def _report(path):
    from . import binding as ago

    data = json.load(open(path))

    def predict(kind, shape, cfg):
        op = {"invres": ago.OP_FUSED_INVRES, "chain": ago.OP_FUSED_CONV_CHAIN, "ffn": ago.OP_FUSED_FFN,
              "attn": ago.OP_FUSED_ATTN}[kind]
        ago.set_tile_config(op, cfg)
        try:
            if kind == "invres":
                n, h, w, ci, ce, co, st, dt, ks = shape
                return ago.fused_invres_plan(n, h, w, ci, ce, co, st, ks, ago.BF16 if dt == "bf16" else ago.F32, 0)
            if kind == "chain":
                return ago.fused_conv_chain_plan(shape[0], shape[1], shape[2], 64)
            if kind == "ffn":
                return ago.fused_ffn_plan(*shape)
            return ago.fused_attn_plan(*shape)
        except (ago.AgoError, ValueError):
            return None
        finally:
            ago.set_tile_config(op, -1)

    out = []
    for kind, title in (("invres", "inverted residual (tile candidates, no channel-split workspace)"),
                        ("chain", "3x3 -> 3x3 chain"), ("attn", "attention chain"), ("ffn", "matmul -> GELU -> matmul")):
        out.append("\n## %s\n" % title)
        if kind == "ffn":
            out.append("| M x K x F x K2 | fused: predicted | measured | two products: predicted | measured | planner says | faster in fact |\n|---|---|---|---|---|---|---|")
        else:
            out.append("| shape | candidates timed | mean / max prediction error | best candidate: id, us | planner's pick: id, us | time lost |\n|---|---|---|---|---|---|")
        errs, losses = [], []
        for row in data[kind]:
            shape, us = row["shape"], row["us"]
            name = "x".join(str(v) for v in shape)
            if kind == "ffn":
                p = predict(kind, shape, -1)
                fused = us.get("3", us.get("-1"))
                errs += [abs(p["predicted_us"] - fused) / fused, abs(p["predicted_unfused_us"] - us["u2"]) / us["u2"]]
                says = "fuse" if p["fuse"] else "two products"
                fact = "fused" if fused <= us["u2"] else "two products"
                losses.append((fused if p["fuse"] else us["u2"]) / min(fused, us["u2"]))
                out.append("| %s | %.1f | %.1f | %.1f | %.1f | %s | %s (%.2fx) |" % (
                    name, p["predicted_us"], fused, p["predicted_unfused_us"], us["u2"], says, fact, max(fused, us["u2"]) / min(fused, us["u2"])))
                continue
            cand = {int(c): t for c, t in us.items() if c not in ("-1", "u2")}
            e = []
            for c, t in cand.items():
                p = predict(kind, shape, c)
                if p is not None:
                    e.append(abs(p["predicted_us"] - t) / t)
            pick = predict(kind, shape, -1)["config"]
            best = min(cand, key=cand.get)
            t_pick = cand.get(pick, us.get("-1"))
            errs += e
            losses.append(t_pick / cand[best])
            out.append("| %s | %d | %.0f%% / %.0f%% | %d, %.1f | %d, %.1f | %.1f%% |" % (
                name, len(cand), 100 * sum(e) / len(e), 100 * max(e), best, cand[best], pick, t_pick, 100 * (t_pick / cand[best] - 1)))
        out.append("\nAll %s rows: mean prediction error %.1f%%, worst %.1f%%; the planner's decision costs %.1f%% on average, %.1f%% at worst, against the best measured alternative.\n"
                   % (kind, 100 * sum(errs) / len(errs), 100 * max(errs), 100 * (sum(losses) / len(losses) - 1), 100 * (max(losses) - 1)))
    print("\n".join(out))


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    sub = ap.add_subparsers(dest="cmd", required=True)
    s = sub.add_parser("sweep")
    s.add_argument("--out", required=True)
    s.add_argument("--iters", type=int, default=30)
    r = sub.add_parser("report")
    r.add_argument("path")
    a = ap.parse_args(argv)
    if a.cmd == "sweep":
        _sweep(a.out, a.iters)
    else:
        _report(a.path)
    return 0


if __name__ == "__main__":
    sys.exit(main())
