"""The paper's fully connected networks as a shape workload (Section V-C, Tables IX and X).  Needs the GPU.

  python -m paper_1702_03192_amd.fcnet --out <dir>/fcnet_report.json [--md <dir>/fcnet_report.md]
  python -m paper_1702_03192_amd.fcnet --profile-steps 20        (config 5's step N times, for a kernel profiler)

Table IX: two families -- "MNIST" (784 inputs, 10 outputs, hidden 2048-1024 / 2048-2048-1024 /
2048-2048-2048-1024) and "synthetic" (26752 inputs and outputs, hidden 4096 x 2 / 3 / 4) -- each
trained at several mini-batch sizes.  Only the layer sizes matter here (N(0,1) inputs stand in for
MNIST images, labels are seeded), since what is measured is the time of the matrix products.  The
paper's figures with the mini-batch sizes are not in its text; the sizes below cover the range it
discusses ("larger than 512", "4096").

For every net, mini-batch size and forward mode (always NT = the paper's baseline framework, MTNN =
mtnn_auto, and always TNN for reference) the forward pass and the whole step are timed; backward =
step - forward.  The summary averages over mini-batch sizes and depths per family, like Table X.
"""
from __future__ import annotations

import argparse
import json
import statistics
import sys

NETS = {
    "mnist": {"in": 784, "out": 10, "hidden": [[2048, 1024], [2048, 2048, 1024], [2048, 2048, 2048, 1024]]},
    "synthetic": {"in": 26752, "out": 26752, "hidden": [[4096, 4096], [4096, 4096, 4096], [4096, 4096, 4096, 4096]]},
}
BATCHES = [128, 256, 512, 1024, 2048, 4096]
MODES = ((1, "nt"), (0, "mtnn"), (-1, "tnn"))


def profile_config5(steps):
    """Config 5's training step (784-4096-4096-4096-10, mini-batch 1024, selector-chosen forward path),
    `steps` times back to back: the workload of the per-kernel profile of the FC step."""
    import torch
    from . import binding as mt
    from . import inputs
    cfg = inputs.CONFIG5
    dims, batch = cfg["dims"], cfg["batch"]
    L = len(dims) - 1
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg["seed"])
    X = torch.randn((batch, dims[0]), generator=gen, device="cuda")
    labels = torch.randint(0, dims[-1], (batch,), generator=gen, device="cuda", dtype=torch.int32)
    W = [torch.from_numpy(inputs.xavier_uniform(cfg["seed"] + 1 + l, 2, dims[l + 1], dims[l])).cuda() for l in range(L)]
    b = [torch.zeros(dims[l + 1], device="cuda") for l in range(L)]
    gW = [torch.empty_like(w) for w in W]
    gb = [torch.empty_like(v) for v in b]
    loss = torch.empty(1, device="cuda")
    ws = torch.empty(mt.mtnn_fc_workspace_bytes(dims, batch), dtype=torch.uint8, device="cuda")
    desc, keep = mt.make_fc_desc(dims, batch, X, labels, W, b, gW, gb, loss, ws, 0.0, 0)
    for _ in range(3):
        mt.mtnn_fc_train_step(desc)
    torch.cuda.synchronize()
    a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        mt.mtnn_fc_train_step(desc)
    e.record()
    torch.cuda.synchronize()
    flops = sum(2.0 * batch * dims[l] * dims[l + 1] * (3 if l > 0 else 2) for l in range(L))
    ms = a.elapsed_time(e) / steps
    print(f"[fcnet] config 5 step x {steps}: {ms:.3f} ms per step, {flops / ms / 1e9:.1f} TFLOP/s of GEMM work", flush=True)
    return 0


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=None)
    ap.add_argument("--md", default=None)
    ap.add_argument("--profile-steps", type=int, default=0,
                    help="run only this many training steps of the config-5 net (after 3 warm-ups) and exit")
    ap.add_argument("--samples", type=int, default=10)
    ap.add_argument("--batches", type=int, nargs="*", default=BATCHES)
    args = ap.parse_args(argv)

    import torch
    from . import binding as mt
    from . import inputs
    from .sweep import _time_batches

    torch.cuda.set_device(0)
    mt.lib()
    if args.profile_steps > 0:
        return profile_config5(args.profile_steps)
    if not args.out:
        ap.error("--out is required")
    stream = torch.cuda.current_stream()
    side = torch.cuda.Stream()                                 # capture stream of the graph timings
    gen = torch.Generator(device="cuda")
    rows = []
    for family, spec in NETS.items():
        for hidden in spec["hidden"]:
            dims = [spec["in"]] + hidden + [spec["out"]]
            L = len(dims) - 1
            gen.manual_seed(9000 + len(hidden))
            W = []
            for l in range(L):
                bound = (6.0 / (dims[l] + dims[l + 1])) ** 0.5
                W.append((torch.rand((dims[l + 1], dims[l]), generator=gen, device="cuda") * 2 - 1) * bound)
            b = [torch.zeros(dims[l + 1], device="cuda") for l in range(L)]
            gW = [torch.empty_like(w) for w in W]
            gb = [torch.empty_like(v) for v in b]
            loss = torch.empty(1, device="cuda")
            for batch in args.batches:
                X = torch.randn((batch, dims[0]), generator=gen, device="cuda")
                labels = torch.randint(0, dims[-1], (batch,), generator=gen, device="cuda", dtype=torch.int32)
                ws = torch.empty(mt.mtnn_fc_workspace_bytes(dims, batch), dtype=torch.uint8, device="cuda")
                fwd_flop = sum(2.0 * batch * dims[l] * dims[l + 1] for l in range(L))
                bwd_flop = sum(2.0 * batch * dims[l] * dims[l + 1] * (2 if l > 0 else 1) for l in range(L))
                rec = {"family": family, "hidden": hidden, "batch": batch, "forward_gflop": fwd_flop / 1e9,
                       "backward_gflop": bwd_flop / 1e9,
                       "forward_nt_shapes": [(batch, dims[l + 1], dims[l]) for l in range(L)],
                       "labels": [mt.mtnn_select(batch, dims[l + 1], dims[l]) for l in range(L)]}
                for mode, name in MODES:
                    desc, keep = mt.make_fc_desc(dims, batch, X, labels, W, b, gW, gb, loss, ws, 0.0, mode)
                    t_f, _ = _time_batches(lambda: mt.mtnn_fc_forward(desc), stream, args.samples, 2000.0)
                    t_s, _ = _time_batches(lambda: mt.mtnn_fc_train_step(desc), stream, args.samples, 2000.0)
                    rec[name] = {"forward_ms": t_f * 1e3, "backward_ms": (t_s - t_f) * 1e3, "total_ms": t_s * 1e3,
                                 "forward_tflops": fwd_flop / t_f / 1e12,
                                 "total_tflops": (fwd_flop + bwd_flop) / t_s / 1e12}
                    if name == "mtnn":
                        # the same step with the bias / ReLU / SGD passes as kernels of their own
                        mt.mtnn_set_fused_epilogues(False)
                        try:
                            t_u, _ = _time_batches(lambda: mt.mtnn_fc_train_step(desc), stream, args.samples, 2000.0)
                        finally:
                            mt.mtnn_set_fused_epilogues(True)
                        rec[name]["total_separate_passes_ms"] = t_u * 1e3
                        # the same step captured once into a HIP graph and replayed: what the launch path costs
                        # (lr is 0 here, so replays leave the weights alone)
                        with torch.cuda.stream(side):          # one-time set-up of this stream (split-k scratch)
                            mt.mtnn_fc_train_step(desc)
                        side.synchronize()
                        graph = torch.cuda.CUDAGraph()
                        with torch.cuda.graph(graph, stream=side):
                            mt.mtnn_fc_train_step(desc)
                        t_g, _ = _time_batches(graph.replay, stream, args.samples, 2000.0)
                        rec[name]["total_graph_ms"] = t_g * 1e3
                        del graph
                rows.append(rec)
                print(f"[fcnet] {family} {hidden} batch {batch}: fwd NT {rec['nt']['forward_ms']:.3f} "
                      f"MTNN {rec['mtnn']['forward_ms']:.3f} TNN {rec['tnn']['forward_ms']:.3f} ms; "
                      f"step NT {rec['nt']['total_ms']:.3f} MTNN {rec['mtnn']['total_ms']:.3f} (graph {rec['mtnn']['total_graph_ms']:.3f}) ms "
                      f"({rec['mtnn']['total_tflops']:.1f} TFLOP/s)", flush=True)
                del X, labels, ws
            del W, b, gW, gb
    summary = {}
    for family in NETS:
        sel = [r for r in rows if r["family"] == family]
        summary[family] = {}
        for phase in ("forward_ms", "backward_ms", "total_ms"):
            nt = statistics.mean(r["nt"][phase] for r in sel)
            mtnn = statistics.mean(r["mtnn"][phase] for r in sel)
            tnn = statistics.mean(r["tnn"][phase] for r in sel)
            summary[family][phase] = {"nt": nt, "mtnn": mtnn, "tnn": tnn, "speedup_mtnn_over_nt": nt / mtnn}
    report = {"device": torch.cuda.get_device_name(0), "rows": rows, "summary": summary}
    with open(args.out, "w") as f:
        json.dump(report, f, indent=1)
    if args.md:
        with open(args.md, "w") as f:
            f.write("Average running time (ms) over mini-batch sizes and depths, as in Table X\n\n")
            f.write("| family | phase | always NT | MTNN | always TNN | MTNN speedup over NT |\n|---|---|---|---|---|---|\n")
            for family in NETS:
                for phase in ("forward_ms", "backward_ms", "total_ms"):
                    s = summary[family][phase]
                    f.write(f"| {family} | {phase[:-3]} | {s['nt']:.3f} | {s['mtnn']:.3f} | {s['tnn']:.3f} | "
                            f"{s['speedup_mtnn_over_nt']:.2f} |\n")
            f.write("\n| family | hidden | batch | fwd NT ms | fwd MTNN ms | fwd TNN ms | step MTNN ms | step from a HIP graph ms | step with separate passes ms | step TFLOP/s | labels |\n")
            f.write("|---|---|---|---|---|---|---|---|---|---|---|\n")
            for r in rows:
                f.write(f"| {r['family']} | {'-'.join(map(str, r['hidden']))} | {r['batch']} | {r['nt']['forward_ms']:.3f} | "
                        f"{r['mtnn']['forward_ms']:.3f} | {r['tnn']['forward_ms']:.3f} | {r['mtnn']['total_ms']:.3f} | "
                        f"{r['mtnn']['total_graph_ms']:.3f} | {r['mtnn']['total_separate_passes_ms']:.3f} | "
                        f"{r['mtnn']['total_tflops']:.1f} | {r['labels']} |\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
