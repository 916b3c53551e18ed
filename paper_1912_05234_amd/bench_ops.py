"""Times the stateless per-operation entry points at the network's layer shapes.

    python -m paper_1912_05234_amd.bench_ops [--batch 10000] [--steps 50]

One JSON line per operation: the average duration of the call's kernels between two HIP events
on the stream the binding launches on, the useful arithmetic (2 flops per multiply-add of the
operation's definition; padding the kernels add is not counted) and its share of the fp32 peak,
the bytes the operation must move (every input read once, every output written once) and their
share of the HBM peak, and which of the two roofs binds (the larger share).  The convolutions are
timed three ways: on the fp32 matrix cores (implicit GEMM), on the fp32 vector unit alone
(`*_valu`, one thread per output; the weight gradient without workspace), and with operands rounded
to bfloat16.  Inputs are synthetic (uniform [-1, 1), seeded) and resident in device memory.
"""
import argparse
import json
import sys

import torch

from . import binding

PEAK_TFLOPS = 157.3  # MI355X, fp32 matrix and vector alike
PEAK_HBM_GBS = 8000.0

# name: (Cin, H, W, Cout, KH, KW) -- the paper's C1 and C2 (Section 3, listing `forward`)
CONVS = {"C1": (1, 28, 28, 6, 5, 5), "C2": (6, 12, 12, 12, 5, 5)}
FC = (192, 10)


def time_call(fn, steps, warmup=5):
    for _ in range(warmup):
        fn()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(steps):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) * 1e3 / steps  # microseconds


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=10000)
    ap.add_argument("--steps", type=int, default=50)
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        sys.exit("bench_ops needs a GPU")
    run(args.batch, args.steps, lambda line: print(json.dumps(line), flush=True))


def run(batch, steps, emit):
    """Times every per-op call at `batch` images and hands each result (a dict) to `emit`."""
    args = argparse.Namespace(batch=batch, steps=steps)
    dev, B = "cuda:0", args.batch
    gen = torch.Generator(device="cpu").manual_seed(7)

    def rnd(*shape):
        return (torch.rand(*shape, generator=gen) * 2 - 1).to(dev)

    def report(layer, op, us, flops, nbytes, extra=None):
        tf, gbs = flops / us / 1e6, nbytes / us / 1e3
        line = {"layer": layer, "op": op, "batch": B, "us": round(us, 2), "tflops": round(tf, 2),
                "frac_of_fp32_peak": round(tf / PEAK_TFLOPS, 4), "gb_per_s": round(gbs, 1),
                "frac_of_hbm_peak": round(gbs / PEAK_HBM_GBS, 4),
                "binding_roof": "hbm" if gbs / PEAK_HBM_GBS > tf / PEAK_TFLOPS else "fp32"}
        line.update(extra or {})
        emit(line)

    def report_bw(layer, op, us, nbytes):
        gbs = nbytes / us / 1e3
        emit({"layer": layer, "op": op, "batch": B, "us": round(us, 2), "gb_per_s": round(gbs, 1),
              "frac_of_hbm_peak": round(gbs / PEAK_HBM_GBS, 4)})

    for name, (Cin, H, W, Cout, KH, KW) in CONVS.items():
        Ho, Wo = H - KH + 1, W - KW + 1
        x, k, b, d = rnd(B, Cin, H, W), rnd(Cout, Cin, KH, KW), rnd(Cout), rnd(B, Cout, Ho, Wo)
        flops = 2.0 * B * Cout * Ho * Wo * Cin * KH * KW
        # outputs and workspace allocated once, outside the timed calls
        out = torch.empty(B, Cout, Ho, Wo, device=dev)
        d_in = torch.empty(B, Cin, H, W, device=dev)
        d_k, d_b = torch.empty_like(k), torch.empty_like(b)
        L = binding.lib()
        nbytes = L.cnn_conv_bwd_weight_workspace_bytes(B, Cin, H, W, Cout, KH, KW)
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=dev)
        p, s = binding._ptr, binding._stream
        calls = {
            "conv_fwd": lambda: L.cnn_conv_fwd(p(x), p(k), p(b), p(out), B, Cin, H, W, Cout, KH, KW, s()),
            "conv_bwd_input": lambda: L.cnn_conv_bwd_input(p(d), p(k), p(d_in), B, Cin, H, W, Cout, KH, KW, s()),
            "conv_bwd_weight": lambda: L.cnn_conv_bwd_weight(p(x), p(d), p(d_k), p(d_b), B, Cin, H, W, Cout, KH,
                                                             KW, p(ws), nbytes, s()),
            # the fp32 vector unit alone
            "conv_fwd_valu": lambda: L.cnn_conv_fwd_valu(p(x), p(k), p(b), p(out), B, Cin, H, W, Cout, KH, KW, s()),
            "conv_bwd_input_valu": lambda: L.cnn_conv_bwd_input_valu(p(d), p(k), p(d_in), B, Cin, H, W, Cout, KH,
                                                                     KW, s()),
            "conv_bwd_weight_valu": lambda: L.cnn_conv_bwd_weight(p(x), p(d), p(d_k), p(d_b), B, Cin, H, W, Cout,
                                                                  KH, KW, None, 0, s()),
        }
        # bytes the operation must move: inputs read once, outputs written once
        sz = {"x": 4 * x.numel(), "d": 4 * d.numel(), "k": 4 * (k.numel() + b.numel())}
        must_move = {"conv_fwd": sz["x"] + sz["k"] + sz["d"], "conv_bwd_input": sz["d"] + sz["k"] + sz["x"],
                     "conv_bwd_weight": sz["x"] + sz["d"] + sz["k"]}
        # reduced precision: operands rounded to bfloat16, fp32 sums (same tensors, same useful flops)
        calls["conv_fwd_bf16"] = lambda: L.cnn_conv_fwd_bf16(p(x), p(k), p(b), p(out), B, Cin, H, W, Cout, KH, KW, s())
        calls["conv_bwd_input_bf16"] = lambda: L.cnn_conv_bwd_input_bf16(p(d), p(k), p(d_in), B, Cin, H, W, Cout, KH,
                                                                         KW, s())
        nbytes16 = L.cnn_conv_bwd_weight_bf16_workspace_bytes(B, Cin, H, W, Cout, KH, KW)
        ws16 = torch.empty(max(nbytes16, 16), dtype=torch.uint8, device=dev)
        calls["conv_bwd_weight_bf16"] = lambda: L.cnn_conv_bwd_weight_bf16(p(x), p(d), p(d_k), p(d_b), B, Cin, H, W,
                                                                           Cout, KH, KW, p(ws16), nbytes16, s())
        for op, fn in calls.items():
            assert fn() == 0, op
            slow = op.endswith("_valu")   # milliseconds each at 10000 images: fewer repeats
            base = op.replace("_valu", "").replace("_bf16", "")
            report(name, op, time_call(fn, max(3, args.steps // 10) if slow else args.steps, 1 if slow else 5), flops,
                   must_move[base])
        # the element-wise layers that follow the convolution: sigmoid, pool, and their backward forms
        act, pooled = torch.empty_like(out), torch.empty(B, Cout, Ho // 2, Wo // 2, device=dev)
        d_act = torch.empty_like(out)
        n = out.numel()
        elementwise = {
            "logistic_fwd": (lambda: L.cnn_logistic_fwd(p(out), p(act), n, s()), 8 * n),
            "avgpool_fwd": (lambda: L.cnn_avgpool_fwd(p(act), p(pooled), B, Cout, Ho, Wo, s()), 5 * n),
            "avgpool_bwd": (lambda: L.cnn_avgpool_bwd(p(pooled), p(d_act), B, Cout, Ho // 2, Wo // 2, s()), 5 * n),
            "logistic_bwd": (lambda: L.cnn_logistic_bwd(p(act), p(d_act), p(d), n, s()), 12 * n),
        }
        for op, (fn, nbytes) in elementwise.items():
            assert fn() == 0, op
            report_bw(name, op, time_call(fn, args.steps), nbytes)
    I, O = FC
    x, w, b, d = rnd(B, I), rnd(O, I), rnd(O), rnd(B, O)
    out, d_in, d_w, d_b = torch.empty(B, O, device=dev), torch.empty(B, I, device=dev), torch.empty_like(w), torch.empty_like(b)
    L = binding.lib()
    nbytes = L.cnn_fc_bwd_weight_workspace_bytes(B, I, O)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=dev)
    p, s = binding._ptr, binding._stream
    calls = {
        "fc_fwd": lambda: L.cnn_fc_fwd(p(x), p(w), p(b), p(out), B, I, O, s()),
        "fc_bwd_input": lambda: L.cnn_fc_bwd_input(p(d), p(w), p(d_in), B, I, O, s()),
        "fc_bwd_weight": lambda: L.cnn_fc_bwd_weight(p(x), p(d), p(d_w), p(d_b), B, I, O, p(ws), nbytes, s()),
    }
    nb = {"fc_fwd": 4 * (x.numel() + w.numel() + b.numel() + out.numel()),
          "fc_bwd_input": 4 * (d.numel() + w.numel() + d_in.numel()),
          "fc_bwd_weight": 4 * (x.numel() + d.numel() + w.numel() + b.numel())}
    for op, fn in calls.items():
        assert fn() == 0, op
        report("FC", op, time_call(fn, args.steps), 2.0 * B * I * O, nb[op])


if __name__ == "__main__":
    main()
