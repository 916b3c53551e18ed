#!/usr/bin/env python3
"""Throughput of one training step (forward, backward, SGD) of the CNN of arXiv 1912.05234 on
one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch 100]

Workload: 60000 synthetic 28x28 fp32 images (uniform [0,1)) with uniform labels, resident in
HBM before the timed region; one step = forward, backward and SGD update over one batch of 100
consecutive images at rate 0.05 (the paper's batch size and rate, Section 4.2), batches taken
round-robin over the 600 of an epoch.  Every step is issued from C by cnn_train_epoch (whole epochs,
then one call over the first n * batch images for the rest), so no per-step Python call sits in the
timed region and the figure does not depend on --steps.  Prints ONE JSON line.  Besides the
contract fields it carries
  roofline      the fused forward+backward kernel's algorithmic flop rate against MI355X's fp32
                peak, from HIP events recorded around that kernel on its own stream;
  cpu_baseline  the single-threaded CPU oracle timed on this host on a bounded sample;
  sweep         the same step at batch 1000 / 10000 / 60000, the forward-only evaluation pass, and the
                stateless per-op calls at the layer shapes (matrix cores, vector unit alone, bf16):
                microseconds per call and the shares of the fp32 and HBM peaks.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FLOP_PER_IMAGE_TRAIN = 2 * 524160     # multiply-adds of C1, C2, FC forward and backward, x2
FLOP_PER_IMAGE_FWD = 2 * 203520
BYTES_PER_IMAGE = 3136 + 4            # pixels + label: the only per-image HBM traffic
PEAK_FP32_TFLOPS = 157.3              # MI355X vector / matrix fp32
PEAK_HBM_GBS = 8000.0
LR = 0.05
N_TRAIN, N_EVAL = 60000, 10000
GROUP_MAX_BATCH = 640                 # batches up to this size run train_group_kernel, larger ones train_kernel
# HBM bytes per launch of the fused kernel from rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this same
# command (profiles/train_group_kernel_batch100.md, profiles/train_kernel_batch60000.md), scaled by
# what the counters read for a plain 256 MiB copy (FETCH x2.0, WRITE x1.0).  Taken from profiles/,
# not read in this run; only for the batch sizes that were profiled with the kernels as they are
# now, null otherwise.
MEASURED_TRAFFIC_BYTES = {100: 2370765, 60000: 305109402}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=6000)
    ap.add_argument("--warmup", type=int, default=600)
    ap.add_argument("--batch", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (a dispatch of known HBM traffic for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: the library is a single-GPU kernel study with no multi-GPU path; "
                 "run it with --gpus 1")

    import numpy as np
    import torch
    from paper_1912_05234_amd import binding, inputs

    dev = "cuda:0"
    torch.cuda.set_device(0)
    images_h, labels_h = inputs.make_batch(N_TRAIN, 1001)
    images = torch.from_numpy(images_h).to(dev)
    labels = torch.from_numpy(labels_h).to(dev)
    weights = inputs.make_weights()
    torch.cuda.synchronize()

    def measure(batch, steps, warmup):
        """-> (images/s, ms per step, mean ms of the fused kernel) for `steps` timed steps."""
        net = binding.CNN(weights, max_batch=batch)
        loss = torch.zeros(1, dtype=torch.float32, device=dev)
        per_epoch = N_TRAIN // batch
        epoch_images, epoch_labels = images[:per_epoch * batch], labels[:per_epoch * batch]

        def go(n):
            # whole epochs, then the first n % per_epoch batches: all through the library's epoch call
            for _ in range(n // per_epoch):
                net.train_epoch(epoch_images, epoch_labels, batch, LR)
            rest = n % per_epoch
            if rest:
                net.train_epoch(epoch_images[:rest * batch], epoch_labels[:rest * batch], batch, LR)

        go(warmup)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        go(steps)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # second pass over the same steps with HIP events around the fused kernel of each step
        cap = min(steps, 4096)
        net.profile_begin(cap)
        go(cap)
        ms = net.profile_read(cap)
        net.profile_begin(0)
        net.train_batch(epoch_images[:batch], epoch_labels[:batch], LR, loss)
        assert bool(torch.isfinite(loss).item())
        net.close()
        return batch * steps / dt, 1e3 * dt / steps, float(np.mean(ms))

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)   # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    value, ms_per_step, kernel_ms = measure(args.batch, args.steps, args.warmup)
    achieved_tflops = FLOP_PER_IMAGE_TRAIN * args.batch / (kernel_ms * 1e-3) / 1e12

    out = {
        "metric": "training images/sec (fwd+bwd+SGD)",
        "value": value,
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[1]: 1 epoch over 60000 synthetic 28x28 fp32 images, batch %d, "
                               "SGD lr 0.05 (steps cycle over the epoch's batches)" % args.batch,
                   "batch": args.batch, "images_resident": N_TRAIN, "lr": LR},
        "roofline": {
            "kernel": "%s (fused forward+backward of one batch)"
                      % ("train_group_kernel" if args.batch <= GROUP_MAX_BATCH else "train_kernel"),
            "bound": "alu",
            "achieved": achieved_tflops,
            "peak": PEAK_FP32_TFLOPS,
            "unit": "TFLOP/s",
            "frac": achieved_tflops / PEAK_FP32_TFLOPS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(args.batch),
            "traffic_unit": "HBM bytes per launch (algorithmic: %d image bytes + %d partial-row bytes)"
                            % (args.batch * BYTES_PER_IMAGE, (args.batch if args.batch <= GROUP_MAX_BATCH else min(args.batch, 256)) * 15616),
            "kernel_ms": kernel_ms,
            "flop_per_launch": FLOP_PER_IMAGE_TRAIN * args.batch,
            "hbm_frac_whole_step": value * BYTES_PER_IMAGE / 1e9 / PEAK_HBM_GBS,
        },
    }

    if not args.no_sweep:
        sweep = {}
        for batch, steps, warm in ((1000, 600, 60), (10000, 60, 6), (60000, 10, 2)):
            v, ms, kms = measure(batch, steps, warm)
            tf = FLOP_PER_IMAGE_TRAIN * batch / (kms * 1e-3) / 1e12
            sweep["train_batch_%d" % batch] = {"images_per_s": v, "ms_per_step": ms, "kernel_ms": kms,
                                               "kernel_tflops": tf, "kernel_frac_fp32_peak": tf / PEAK_FP32_TFLOPS,
                                               "step_frac_fp32_peak": v * FLOP_PER_IMAGE_TRAIN / 1e12 / PEAK_FP32_TFLOPS}
        ev_images, ev_labels = inputs.make_batch(N_EVAL, 1002)
        ev_i, ev_l = torch.from_numpy(ev_images).to(dev), torch.from_numpy(ev_labels).to(dev)
        net = binding.CNN(weights, max_batch=N_EVAL)
        for _ in range(3):
            net.evaluate(ev_i, ev_l)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 20
        for _ in range(reps):
            net.evaluate(ev_i, ev_l)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / reps
        sweep["evaluate_10000"] = {"images_per_s": N_EVAL / dt, "ms_per_pass": 1e3 * dt,
                                   "frac_fp32_peak": N_EVAL / dt * FLOP_PER_IMAGE_FWD / 1e12 / PEAK_FP32_TFLOPS}
        net.close()
        # the stateless per-op calls at the layer shapes (10000 images): microseconds per call
        from paper_1912_05234_amd import bench_ops
        per_op = {}
        keep = ("us", "frac_of_fp32_peak", "frac_of_hbm_peak", "binding_roof")
        bench_ops.run(10000, 20, lambda line: per_op.__setitem__("%s.%s" % (line["layer"], line["op"]),
                                                                  {k: line[k] for k in keep if k in line}))
        sweep["per_op_batch_10000"] = per_op
        out["sweep"] = sweep

    if not args.no_cpu_baseline:
        import oracle
        n_steps = 600  # one epoch: about 18 s on one core
        w = inputs.flatten(weights)
        oracle.train_batch(images_h[:100], labels_h[:100], LR, w.copy())  # page in
        t0 = time.perf_counter()
        for s in range(n_steps):
            oracle.train_batch(images_h[s * 100:(s + 1) * 100], labels_h[s * 100:(s + 1) * 100], LR, w)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": n_steps * 100 / dt, "unit": "images/s", "cores": 1, "kind": "oracle",
                               "sample": "%d training steps of batch 100 (%d of the 60000 images), "
                                         "single-threaded C++ oracle; host has %d cores"
                                         % (n_steps, n_steps * 100, os.cpu_count())}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
