#!/usr/bin/env python3
"""Writes the stored expected values of the full-size training configurations.

Calls ONLY the CPU oracle (oracle/) and the seeded input generator; nothing here touches the GPU
library.  Workload (the full-MNIST-sized configurations): 60000 synthetic training images and 10000 evaluation
images (paper_1912_05234_amd/inputs.py, seeds below), batch 100, rate 0.05, weights from the default
seed.  Outputs, all float64/int64 in one .npz beside this script:
  grad_1000 / grad_10000 / grad_60000, loss_*   summed gradient and loss of the first 1000 / 10000 /
                                                all 60000 images at the initial weights (config 4);
  w_epoch1, w_epoch10                           flat weights [3898] after 1 and after 10 epochs of
                                                600 steps each (configs 2 and 3);
  loss_epoch[10]                                summed training loss of every epoch;
  eval1_correct, eval1_loss, eval1_yhat_head    evaluation of the 10000 images with w_epoch1
                                                (count, loss, first 64 output rows).
Run time: about 20 minutes on one core (the oracle is single-threaded by design).

    python tests/golden/make_training_golden.py [--epochs 10]
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_1912_05234_amd import inputs  # noqa: E402

TRAIN_SEED, EVAL_SEED, BATCH, RATE = 1001, 1002, 100, float(np.float32(0.05))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--epochs", type=int, default=10)
    ap.add_argument("--out", default=os.path.join(os.path.dirname(os.path.abspath(__file__)), "training_golden.npz"))
    args = ap.parse_args()
    images, labels = inputs.make_batch(60000, TRAIN_SEED)
    ev_images, ev_labels = inputs.make_batch(10000, EVAL_SEED)
    w0 = inputs.flatten(inputs.make_weights())
    out = {}

    t0 = time.time()
    g = np.zeros(oracle.NPARAM)
    loss = 0.0
    for c in range(60):
        w = w0.copy()
        l_c, g_c = oracle.train_batch(images[c * 1000:(c + 1) * 1000], labels[c * 1000:(c + 1) * 1000], 0.0, w,
                                      want_grad=True)
        g += g_c
        loss += l_c
        if c + 1 in (1, 10, 60):
            out["grad_%d" % ((c + 1) * 1000)] = g.copy()
            out["loss_%d" % ((c + 1) * 1000)] = np.float64(loss)
    print("gradients done in %.0f s" % (time.time() - t0), flush=True)

    w = w0.copy()
    epoch_loss = []
    for e in range(args.epochs):
        tot = 0.0
        for s in range(600):
            tot += oracle.train_batch(images[s * BATCH:(s + 1) * BATCH], labels[s * BATCH:(s + 1) * BATCH], RATE, w)
        epoch_loss.append(tot)
        print("epoch %d loss %.6f (%.0f s)" % (e + 1, tot, time.time() - t0), flush=True)
        if e == 0:
            out["w_epoch1"] = w.astype(np.float64)
            yhat, n_ok, ev_loss = oracle.evaluate(ev_images, ev_labels, w)
            out["eval1_correct"] = np.int64(n_ok)
            out["eval1_loss"] = np.float64(ev_loss)
            out["eval1_yhat_head"] = yhat[:64].astype(np.float64)
        np.savez(args.out, loss_epoch=np.array(epoch_loss), epochs_done=np.int64(e + 1),
                 **{"w_epoch%d" % (e + 1) if False else k: v for k, v in out.items()},
                 w_last=w.astype(np.float64))
    out["w_epoch%d" % args.epochs] = w.astype(np.float64)
    np.savez(args.out, loss_epoch=np.array(epoch_loss), epochs_done=np.int64(args.epochs), **out)
    print("wrote", args.out)


if __name__ == "__main__":
    main()
