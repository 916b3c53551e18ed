"""Trains the paper's network for some epochs and classifies a test set after each (Section 4.2:
60000 training images in batches of 100 at rate 0.05, ten epochs, then 10000 test images).

    python -m paper_1912_05234_amd.train --synthetic [--epochs 10]
    python -m paper_1912_05234_amd.train --train-images train-images-idx3-ubyte.gz \
        --train-labels train-labels-idx1-ubyte.gz --test-images t10k-images-idx3-ubyte.gz \
        --test-labels t10k-labels-idx1-ubyte.gz

Prints one JSON line per epoch: mean training loss of the epoch, test accuracy and loss, seconds
spent in the training pass.  `--synthetic` uses the seeded stand-in digits of inputs.make_digits.
"""
import argparse
import json
import sys
import time

import numpy as np
import torch

from . import binding, inputs, mnist


def run(train, test, epochs, batch=100, lr=0.05, seed=inputs.DEFAULT_SEED, report=print):
    """Returns the list of per-epoch records; `train` and `test` are (images, labels) numpy pairs."""
    dev = "cuda:0"
    xi, xl = (torch.from_numpy(np.ascontiguousarray(a)).to(dev) for a in train)
    ti, tl = (torch.from_numpy(np.ascontiguousarray(a)).to(dev) for a in test)
    net = binding.CNN(inputs.make_weights(seed), max_batch=max(batch, min(len(test[0]), 10000)))
    steps = -(-len(train[0]) // batch)
    losses = torch.zeros(steps, device=dev)
    records = []
    chunk = min(len(test[0]), 10000)
    for epoch in range(1, epochs + 1):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        net.train_epoch(xi, xl, batch, lr, losses)
        torch.cuda.synchronize()
        seconds = time.perf_counter() - t0
        correct, test_loss = 0, 0.0
        for lo in range(0, len(test[0]), chunk):
            c, l = net.evaluate(ti[lo:lo + chunk], tl[lo:lo + chunk])
            correct += int(c.item())
            test_loss += float(l.item())
        rec = {"epoch": epoch, "train_loss": float(losses.sum().item()) / len(train[0]),
               "test_accuracy": correct / len(test[0]), "test_loss": test_loss / len(test[0]),
               "train_seconds": round(seconds, 4)}
        records.append(rec)
        report(json.dumps(rec))
    net.close()
    return records


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--synthetic", action="store_true")
    ap.add_argument("--train-images"), ap.add_argument("--train-labels")
    ap.add_argument("--test-images"), ap.add_argument("--test-labels")
    ap.add_argument("--epochs", type=int, default=10)
    ap.add_argument("--batch", type=int, default=100)
    ap.add_argument("--lr", type=float, default=0.05)
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        sys.exit("train needs a GPU")
    if args.synthetic:
        train, test = inputs.make_digits(60000, 1), inputs.make_digits(10000, 2)
    else:
        if not all((args.train_images, args.train_labels, args.test_images, args.test_labels)):
            sys.exit("give the four IDX files or --synthetic")
        train = mnist.load_images(args.train_images), mnist.load_labels(args.train_labels)
        test = mnist.load_images(args.test_images), mnist.load_labels(args.test_labels)
    run(train, test, args.epochs, args.batch, args.lr)


if __name__ == "__main__":
    main()
