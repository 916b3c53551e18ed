"""Seeded synthetic inputs shaped like the paper's workload (Section 4.2:
MNIST digits, 28x28 pixels, 10 classes, batches of 100, rate 0.05).

This module only draws numbers.  It contains none of the network's
arithmetic and is the one piece of code that both the GPU library's callers
and the CPU oracle's callers may use.

Recipe (one numpy PCG64 stream per call, draw order fixed):
  weights: k1[6,5,5], k2[12,6,5,5], fc[10,12,1,4,4] uniform in
           [-1/sqrt(fan_in), +1/sqrt(fan_in)) with fan_in 25 / 150 / 192,
           drawn in that order; biases b1, b2, b are zero;
  images:  float32 uniform [0, 1);
  labels:  int32 uniform over {0..9}, drawn after the images of the same call;
  digits:  a learnable stand-in for MNIST (`make_digits`): ten fixed prototypes, each the sum of six
           Gaussian strokes at positions drawn once from the prototype seed, and per sample a label,
           a shift of up to two pixels each way and uniform pixel noise, clipped to [0, 1].
"""
import numpy as np

PARAM_SHAPES = (("k1", (6, 5, 5)), ("b1", (6,)), ("k2", (12, 6, 5, 5)), ("b2", (12,)),
                ("fc", (10, 12, 1, 4, 4)), ("b", (10,)))
NPARAM = 3898
DEFAULT_SEED = 191205234


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def make_weights(seed=DEFAULT_SEED):
    """dict name -> float32 array, layout as in the paper's `forward` signature."""
    rng = _rng(seed)
    out = {}
    for name, shp in PARAM_SHAPES:
        if name in ("b1", "b2", "b"):
            out[name] = np.zeros(shp, np.float32)
    for name, fan_in in (("k1", 25), ("k2", 150), ("fc", 192)):
        shp = dict(PARAM_SHAPES)[name]
        bound = 1.0 / np.sqrt(float(fan_in))
        u = rng.random(shp, dtype=np.float64)
        out[name] = ((2.0 * u - 1.0) * bound).astype(np.float32)
    return {name: out[name] for name, _ in PARAM_SHAPES}


def make_random_biases(weights, seed):
    """Copy of `weights` with small non-zero biases (tests that must see the bias path)."""
    rng = _rng(seed)
    w = {k: v.copy() for k, v in weights.items()}
    for name in ("b1", "b2", "b"):
        w[name] = ((rng.random(w[name].shape) - 0.5) * 0.2).astype(np.float32)
    return w


def make_batch(n, seed):
    """(images float32 [n,28,28] in [0,1), labels int32 [n] in 0..9)."""
    rng = _rng(seed)
    images = rng.random((n, 28, 28), dtype=np.float32)
    labels = rng.integers(0, 10, size=n, dtype=np.int32)
    return images, labels


PROTOTYPE_SEED = 28281010


def digit_prototypes():
    """float32 [10, 32, 32]: one blob pattern per class on a canvas with a two-pixel margin."""
    rng = _rng(PROTOTYPE_SEED)
    yy, xx = np.mgrid[0:32, 0:32].astype(np.float64)
    protos = np.zeros((10, 32, 32))
    for c in range(10):
        for _ in range(6):
            cy, cx = rng.uniform(7.0, 25.0, size=2)
            sy, sx = rng.uniform(1.5, 4.0, size=2)
            protos[c] += np.exp(-0.5 * (((yy - cy) / sy) ** 2 + ((xx - cx) / sx) ** 2))
        protos[c] /= protos[c].max()
    return protos.astype(np.float32)


def make_digits(n, seed, noise=0.25):
    """(images float32 [n,28,28] in [0,1], labels int32 [n]): shifted, noisy class prototypes."""
    rng = _rng(seed)
    protos = digit_prototypes()
    labels = rng.integers(0, 10, size=n, dtype=np.int32)
    dy = rng.integers(0, 5, size=n)
    dx = rng.integers(0, 5, size=n)
    images = np.empty((n, 28, 28), np.float32)
    for i in range(n):
        images[i] = protos[labels[i], dy[i]:dy[i] + 28, dx[i]:dx[i] + 28]
    images += (rng.random((n, 28, 28), dtype=np.float32) - 0.5) * np.float32(2.0 * noise)
    np.clip(images, 0.0, 1.0, out=images)
    return images, labels


def make_signed(shape, seed):
    """float32 uniform [-1, 1): operands of the per-layer micro-benchmarks."""
    rng = _rng(seed)
    return (2.0 * rng.random(shape, dtype=np.float32) - 1.0).astype(np.float32)


def flatten(weights, dtype=np.float32):
    return np.ascontiguousarray(
        np.concatenate([np.asarray(weights[n], dtype=dtype).ravel() for n, _ in PARAM_SHAPES]))


def unflatten(flat):
    out, off = {}, 0
    for name, shp in PARAM_SHAPES:
        n = int(np.prod(shp))
        out[name] = flat[off:off + n].reshape(shp)
        off += n
    return out
