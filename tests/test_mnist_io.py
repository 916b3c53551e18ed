"""CPU tests of the IDX reader and of the learnable synthetic digits (the stand-in for MNIST,
Section 4.2), including that the oracle learns them."""
import numpy as np
import pytest

import oracle
from paper_1912_05234_amd import inputs, mnist


@pytest.mark.parametrize("name", ["images.idx3-ubyte", "images.idx3-ubyte.gz"])
def test_idx_round_trip(tmp_path, name):
    rng = np.random.default_rng(3)
    pixels = rng.integers(0, 256, size=(7, 28, 28), dtype=np.uint8)
    labels = rng.integers(0, 10, size=7, dtype=np.uint8)
    ip, lp = tmp_path / name, tmp_path / name.replace("images.idx3", "labels.idx1")
    mnist.write_idx(ip, pixels)
    mnist.write_idx(lp, labels)
    np.testing.assert_array_equal(mnist.read_idx(ip), pixels)
    img, lab = mnist.load_images(ip), mnist.load_labels(lp)
    assert img.dtype == np.float32 and img.shape == (7, 28, 28) and lab.dtype == np.int32
    np.testing.assert_array_equal(lab, labels)
    np.testing.assert_array_equal(img, pixels.astype(np.float32) / np.float32(255))
    assert img.min() >= 0.0 and img.max() <= 1.0
    # the published header of an image file: 0x00000803, then count, rows, columns, big-endian
    raw = (__import__("gzip").open if name.endswith(".gz") else open)(ip, "rb").read()
    assert raw[:16] == bytes([0, 0, 8, 3, 0, 0, 0, 7, 0, 0, 0, 28, 0, 0, 0, 28])


def test_idx_errors(tmp_path):
    p = tmp_path / "bad"
    p.write_bytes(b"\x00\x00\x0d\x01\x00\x00\x00\x01\x00")          # float type code
    with pytest.raises(ValueError):
        mnist.read_idx(p)
    p.write_bytes(b"\x00\x00\x08\x01\x00\x00\x00\x05\x01\x02")      # promises 5 items, holds 2
    with pytest.raises(ValueError):
        mnist.read_idx(p)
    p.write_bytes(b"\x00\x00")
    with pytest.raises(ValueError):
        mnist.read_idx(p)
    mnist.write_idx(p, np.zeros((3, 27, 28), np.uint8))
    with pytest.raises(ValueError):
        mnist.load_images(p)
    mnist.write_idx(p, np.array([1, 2, 10], np.uint8))
    with pytest.raises(ValueError):
        mnist.load_labels(p)


def test_digits_are_seeded_bounded_and_class_dependent():
    a, la = inputs.make_digits(400, 5)
    b, lb = inputs.make_digits(400, 5)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(la, lb)
    assert a.shape == (400, 28, 28) and a.dtype == np.float32 and la.dtype == np.int32
    assert a.min() >= 0.0 and a.max() <= 1.0 and set(np.unique(la)) <= set(range(10))
    c, lc = inputs.make_digits(400, 6)
    assert not np.array_equal(a, c)
    # images of one class are closer to their class mean than to the other class means
    means = np.stack([a[la == k].mean(0) for k in range(10)])
    d = ((c[:, None] - means[None]) ** 2).sum((2, 3))
    assert (d.argmin(1) == lc).mean() > 0.9


def test_oracle_loss_falls_on_the_digits():
    """Fifteen oracle steps on one fixed batch at rate 2: the summed loss falls below half its
    initial value (the long plateau that follows, before the classes separate, needs hundreds
    of steps and is covered on the GPU)."""
    images, labels = inputs.make_digits(40, 11)
    w = inputs.flatten(inputs.make_weights())
    losses = [oracle.train_batch(images, labels, 2.0, w) for _ in range(15)]
    assert losses[-1] < 0.5 * losses[0] and all(np.isfinite(losses))
