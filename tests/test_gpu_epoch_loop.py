"""Device-side epoch loop (cnn_epoch_mode(ctx, 1, ...)): bitwise the weights and losses of the
two-kernel step, the oracle's to parity.RTOL_W, reproducible, and a give-up path that can be forced from the
host so that every kernel still exits normally."""
import numpy as np
import pytest
import torch

import oracle
from paper_1912_05234_amd import binding, inputs
from parity import RTOL_W, assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LR = 0.05
ETIMEOUT = -5


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def weights(seed=5):
    w = inputs.make_weights(seed)
    rng = np.random.default_rng(seed + 1)
    for name in ("b1", "b2", "b"):
        w[name] = rng.uniform(-0.1, 0.1, w[name].shape).astype(np.float32)
    return w


def run(images, labels, batch, device_loop, n_losses):
    net = binding.CNN(weights(), max_batch=batch)
    net.epoch_mode(device_loop, 1.0)
    losses = torch.zeros(n_losses, dtype=torch.float32, device=DEV)
    net.train_epoch(images, labels, batch, LR, losses)
    assert net.epoch_status() == 0
    return host(net.get_weights_flat()), host(losses), net


@pytest.mark.parametrize("N,batch", [(1000, 100), (1050, 100), (96, 8), (512, 256), (600, 1), (999, 37)])
def test_device_loop_equals_the_two_kernel_step_bitwise(N, batch):
    images, labels = inputs.make_batch(N, 51)
    d_im, d_lb = dev(images), dev(labels)
    steps = -(-N // batch)
    w_loop, l_loop, _ = run(d_im, d_lb, batch, 0, steps)
    w_dev, l_dev, net = run(d_im, d_lb, batch, 1, steps)
    assert np.array_equal(w_dev, w_loop) and np.array_equal(l_dev, l_loop)
    assert np.abs(w_dev - inputs.flatten(weights())).max() > 0
    # a second epoch on the same context (the barrier counts go on), against a second two-kernel epoch
    net.train_epoch(d_im, d_lb, batch, LR)
    assert net.epoch_status() == 0
    ref = binding.CNN(weights(), max_batch=batch)
    ref.train_epoch(d_im, d_lb, batch, LR)
    ref.train_epoch(d_im, d_lb, batch, LR)
    assert np.array_equal(host(net.get_weights_flat()), host(ref.get_weights_flat()))


def test_device_loop_against_the_oracle():
    images, labels = inputs.make_batch(1000, 52)
    w_dev, l_dev, _ = run(dev(images), dev(labels), 100, 1, 10)
    w_ref = inputs.flatten(weights())
    ref_losses = [oracle.train_batch(images[k:k + 100], labels[k:k + 100], float(np.float32(LR)), w_ref)
                  for k in range(0, 1000, 100)]
    g, r = inputs.unflatten(w_dev), inputs.unflatten(w_ref)
    for name in g:
        assert_close(g[name], r[name], RTOL_W, "weights %s after ten steps in one kernel" % name)
    np.testing.assert_allclose(l_dev, ref_losses, rtol=1e-5)


def test_batches_that_do_not_fit_fall_back():
    images, labels = inputs.make_batch(514, 53)
    d_im, d_lb = dev(images), dev(labels)
    w_loop, _, _ = run(d_im, d_lb, 257, 0, 2)
    w_dev, _, _ = run(d_im, d_lb, 257, 1, 2)   # more workgroups than the loop takes: two-kernel steps
    assert np.array_equal(w_dev, w_loop)


def test_give_up_path_forced_from_the_host():
    """Every barrier also waits for a workgroup that does not exist, for at most 2 ms: all workgroups
    give up at the first barrier (before any update), the kernel ends, the status call reports it
    once, and the context trains normally afterwards."""
    images, labels = inputs.make_batch(1000, 54)
    d_im, d_lb = dev(images), dev(labels)
    net = binding.CNN(weights(), max_batch=100)
    before = host(net.get_weights_flat())
    net.epoch_mode(1, 0.002, never_arrives=True)
    net.train_epoch(d_im, d_lb, 100, LR)
    assert net.epoch_status() == ETIMEOUT
    assert b"given up" in binding.lib().cnn_strerror(ETIMEOUT)
    assert np.array_equal(host(net.get_weights_flat()), before)     # gave up before the first update
    assert net.epoch_status() == 0                                  # reported once, state re-armed
    # a kernel launched while the error word is still set does nothing
    net.train_epoch(d_im, d_lb, 100, LR)
    net.train_epoch(d_im, d_lb, 100, LR)
    assert net.epoch_status() == ETIMEOUT
    assert np.array_equal(host(net.get_weights_flat()), before)
    net.epoch_mode(1, 1.0)
    net.train_epoch(d_im, d_lb, 100, LR)
    assert net.epoch_status() == 0
    w_loop, _, _ = run(d_im, d_lb, 100, 0, 10)
    assert np.array_equal(host(net.get_weights_flat()), w_loop)
