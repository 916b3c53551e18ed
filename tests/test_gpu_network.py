"""GPU parity of the fused forward / backward / SGD path against the CPU oracle (through the
C ABI): activations, per-batch gradients, the small training configuration, evaluation,
reproducibility and edge cases."""
import numpy as np
import pytest
import torch

import oracle
from paper_1912_05234_amd import binding, inputs
from parity import RTOL_GRAD, RTOL_ACT, RTOL_W, assert_close, assert_close_elementwise

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LR = 0.05


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def weights(seed=inputs.DEFAULT_SEED, biases=False):
    w = inputs.make_weights(seed)
    return inputs.make_random_biases(w, seed + 1) if biases else w


def oracle_grad(images, labels, wflat):
    w = wflat.copy()
    loss, g = oracle.train_batch(images, labels, 0.0, w, want_grad=True)
    return loss, g


# 6149 = 2 * 3072 + 5: more images than the forward kernel has waves, so every wave walks several
# images (the hand-over of the prefetched pixels, the activation dump of later images) and the last
# round is ragged; every image is compared
@pytest.mark.parametrize("B", [1, 7, 64, 6149])
def test_forward_activations(B):
    images, _ = inputs.make_batch(B, 21)
    w = weights(biases=True)
    net = binding.CNN(w, max_batch=B)
    acts = {k: host(v) for k, v in net.forward_activations(dev(images)).items()}
    yhat = host(net.forward(dev(images)))
    wflat = inputs.flatten(w)
    for n in range(B):
        ref = oracle.forward(images[n], wflat)
        for name in ("c1", "s1", "c2", "s2", "y"):
            assert_close(acts[name][n], ref[name], RTOL_ACT, "%s[%d]" % (name, n))
            assert_close_elementwise(acts[name][n], ref[name], RTOL_ACT, "%s[%d]" % (name, n))
        np.testing.assert_array_equal(yhat[n], acts["y"][n])


# 640 is the last size of the small-batch kernel; 1023 / 1025 / 1500 straddle one image per wave
@pytest.mark.parametrize("B", [1, 3, 63, 100, 257, 512, 640, 641, 1023, 1025, 1500])
def test_batch_gradient(B):
    images, labels = inputs.make_batch(B, 22)
    w = weights(biases=True)
    net = binding.CNN(w, max_batch=B)
    grad, loss = net.gradient(dev(images), dev(labels))
    ref_loss, ref_g = oracle_grad(images, labels, inputs.flatten(w))
    g = inputs.unflatten(host(grad))
    r = inputs.unflatten(ref_g)
    for name in ("k1", "b1", "k2", "b2", "fc", "b"):
        assert_close(g[name], r[name], RTOL_GRAD, "grad %s (B=%d)" % (name, B))
    assert abs(host(loss)[0] - ref_loss) <= 1e-5 * ref_loss
    # the weights were not touched
    np.testing.assert_array_equal(host(net.get_weights_flat()), inputs.flatten(w))


@pytest.mark.parametrize("B", [640, 700])
def test_gradient_of_a_repeated_image(B):
    """B copies of ONE image: the batch gradient is B times that image's gradient, so every layer's
    error array of the single image (the bias gradients are its sums per map) is checked against
    the oracle's, in the small-batch kernel (640) and in the one-wave-per-image kernel (700)."""
    image, label = inputs.make_batch(1, 27)
    images, labels = np.repeat(image, B, axis=0), np.repeat(label, B)
    w = weights(biases=True)
    net = binding.CNN(w, max_batch=B)
    grad, loss = net.gradient(dev(images), dev(labels))
    ref_loss, ref_g = oracle_grad(image, label, inputs.flatten(w))
    g, r = inputs.unflatten(host(grad) / B), inputs.unflatten(ref_g)
    for name in ("b", "b2", "b1", "fc", "k2", "k1"):
        assert_close(g[name], r[name], RTOL_GRAD, "single-image grad %s via %d copies" % (name, B))
    assert abs(host(loss)[0] / B - ref_loss) <= 1e-5 * ref_loss


def test_zero_weights_closed_form():
    # all activations 1/2, loss 1.25 per image, only fc and b receive gradient
    B = 10
    images, labels = inputs.make_batch(B, 23)
    net = binding.CNN({}, max_batch=B)
    yhat = host(net.forward(dev(images)))
    assert np.all(yhat == 0.5)
    grad, loss = net.gradient(dev(images), dev(labels))
    g = inputs.unflatten(host(grad))
    assert host(loss)[0] == 1.25 * B
    delta = np.full((B, 10), 0.125, np.float32)
    delta[np.arange(B), labels] = -0.125
    np.testing.assert_array_equal(g["b"], delta.sum(0))
    np.testing.assert_array_equal(g["fc"].reshape(10, 192), np.repeat(delta.sum(0)[:, None] * 0.5, 192, 1))
    for name in ("k1", "b1", "k2", "b2"):
        assert np.all(g[name] == 0)


def run_training(net, images, labels, batch, lr):
    img_d, lab_d = dev(images), dev(labels)
    losses = torch.zeros(len(images) // batch, dtype=torch.float32, device=DEV)
    for s in range(len(images) // batch):
        sl = slice(s * batch, (s + 1) * batch)
        net.train_batch(img_d[sl], lab_d[sl], lr, losses[s:s + 1])
    return host(net.get_weights_flat()), host(losses)


def test_small_training_configuration():
    """1000 images, batch 100, rate 0.05, one epoch: every weight within parity.RTOL_W (1e-5) of the oracle."""
    images, labels = inputs.make_batch(1000, 24)
    w = weights()
    net = binding.CNN(w, max_batch=100)
    w_gpu, losses = run_training(net, images, labels, 100, LR)
    w_ref = inputs.flatten(w)
    ref_losses = []
    for s in range(10):
        sl = slice(s * 100, (s + 1) * 100)
        ref_losses.append(oracle.train_batch(images[sl], labels[sl], float(np.float32(LR)), w_ref))
    g, r = inputs.unflatten(w_gpu), inputs.unflatten(w_ref)
    for name in g:
        assert_close(g[name], r[name], RTOL_W, "weights %s after the epoch" % name)
    assert_close_elementwise(w_gpu[np.abs(w_ref) > 1e-3], w_ref[np.abs(w_ref) > 1e-3], RTOL_W, "weights")
    np.testing.assert_allclose(losses, ref_losses, rtol=1e-5)
    # the update moved the weights by far more than the tolerance (the test can fail)
    assert np.abs(w_ref - inputs.flatten(w)).max() > 100 * RTOL_W * np.abs(w_ref).max()
    # evaluation on fresh images with the trained weights
    ev_images, ev_labels = inputs.make_batch(500, 25)
    net_e = binding.CNN(inputs.unflatten(w_ref), max_batch=500)
    n_ok, loss = net_e.evaluate(dev(ev_images), dev(ev_labels))
    yhat = host(net_e.forward(dev(ev_images)))
    ref_y, ref_ok, ref_loss = oracle.evaluate(ev_images, ev_labels, w_ref)
    assert_close(yhat, ref_y, RTOL_ACT, "yhat")
    # the count may differ only on images whose two largest outputs tie to within the tolerance
    top2 = np.sort(ref_y, axis=1)[:, -2:]
    near_ties = int((top2[:, 1] - top2[:, 0] <= 2 * RTOL_ACT).sum())
    assert abs(int(host(n_ok)[0]) - ref_ok) <= near_ties
    assert int(host(n_ok)[0]) == int((yhat.argmax(1) == ev_labels).sum())
    assert abs(host(loss)[0] - ref_loss) <= 1e-5 * ref_loss


def test_epoch_call_matches_the_oracle_and_the_per_batch_calls():
    """cnn_train_epoch over 450 images in batches of 100 (last batch 50): weights within parity.RTOL_W (1e-5) of the
    oracle's five steps, per-step losses, and bitwise equal to five cnn_train_batch calls."""
    images, labels = inputs.make_batch(450, 31)
    w = weights(biases=True)
    d_im, d_lb = dev(images), dev(labels)
    net = binding.CNN(w, max_batch=100)
    losses = torch.zeros(5, dtype=torch.float32, device=DEV)
    net.train_epoch(d_im, d_lb, 100, LR, losses)
    w_epoch = host(net.get_weights_flat())
    w_ref = inputs.flatten(w)
    ref_losses = []
    for first in range(0, 450, 100):
        sl = slice(first, min(450, first + 100))
        ref_losses.append(oracle.train_batch(images[sl], labels[sl], float(np.float32(LR)), w_ref))
    g, r = inputs.unflatten(w_epoch), inputs.unflatten(w_ref)
    for name in g:
        assert_close(g[name], r[name], RTOL_W, "weights %s after the epoch call" % name)
    np.testing.assert_allclose(host(losses), ref_losses, rtol=1e-5)
    net2 = binding.CNN(w, max_batch=100)
    loss1 = torch.zeros(1, dtype=torch.float32, device=DEV)
    for first in range(0, 450, 100):
        net2.train_batch(d_im[first:first + 100], d_lb[first:first + 100], LR, loss1)
    w_steps = host(net2.get_weights_flat())
    assert np.array_equal(w_epoch, w_steps)
    # argument checks
    with pytest.raises(binding.CnnError):
        net.train_epoch(d_im, d_lb, 101, LR)      # batch above max_batch
    with pytest.raises(ValueError):
        net.train_epoch(d_im, d_lb, 100, LR, torch.zeros(4, dtype=torch.float32, device=DEV))


def test_operand_table_follows_the_weights_through_updates():
    """The kernels read the weights from a copy laid out as matrix operands that the update kernel
    patches in place.  After several steps (small-batch and large-batch kernels, biases moving too)
    a context rebuilt from the current weights must give bitwise the same outputs and gradients."""
    images, labels = inputs.make_batch(1800, 41)
    d_im, d_lb = dev(images), dev(labels)
    net = binding.CNN(weights(biases=True), max_batch=1000)
    for first, size in ((0, 100), (100, 37), (137, 700), (837, 963)):   # 700 and 963 use the large-batch kernel
        net.train_batch(d_im[first:first + size], d_lb[first:first + size], LR)
    fresh = binding.CNN({k: host(v) for k, v in net.get_weights().items()}, max_batch=1000)
    probe_im, probe_lb = d_im[:1000], d_lb[:1000]
    assert np.array_equal(host(net.forward(probe_im)), host(fresh.forward(probe_im)))
    for size in (64, 1000):
        g_a, l_a = net.gradient(probe_im[:size], probe_lb[:size])
        g_b, l_b = fresh.gradient(probe_im[:size], probe_lb[:size])
        assert np.array_equal(host(g_a), host(g_b)) and np.array_equal(host(l_a), host(l_b))
    # and set_weights rebuilds it too
    net.set_weights(weights(seed=77))
    ref = binding.CNN(weights(seed=77), max_batch=1000)
    assert np.array_equal(host(net.forward(probe_im)), host(ref.forward(probe_im)))


def test_step_is_bitwise_reproducible_and_zero_rate_is_identity():
    images, labels = inputs.make_batch(300, 26)
    w = weights(biases=True)
    runs = []
    for _ in range(2):
        net = binding.CNN(w, max_batch=300)
        runs.append(run_training(net, images, labels, 150, LR)[0])
    np.testing.assert_array_equal(runs[0], runs[1])
    net = binding.CNN(w, max_batch=300)
    net.train_batch(dev(images), dev(labels), 0.0)
    np.testing.assert_array_equal(host(net.get_weights_flat()), inputs.flatten(w))


def test_batch_invariants_on_gpu():
    images, labels = inputs.make_batch(6, 27)
    w = weights(biases=True)
    net = binding.CNN(w, max_batch=64)
    g_all, _ = net.gradient(dev(images), dev(labels))
    g_sum = np.zeros(oracle.NPARAM)
    for n in range(6):
        g_n, _ = net.gradient(dev(images[n:n + 1]), dev(labels[n:n + 1]))
        g_sum += host(g_n)
    assert_close(host(g_all), g_sum, 1e-6, "sum of single-image gradients")
    # B copies of one image: B times its gradient
    g_rep, _ = net.gradient(dev(np.repeat(images[:1], 5, 0)), dev(np.repeat(labels[:1], 5)))
    g_one, _ = net.gradient(dev(images[:1]), dev(labels[:1]))
    assert_close(host(g_rep), 5 * host(g_one), 1e-6, "repeated image")


def test_ragged_batch_beyond_the_workgroup_cap():
    """More images than gradient partials: workgroups loop, the last round is ragged."""
    B = 2 * 1024 + 37
    images, labels = inputs.make_batch(B, 28)
    w = weights(biases=True)
    net = binding.CNN(w, max_batch=B)
    wflat = inputs.flatten(w)
    yhat = host(net.forward(dev(images)))
    for n in (0, 1023, 1024, 2047, 2048, B - 1):
        assert_close(yhat[n], oracle.forward(images[n], wflat)["y"], RTOL_ACT, "yhat[%d]" % n)
    grad, loss = net.gradient(dev(images), dev(labels))
    ref_loss, ref_g = oracle_grad(images, labels, wflat)
    assert_close(host(grad), ref_g, RTOL_GRAD, "gradient")
    assert abs(host(loss)[0] - ref_loss) <= 1e-5 * ref_loss
    n_ok, _ = net.evaluate(dev(images), dev(labels))
    assert int(host(n_ok)[0]) == int((yhat.argmax(1) == labels).sum())


@pytest.mark.parametrize("B", [5, 700])   # small-batch and large-batch kernels
def test_saturated_sigmoids_stay_finite(B):
    """Weights fifty times the usual size drive every sigmoid to 0 or 1: exp overflows to inf and the
    reciprocal must give exactly 0, never NaN; outputs and gradients still match the oracle."""
    images, labels = inputs.make_batch(B, 47)
    w = {k: (50.0 * v).astype(np.float32) for k, v in weights(biases=True).items()}
    net = binding.CNN(w, max_batch=B)
    yhat = host(net.forward(dev(images)))
    grad, loss = net.gradient(dev(images), dev(labels))
    assert np.isfinite(yhat).all() and np.isfinite(host(grad)).all() and np.isfinite(host(loss)).all()
    wflat = inputs.flatten(w)
    ref_y = np.stack([oracle.forward(images[n], wflat)["y"] for n in range(min(B, 16))])
    assert_close(yhat[:len(ref_y)], ref_y, RTOL_ACT, "saturated yhat")
    ref_loss, ref_g = oracle_grad(images, labels, wflat)
    assert_close(host(grad), ref_g, RTOL_GRAD, "saturated gradient")
    assert abs(host(loss)[0] - ref_loss) <= 1e-5 * max(ref_loss, 1.0)


def test_kernel_timing_aid():
    """cnn_profile_begin / cnn_profile_read: one reading per recorded step, only the first
    `capacity` steps are recorded, readings are positive and of a plausible size, and recording
    does not change the result."""
    images, labels = inputs.make_batch(300, 43)
    d_im, d_lb = dev(images), dev(labels)
    w = weights()
    plain, timed = binding.CNN(w, max_batch=100), binding.CNN(w, max_batch=100)
    timed.profile_begin(4)
    for net in (plain, timed):
        for first in (0, 100, 200):
            net.train_batch(d_im[first:first + 100], d_lb[first:first + 100], LR)
    ms = timed.profile_read(4)
    assert len(ms) == 3 and all(0.0 < t < 5.0 for t in ms)
    for first in (0, 100, 200, 0, 100, 200):      # six steps, capacity four
        timed.train_batch(d_im[first:first + 100], d_lb[first:first + 100], LR)
        plain.train_batch(d_im[first:first + 100], d_lb[first:first + 100], LR)
    assert len(timed.profile_read(4)) == 4
    timed.profile_begin(0)
    assert timed.profile_read(4) == []
    assert np.array_equal(host(plain.get_weights_flat()), host(timed.get_weights_flat()))


def test_context_errors():
    net = binding.CNN(weights(), max_batch=8)
    images, labels = inputs.make_batch(9, 29)
    with pytest.raises(binding.CnnError) as e:
        net.forward(dev(images))             # B > max_batch
    assert e.value.code == -1
    with pytest.raises(binding.CnnError):
        net.train_batch(dev(images), dev(labels), LR)
    with pytest.raises(binding.CnnError):
        net.forward(dev(images[:0]))         # empty batch
    # weights round trip
    w2 = weights(seed=5, biases=True)
    net.set_weights(w2)
    np.testing.assert_array_equal(host(net.get_weights_flat()), inputs.flatten(w2))



def test_training_learns_the_synthetic_digits():
    """End to end on the learnable stand-in for MNIST: one epoch of 600 steps at rate 1 (the
    batch-mean update makes that a summed update at 0.01) and the held-out accuracy is above
    95 %; the first three steps at that rate also match the oracle."""
    from paper_1912_05234_amd import train
    tr, te = inputs.make_digits(60000, 1), inputs.make_digits(10000, 2)
    recs = train.run(tr, te, epochs=2, batch=100, lr=1.0, report=lambda line: None)
    assert recs[0]["test_accuracy"] > 0.95 and recs[1]["test_accuracy"] >= recs[0]["test_accuracy"] - 0.01
    assert recs[1]["train_loss"] < recs[0]["train_loss"] and recs[1]["test_loss"] < 0.1
    net = binding.CNN(inputs.make_weights(), max_batch=100)
    w_ref = inputs.flatten(inputs.make_weights())
    d_im, d_lb = dev(tr[0][:300]), dev(tr[1][:300])
    for s in range(3):
        net.train_batch(d_im[100 * s:100 * s + 100], d_lb[100 * s:100 * s + 100], 1.0)
        oracle.train_batch(tr[0][100 * s:100 * s + 100], tr[1][100 * s:100 * s + 100], 1.0, w_ref)
    assert_close(host(net.get_weights_flat()), w_ref, RTOL_W, "weights after three steps at rate 1")
    net.close()

