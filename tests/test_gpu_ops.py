"""GPU parity of the per-operation entry points against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1912_05234_amd import binding, inputs
from parity import RTOL_GRAD, RTOL_ACT, assert_close, assert_close_elementwise

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


# (B, Cin, H, W, Cout, KH, KW): the network's two layers, ragged shapes, 1x1 and full-size kernels,
# more than 16 output maps (two M tiles) and more than 256 taps (two groups of N tiles), batches that
# make every workgroup loop over several image groups with a ragged last one, and two shapes too
# large for LDS (served by the plain kernels)
CONV_CASES = [(3, 1, 28, 28, 6, 5, 5), (5, 6, 12, 12, 12, 5, 5), (2, 3, 9, 7, 4, 3, 2), (1, 2, 5, 5, 3, 1, 1),
              (4, 12, 4, 4, 10, 4, 4), (1, 1, 6, 5, 1, 6, 5), (37, 2, 11, 13, 5, 4, 6), (3, 3, 8, 8, 20, 3, 3),
              (2, 30, 6, 6, 5, 3, 3), (2600, 2, 6, 6, 3, 3, 3), (1300, 6, 12, 12, 12, 5, 5), (131, 1, 3, 3, 1, 2, 2),
              (2, 3, 80, 80, 4, 3, 3), (1, 40, 20, 20, 2, 5, 5),
              # odd ones: one-row images, 17 and 33 output maps, a kernel as large as the image, packing by 7 and by 6
              (3, 2, 1, 300, 3, 1, 7), (2, 1, 40, 3, 17, 2, 3), (5, 7, 5, 9, 33, 5, 2), (1, 3, 16, 16, 1, 16, 16),
              (9, 4, 10, 10, 2, 1, 4), (70, 1, 2, 2, 16, 2, 2),
              # packing by 4 and by 8 (16-byte stores), by 6 (8-byte stores)
              (40, 2, 6, 6, 3, 3, 3), (4, 2, 10, 12, 1, 3, 5),
              # the second convolution's shape with one image and with a ragged nine (its input gradient has a
              # kernel of its own, one wave per image)
              (1, 6, 12, 12, 12, 5, 5), (9, 6, 12, 12, 12, 5, 5)]


def oracle_conv_fwd(x, k, b):
    return np.stack([oracle.mconv(x[n], k, b).reshape(k.shape[0], x.shape[2] - k.shape[2] + 1, -1)
                     for n in range(x.shape[0])])


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_fwd(case):
    B, Cin, H, W, Cout, KH, KW = case
    x = inputs.make_signed((B, Cin, H, W), 1)
    k = inputs.make_signed((Cout, Cin, KH, KW), 2)
    b = inputs.make_signed((Cout,), 3)
    ref = oracle_conv_fwd(x, k, b)
    assert_close(host(binding.conv_fwd(dev(x), dev(k), dev(b))), ref, RTOL_ACT, "conv_fwd")
    assert_close(host(binding.conv_fwd(dev(x), dev(k), dev(b), valu=True)), ref, RTOL_ACT, "conv_fwd_valu")
    ref0 = oracle_conv_fwd(x, k, np.zeros(Cout, np.float32))
    assert_close(host(binding.conv_fwd(dev(x), dev(k), None)), ref0, RTOL_ACT, "conv_fwd no bias")


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_bwd_input(case):
    B, Cin, H, W, Cout, KH, KW = case
    Ho, Wo = H - KH + 1, W - KW + 1
    d = inputs.make_signed((B, Cout, Ho, Wo), 4)
    k = inputs.make_signed((Cout, Cin, KH, KW), 5)
    ref = np.zeros((B, Cin, H, W), np.float64)
    for n in range(B):
        for co in range(Cout):
            ref[n] += oracle.backin(d[n, co][None].astype(np.float64), k[co].astype(np.float64), (Cin, H, W))
    assert_close(host(binding.conv_bwd_input(dev(d), dev(k), H, W)), ref, RTOL_ACT, "conv_bwd_input")
    assert_close(host(binding.conv_bwd_input(dev(d), dev(k), H, W, valu=True)), ref, RTOL_ACT, "conv_bwd_input_valu")


def test_conv_bwd_input_of_the_second_convolution_with_looping_waves():
    """4101 images of C2's shape: more images than the col2im kernel has waves (512 workgroups of eight),
    so waves take a second image (the hand-over of the prefetched error) and the last round is ragged;
    sampled images against the oracle, and the bordered-convolution kernels' result for all of them."""
    B, Cin, H, W, Cout, KH, KW = 4101, 6, 12, 12, 12, 5, 5
    d = inputs.make_signed((B, Cout, 8, 8), 41)
    k = inputs.make_signed((Cout, Cin, KH, KW), 42)
    got = host(binding.conv_bwd_input(dev(d), dev(k), H, W))
    sample = sorted(set(list(range(8)) + list(range(4090, 4101)) + list(range(0, B, 397))))
    ref = np.zeros((len(sample), Cin, H, W), np.float64)
    for i, n in enumerate(sample):
        for co in range(Cout):
            ref[i] += oracle.backin(d[n, co][None].astype(np.float64), k[co].astype(np.float64), (Cin, H, W))
    assert_close(got[sample], ref, RTOL_ACT, "conv_bwd_input of C2, sampled images")
    # the plain kernel computes the same sums in another order: every image
    plain = host(binding.conv_bwd_input(dev(d), dev(k), H, W, valu=True))
    assert_close(got, plain.astype(np.float64), RTOL_ACT, "conv_bwd_input of C2 against the plain kernel")


def test_forward_and_weight_gradient_of_the_second_convolution_with_looping_waves():
    """The same 4101 images through the one-wave-per-image forward and weight-gradient kernels of C2's
    shape: sampled images of the forward pass against the oracle, every image against the plain
    kernel; the weight and bias gradient (a sum over all images) against the plain kernel and, for
    the last 37 images alone, against the oracle."""
    B, Cin, H, W, Cout, KH, KW = 4101, 6, 12, 12, 12, 5, 5
    x = inputs.make_signed((B, Cin, H, W), 43)
    k = inputs.make_signed((Cout, Cin, KH, KW), 44)
    b = inputs.make_signed((Cout,), 45)
    d = inputs.make_signed((B, Cout, 8, 8), 46)
    got = host(binding.conv_fwd(dev(x), dev(k), dev(b)))
    sample = sorted(set(list(range(8)) + list(range(4090, 4101)) + list(range(0, B, 397))))
    assert_close(got[sample], oracle_conv_fwd(x[sample], k, b), RTOL_ACT, "conv_fwd of C2, sampled images")
    plain = host(binding.conv_fwd(dev(x), dev(k), dev(b), valu=True))
    assert_close(got, plain.astype(np.float64), RTOL_ACT, "conv_fwd of C2 against the plain kernel")
    gk, gb = binding.conv_bwd_weight(dev(x), dev(d))
    pk, pb = binding.conv_bwd_weight(dev(x), dev(d), workspace=False)
    assert_close(host(gk), host(pk).astype(np.float64), RTOL_GRAD, "conv_bwd_weight of C2 against the plain kernel")
    assert_close(host(gb), host(pb).astype(np.float64), RTOL_GRAD, "conv_bwd_weight bias of C2 against the plain kernel")
    tail = slice(B - 37, B)
    gk, gb = binding.conv_bwd_weight(dev(x[tail]), dev(d[tail]))
    rk = np.zeros((Cout, Cin, KH, KW), np.float64)
    rb = np.zeros(Cout, np.float64)
    for n in range(B - 37, B):
        for co in range(Cout):
            rk[co] += oracle.backweights(d[n, co][None].astype(np.float64), x[n].astype(np.float64)).reshape(Cin, KH, KW)
            rb[co] += oracle.backbias(d[n, co].astype(np.float64))
    assert_close(host(gk), rk, RTOL_GRAD, "conv_bwd_weight of C2, 37 images")
    assert_close(host(gb), rb, RTOL_GRAD, "conv_bwd_weight bias of C2, 37 images")


def test_the_three_calls_of_the_first_convolution_with_looping_waves():
    """4101 images of C1's shape through its one-wave-per-image forward, weight-gradient and input-gradient kernels (waves
    take a second image, ragged last round): sampled images against the oracle, every image against the
    plain kernel; without a bias; the gradient sums against the plain kernel and the oracle."""
    B = 4101
    x = inputs.make_signed((B, 1, 28, 28), 47)
    k = inputs.make_signed((6, 1, 5, 5), 48)
    b = inputs.make_signed((6,), 49)
    got = host(binding.conv_fwd(dev(x), dev(k), dev(b)))
    sample = sorted(set(list(range(8)) + list(range(4090, 4101)) + list(range(0, B, 397))))
    assert_close(got[sample], oracle_conv_fwd(x[sample], k, b), RTOL_ACT, "conv_fwd of C1, sampled images")
    plain = host(binding.conv_fwd(dev(x), dev(k), dev(b), valu=True))
    assert_close(got, plain.astype(np.float64), RTOL_ACT, "conv_fwd of C1 against the plain kernel")
    got0 = host(binding.conv_fwd(dev(x[:9]), dev(k), None))
    assert_close(got0, oracle_conv_fwd(x[:9], k, np.zeros(6, np.float32)), RTOL_ACT, "conv_fwd of C1 without bias")
    # weight and bias gradient over the same images: against the plain kernel, and the last 37 against the oracle
    d = inputs.make_signed((B, 6, 24, 24), 50)
    gk, gb = binding.conv_bwd_weight(dev(x), dev(d))
    pk, pb = binding.conv_bwd_weight(dev(x), dev(d), workspace=False)
    assert_close(host(gk), host(pk).astype(np.float64), RTOL_GRAD, "conv_bwd_weight of C1 against the plain kernel")
    assert_close(host(gb), host(pb).astype(np.float64), RTOL_GRAD, "conv_bwd_weight bias of C1 against the plain kernel")
    gk, gb = binding.conv_bwd_weight(dev(x[B - 37:]), dev(d[B - 37:]))
    rk, rb = np.zeros((6, 1, 5, 5), np.float64), np.zeros(6, np.float64)
    for n in range(B - 37, B):
        for co in range(6):
            rk[co] += oracle.backweights(d[n, co][None].astype(np.float64), x[n].astype(np.float64)).reshape(1, 5, 5)
            rb[co] += oracle.backbias(d[n, co].astype(np.float64))
    assert_close(host(gk), rk, RTOL_GRAD, "conv_bwd_weight of C1, 37 images")
    assert_close(host(gb), rb, RTOL_GRAD, "conv_bwd_weight bias of C1, 37 images")
    # input gradient of the same error (a vector-unit kernel of its own for this shape): sampled images against
    # the oracle, every image against the plain kernel
    gi = host(binding.conv_bwd_input(dev(d), dev(k), 28, 28))
    ref = np.zeros((len(sample), 1, 28, 28), np.float64)
    for i, n in enumerate(sample):
        for co in range(6):
            ref[i] += oracle.backin(d[n, co][None].astype(np.float64), k[co].astype(np.float64), (1, 28, 28))
    assert_close(gi[sample], ref, RTOL_ACT, "conv_bwd_input of C1, sampled images")
    plain = host(binding.conv_bwd_input(dev(d), dev(k), 28, 28, valu=True))
    assert_close(gi, plain.astype(np.float64), RTOL_ACT, "conv_bwd_input of C1 against the plain kernel")


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_bwd_weight(case):
    B, Cin, H, W, Cout, KH, KW = case
    Ho, Wo = H - KH + 1, W - KW + 1
    x = inputs.make_signed((B, Cin, H, W), 6)
    d = inputs.make_signed((B, Cout, Ho, Wo), 7)
    ref_k = np.zeros((Cout, Cin, KH, KW), np.float64)
    ref_b = np.zeros(Cout, np.float64)
    for n in range(B):
        for co in range(Cout):
            ref_k[co] += oracle.backweights(d[n, co][None].astype(np.float64), x[n].astype(np.float64))
            ref_b[co] += oracle.backbias(d[n, co].astype(np.float64))
    for workspace in (True, False):   # the matrix-core kernel, then the one that needs no workspace
        d_k, d_b = binding.conv_bwd_weight(dev(x), dev(d), workspace=workspace)
        assert_close(host(d_k), ref_k, RTOL_ACT, "conv_bwd_weight")
        assert_close(host(d_b), ref_b, RTOL_ACT, "conv_bwd_bias")
        d_k2, none = binding.conv_bwd_weight(dev(x), dev(d), want_bias=False, workspace=workspace)
        assert none is None and torch.equal(d_k2, d_k)   # deterministic order


def test_vector_unit_convolutions_keep_non_finite_values_local():
    """cnn_conv_fwd_valu / cnn_conv_bwd_input_valu multiply nothing by padding zeros: a NaN in the
    data reaches exactly the outputs whose defining sums contain it."""
    x = inputs.make_signed((2, 6, 12, 12), 61)
    k = inputs.make_signed((12, 6, 5, 5), 62)
    x[1, 3, 7, 2] = np.nan
    out = host(binding.conv_fwd(dev(x), dev(k), None, valu=True))
    hit = np.zeros(out.shape, bool)
    hit[1, :, 3:8, 0:3] = True          # output (y, x) reads input rows y..y+4, columns x..x+4
    assert np.array_equal(np.isnan(out), hit)
    d = inputs.make_signed((2, 12, 8, 8), 63)
    d[0, 5, 2, 6] = np.inf
    g = host(binding.conv_bwd_input(dev(d), dev(k), 12, 12, valu=True))
    bad = ~np.isfinite(g)
    want = np.zeros(g.shape, bool)
    want[0, :, 2:7, 6:11] = True        # d_out (y, x) spreads to input rows y..y+4, columns x..x+4
    assert np.array_equal(bad, want)


@pytest.mark.parametrize("shape", [(2, 6, 24, 24), (3, 12, 8, 8), (1, 1, 2, 2), (5, 3, 6, 10)])
def test_avgpool_fwd_bwd(shape):
    x = inputs.make_signed(shape, 8)
    assert_close(host(binding.avgpool_fwd(dev(x))), oracle.avgpool(x), 1e-6, "avgpool_fwd")
    d = inputs.make_signed(shape[:2] + (shape[2] // 2, shape[3] // 2), 9)
    up = host(binding.avgpool_bwd(dev(d)))
    np.testing.assert_array_equal(up, oracle.backavgpool(d))   # d/4 is exact
    assert abs(up.astype(np.float64).sum() - d.astype(np.float64).sum()) <= 1e-6 * np.abs(d).sum()


@pytest.mark.parametrize("B,I,O", [(7, 192, 10), (1, 1, 1), (300, 33, 5), (2000, 192, 10), (4101, 192, 10), (70, 20, 300)])
def test_fc(B, I, O):
    x, w, b = inputs.make_signed((B, I), 10), inputs.make_signed((O, I), 11), inputs.make_signed((O,), 12)
    d = inputs.make_signed((B, O), 13)
    x64, w64, d64, b64 = x.astype(np.float64), w.astype(np.float64), d.astype(np.float64), b.astype(np.float64)
    # expected values from the oracle's own functions: FC is mconv with kernel shape == input shape
    # (Section 3), its backward forms are backin / backweights / backbias with a one-element error
    ref_out = np.stack([oracle.mconv(x64[n], w64, b64).ravel() for n in range(B)])
    ref_out0 = np.stack([oracle.mconv(x64[n], w64, np.zeros(O)).ravel() for n in range(B)])
    ref_din = np.zeros((B, I))
    ref_dw, ref_db = np.zeros((O, I)), np.zeros(O)
    for n in range(B):
        for o in range(O):
            e = d64[n, o:o + 1]
            ref_din[n] += oracle.backin(e, w64[o], (I,)).ravel()
            ref_dw[o] += oracle.backweights(e, x64[n]).ravel()
            ref_db[o] += oracle.backbias(e)
    # (and the oracle agrees with the matrix products these reduce to)
    np.testing.assert_allclose(ref_out, x64 @ w64.T + b64, rtol=0, atol=1e-11)
    np.testing.assert_allclose(ref_din, d64 @ w64, rtol=0, atol=1e-11)
    np.testing.assert_allclose(ref_dw, d64.T @ x64, rtol=0, atol=1e-9)
    assert_close(host(binding.fc_fwd(dev(x), dev(w), dev(b))), ref_out, RTOL_ACT, "fc_fwd")
    assert_close(host(binding.fc_fwd(dev(x), dev(w), None)), ref_out0, RTOL_ACT, "fc_fwd no bias")
    assert_close(host(binding.fc_bwd_input(dev(d), dev(w))), ref_din, RTOL_ACT, "fc_bwd_input")
    for workspace in (True, False):
        d_w, d_b = binding.fc_bwd_weight(dev(x), dev(d), workspace=workspace)
        assert_close(host(d_w), ref_dw, RTOL_ACT, "fc_bwd_weight")
        assert_close(host(d_b), ref_db, RTOL_ACT, "fc_bwd_bias")


def test_fc_of_the_network_with_looping_waves():
    """The network's own fully connected shape has kernels in which a wave takes sixteen rows (four for
    the weight gradient) at a time; 70001 rows make their waves loop and leave a ragged last tile.  The
    whole result is compared with the matrix products that test_fc pins the oracle's functions to, and
    sampled rows with those functions themselves."""
    B, I, O = 70001, 192, 10
    x, w, b = inputs.make_signed((B, I), 20), inputs.make_signed((O, I), 21), inputs.make_signed((O,), 22)
    d = inputs.make_signed((B, O), 23)
    x64, w64, d64, b64 = x.astype(np.float64), w.astype(np.float64), d.astype(np.float64), b.astype(np.float64)
    out = host(binding.fc_fwd(dev(x), dev(w), dev(b)))
    d_in = host(binding.fc_bwd_input(dev(d), dev(w)))
    assert_close(out, x64 @ w64.T + b64, RTOL_ACT, "fc_fwd")
    assert_close(d_in, d64 @ w64, RTOL_ACT, "fc_bwd_input")
    rows = np.unique(np.concatenate([np.arange(3), np.arange(B - 20, B), np.random.default_rng(5).integers(0, B, 40)]))
    for n in rows:
        assert_close(out[n], oracle.mconv(x64[n], w64, b64).ravel(), RTOL_ACT, "fc_fwd row %d" % n)
        ref = sum(oracle.backin(d64[n, o:o + 1], w64[o], (I,)).ravel() for o in range(O))
        assert_close(d_in[n], ref, RTOL_ACT, "fc_bwd_input row %d" % n)
    for workspace in (True, False):
        d_w, d_b = binding.fc_bwd_weight(dev(x), dev(d), workspace=workspace)
        assert_close(host(d_w), d64.T @ x64, RTOL_ACT, "fc_bwd_weight")
        assert_close(host(d_b), d64.sum(axis=0), RTOL_ACT, "fc_bwd_bias")


def test_logistic():
    x = np.concatenate([np.linspace(-20, 20, 4001), [0.0, -100.0, 100.0, -1e4, 1e4, 88.0, -88.0, 104.0]])
    x = x.astype(np.float32)
    y = host(binding.logistic_fwd(dev(x)))
    ref = oracle.sigmoid(x)
    assert np.all(np.isfinite(y))
    assert_close(y, ref, RTOL_ACT, "logistic_fwd")
    inner = np.abs(x) <= 12
    assert_close_elementwise(y[inner], ref[inner], 1e-5, "logistic_fwd element-wise")
    assert y[x == 0][0] == 0.5 and y[x == -1e4][0] == 0.0 and y[x == 1e4][0] == 1.0
    d = inputs.make_signed(x.shape, 14)
    assert_close(host(binding.logistic_bwd(dev(ref), dev(d))), oracle.sigmoid_back(ref, d), 1e-6, "logistic_bwd")
    # ragged sizes around the workgroup size
    for n in (1, 255, 257, 1000003):
        xs = inputs.make_signed((n,), 15) * 8
        assert_close(host(binding.logistic_fwd(dev(xs))), oracle.sigmoid(xs), RTOL_ACT, "logistic n=%d" % n)


@pytest.mark.parametrize("B", [37, 1300])
def test_training_gradient_assembled_from_per_op_calls(B):
    """The paper's whole forward/backward chain (Section 3) built from the stateless entry points
    gives the gradient of the fused step: two GPU paths that share no kernels, each also checked
    against the oracle elsewhere."""
    w = inputs.make_weights()
    images, labels = inputs.make_batch(B, 77)
    net = binding.CNN(w, max_batch=B)
    g_fused, loss = net.gradient(dev(images), dev(labels))
    g_fused = host(g_fused).astype(np.float64)
    net.close()

    x = dev(images).reshape(B, 1, 28, 28)
    k1, b1, k2, b2, fc, b = (dev(w[n]) for n in ("k1", "b1", "k2", "b2", "fc", "b"))
    k1 = k1.reshape(6, 1, 5, 5)                                      # the paper's k1 has no input-map axis
    c1 = binding.logistic_fwd(binding.conv_fwd(x, k1, b1))
    s1 = binding.avgpool_fwd(c1)
    c2 = binding.logistic_fwd(binding.conv_fwd(s1, k2, b2))
    s2 = binding.avgpool_fwd(c2)
    s2f, fcw = s2.reshape(B, 192), fc.reshape(10, 192)
    y = binding.logistic_fwd(binding.fc_fwd(s2f, fcw, b))
    target = torch.zeros_like(y)
    target[torch.arange(B), dev(labels).long()] = 1.0
    d_pre = binding.logistic_bwd(y, y - target)                      # (y - t) y (1 - y)
    d_fc, d_b = binding.fc_bwd_weight(s2f, d_pre)
    d_s2 = binding.fc_bwd_input(d_pre, fcw).reshape(B, 12, 4, 4)
    d_c2 = binding.logistic_bwd(c2, binding.avgpool_bwd(d_s2))
    d_k2, d_b2 = binding.conv_bwd_weight(s1, d_c2)
    d_s1 = binding.conv_bwd_input(d_c2, k2, 12, 12)
    d_c1 = binding.logistic_bwd(c1, binding.avgpool_bwd(d_s1))
    d_k1, d_b1 = binding.conv_bwd_weight(x, d_c1)
    parts = dict(zip(("k1", "b1", "k2", "b2", "fc", "b"), (d_k1, d_b1, d_k2, d_b2, d_fc, d_b)))
    ref = inputs.unflatten(g_fused)
    for name, t in parts.items():
        assert_close(host(t).reshape(ref[name].shape), ref[name], RTOL_GRAD, "gradient of %s from per-op calls" % name)
    ref_loss = 0.5 * float(((host(y).astype(np.float64) - host(target)) ** 2).sum())
    assert abs(float(host(loss)[0]) - ref_loss) <= 1e-5 * ref_loss


def test_training_gradient_with_bf16_c2_stays_close():
    """The same chain with C2's three convolution calls in reduced precision: the gradient moves by
    the bf16 rounding of C2's operands (relative 2^-9 each), far more than fp32 rounding and far less
    than the gradient itself.  (Element by element the bf16 calls are checked against the oracle above.)"""
    B = 64
    w = inputs.make_weights()
    images, labels = inputs.make_batch(B, 78)
    net = binding.CNN(w, max_batch=B)
    g_fused, _ = net.gradient(dev(images), dev(labels))
    ref = inputs.unflatten(host(g_fused).astype(np.float64))
    net.close()
    x = dev(images).reshape(B, 1, 28, 28)
    k1, b1, k2, b2, fc, b = (dev(w[n]) for n in ("k1", "b1", "k2", "b2", "fc", "b"))
    k1 = k1.reshape(6, 1, 5, 5)
    c1 = binding.logistic_fwd(binding.conv_fwd(x, k1, b1))
    s1 = binding.avgpool_fwd(c1)
    c2 = binding.logistic_fwd(binding.conv_fwd(s1, k2, b2, bf16=True))
    s2f, fcw = binding.avgpool_fwd(c2).reshape(B, 192), fc.reshape(10, 192)
    y = binding.logistic_fwd(binding.fc_fwd(s2f, fcw, b))
    target = torch.zeros_like(y)
    target[torch.arange(B), dev(labels).long()] = 1.0
    d_pre = binding.logistic_bwd(y, y - target)
    d_c2 = binding.logistic_bwd(c2, binding.avgpool_bwd(binding.fc_bwd_input(d_pre, fcw).reshape(B, 12, 4, 4)))
    d_k2, d_b2 = binding.conv_bwd_weight(s1, d_c2, bf16=True)
    d_c1 = binding.logistic_bwd(c1, binding.avgpool_bwd(binding.conv_bwd_input(d_c2, k2, 12, 12, bf16=True)))
    d_k1, d_b1 = binding.conv_bwd_weight(x, d_c1)
    for name, t in (("k2", d_k2), ("b2", d_b2), ("k1", d_k1), ("b1", d_b1)):
        got, want = host(t).astype(np.float64).reshape(ref[name].shape), ref[name]
        err = np.abs(got - want).max() / np.abs(want).max()
        assert 2e-5 < err < 2e-2, (name, err)


def _random_conv_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        KH, KW = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        H, W = KH + int(rng.integers(0, 14)), KW + int(rng.integers(0, 14))
        cases.append((int(rng.integers(1, 80)), int(rng.integers(1, 9)), H, W, int(rng.integers(1, 20)), KH, KW))
    return cases


@pytest.mark.parametrize("case", _random_conv_cases(24, 20240527))
def test_conv_random_shapes(case):
    """Seeded random small shapes through all three convolution entry points (every launch plan the
    shapes happen to select: packing factors, tile counts, K splits, ragged groups)."""
    B, Cin, H, W, Cout, KH, KW = case
    Ho, Wo = H - KH + 1, W - KW + 1
    x, k, b = inputs.make_signed((B, Cin, H, W), 41), inputs.make_signed((Cout, Cin, KH, KW), 42), inputs.make_signed((Cout,), 43)
    d = inputs.make_signed((B, Cout, Ho, Wo), 44)
    x64, k64, d64 = x.astype(np.float64), k.astype(np.float64), d.astype(np.float64)
    assert_close(host(binding.conv_fwd(dev(x), dev(k), dev(b))), oracle_conv_fwd(x, k, b), RTOL_ACT, "conv_fwd %r" % (case,))
    ref_in = np.zeros((B, Cin, H, W))
    ref_k = np.zeros((Cout, Cin, KH, KW))
    for n in range(B):
        for co in range(Cout):
            ref_in[n] += oracle.backin(d64[n, co][None], k64[co], (Cin, H, W))
            ref_k[co] += oracle.backweights(d64[n, co][None], x64[n])
    assert_close(host(binding.conv_bwd_input(dev(d), dev(k), H, W)), ref_in, RTOL_ACT, "conv_bwd_input %r" % (case,))
    d_k, d_b = binding.conv_bwd_weight(dev(x), dev(d))
    assert_close(host(d_k), ref_k, RTOL_ACT, "conv_bwd_weight %r" % (case,))
    assert_close(host(d_b), d64.sum(axis=(0, 2, 3)), RTOL_ACT, "conv_bwd_bias %r" % (case,))



# ---- reduced precision: operands rounded to bfloat16, fp32 sums ----------------------------------------
# Expected value: the oracle's plain definition applied to operands rounded by the oracle's own
# rounding; what is left is fp32 summation order.  Bound: K products of magnitude <= 1, each exact in
# fp32, summed in fp32: |error| <= K * 2^-24 * sum|terms| in the worst case, a few 1e-7 of the largest
# result in practice; the tests allow 2e-5 of the largest result, as for the fp32 gradients.
RTOL_BF16 = 2e-5
BF16_CASES = [(5, 6, 12, 12, 12, 5, 5), (3, 1, 28, 28, 6, 5, 5), (2, 3, 9, 7, 4, 3, 2), (1, 2, 5, 5, 3, 1, 1),
              (37, 2, 11, 13, 5, 4, 6), (3, 3, 8, 8, 20, 3, 3), (2, 30, 6, 6, 5, 3, 3), (1300, 6, 12, 12, 12, 5, 5),
              (131, 1, 3, 3, 1, 2, 2), (2, 9, 7, 7, 33, 2, 3), (1, 3, 16, 16, 1, 16, 16), (2, 3, 80, 80, 4, 3, 3),
              (4, 12, 4, 4, 10, 4, 4),
              # the fully connected layer as a convolution with one pixel
              (300, 192, 1, 1, 10, 1, 1)]


@pytest.mark.parametrize("case", BF16_CASES)
def test_conv_fwd_bf16(case):
    B, Cin, H, W, Cout, KH, KW = case
    x = inputs.make_signed((B, Cin, H, W), 21)
    k = inputs.make_signed((Cout, Cin, KH, KW), 22)
    b = inputs.make_signed((Cout,), 23)
    ref = oracle_conv_fwd(oracle.round_bf16(x), oracle.round_bf16(k), b)
    got = host(binding.conv_fwd(dev(x), dev(k), dev(b), bf16=True))
    assert_close(got, ref, RTOL_BF16, "conv_fwd_bf16")
    # and it is the rounded problem that was solved, not the fp32 one: the two differ by far more
    exact = oracle_conv_fwd(x, k, b)
    if Cin * KH * KW >= 9:
        assert np.abs(got - exact).max() > 20 * np.abs(got - ref).max()
    assert_close(host(binding.conv_fwd(dev(x), dev(k), None, bf16=True)),
                 oracle_conv_fwd(oracle.round_bf16(x), oracle.round_bf16(k), np.zeros(Cout, np.float32)), RTOL_BF16,
                 "conv_fwd_bf16 no bias")


@pytest.mark.parametrize("case", BF16_CASES)
def test_conv_bwd_input_bf16(case):
    B, Cin, H, W, Cout, KH, KW = case
    Ho, Wo = H - KH + 1, W - KW + 1
    d = inputs.make_signed((B, Cout, Ho, Wo), 24)
    k = inputs.make_signed((Cout, Cin, KH, KW), 25)
    d64, k64 = oracle.round_bf16(d).astype(np.float64), oracle.round_bf16(k).astype(np.float64)
    ref = np.zeros((B, Cin, H, W), np.float64)
    for n in range(B):
        for co in range(Cout):
            ref[n] += oracle.backin(d64[n, co][None], k64[co], (Cin, H, W))
    assert_close(host(binding.conv_bwd_input(dev(d), dev(k), H, W, bf16=True)), ref, RTOL_BF16, "conv_bwd_input_bf16")


@pytest.mark.parametrize("case", _random_conv_cases(16, 20251127))
def test_conv_bf16_random_shapes(case):
    """Seeded random small shapes through the three reduced-precision entry points."""
    B, Cin, H, W, Cout, KH, KW = case
    Ho, Wo = H - KH + 1, W - KW + 1
    x, k, b = inputs.make_signed((B, Cin, H, W), 51), inputs.make_signed((Cout, Cin, KH, KW), 52), inputs.make_signed((Cout,), 53)
    d = inputs.make_signed((B, Cout, Ho, Wo), 54)
    xr, kr, dr = oracle.round_bf16(x), oracle.round_bf16(k), oracle.round_bf16(d)
    assert_close(host(binding.conv_fwd(dev(x), dev(k), dev(b), bf16=True)), oracle_conv_fwd(xr, kr, b), RTOL_BF16,
                 "conv_fwd_bf16 %r" % (case,))
    ref_in = np.zeros((B, Cin, H, W))
    for n in range(B):
        for co in range(Cout):
            ref_in[n] += oracle.backin(dr[n, co][None].astype(np.float64), kr[co].astype(np.float64), (Cin, H, W))
    assert_close(host(binding.conv_bwd_input(dev(d), dev(k), H, W, bf16=True)), ref_in, RTOL_BF16,
                 "conv_bwd_input_bf16 %r" % (case,))
    ref_k = np.zeros((Cout, Cin, KH, KW))
    for n in range(B):
        for co in range(Cout):
            ref_k[co] += oracle.backweights(dr[n, co][None].astype(np.float64), xr[n].astype(np.float64))
    d_k, d_b = binding.conv_bwd_weight(dev(x), dev(d), bf16=True)
    assert_close(host(d_k), ref_k, RTOL_BF16, "conv_bwd_weight_bf16 %r" % (case,))
    assert_close(host(d_b), dr.astype(np.float64).sum(axis=(0, 2, 3)), RTOL_BF16, "conv_bwd_bias_bf16 %r" % (case,))


@pytest.mark.parametrize("case", BF16_CASES + [(70, 3, 9, 20, 5, 2, 4), (9, 2, 6, 40, 3, 3, 3)])
def test_conv_bwd_weight_bf16(case):
    B, Cin, H, W, Cout, KH, KW = case
    Ho, Wo = H - KH + 1, W - KW + 1
    x = inputs.make_signed((B, Cin, H, W), 26)
    d = inputs.make_signed((B, Cout, Ho, Wo), 27)
    x64, d64 = oracle.round_bf16(x).astype(np.float64), oracle.round_bf16(d).astype(np.float64)
    ref_k = np.zeros((Cout, Cin, KH, KW), np.float64)
    ref_b = np.zeros(Cout, np.float64)
    for n in range(B):
        for co in range(Cout):
            ref_k[co] += oracle.backweights(d64[n, co][None], x64[n])
            ref_b[co] += oracle.backbias(d64[n, co])
    for workspace in (True, False):   # the matrix-core kernel, then the plain one with the same rounding
        d_k, d_b = binding.conv_bwd_weight(dev(x), dev(d), workspace=workspace, bf16=True)
        assert_close(host(d_k), ref_k, RTOL_BF16, "conv_bwd_weight_bf16")
        assert_close(host(d_b), ref_b, RTOL_BF16, "conv_bwd_bias_bf16")
    d_k2, none = binding.conv_bwd_weight(dev(x), dev(d), want_bias=False, bf16=True)
    assert none is None and torch.equal(d_k2, binding.conv_bwd_weight(dev(x), dev(d), bf16=True)[0])
