"""Pins for the per-operation functions of the CPU oracle (oracle/cnn_oracle.cpp).

Every check compares the oracle with something other than itself: brute-force
loops written here from the paper's sentence, closed forms, a library routine
(scipy.signal), adjoint identities and invariants.  Citations: arXiv
1912.05234, Section 3 (CNN).
"""
import itertools
import os

import numpy as np
import pytest
import scipy.signal

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(shape, seed, dtype=np.float64):
    return np.random.default_rng(seed).uniform(-1, 1, size=shape).astype(dtype)


def read_shapes():
    rows = {}
    for line in open(os.path.join(GOLDEN, "paper_shapes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, a, b, c, _ = [f.strip() for f in line.split("|")]
        tup = lambda s: None if s == "-" else tuple(int(x) for x in s.split(","))
        rows[name] = (tup(a), tup(b), tup(c))
    return rows


# --------------------------------------------------------------------------- conv
def brute_conv(I, k):
    """out[iv] = sum_ov I[iv+ov]*k[ov]; Section 3, Convolution.  Index-vector form."""
    oshape = tuple(a - b + 1 for a, b in zip(I.shape, k.shape))
    out = np.zeros(oshape)
    for iv in itertools.product(*[range(n) for n in oshape]):
        s = 0.0
        for ov in itertools.product(*[range(n) for n in k.shape]):
            s += I[tuple(i + o for i, o in zip(iv, ov))] * k[ov]
        out[iv] = s
    return out


@pytest.mark.parametrize("ishape,kshape", [((4, 4), (2, 2)), ((5, 7), (3, 2)), ((3, 5, 4), (3, 2, 2)),
                                           ((3, 4, 5), (2, 2, 3)), ((2, 3, 4, 4), (2, 3, 4, 4)),
                                           ((6,), (3,))])
def test_conv_brute_force(ishape, kshape):
    I, k = rnd(ishape, 1), rnd(kshape, 2)
    np.testing.assert_allclose(oracle.conv(I, k), brute_conv(I, k), rtol=0, atol=1e-14)


def test_conv_is_correlation_not_convolution():
    # library special case: valid cross-correlation (no kernel flip)
    I, k = rnd((9, 8), 3), rnd((5, 3), 4)
    np.testing.assert_allclose(oracle.conv(I, k), scipy.signal.correlate(I, k, mode="valid"),
                               rtol=0, atol=1e-13)
    I, k = rnd((6, 12, 12), 5), rnd((6, 5, 5), 6)
    np.testing.assert_allclose(oracle.conv(I, k), scipy.signal.correlate(I, k, mode="valid"),
                               rtol=0, atol=1e-12)
    flipped = scipy.signal.convolve(I, k, mode="valid")
    assert np.abs(oracle.conv(I, k) - flipped).max() > 1e-3


def test_conv_closed_forms():
    # all ones: every output is prod(shape(k))
    out = oracle.conv(np.ones((7, 9)), np.ones((3, 4)))
    assert out.shape == (5, 6) and np.all(out == 12.0)
    # unit impulse kernel: a shifted crop of the input
    I = rnd((8, 8), 7)
    k = np.zeros((3, 3))
    k[1, 2] = 1.0
    np.testing.assert_array_equal(oracle.conv(I, k), I[1:7, 2:8])
    # kernel shape == input shape: one dot product (the paper's FC claim)
    a, b = rnd((12, 1, 4, 4), 8), rnd((12, 1, 4, 4), 9)
    out = oracle.conv(a, b)
    assert out.shape == (1, 1, 1, 1)
    np.testing.assert_allclose(out.ravel()[0], np.dot(a.ravel(), b.ravel()), rtol=1e-14)


def test_conv_f32_rounds_once_from_double_sum():
    I, k = rnd((12, 12), 10, np.float32), rnd((5, 5), 11, np.float32)
    exact = scipy.signal.correlate(I.astype(np.float64), k.astype(np.float64), mode="valid")
    np.testing.assert_array_equal(oracle.conv(I, k), exact.astype(np.float32))


def test_paper_shapes_conv():
    s = read_shapes()
    i, k, o = s["conv_c1"]
    assert oracle.conv(np.zeros(i), np.zeros(k)).shape == o
    i, k, o = s["conv_c2"]
    assert oracle.conv(np.zeros(i), np.zeros(k)).shape == o
    i, k, o = s["mconv_c1"]
    assert oracle.mconv(np.zeros(i), np.zeros(k), np.zeros(k[0])).shape == o
    i, k, o = s["mconv_c2"]
    assert oracle.mconv(np.zeros(i), np.zeros(k), np.zeros(k[0])).shape == o
    # rank 5 of the paper's FC ([12,1,4,4] with unit axis) is rank 4 once the unit axis of the
    # *result* list is dropped; the oracle works at rank <= 4, so check it at that rank.
    i, k, o = s["mconv_fc"]
    assert oracle.mconv(np.zeros(i), np.zeros(k), np.zeros(k[0])).shape == o


def test_mconv_is_conv_plus_bias_per_map():
    I, k, b = rnd((6, 12, 12), 12), rnd((12, 6, 5, 5), 13), rnd((12,), 14)
    out = oracle.mconv(I, k, b)
    for j in range(12):
        np.testing.assert_allclose(out[j], scipy.signal.correlate(I, k[j], mode="valid") + b[j],
                                   rtol=0, atol=1e-12)
    # every C2 map sums over all six input maps: zeroing one input map changes every output map
    I2 = I.copy()
    I2[3] = 0
    assert np.all(np.abs(oracle.mconv(I2, k, b) - out).reshape(12, -1).max(axis=1) > 1e-6)


# ------------------------------------------------------------------------ sigmoid
def test_sigmoid_pins():
    x = np.linspace(-30, 30, 2001)
    y = oracle.sigmoid(x)
    assert oracle.sigmoid(np.zeros(1))[0] == 0.5
    np.testing.assert_allclose(y + oracle.sigmoid(-x), 1.0, rtol=0, atol=1e-15)
    np.testing.assert_allclose(y, 0.5 * (1 + np.tanh(x / 2)), rtol=0, atol=5e-16)
    big = oracle.sigmoid(np.array([-800.0, 800.0, -100.0, 100.0], np.float32))
    assert np.all(np.isfinite(big)) and big[0] == 0.0 and big[1] == 1.0
    x32 = x.astype(np.float32)
    np.testing.assert_array_equal(oracle.sigmoid(x32),
                                  (1.0 / (1.0 + np.exp(-x32.astype(np.float64)))).astype(np.float32))


def test_sigmoid_back_is_derivative():
    x = np.linspace(-6, 6, 241)
    h = 1e-6
    fd = (oracle.sigmoid(x + h) - oracle.sigmoid(x - h)) / (2 * h)
    d = rnd(x.shape, 15)
    np.testing.assert_allclose(oracle.sigmoid_back(oracle.sigmoid(x), d), d * fd, rtol=1e-8, atol=1e-10)


# ------------------------------------------------------------------------ pooling
def test_avgpool_brute_constant_and_shape():
    x = rnd((3, 6, 8), 16)
    out = oracle.avgpool(x)
    assert out.shape == (3, 3, 4)
    for m in range(3):
        for p in range(3):
            for q in range(4):
                blk = x[m, 2 * p:2 * p + 2, 2 * q:2 * q + 2]
                assert abs(out[m, p, q] - blk.sum() / 4) < 1e-15
    assert np.all(oracle.avgpool(np.full((2, 4, 4), 0.37)) == 0.37)
    s = read_shapes()
    for name in ("avgpool_s1", "avgpool_s2"):
        i, _, o = s[name]
        assert oracle.avgpool(np.zeros(i)).shape == o
    # the generic version maps over all leading axes
    y = rnd((2, 3, 4, 6), 17)
    np.testing.assert_array_equal(oracle.avgpool(y)[1, 2], oracle.avgpool(y[1, 2]))


def test_backavgpool_definition_mass_and_adjoint():
    d = rnd((12, 4, 4), 18)
    up = oracle.backavgpool(d)
    s = read_shapes()
    assert up.shape == s["backavgpool"][2]
    for y in range(8):
        for x in range(8):
            np.testing.assert_array_equal(up[:, y, x], d[:, y // 2, x // 2] / 4)
    # gradient mass is conserved
    np.testing.assert_allclose(up.sum(), d.sum(), rtol=1e-13)
    # <avgpool(x), d> == <x, backavgpool(d)>
    x = rnd((12, 8, 8), 19)
    np.testing.assert_allclose(np.vdot(oracle.avgpool(x), d), np.vdot(x, up), rtol=1e-12)


# ------------------------------------------------------------- backweights/backbias
def test_backweights_is_conv_of_input_with_error_and_adjoint():
    I, k, d = rnd((6, 12, 12), 20), rnd((6, 5, 5), 21), rnd((1, 8, 8), 22)
    gw = oracle.backweights(d, I)
    assert gw.shape == k.shape
    np.testing.assert_allclose(gw, scipy.signal.correlate(I, d, mode="valid"), rtol=0, atol=1e-12)
    # <conv(I,k), d> == <k, backweights(d, I)>
    np.testing.assert_allclose(np.vdot(oracle.conv(I, k), d), np.vdot(k, gw), rtol=1e-12)
    # explicit Jacobian: conv is linear in k, so conv(I, e_ov) is the column for weight ov
    I2, d2 = rnd((5, 6), 23), rnd((3, 3), 24)
    gw2 = oracle.backweights(d2, I2)
    for ov in itertools.product(range(3), range(4)):
        e = np.zeros((3, 4))
        e[ov] = 1.0
        assert abs(np.vdot(oracle.conv(I2, e), d2) - gw2[ov]) < 1e-13


def test_backbias_is_sum():
    d = rnd((8, 8), 25)
    assert abs(oracle.backbias(d) - d.sum()) < 1e-13
    d32 = rnd((24, 24), 26, np.float32)
    assert oracle.backbias(d32) == np.float32(d32.astype(np.float64).sum())


# -------------------------------------------------------------------------- backin
CASES_BACKIN = [((5, 6), (3, 3)),          # d_out larger than k-1 on both axes
                ((4, 4), (4, 4)),          # d_out is a single element (the FC case)
                ((6, 7), (5, 6)),          # d_out smaller than k-1 (where the printed bounds fail)
                ((6, 12, 12), (6, 5, 5)),  # C2: channel axis has d_out extent 1
                ((2, 3, 4, 4), (2, 3, 4, 4))]


@pytest.mark.parametrize("ishape,kshape", CASES_BACKIN)
def test_backin_is_exact_adjoint_of_conv(ishape, kshape):
    dshape = tuple(a - b + 1 for a, b in zip(ishape, kshape))
    k, d = rnd(kshape, 27), rnd(dshape, 28)
    din = oracle.backin(d, k, ishape)
    assert din.shape == ishape
    # explicit Jacobian of conv w.r.t. its input: column for input element iv is conv(e_iv, k)
    if np.prod(ishape) <= 200:
        for iv in itertools.product(*[range(n) for n in ishape]):
            e = np.zeros(ishape)
            e[iv] = 1.0
            assert abs(np.vdot(oracle.conv(e, k), d) - din[iv]) < 1e-13
    x = rnd(ishape, 29)
    np.testing.assert_allclose(np.vdot(oracle.conv(x, k), d), np.vdot(x, din), rtol=1e-11)


@pytest.mark.parametrize("ishape,kshape", CASES_BACKIN)
def test_backin_equals_zero_embedding_formulation(ishape, kshape):
    # the alternative the paper names: embed the error in a larger array of zeros and run a
    # convolution over it, i.e. the "full" convolution of d_out with k (library routine)
    dshape = tuple(a - b + 1 for a, b in zip(ishape, kshape))
    k, d = rnd(kshape, 30), rnd(dshape, 31)
    np.testing.assert_allclose(oracle.backin(d, k, ishape), scipy.signal.convolve(d, k, mode="full"),
                               rtol=0, atol=1e-12)
    # and by hand: zero-pad by shape(k)-1 on each side, valid correlation with the reversed kernel
    pad = np.pad(d, [(n - 1, n - 1) for n in kshape])
    np.testing.assert_allclose(oracle.backin(d, k, ishape),
                               brute_conv(pad, k[tuple(slice(None, None, -1) for _ in kshape)])
                               if np.prod(ishape) <= 200 else
                               scipy.signal.correlate(pad, k[tuple(slice(None, None, -1) for _ in kshape)],
                                                      mode="valid"),
                               rtol=0, atol=1e-12)


def test_backin_inner_elements_see_every_weight():
    # all ones: an inner element sums prod(shape(k)) products, a corner exactly one
    din = oracle.backin(np.ones((8, 8)), np.ones((5, 5)), (12, 12))
    assert din[6, 6] == 25.0 and din[0, 0] == 1.0 and din[11, 11] == 1.0 and din[0, 11] == 1.0
    assert din[4, 0] == 5.0 and din[7, 11] == 5.0
    assert din.sum() == 64 * 25


# ---- bfloat16 rounding (states what the reduced-precision convolution computes) ----------------------

def test_round_bf16_hand_values():
    """1 sign, 8 exponent, 7 fraction bits: the spacing in [1, 2) is 2^-7; ties go to the even significand."""
    u = 2.0 ** -7
    cases = [(1.0, 1.0), (1.0 + u, 1.0 + u), (1.0 + u / 2, 1.0),              # tie between 1 (even) and 1+u (odd)
             (1.0 + 3 * u / 2, 1.0 + 2 * u),                                   # tie between 1+u (odd) and 1+2u (even)
             (1.0 + u / 2 + 2.0 ** -23, 1.0 + u), (1.0 + u / 2 - 2.0 ** -23, 1.0),
             (2.0 - u / 4, 2.0), (-1.0 - 3 * u / 2, -1.0 - 2 * u),
             (0.0, 0.0), (2.0 ** -126, 2.0 ** -126), (2.0 ** -133, 2.0 ** -133), (2.0 ** -134, 0.0),
             (3 * 2.0 ** -134, 2.0 ** -132), (0.1, 0.10009765625)]
    got = oracle.round_bf16(np.array([a for a, _ in cases], np.float32))
    np.testing.assert_array_equal(got, np.array([b for _, b in cases], np.float32))


def test_round_bf16_against_library_and_properties():
    import torch
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.uniform(-1, 1, 20000), rng.standard_normal(20000) * 1e-3,
                        np.ldexp(rng.uniform(0.5, 1, 4000), rng.integers(-140, 120, 4000)) * rng.choice([-1, 1], 4000)])
    x = x.astype(np.float32)
    r = oracle.round_bf16(x)
    lib = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()   # an independent conversion
    np.testing.assert_array_equal(r, lib)
    np.testing.assert_array_equal(oracle.round_bf16(r), r)                    # idempotent
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)                          # low 16 bits of the float are clear
    nz = x != 0
    assert np.all(np.abs(r[nz].astype(np.float64) - x[nz]) <= np.abs(x[nz]).astype(np.float64) * 2.0 ** -8 + 2.0 ** -134)
    assert np.all(np.sign(r) * np.sign(x) >= 0) and np.all(np.diff(oracle.round_bf16(np.sort(x))) >= 0)  # monotone
