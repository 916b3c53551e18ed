"""cnn_conv_bwd_weight_static (the entry point for callers that cannot allocate) against
cnn_conv_bwd_weight with a caller workspace, through the C ABI: same kernels and summation order, so
the results must be bitwise equal; and against the CPU oracle to the per-op tolerance.  Two calls in a
row share the library's built-in buffer, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_1912_05234_amd import binding, inputs
from parity import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def oracle_wgrad(x, d):
    """backweights / backbias of Section 3 per output map, summed over the batch."""
    B, Cin, H, W = x.shape
    Cout, Ho, Wo = d.shape[1:]
    gk = np.zeros((Cout, Cin, H - Ho + 1, W - Wo + 1), np.float64)
    gb = np.zeros(Cout, np.float64)
    for n in range(B):
        for co in range(Cout):
            gk[co] += oracle.backweights(d[n, co][None].astype(np.float64), x[n].astype(np.float64)).reshape(gk.shape[1:])
            gb[co] += oracle.backbias(d[n, co].astype(np.float64))
    return gk, gb


# first the larger call, then a smaller one that leaves most of the buffer's old contents in place;
# (B, Cin, H, W, Cout, KH, KW): C2's shape with looping workgroups, C1's packed shape, a ragged one
SEQUENCES = [[(1300, 6, 12, 12, 12, 5, 5), (37, 6, 12, 12, 12, 5, 5)],
             [(300, 1, 28, 28, 6, 5, 5), (3, 1, 28, 28, 6, 5, 5)],
             [(37, 2, 11, 13, 5, 4, 6), (2, 3, 9, 7, 4, 3, 2)]]


@pytest.mark.parametrize("seq", SEQUENCES)
def test_static_scratch_matches_workspace_call(seq):
    for i, (B, Cin, H, W, Cout, KH, KW) in enumerate(seq):
        x = inputs.make_signed((B, Cin, H, W), 21 + i)
        d = inputs.make_signed((B, Cout, H - KH + 1, W - KW + 1), 23 + i)
        xd, dd = dev(x), dev(d)
        assert binding.lib().cnn_conv_bwd_weight_workspace_bytes(B, Cin, H, W, Cout, KH, KW) > 0
        ref_k, ref_b = binding.conv_bwd_weight(xd, dd)          # caller workspace
        got_k = torch.full_like(ref_k, float("nan"))
        got_b = torch.full_like(ref_b, float("nan"))
        binding.conv_bwd_weight_static(xd, dd, got_k, got_b)    # built-in scratch
        torch.cuda.synchronize()
        assert torch.equal(got_k, ref_k) and torch.equal(got_b, ref_b), (i, B)
        if B <= 64:  # the oracle takes seconds here
            ok, ob = oracle_wgrad(x, d)
            assert_close(got_k.cpu().numpy(), ok, 2e-5, "d_k")
            assert_close(got_b.cpu().numpy(), ob, 2e-5, "d_bias")


def test_static_scratch_without_bias_and_plain_shape():
    # no bias output; and a shape only the kernel without partial sums serves (needs no scratch)
    x, d = inputs.make_signed((5, 6, 12, 12), 31), inputs.make_signed((5, 12, 8, 8), 32)
    ref_k, _ = binding.conv_bwd_weight(dev(x), dev(d), want_bias=False)
    got_k = torch.empty_like(ref_k)
    binding.conv_bwd_weight_static(dev(x), dev(d), got_k, None)
    torch.cuda.synchronize()
    assert torch.equal(got_k, ref_k)
    x, d = inputs.make_signed((2, 3, 80, 80), 33), inputs.make_signed((2, 4, 78, 78), 34)
    assert binding.lib().cnn_conv_bwd_weight_workspace_bytes(2, 3, 80, 80, 4, 3, 3) == 0
    ref_k, ref_b = binding.conv_bwd_weight(dev(x), dev(d))
    got_k, got_b = torch.empty_like(ref_k), torch.empty_like(ref_b)
    binding.conv_bwd_weight_static(dev(x), dev(d), got_k, got_b)
    torch.cuda.synchronize()
    assert torch.equal(got_k, ref_k) and torch.equal(got_b, ref_b)


def test_static_scratch_rejects_what_does_not_fit():
    # 32 output maps x 200 taps at a batch that fills every partial column: 26 tiles x 1024 columns
    L = binding.lib()
    need = L.cnn_conv_bwd_weight_workspace_bytes(8192, 8, 12, 12, 32, 5, 5)
    assert need > 16 << 20
    t = torch.zeros(64, dtype=torch.float32, device=DEV)   # never touched: the size check comes first
    p = ctypes.c_void_p(t.data_ptr())
    assert L.cnn_conv_bwd_weight_static(p, p, p, None, 8192, 8, 12, 12, 32, 5, 5, None) == -4
    assert b"scratch" in L.cnn_strerror(-4)
