"""CPU-side checks of the C ABI: the built library loads without a GPU, exports every
function include/cnn.h declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_1912_05234_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cnn_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_list_the_same_functions():
    names = declared_functions()
    assert len(names) >= 20
    assert names == sorted(binding.SIGNATURES)


def test_library_exports_every_declared_symbol():
    handle = binding.lib()
    for name in declared_functions():
        assert hasattr(handle, name), name


def test_error_strings_and_workspace_size():
    L = binding.lib()
    assert L.cnn_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert len(L.cnn_strerror(code)) > 0
    assert L.cnn_workspace_bytes(0) == 0 and L.cnn_workspace_bytes(-5) == 0
    small, big = L.cnn_workspace_bytes(1), L.cnn_workspace_bytes(60000)
    assert 0 < small <= big
    # the partial count is capped; beyond it the size grows by one KiB per image (the per-image history rows)
    assert L.cnn_workspace_bytes(10 ** 7) - L.cnn_workspace_bytes(10 ** 6) == 1024 * (10 ** 7 - 10 ** 6)


def test_bad_arguments_are_rejected_on_the_host():
    L = binding.lib()
    ctx = ctypes.c_void_p()
    nul = ctypes.c_void_p(None)
    fake = ctypes.c_void_p(0x1000)       # never dereferenced: the checks below fail first
    odd = ctypes.c_void_p(0x1004)
    EINVAL, EWS = -1, -2
    assert L.cnn_init(None, fake, 1 << 30, 10, nul, nul, nul, nul, nul, nul, nul) == EINVAL
    assert L.cnn_init(ctypes.byref(ctx), nul, 1 << 30, 10, nul, nul, nul, nul, nul, nul, nul) == EINVAL
    assert L.cnn_init(ctypes.byref(ctx), odd, 1 << 30, 10, nul, nul, nul, nul, nul, nul, nul) == EINVAL
    assert L.cnn_init(ctypes.byref(ctx), fake, 1 << 30, 0, nul, nul, nul, nul, nul, nul, nul) == EINVAL
    assert L.cnn_init(ctypes.byref(ctx), fake, 16, 10, nul, nul, nul, nul, nul, nul, nul) == EWS
    assert not ctx.value
    assert L.cnn_forward(nul, fake, 1, fake) == EINVAL
    assert L.cnn_train_batch(nul, fake, fake, 1, 0.05, nul) == EINVAL
    assert L.cnn_train_epoch(nul, fake, fake, 10, 5, 0.05, nul) == EINVAL
    assert L.cnn_epoch_mode(nul, 1, 1.0, 0) == EINVAL
    assert L.cnn_epoch_status(nul) == EINVAL
    assert L.cnn_evaluate(nul, fake, fake, 1, fake, nul) == EINVAL
    assert L.cnn_gradient(nul, fake, fake, 1, fake, nul) == EINVAL
    assert L.cnn_get_weights(nul, nul, nul, nul, nul, nul, nul) == EINVAL
    L.cnn_destroy(nul)
    # per-op: null, misaligned, bad shapes
    assert L.cnn_conv_fwd(nul, fake, nul, fake, 1, 1, 8, 8, 1, 3, 3, nul) == EINVAL
    assert L.cnn_conv_fwd(odd, fake, nul, fake, 1, 1, 8, 8, 1, 3, 3, nul) == EINVAL
    assert L.cnn_conv_fwd(fake, fake, nul, fake, 1, 1, 2, 8, 1, 3, 3, nul) == EINVAL   # H < KH
    assert L.cnn_conv_fwd(fake, fake, nul, fake, 0, 1, 8, 8, 1, 3, 3, nul) == EINVAL   # B < 1
    assert L.cnn_conv_bwd_input(fake, nul, fake, 1, 1, 8, 8, 1, 3, 3, nul) == EINVAL
    assert L.cnn_conv_fwd_bf16(fake, fake, nul, odd, 1, 1, 8, 8, 1, 3, 3, nul) == EINVAL
    assert L.cnn_conv_fwd_bf16(fake, fake, nul, fake, 1, 1, 8, 2, 1, 3, 3, nul) == EINVAL   # W < KW
    assert L.cnn_conv_bwd_input_bf16(fake, fake, nul, 1, 1, 8, 8, 1, 3, 3, nul) == EINVAL
    assert L.cnn_conv_bwd_weight(fake, fake, nul, nul, 1, 1, 8, 8, 1, 3, 3, nul, 0, nul) == EINVAL
    assert L.cnn_conv_bwd_weight(fake, fake, fake, nul, 1, 1, 8, 8, 1, 3, 3, odd, 1 << 20, nul) == EINVAL  # workspace alignment
    assert L.cnn_conv_bwd_weight_workspace_bytes(1, 1, 8, 8, 1, 9, 3) == 0               # kernel larger than input
    assert L.cnn_conv_bwd_weight_static(fake, fake, nul, nul, 1, 1, 8, 8, 1, 3, 3, nul) == EINVAL
    assert L.cnn_conv_bwd_weight_static(fake, odd, fake, nul, 1, 1, 8, 8, 1, 3, 3, nul) == EINVAL
    # more partial sums than the built-in buffer holds: refused before anything touches the device
    assert L.cnn_conv_bwd_weight_workspace_bytes(8192, 8, 12, 12, 32, 5, 5) > 16 << 20
    assert L.cnn_conv_bwd_weight_static(fake, fake, fake, nul, 8192, 8, 12, 12, 32, 5, 5, nul) == -4
    assert L.cnn_conv_bwd_weight_bf16(fake, fake, nul, nul, 1, 1, 8, 8, 1, 3, 3, nul, 0, nul) == EINVAL
    assert L.cnn_conv_bwd_weight_bf16(fake, fake, fake, nul, 1, 1, 8, 8, 1, 3, 3, odd, 1 << 20, nul) == EINVAL
    assert L.cnn_conv_bwd_weight_bf16_workspace_bytes(1, 1, 8, 8, 1, 9, 3) == 0
    assert L.cnn_conv_bwd_weight_bf16_workspace_bytes(100, 6, 12, 12, 12, 5, 5) % ((10 * 256 + 16) * 4) == 0
    assert L.cnn_avgpool_fwd(fake, fake, 1, 1, 7, 8, nul) == EINVAL                     # odd extent
    assert L.cnn_avgpool_bwd(fake, nul, 1, 1, 4, 4, nul) == EINVAL
    assert L.cnn_fc_fwd(fake, fake, nul, fake, 1, 0, 10, nul) == EINVAL
    assert L.cnn_fc_bwd_input(nul, fake, fake, 1, 4, 4, nul) == EINVAL
    assert L.cnn_fc_bwd_weight(fake, fake, fake, odd, 1, 4, 4, nul, 0, nul) == EINVAL
    assert L.cnn_logistic_fwd(fake, fake, 0, nul) == EINVAL
    assert L.cnn_logistic_bwd(fake, nul, fake, 4, nul) == EINVAL


def test_weight_gradient_workspace_query():
    """Host-only logic: the size query follows the launch plan and rejects what the call rejects."""
    L = binding.lib()
    q = L.cnn_conv_bwd_weight_workspace_bytes
    c2 = q(100, 6, 12, 12, 12, 5, 5)
    assert c2 > 0 and c2 % 4 == 0
    # per partial-sum column: one 16 x 16 tile per 16 output maps and 16 taps, plus 16 bias sums
    per_column = (10 * 256 + 16) * 4
    assert c2 % per_column == 0 and c2 // per_column <= 100
    big = q(100000, 6, 12, 12, 12, 5, 5)
    assert big % per_column == 0 and c2 // per_column <= big // per_column <= 1024   # the column count is capped
    assert q(200000, 6, 12, 12, 12, 5, 5) == big
    assert q(2, 3, 80, 80, 4, 3, 3) == 0      # does not fit in LDS: the plain kernel needs no workspace
    assert q(0, 6, 12, 12, 12, 5, 5) == 0     # invalid batch
    assert q(1, 1, 8, 8, 1, 9, 3) == 0        # kernel larger than the input
    assert L.cnn_fc_bwd_weight_workspace_bytes(100, 192, 10) == q(100, 192, 1, 1, 10, 1, 1) > 0

