"""Comparison rule used by the GPU parity tests.

Floating-point results of the GPU path and of the oracle differ only by fp32 rounding and
summation order.  A tensor passes when max|gpu - ref| <= rtol * max|ref| (error relative to the
tensor's scale: element-wise relative error is ill-posed for gradients and error arrays, whose
elements pass through zero).  The element-wise figure |gpu-ref| / (|ref| + rtol*max|ref|) is
returned too so that tests can bound it where it is meaningful (activations in (0,1)).
"""
import re

import numpy as np

# Limits, about ten times what the kernels reach (the summary at the end of a GPU run prints the
# largest error of every compared quantity): activations and per-op results reach <= 1e-6 of their
# scale, gradients <= 8e-7 (2.3e-6 with saturated units), weights 3e-7 after one epoch of 600 steps
# and 1.4e-6 after ten.  The stated bars of the method are 1e-5 on activations and 1e-4 on weights
# after one epoch; the weight limit used here is ten times tighter than that bar.
RTOL_ACT = 1e-5     # activations, per-op results
RTOL_GRAD = 1e-5    # gradients summed over a batch
RTOL_W = 1e-5       # weights after training

# largest error seen per kind of quantity in this run, relative to the tensor's scale (printed in the
# test summary: the limits above are checked against what the kernels actually reach)
OBSERVED = {}


def _note(what, rel):
    key = re.sub(r"[\[(].*", "", what).strip() or "?"
    key = re.sub(r"\d+", "#", key)
    OBSERVED[key] = max(OBSERVED.get(key, 0.0), float(rel))


def errors(gpu, ref):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    assert np.all(np.isfinite(gpu))
    scale = max(np.abs(ref).max(), 1e-30) if ref.size else 1.0
    diff = np.abs(gpu - ref)
    return (diff.max() / scale if ref.size else 0.0), scale, diff


def assert_close(gpu, ref, rtol, what=""):
    rel, scale, diff = errors(gpu, ref)
    _note(what, rel)
    assert rel <= rtol, "%s: max|gpu-ref| = %.3e is %.3e of scale %.3e (allowed %.1e)" % (
        what, diff.max(), rel, scale, rtol)
    return rel


def assert_close_elementwise(gpu, ref, rtol, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rel = np.abs(gpu - ref) / np.maximum(np.abs(ref), 1e-30)
    _note(what + " element-wise", rel.max())
    assert rel.max() <= rtol, "%s: element-wise relative error %.3e (allowed %.1e)" % (what, rel.max(), rtol)
    return rel.max()
