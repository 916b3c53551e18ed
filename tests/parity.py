"""Comparison rule used by the GPU parity tests.

Floating-point results of the GPU path and of the oracle differ only by fp32 rounding and
summation order.  A tensor passes when max|gpu - ref| <= rtol * max|ref| (error relative to the
tensor's scale: element-wise relative error is ill-posed for gradients and error arrays, whose
elements pass through zero).  The element-wise figure |gpu-ref| / (|ref| + rtol*max|ref|) is
returned too so that tests can bound it where it is meaningful (activations in (0,1)).
"""
import numpy as np

RTOL_ACT = 1e-5     # activations
RTOL_W = 1e-4       # weights after training


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
    assert rel <= rtol, "%s: max|gpu-ref| = %.3e is %.3e of scale %.3e (allowed %.1e)" % (
        what, diff.max(), rel, scale, rtol)
    return rel


def assert_close_elementwise(gpu, ref, rtol, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rel = np.abs(gpu - ref) / np.maximum(np.abs(ref), 1e-30)
    assert rel.max() <= rtol, "%s: element-wise relative error %.3e (allowed %.1e)" % (what, rel.max(), rtol)
    return rel.max()
