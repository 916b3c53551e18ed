"""ctypes binding over the C ABI in include/cnn.h (same names, argument marshalling only).

PyTorch supplies device memory (tensors) and the stream handle; every step of
the computation runs inside the library's HIP kernels.  The built library must
be present (python -m paper_1912_05234_amd.build): there is no fallback path.
"""
import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcnn_mi355x.so")

NPARAM = 3898
PARAM_SHAPES = (("k1", (6, 5, 5)), ("b1", (6,)), ("k2", (12, 6, 5, 5)), ("b2", (12,)),
                ("fc", (10, 12, 1, 4, 4)), ("b", (10,)))

_vp, _i, _f, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t

# name -> (restype, argtypes); one entry per declaration in include/cnn.h
SIGNATURES = {
    "cnn_strerror": (ctypes.c_char_p, [_i]),
    "cnn_workspace_bytes": (_sz, [_i]),
    "cnn_init": (_i, [ctypes.POINTER(_vp), _vp, _sz, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "cnn_destroy": (None, [_vp]),
    "cnn_get_weights": (_i, [_vp] * 7),
    "cnn_set_weights": (_i, [_vp] * 7),
    "cnn_forward": (_i, [_vp, _vp, _i, _vp]),
    "cnn_forward_activations": (_i, [_vp, _vp, _i, _vp, _vp, _vp, _vp, _vp]),
    "cnn_gradient": (_i, [_vp, _vp, _vp, _i, _vp, _vp]),
    "cnn_train_batch": (_i, [_vp, _vp, _vp, _i, _f, _vp]),
    "cnn_train_epoch": (_i, [_vp, _vp, _vp, _i, _i, _f, _vp]),
    "cnn_epoch_mode": (_i, [_vp, _i, ctypes.c_double, _i]),
    "cnn_epoch_status": (_i, [_vp]),
    "cnn_evaluate": (_i, [_vp, _vp, _vp, _i, _vp, _vp]),
    "cnn_profile_begin": (_i, [_vp, _i]),
    "cnn_profile_read": (_i, [_vp, _vp, _i, ctypes.POINTER(_i)]),
    "cnn_conv_fwd": (_i, [_vp, _vp, _vp, _vp] + [_i] * 7 + [_vp]),
    "cnn_conv_bwd_input": (_i, [_vp, _vp, _vp] + [_i] * 7 + [_vp]),
    "cnn_conv_fwd_valu": (_i, [_vp, _vp, _vp, _vp] + [_i] * 7 + [_vp]),
    "cnn_conv_bwd_input_valu": (_i, [_vp, _vp, _vp] + [_i] * 7 + [_vp]),
    "cnn_conv_fwd_bf16": (_i, [_vp, _vp, _vp, _vp] + [_i] * 7 + [_vp]),
    "cnn_conv_bwd_input_bf16": (_i, [_vp, _vp, _vp] + [_i] * 7 + [_vp]),
    "cnn_conv_bwd_weight_workspace_bytes": (_sz, [_i] * 7),
    "cnn_conv_bwd_weight_bf16_workspace_bytes": (_sz, [_i] * 7),
    "cnn_conv_bwd_weight_bf16": (_i, [_vp, _vp, _vp, _vp] + [_i] * 7 + [_vp, _sz, _vp]),
    "cnn_conv_bwd_weight": (_i, [_vp, _vp, _vp, _vp] + [_i] * 7 + [_vp, _sz, _vp]),
    "cnn_conv_bwd_weight_static": (_i, [_vp, _vp, _vp, _vp] + [_i] * 7 + [_vp]),
    "cnn_avgpool_fwd": (_i, [_vp, _vp, _i, _i, _i, _i, _vp]),
    "cnn_avgpool_bwd": (_i, [_vp, _vp, _i, _i, _i, _i, _vp]),
    "cnn_fc_fwd": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _vp]),
    "cnn_fc_bwd_input": (_i, [_vp, _vp, _vp, _i, _i, _i, _vp]),
    "cnn_fc_bwd_weight_workspace_bytes": (_sz, [_i] * 3),
    "cnn_fc_bwd_weight": (_i, [_vp, _vp, _vp, _vp, _i, _i, _i, _vp, _sz, _vp]),
    "cnn_logistic_fwd": (_i, [_vp, _vp, _sz, _vp]),
    "cnn_logistic_bwd": (_i, [_vp, _vp, _vp, _sz, _vp]),
}

_lib = None


class CnnError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = lib().cnn_strerror(code).decode()
        super().__init__("%s failed: %s (code %d)" % (where, msg, code))


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is missing: build it with `python -m paper_1912_05234_amd.build`; "
                               "there is no fallback implementation" % LIB_PATH)
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def _check(code, where):
    if code != 0:
        raise CnnError(code, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _dev(t, dtype=torch.float32):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise ValueError("expected a contiguous %s tensor on the GPU" % dtype)
    return t


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class CNN:
    """Owns a library context plus the device workspace it lives in."""

    def __init__(self, weights, max_batch, device="cuda:0"):
        self.device = torch.device(device)
        self.max_batch = int(max_batch)
        L = lib()
        nbytes = L.cnn_workspace_bytes(self.max_batch)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        w = {k: _dev(torch.as_tensor(v, dtype=torch.float32).contiguous().to(self.device))
             for k, v in weights.items()}
        self._ctx = ctypes.c_void_p()
        with torch.cuda.device(self.device):
            self._stream_obj = torch.cuda.current_stream()
            _check(L.cnn_init(ctypes.byref(self._ctx), _ptr(self.workspace), nbytes, self.max_batch,
                              *[_ptr(w.get(n)) for n, _ in PARAM_SHAPES], _stream()), "cnn_init")
            torch.cuda.current_stream().synchronize()  # the staging copies of `w` may now be freed

    def close(self):
        if self._ctx:
            lib().cnn_destroy(self._ctx)
            self._ctx = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def get_weights(self):
        out = {n: torch.empty(s, dtype=torch.float32, device=self.device) for n, s in PARAM_SHAPES}
        _check(lib().cnn_get_weights(self._ctx, *[_ptr(out[n]) for n, _ in PARAM_SHAPES]), "cnn_get_weights")
        return out

    def get_weights_flat(self):
        w = self.get_weights()
        return torch.cat([w[n].reshape(-1) for n, _ in PARAM_SHAPES])

    def set_weights(self, weights):
        w = {k: _dev(torch.as_tensor(v, dtype=torch.float32).contiguous().to(self.device))
             for k, v in weights.items()}
        _check(lib().cnn_set_weights(self._ctx, *[_ptr(w.get(n)) for n, _ in PARAM_SHAPES]), "cnn_set_weights")
        self._stream_obj.synchronize()

    def forward(self, images, yhat=None):
        images = _dev(images)
        B = images.shape[0]
        if yhat is None:
            yhat = torch.empty((B, 10), dtype=torch.float32, device=self.device)
        _check(lib().cnn_forward(self._ctx, _ptr(images), B, _ptr(_dev(yhat))), "cnn_forward")
        return yhat

    def forward_activations(self, images):
        images = _dev(images)
        B = images.shape[0]
        mk = lambda *s: torch.empty((B,) + s, dtype=torch.float32, device=self.device)
        a = {"c1": mk(6, 24, 24), "s1": mk(6, 12, 12), "c2": mk(12, 8, 8), "s2": mk(12, 4, 4), "y": mk(10)}
        _check(lib().cnn_forward_activations(self._ctx, _ptr(images), B, _ptr(a["c1"]), _ptr(a["s1"]),
                                             _ptr(a["c2"]), _ptr(a["s2"]), _ptr(a["y"])),
               "cnn_forward_activations")
        return a

    def gradient(self, images, labels):
        images, labels = _dev(images), _dev(labels, torch.int32)
        B = images.shape[0]
        grad = torch.empty(NPARAM, dtype=torch.float32, device=self.device)
        loss = torch.empty(1, dtype=torch.float32, device=self.device)
        _check(lib().cnn_gradient(self._ctx, _ptr(images), _ptr(labels), B, _ptr(grad), _ptr(loss)),
               "cnn_gradient")
        return grad, loss

    def train_batch(self, images, labels, lr, loss_sum=None):
        images, labels = _dev(images), _dev(labels, torch.int32)
        _check(lib().cnn_train_batch(self._ctx, _ptr(images), _ptr(labels), images.shape[0], float(lr),
                                     _ptr(_dev(loss_sum))), "cnn_train_batch")
        return loss_sum

    def train_epoch(self, images, labels, batch, lr, loss_sums=None):
        """One pass over `images` in consecutive batches of `batch` (the last may be shorter)."""
        images, labels = _dev(images), _dev(labels, torch.int32)
        if loss_sums is not None and loss_sums.numel() < -(-images.shape[0] // int(batch)):
            raise ValueError("loss_sums needs one float per step")
        _check(lib().cnn_train_epoch(self._ctx, _ptr(images), _ptr(labels), images.shape[0], int(batch),
                                     float(lr), _ptr(_dev(loss_sums))), "cnn_train_epoch")
        return loss_sums

    def epoch_mode(self, device_loop, wait_seconds=1.0, never_arrives=False):
        _check(lib().cnn_epoch_mode(self._ctx, int(device_loop), float(wait_seconds), int(never_arrives)),
               "cnn_epoch_mode")

    def epoch_status(self):
        """Waits for the stream; 0, or the (negative) code of a device-side loop that gave up."""
        return lib().cnn_epoch_status(self._ctx)

    def evaluate(self, images, labels):
        images, labels = _dev(images), _dev(labels, torch.int32)
        n_ok = torch.empty(1, dtype=torch.int64, device=self.device)
        loss = torch.empty(1, dtype=torch.float32, device=self.device)
        _check(lib().cnn_evaluate(self._ctx, _ptr(images), _ptr(labels), images.shape[0], _ptr(n_ok),
                                  _ptr(loss)), "cnn_evaluate")
        return n_ok, loss


    def profile_begin(self, capacity):
        _check(lib().cnn_profile_begin(self._ctx, int(capacity)), "cnn_profile_begin")

    def profile_read(self, capacity):
        """Per-step milliseconds of the fused forward+backward kernel (host list)."""
        buf = (ctypes.c_float * max(1, capacity))()
        n = ctypes.c_int(0)
        _check(lib().cnn_profile_read(self._ctx, ctypes.cast(buf, _vp), int(capacity), ctypes.byref(n)),
               "cnn_profile_read")
        return [buf[i] for i in range(n.value)]


# ---- per-operation entry points -------------------------------------------------
def conv_fwd(inp, k, bias=None, bf16=False, valu=False):
    inp, k, bias = _dev(inp), _dev(k), _dev(bias)
    B, Cin, H, W = inp.shape
    Cout, _, KH, KW = k.shape
    out = torch.empty((B, Cout, H - KH + 1, W - KW + 1), dtype=torch.float32, device=inp.device)
    name = "cnn_conv_fwd_bf16" if bf16 else "cnn_conv_fwd_valu" if valu else "cnn_conv_fwd"
    _check(getattr(lib(), name)(_ptr(inp), _ptr(k), _ptr(bias), _ptr(out), B, Cin, H, W, Cout, KH, KW,
                                _stream()), name)
    return out


def conv_bwd_input(d_out, k, H, W, bf16=False, valu=False):
    d_out, k = _dev(d_out), _dev(k)
    B = d_out.shape[0]
    Cout, Cin, KH, KW = k.shape
    d_in = torch.empty((B, Cin, H, W), dtype=torch.float32, device=d_out.device)
    name = "cnn_conv_bwd_input_bf16" if bf16 else "cnn_conv_bwd_input_valu" if valu else "cnn_conv_bwd_input"
    _check(getattr(lib(), name)(_ptr(d_out), _ptr(k), _ptr(d_in), B, Cin, H, W, Cout, KH, KW, _stream()), name)
    return d_in


def _workspace(nbytes, device, use):
    if not use or nbytes == 0:
        return None, 0
    return torch.empty((nbytes,), dtype=torch.uint8, device=device), nbytes


def conv_bwd_weight(inp, d_out, want_bias=True, workspace=True, bf16=False):
    """workspace=False passes none, which selects the kernel that needs no partial sums."""
    suffix = "_bf16" if bf16 else ""
    inp, d_out = _dev(inp), _dev(d_out)
    B, Cin, H, W = inp.shape
    Cout, Ho, Wo = d_out.shape[1:]
    KH, KW = H - Ho + 1, W - Wo + 1
    d_k = torch.empty((Cout, Cin, KH, KW), dtype=torch.float32, device=inp.device)
    d_b = torch.empty((Cout,), dtype=torch.float32, device=inp.device) if want_bias else None
    query = getattr(lib(), "cnn_conv_bwd_weight%s_workspace_bytes" % suffix)
    ws, nbytes = _workspace(query(B, Cin, H, W, Cout, KH, KW), inp.device, workspace)
    name = "cnn_conv_bwd_weight" + suffix
    _check(getattr(lib(), name)(_ptr(inp), _ptr(d_out), _ptr(d_k), _ptr(d_b), B, Cin, H, W, Cout, KH, KW,
                                _ptr(ws), nbytes, _stream()), name)
    return d_k, d_b


def conv_bwd_weight_static(inp, d_out, d_k, d_b=None):
    """cnn_conv_bwd_weight_static into the caller's d_k / d_b (this wrapper allocates nothing either)."""
    inp, d_out, d_k, d_b = _dev(inp), _dev(d_out), _dev(d_k), _dev(d_b)
    B, Cin, H, W = inp.shape
    Cout, Ho, Wo = d_out.shape[1:]
    KH, KW = H - Ho + 1, W - Wo + 1
    _check(lib().cnn_conv_bwd_weight_static(_ptr(inp), _ptr(d_out), _ptr(d_k), _ptr(d_b), B, Cin, H, W, Cout,
                                            KH, KW, _stream()), "cnn_conv_bwd_weight_static")
    return d_k, d_b


def avgpool_fwd(inp):
    inp = _dev(inp)
    B, C, H, W = inp.shape
    out = torch.empty((B, C, H // 2, W // 2), dtype=torch.float32, device=inp.device)
    _check(lib().cnn_avgpool_fwd(_ptr(inp), _ptr(out), B, C, H, W, _stream()), "cnn_avgpool_fwd")
    return out


def avgpool_bwd(d_out):
    d_out = _dev(d_out)
    B, C, Ho, Wo = d_out.shape
    d_in = torch.empty((B, C, 2 * Ho, 2 * Wo), dtype=torch.float32, device=d_out.device)
    _check(lib().cnn_avgpool_bwd(_ptr(d_out), _ptr(d_in), B, C, Ho, Wo, _stream()), "cnn_avgpool_bwd")
    return d_in


def fc_fwd(inp, w, bias=None):
    inp, w, bias = _dev(inp), _dev(w), _dev(bias)
    B, I = inp.shape
    O = w.shape[0]
    out = torch.empty((B, O), dtype=torch.float32, device=inp.device)
    _check(lib().cnn_fc_fwd(_ptr(inp), _ptr(w), _ptr(bias), _ptr(out), B, I, O, _stream()), "cnn_fc_fwd")
    return out


def fc_bwd_input(d_out, w):
    d_out, w = _dev(d_out), _dev(w)
    B, O = d_out.shape
    I = w.shape[1]
    d_in = torch.empty((B, I), dtype=torch.float32, device=d_out.device)
    _check(lib().cnn_fc_bwd_input(_ptr(d_out), _ptr(w), _ptr(d_in), B, I, O, _stream()), "cnn_fc_bwd_input")
    return d_in


def fc_bwd_weight(inp, d_out, want_bias=True, workspace=True):
    inp, d_out = _dev(inp), _dev(d_out)
    B, I = inp.shape
    O = d_out.shape[1]
    d_w = torch.empty((O, I), dtype=torch.float32, device=inp.device)
    d_b = torch.empty((O,), dtype=torch.float32, device=inp.device) if want_bias else None
    ws, nbytes = _workspace(lib().cnn_fc_bwd_weight_workspace_bytes(B, I, O), inp.device, workspace)
    _check(lib().cnn_fc_bwd_weight(_ptr(inp), _ptr(d_out), _ptr(d_w), _ptr(d_b), B, I, O, _ptr(ws), nbytes,
                                   _stream()), "cnn_fc_bwd_weight")
    return d_w, d_b


def logistic_fwd(x):
    x = _dev(x)
    y = torch.empty_like(x)
    _check(lib().cnn_logistic_fwd(_ptr(x), _ptr(y), x.numel(), _stream()), "cnn_logistic_fwd")
    return y


def logistic_bwd(y, d_y):
    y, d_y = _dev(y), _dev(d_y)
    d_x = torch.empty_like(y)
    _check(lib().cnn_logistic_bwd(_ptr(y), _ptr(d_y), _ptr(d_x), y.numel(), _stream()), "cnn_logistic_bwd")
    return d_x
