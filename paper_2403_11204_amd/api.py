"""Python names for the C ABI in include/slp.h -- argument marshalling only.

Every function here packs its arguments, calls the library entry point of the
same name and raises ``SlpError`` on a non-zero status.  Tensors are torch CUDA
tensors used as raw device memory; the stream passed to the library is torch's
current stream, so ordinary torch stream semantics apply.
"""

import ctypes
import os

import torch

UNIFORM01, UNIFORM_PM1, NORMAL, BINARY_PM1 = 0, 1, 2, 3
F32, BF16 = 0, 1
RELU_ALL, RELU_HIDDEN_IDENTITY_LAST = 0, 1
MSE_SIL, SOFTMAX_XENT = 0, 1

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libslp.so")
_lib = None


class SlpError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("slp error %d: %s" % (code, message))
        self.code = code


class _Opts(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int), ("max_batch", ctypes.c_int), ("lr", ctypes.c_float), ("momentum", ctypes.c_float),
                ("input_grad", ctypes.c_int)]


def lib():
    """Loads libslp.so once.  Fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("%s is missing: build it with `python -m paper_2403_11204_amd.build` "
                           "(there is no fallback path)" % _LIB_PATH)
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, u64, f32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_uint64, ctypes.c_float, ctypes.c_size_t
    sig = {
        "slp_last_error": (ctypes.c_char_p, []),
        "slp_make_synthetic_labels": (i32, [u64, i32, i32, i32, f32, vp, i32, vp]),
        "slp_make_segment_inputs": (i32, [u64, vp, i32, vp, i64, i32, i32, f32, vp, i32, vp]),
        "slp_segment_create": (i32, [ctypes.POINTER(i32), i32, i32, i32, ctypes.POINTER(_Opts), ctypes.POINTER(vp)]),
        "slp_segment_destroy": (None, [vp]),
        "slp_segment_param_bytes": (sz, [vp]),
        "slp_segment_workspace_bytes": (sz, [vp]),
        "slp_segment_bind": (i32, [vp, vp, sz, vp, sz, vp]),
        "slp_segment_init": (i32, [vp, u64, vp]),
        "slp_segment_set_params": (i32, [vp, i32, vp, vp, i32, vp]),
        "slp_segment_get_params": (i32, [vp, i32, vp, vp, i32, vp]),
        "slp_segment_get_grads": (i32, [vp, i32, vp, vp, i32, vp]),
        "slp_segment_get_momentum": (i32, [vp, i32, vp, vp, i32, vp]),
        "slp_segment_get_activation": (i32, [vp, i32, i32, i32, vp, vp]),
        "slp_segment_set_lr": (i32, [vp, f32, f32]),
        "slp_segment_set_labels": (i32, [vp, vp, i32, i32]),
        "slp_segment_step": (i32, [vp, vp, vp, i32, vp, vp]),
        "slp_segment_forward": (i32, [vp, vp, i32, vp, vp]),
        "slp_segment_input_grad": (i32, [vp, vp, vp, i32, vp, vp, vp]),
        "slp_segment_step_external": (i32, [vp, vp, vp, i32, vp]),
        "slp_segment_profile_enable": (i32, [vp, i32]),
        "slp_segment_set_graph": (i32, [vp, i32]),
        "slp_segment_set_overlap": (i32, [vp, i32]),
        "slp_segment_set_fused_update": (i32, [vp, i32]),
        "slp_segment_target_errors": (i32, [vp, ctypes.POINTER(i64), vp]),
        "slp_segment_join": (i32, [vp, vp]),
        "slp_segment_profile_read": (i32, [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64), ctypes.POINTER(ctypes.c_double)]),
        "slp_probe_mfma_rate": (i32, [i32, i32, vp, sz, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double), vp]),
        "slp_count_correct": (i32, [vp, vp, i32, i32, i32, vp, sz, i32, vp, vp]),
        "slp_mean_loss": (i32, [vp, i32, vp, vp]),
        "slp_count_correct_static": (i32, [vp, vp, i32, i32, i32, i32, vp, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


EXPORTS = ["slp_last_error", "slp_make_synthetic_labels", "slp_make_segment_inputs", "slp_segment_create",
           "slp_segment_destroy", "slp_segment_param_bytes", "slp_segment_workspace_bytes", "slp_segment_bind",
           "slp_segment_init", "slp_segment_set_params", "slp_segment_get_params", "slp_segment_get_grads",
           "slp_segment_get_momentum", "slp_segment_get_activation", "slp_segment_set_lr", "slp_segment_set_labels",
           "slp_segment_step", "slp_segment_forward", "slp_segment_input_grad", "slp_segment_step_external",
           "slp_segment_profile_enable", "slp_segment_profile_read", "slp_probe_mfma_rate",
           "slp_segment_set_graph", "slp_segment_set_overlap", "slp_segment_join", "slp_count_correct", "slp_mean_loss",
           "slp_count_correct_static", "slp_segment_set_fused_update", "slp_segment_target_errors"]


def _check(code):
    if code != 0:
        raise SlpError(code, lib().slp_last_error().decode())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _torch_dtype(dt):
    return torch.bfloat16 if dt == BF16 else torch.float32


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def make_synthetic_labels(seed, classes, dim, dist, kappa=1.0, dtype=F32, device="cuda"):
    """slp_make_synthetic_labels: table[classes, dim] on the device."""
    out = torch.empty((classes, dim), dtype=_torch_dtype(dtype), device=device)
    _check(lib().slp_make_synthetic_labels(seed, classes, dim, dist, kappa, _ptr(out), dtype, _stream()))
    return out


def make_segment_inputs(seed, table, y, first_sample, sigma, dtype=F32):
    """slp_make_segment_inputs: out[n] = table[y[n]] + sigma * N(0,1)."""
    assert table.dtype == torch.float32 and table.is_contiguous() and y.dtype == torch.int32
    out = torch.empty((y.numel(), table.shape[1]), dtype=_torch_dtype(dtype), device=table.device)
    _check(lib().slp_make_segment_inputs(seed, _ptr(table), table.shape[0], _ptr(y), first_sample, y.numel(),
                                         table.shape[1], sigma, _ptr(out), dtype, _stream()))
    return out


def probe_mfma_rate(dtype=BF16, iters=20000, device="cuda"):
    """slp_probe_mfma_rate: (TFLOP/s, ms) of the register-only MFMA loop on the current device."""
    scratch = torch.empty(1 << 20, dtype=torch.float32, device=device)      # 4 MiB >= 2048 B per compute unit
    tf, ms = ctypes.c_double(), ctypes.c_double()
    _check(lib().slp_probe_mfma_rate(dtype, iters, _ptr(scratch), scratch.numel() * 4, ctypes.byref(tf), ctypes.byref(ms), _stream()))
    return tf.value, ms.value


def count_correct(logits, targets, out=None, accumulate=False):
    """slp_count_correct: rows whose arg-max logit is the row's class, as a device int64 scalar (added to `out`
    when accumulate is set)."""
    assert logits.is_cuda and logits.is_contiguous() and logits.dim() == 2 and logits.dtype in (torch.float32, torch.bfloat16)
    assert targets.dtype == torch.int32 and targets.numel() == logits.shape[0]
    if out is None:
        assert not accumulate
        out = torch.empty(1, dtype=torch.int64, device=logits.device)
    scratch = torch.empty((logits.shape[0] + 3) // 4, dtype=torch.int32, device=logits.device)
    _check(lib().slp_count_correct(_ptr(logits), _ptr(targets), logits.shape[0], logits.shape[1],
                                   BF16 if logits.dtype == torch.bfloat16 else F32, _ptr(scratch), scratch.numel() * 4,
                                   int(bool(accumulate)), _ptr(out), _stream()))
    return out


def count_correct_static(logits, targets, out, accumulate=False):
    """slp_count_correct_static: the same count with the partial counts in the library's static device array; `out`
    (one int64 on the device) is the caller's, nothing is allocated here or in the library."""
    assert logits.is_cuda and logits.is_contiguous() and logits.dim() == 2 and logits.dtype in (torch.float32, torch.bfloat16)
    assert targets.dtype == torch.int32 and targets.numel() == logits.shape[0]
    assert out.is_cuda and out.dtype == torch.int64 and out.numel() == 1
    _check(lib().slp_count_correct_static(_ptr(logits), _ptr(targets), logits.shape[0], logits.shape[1],
                                          BF16 if logits.dtype == torch.bfloat16 else F32, int(bool(accumulate)), _ptr(out),
                                          _stream()))
    return out


def mean_loss(losses, out=None):
    """slp_mean_loss: mean of a contiguous run of float32 device scalars, as a device scalar."""
    assert losses.is_cuda and losses.is_contiguous() and losses.dtype == torch.float32
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=losses.device)
    _check(lib().slp_mean_loss(_ptr(losses), losses.numel(), _ptr(out), _stream()))
    return out


class Segment:
    """One network segment: owns the handle and the two torch buffers bound to it."""

    def __init__(self, widths, act, loss, max_batch, dtype=F32, lr=0.01, momentum=0.9, input_grad=False, device="cuda"):
        self.widths, self.act, self.loss, self.dtype, self.max_batch = list(widths), act, loss, dtype, max_batch
        self.L = len(widths) - 1
        self.device = torch.device(device)
        arr = (ctypes.c_int * len(widths))(*widths)
        opts = _Opts(dtype, max_batch, lr, momentum, int(input_grad))
        h = ctypes.c_void_p()
        self._h = None
        _check(lib().slp_segment_create(arr, len(widths), act, loss, ctypes.byref(opts), ctypes.byref(h)))
        self._h = h
        self.param_bytes = lib().slp_segment_param_bytes(h)
        self.workspace_bytes = lib().slp_segment_workspace_bytes(h)
        self._params = torch.empty(self.param_bytes, dtype=torch.uint8, device=self.device)
        self._work = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=self.device)
        _check(lib().slp_segment_bind(h, _ptr(self._params), self.param_bytes, _ptr(self._work), self.workspace_bytes, _stream()))
        self._table = None
        self._loss = torch.zeros(1, dtype=torch.float32, device=self.device)

    def __del__(self):
        if getattr(self, "_h", None) is not None and _lib is not None:
            _lib.slp_segment_destroy(self._h)
            self._h = None

    def init(self, seed):
        _check(lib().slp_segment_init(self._h, seed, _stream()))

    def set_lr(self, lr, momentum):
        _check(lib().slp_segment_set_lr(self._h, lr, momentum))

    def set_labels(self, table):
        assert table.dtype == torch.float32 and table.is_contiguous()
        self._table = table     # keep it alive: the library only borrows it
        _check(lib().slp_segment_set_labels(self._h, _ptr(table), table.shape[0], table.shape[1]))

    def set_params(self, layer, W, b):
        W = None if W is None else W.to(torch.float32).contiguous()
        b = None if b is None else b.to(torch.float32).contiguous()
        on_dev = int((W if W is not None else b).is_cuda)
        _check(lib().slp_segment_set_params(self._h, layer, _ptr(W), _ptr(b), on_dev, _stream()))

    def _get(self, fn, layer):
        W = torch.empty((self.widths[layer + 1], self.widths[layer]), dtype=torch.float32, device=self.device)
        b = torch.empty((self.widths[layer + 1],), dtype=torch.float32, device=self.device)
        _check(fn(self._h, layer, _ptr(W), _ptr(b), 1, _stream()))
        return W, b

    def get_params(self, layer):
        return self._get(lib().slp_segment_get_params, layer)

    def get_grads(self, layer):
        return self._get(lib().slp_segment_get_grads, layer)

    def get_bias_grad(self, layer):
        """slp_segment_get_grads for the bias alone (the only stored gradient while the fused update is on)."""
        b = torch.empty((self.widths[layer + 1],), dtype=torch.float32, device=self.device)
        _check(lib().slp_segment_get_grads(self._h, layer, None, _ptr(b), 1, _stream()))
        return b

    def get_momentum(self, layer):
        return self._get(lib().slp_segment_get_momentum, layer)

    def get_activation(self, layer, batch, kind=0):
        out = torch.empty((batch, self.widths[layer]), dtype=_torch_dtype(self.dtype), device=self.device)
        _check(lib().slp_segment_get_activation(self._h, layer, kind, batch, _ptr(out), _stream()))
        return out

    def step(self, X, targets, want_loss=True, loss_out=None):
        """slp_segment_step; returns the device scalar holding the batch loss (loss_out, a one-element float32 device
        tensor such as a slot of a loss curve, or the handle's own scalar)."""
        assert X.is_cuda and X.is_contiguous() and X.dtype == _torch_dtype(self.dtype) and X.shape[1] == self.widths[0]
        assert targets.dtype == torch.int32 and targets.numel() == X.shape[0]
        dst = self._loss if loss_out is None else loss_out
        assert dst.dtype == torch.float32 and dst.numel() == 1 and dst.is_cuda
        _check(lib().slp_segment_step(self._h, _ptr(X), _ptr(targets), X.shape[0], _ptr(dst) if want_loss else None,
                                      _stream()))
        return dst

    def forward(self, X, out=None):
        assert X.is_cuda and X.is_contiguous() and X.dtype == _torch_dtype(self.dtype) and X.shape[1] == self.widths[0]
        if out is None:
            out = torch.empty((X.shape[0], self.widths[-1]), dtype=X.dtype, device=X.device)
        _check(lib().slp_segment_forward(self._h, _ptr(X), X.shape[0], _ptr(out), _stream()))
        return out

    def input_grad(self, X, targets, loss_out=None):
        """slp_segment_input_grad: (d loss / d X, device scalar loss); parameters untouched."""
        assert X.is_cuda and X.is_contiguous() and X.dtype == _torch_dtype(self.dtype) and X.shape[1] == self.widths[0]
        assert targets.dtype == torch.int32 and targets.numel() == X.shape[0]
        dst = self._loss if loss_out is None else loss_out
        assert dst.dtype == torch.float32 and dst.numel() == 1 and dst.is_cuda
        dX = torch.empty_like(X)
        _check(lib().slp_segment_input_grad(self._h, _ptr(X), _ptr(targets), X.shape[0], _ptr(dX), _ptr(dst), _stream()))
        return dX, dst

    def step_external(self, X, dA_out):
        """slp_segment_step_external: training step from a gradient w.r.t. the segment output."""
        assert X.is_cuda and X.is_contiguous() and X.dtype == _torch_dtype(self.dtype) and X.shape[1] == self.widths[0]
        assert dA_out.is_contiguous() and dA_out.dtype == X.dtype and tuple(dA_out.shape) == (X.shape[0], self.widths[-1])
        _check(lib().slp_segment_step_external(self._h, _ptr(X), _ptr(dA_out), X.shape[0], _stream()))

    def profile_enable(self, on=True):
        _check(lib().slp_segment_profile_enable(self._h, int(on)))

    def set_graph(self, on=True):
        """slp_segment_set_graph: replay captured launch sequences of step() (for launch-bound segments)."""
        _check(lib().slp_segment_set_graph(self._h, int(bool(on))))

    def set_overlap(self, on=True):
        """slp_segment_set_overlap: step() returns with the parameter updates still running beside the caller's next work."""
        _check(lib().slp_segment_set_overlap(self._h, int(bool(on))))

    def set_fused_update(self, on=True):
        """slp_segment_set_fused_update: the weight-gradient products apply the SGD step in their epilogue."""
        _check(lib().slp_segment_set_fused_update(self._h, int(on)))

    def target_errors(self):
        """slp_segment_target_errors: rows with an out-of-range class id seen since bind (synchronises the stream)."""
        n = ctypes.c_int64()
        _check(lib().slp_segment_target_errors(self._h, ctypes.byref(n), _stream()))
        return n.value

    def join(self):
        """slp_segment_join: the current stream waits for updates a step with overlap on left running."""
        _check(lib().slp_segment_join(self._h, _stream()))

    def profile_read(self):
        ms, n, fl = ctypes.c_double(), ctypes.c_int64(), ctypes.c_double()
        _check(lib().slp_segment_profile_read(self._h, ctypes.byref(ms), ctypes.byref(n), ctypes.byref(fl)))
        return ms.value, n.value, fl.value
