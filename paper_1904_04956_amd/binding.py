"""ctypes binding of libblstm_mi355.so: argument marshalling only.

Every function has the name and the argument order of its C declaration in
include/blstm_mi355.h.  Device buffers are torch tensors (PyTorch is used for
device memory and streams, nothing else) or raw integer addresses.  There is no
CPU fallback: a missing library or a non-zero status raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_double, c_float, c_int, c_int32, c_int64, c_size_t, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libblstm_mi355.so")

BLSTM_WX, BLSTM_UH, BLSTM_B, BLSTM_WP, BLSTM_BP, BLSTM_WS, BLSTM_BS = range(7)
BLSTM_MAX_REPLICAS = 64

EXPORTS = [
    "blstm_create", "blstm_destroy", "blstm_param_count", "blstm_workspace_bytes", "blstm_param_offset",
    "blstm_bind", "blstm_forward", "softmax_xent_fwd_bwd", "softmax_xent_fwd_bwd_noalloc", "blstm_backward", "sgd_step", "adpsgd_mix",
    "sgd_mix_pair", "sync_average", "blstm_lr_schedule",
    "adpsgd_ring_partner", "blstm_shadow_refresh", "blstm_set_option", "blstm_weights_changed", "blstm_device_status", "blstm_profile_enable", "blstm_profile_read",
    "blstm_profile_classes", "blstm_profile_name", "blstm_last_error",
]


class BlstmError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"blstm_mi355 status {code}: {text}")
        self.code = code


class blstm_config(ctypes.Structure):
    _fields_ = [("T", c_int32), ("B", c_int32), ("D", c_int32), ("H", c_int32), ("L", c_int32),
                ("P", c_int32), ("V", c_int32), ("mode", c_int32), ("loss_scale", c_float)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_1904_04956_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_1904_04956_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    L.blstm_create.argtypes = [POINTER(blstm_config), POINTER(c_void_p)]
    L.blstm_create.restype = c_int
    L.blstm_destroy.argtypes = [c_void_p]
    L.blstm_destroy.restype = None
    L.blstm_param_count.argtypes = [c_void_p]
    L.blstm_param_count.restype = c_size_t
    L.blstm_workspace_bytes.argtypes = [c_void_p]
    L.blstm_workspace_bytes.restype = c_size_t
    L.blstm_param_offset.argtypes = [c_void_p, c_int, c_int, c_int, POINTER(c_size_t), POINTER(c_size_t)]
    L.blstm_param_offset.restype = c_int
    L.blstm_bind.argtypes = [c_void_p, c_void_p, c_size_t]
    L.blstm_bind.restype = c_int
    L.blstm_forward.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    L.blstm_forward.restype = c_int
    L.softmax_xent_fwd_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    L.softmax_xent_fwd_bwd.restype = c_int
    L.softmax_xent_fwd_bwd_noalloc.argtypes = L.softmax_xent_fwd_bwd.argtypes
    L.softmax_xent_fwd_bwd_noalloc.restype = c_int
    L.blstm_backward.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
    L.blstm_backward.restype = c_int
    L.sgd_step.argtypes = [c_void_p, c_void_p, c_void_p, c_size_t, c_float, c_float, c_void_p, c_void_p]
    L.sgd_step.restype = c_int
    L.adpsgd_mix.argtypes = [POINTER(c_void_p), POINTER(c_void_p), c_size_t, c_int, POINTER(c_int32), c_void_p]
    L.adpsgd_mix.restype = c_int
    L.sgd_mix_pair.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_float, c_float,
                               c_void_p, c_void_p, c_void_p]
    L.sgd_mix_pair.restype = c_int
    L.sync_average.argtypes = [POINTER(c_void_p), POINTER(c_void_p), c_size_t, c_int, c_void_p]
    L.sync_average.restype = c_int
    L.blstm_lr_schedule.argtypes = [c_int, c_double, c_double, c_int, c_int]
    L.blstm_lr_schedule.restype = c_double
    L.adpsgd_ring_partner.argtypes = [c_int, c_int64, POINTER(c_int32)]
    L.adpsgd_ring_partner.restype = c_int
    L.blstm_shadow_refresh.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p]
    L.blstm_shadow_refresh.restype = c_int
    L.blstm_set_option.argtypes = [c_void_p, c_int, c_int]
    L.blstm_set_option.restype = c_int
    L.blstm_weights_changed.argtypes = [c_void_p]
    L.blstm_weights_changed.restype = c_int
    L.blstm_device_status.argtypes = [c_void_p, c_void_p]
    L.blstm_device_status.restype = c_int
    L.blstm_profile_enable.argtypes = [c_void_p, c_int]
    L.blstm_profile_enable.restype = c_int
    L.blstm_profile_read.argtypes = [c_void_p, POINTER(c_double), POINTER(c_int64), c_int]
    L.blstm_profile_read.restype = c_int
    L.blstm_profile_classes.argtypes = []
    L.blstm_profile_classes.restype = c_int
    L.blstm_profile_name.argtypes = [c_int]
    L.blstm_profile_name.restype = c_char_p
    L.blstm_last_error.argtypes = []
    L.blstm_last_error.restype = c_char_p
    _lib = L
    return L


def _check(rc):
    if rc != 0:
        raise BlstmError(rc, lib().blstm_last_error().decode())
    return rc


def _ptr(t):
    """Address of a torch tensor's storage, a raw address, or NULL for None."""
    if t is None:
        return None
    if isinstance(t, int):
        return c_void_p(t)
    return c_void_p(t.data_ptr())


def _stream(stream):
    """hipStream_t handle: None = torch's current stream, int = raw handle, else a torch stream."""
    if stream is None:
        import torch
        return c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return c_void_p(stream)
    return c_void_p(stream.cuda_stream)


# --------------------------------------------------------------------------- context

def blstm_create(T, B, D, H, L, P, V, mode, loss_scale=0.0):
    cfg = blstm_config(T, B, D, H, L, P, V, mode, loss_scale)
    h = c_void_p()
    _check(lib().blstm_create(byref(cfg), byref(h)))
    return h


def blstm_destroy(ctx):
    lib().blstm_destroy(ctx)


def blstm_param_count(ctx):
    return int(lib().blstm_param_count(ctx))


def blstm_workspace_bytes(ctx):
    return int(lib().blstm_workspace_bytes(ctx))


def blstm_param_offset(ctx, layer, direction, which):
    off, ln = c_size_t(), c_size_t()
    _check(lib().blstm_param_offset(ctx, layer, direction, which, byref(off), byref(ln)))
    return int(off.value), int(ln.value)


def blstm_bind(ctx, workspace, nbytes=None):
    if nbytes is None:
        nbytes = workspace.numel() * workspace.element_size()
    return _check(lib().blstm_bind(ctx, _ptr(workspace), nbytes))


# --------------------------------------------------------------------------- the five calls of the hot path

def blstm_forward(ctx, theta, x, z_out, stream=None):
    return _check(lib().blstm_forward(ctx, _ptr(theta), _ptr(x), _ptr(z_out), _stream(stream)))


def softmax_xent_fwd_bwd(ctx, theta, z, labels, loss_dev, dz, grad, stream=None):
    return _check(lib().softmax_xent_fwd_bwd(ctx, _ptr(theta), _ptr(z), _ptr(labels), _ptr(loss_dev), _ptr(dz),
                                             _ptr(grad), _stream(stream)))


def softmax_xent_fwd_bwd_noalloc(ctx, theta, z, labels, loss_dev, dz, grad, stream=None):
    return _check(lib().softmax_xent_fwd_bwd_noalloc(ctx, _ptr(theta), _ptr(z), _ptr(labels), _ptr(loss_dev), _ptr(dz),
                                                     _ptr(grad), _stream(stream)))


def blstm_backward(ctx, theta, x, dz, grad, stream=None):
    return _check(lib().blstm_backward(ctx, _ptr(theta), _ptr(x), _ptr(dz), _ptr(grad), _stream(stream)))


def sgd_step(theta_master, theta_bf16_or_null, grad, n, lr, momentum=0.0, velocity_or_null=None, stream=None):
    return _check(lib().sgd_step(_ptr(theta_master), _ptr(theta_bf16_or_null), _ptr(grad), n, lr, momentum,
                                 _ptr(velocity_or_null), _stream(stream)))


def adpsgd_mix(theta_master, theta_bf16_or_null, n, R, partner, stream=None):
    masters = (c_void_p * R)(*[_ptr(t) for t in theta_master])
    shadows = None
    if theta_bf16_or_null is not None:
        shadows = (c_void_p * R)(*[_ptr(t) for t in theta_bf16_or_null])
    part = (c_int32 * R)(*[int(p) for p in partner])
    return _check(lib().adpsgd_mix(masters, shadows, n, R, part, _stream(stream)))


def sgd_mix_pair(theta_i, theta_j, theta_bf16_i_or_null, theta_bf16_j_or_null, grad_i, grad_j, n, lr, momentum=0.0,
                 velocity_i_or_null=None, velocity_j_or_null=None, stream=None):
    return _check(lib().sgd_mix_pair(_ptr(theta_i), _ptr(theta_j), _ptr(theta_bf16_i_or_null), _ptr(theta_bf16_j_or_null),
                                     _ptr(grad_i), _ptr(grad_j), n, lr, momentum, _ptr(velocity_i_or_null),
                                     _ptr(velocity_j_or_null), _stream(stream)))


def sync_average(theta_master, theta_bf16_or_null, n, R, stream=None):
    masters = (c_void_p * R)(*[_ptr(t) for t in theta_master])
    shadows = None
    if theta_bf16_or_null is not None:
        shadows = (c_void_p * R)(*[_ptr(t) for t in theta_bf16_or_null])
    return _check(lib().sync_average(masters, shadows, n, R, _stream(stream)))


def blstm_lr_schedule(epoch, base_lr, peak_lr, warmup_epochs=10, anneal_from=11):
    return float(lib().blstm_lr_schedule(int(epoch), float(base_lr), float(peak_lr), int(warmup_epochs), int(anneal_from)))


def adpsgd_ring_partner(R, step):
    out = (c_int32 * max(R, 1))()
    _check(lib().adpsgd_ring_partner(R, step, out))
    return [int(v) for v in out[:R]]


def blstm_shadow_refresh(theta_master, theta_bf16, n, stream=None):
    return _check(lib().blstm_shadow_refresh(_ptr(theta_master), _ptr(theta_bf16), n, _stream(stream)))


BLSTM_OPT_RECURRENT_PATH = 1
BLSTM_OPT_RECURRENT_SYNC = 2
BLSTM_OPT_KEEP_WEIGHT_COPIES = 3
BLSTM_OPT_TEST_ABORT = 4
BLSTM_OPT_DEFER_SOFTMAX_WGRAD = 5
BLSTM_NOALLOC_SCRATCH_BYTES = 32 << 20


def blstm_set_option(ctx, option, value):
    return _check(lib().blstm_set_option(ctx, option, value))


def blstm_weights_changed(ctx):
    return _check(lib().blstm_weights_changed(ctx))


def blstm_device_status(ctx, stream=None):
    return _check(lib().blstm_device_status(ctx, _stream(stream)))


# --------------------------------------------------------------------------- per-kernel-class timing

def blstm_profile_enable(ctx, enable):
    return _check(lib().blstm_profile_enable(ctx, int(bool(enable))))


def blstm_profile_read(ctx):
    """{class name: (milliseconds, launches)} accumulated since profiling was enabled."""
    k = lib().blstm_profile_classes()
    ms = (c_double * k)()
    cnt = (c_int64 * k)()
    _check(lib().blstm_profile_read(ctx, ms, cnt, k))
    return {lib().blstm_profile_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(k)}


def blstm_last_error():
    return lib().blstm_last_error().decode()
