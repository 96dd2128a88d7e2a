"""Thin ctypes binding over the whole-layer entry points of libgswa.so (see include/astl.h).

Argument marshalling only; the functions carry the names of the C entry points.  The library is
the one ``gswa.lib()`` loads: a missing library is an error, there is no fallback path.
"""
import ctypes

from . import gswa
from .gswa import _check, _ptr, _stream

EXPORTS = ("astl_query_bytes", "astl_forward", "astl_backward",
           "astl_stack_query_bytes", "astl_stack_forward", "astl_stack_backward",
           "astl_stack_tiled_query_bytes", "astl_stack_forward_tiled")
PARAM_FIELDS = ("ln1_w", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj", "bias_table",
                "ln2_w", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


class astl_desc(ctypes.Structure):
    _fields_ = [("attn", gswa.gswa_desc), ("hidden", ctypes.c_int32), ("eps", ctypes.c_float)]


class astl_params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in PARAM_FIELDS]


class astl_grads(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in PARAM_FIELDS]


class astl_stack_desc(ctypes.Structure):
    _fields_ = [("layer", astl_desc), ("n_layers", ctypes.c_int32), ("shift", ctypes.c_int32),
                ("checkpoint_every", ctypes.c_int32)]


_ready = False


def lib():
    global _ready
    L = gswa.lib()
    if not _ready:
        vp, sp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t)
        dp = ctypes.POINTER(astl_desc)
        L.astl_query_bytes.argtypes = [dp, sp, sp, sp]
        L.astl_query_bytes.restype = ctypes.c_int
        L.astl_forward.argtypes = [dp, vp, ctypes.POINTER(astl_params), vp, vp, vp, vp]
        L.astl_forward.restype = ctypes.c_int
        L.astl_backward.argtypes = [dp, vp, vp, ctypes.POINTER(astl_params), vp, vp,
                                    ctypes.POINTER(astl_grads), vp, vp]
        L.astl_backward.restype = ctypes.c_int
        sd = ctypes.POINTER(astl_stack_desc)
        L.astl_stack_query_bytes.argtypes = [sd, sp, sp, sp]
        L.astl_stack_query_bytes.restype = ctypes.c_int
        L.astl_stack_forward.argtypes = [sd, vp, ctypes.POINTER(astl_params), vp, vp, vp, vp]
        L.astl_stack_forward.restype = ctypes.c_int
        L.astl_stack_backward.argtypes = [sd, vp, vp, ctypes.POINTER(astl_params), vp, vp,
                                          ctypes.POINTER(astl_grads), vp, vp]
        L.astl_stack_backward.restype = ctypes.c_int
        L.astl_stack_tiled_query_bytes.argtypes = [sd, ctypes.c_int32, sp]
        L.astl_stack_tiled_query_bytes.restype = ctypes.c_int
        L.astl_stack_forward_tiled.argtypes = [sd, vp, ctypes.POINTER(astl_params), vp, ctypes.c_int32, vp, vp]
        L.astl_stack_forward_tiled.restype = ctypes.c_int
        _ready = True
    return L


def make_desc(B, H, W, C, heads, groups, window, shift, dtype, hidden, eps=1e-5, flags=0, dqk=0):
    return astl_desc(gswa.make_desc(B, H, W, C, heads, groups, window, shift, dtype, flags, dqk),
                     hidden, eps)


def _fill(struct, tensors):
    """Struct of device pointers from a mapping field name -> tensor / address / None."""
    return struct(**{n: _ptr(tensors.get(n)) for n in PARAM_FIELDS})


def astl_query_bytes(desc):
    """(saved_bytes, fwd_ws_bytes, bwd_ws_bytes) for the layer."""
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().astl_query_bytes(ctypes.byref(desc), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def astl_forward(desc, x, params, y, saved, ws, stream=None):
    """params: mapping with the fields of astl_params (tensors or raw device addresses)."""
    p = _fill(astl_params, params)
    _check(lib().astl_forward(ctypes.byref(desc), _ptr(x), ctypes.byref(p), _ptr(y), _ptr(saved),
                              _ptr(ws), _stream(stream)))


def astl_backward(desc, x, dy, params, saved, dx, grads, ws, stream=None):
    p, g = _fill(astl_params, params), _fill(astl_grads, grads)
    _check(lib().astl_backward(ctypes.byref(desc), _ptr(x), _ptr(dy), ctypes.byref(p), _ptr(saved),
                               _ptr(dx), ctypes.byref(g), _ptr(ws), _stream(stream)))


def make_stack_desc(B, H, W, C, heads, groups, window, shift, dtype, hidden, n_layers, checkpoint_every=0,
                    eps=1e-5, flags=0, dqk=0):
    """``shift`` is the shift of the odd layers (even layers are unshifted)."""
    return astl_stack_desc(make_desc(B, H, W, C, heads, groups, window, 0, dtype, hidden, eps, flags, dqk),
                           n_layers, shift, checkpoint_every)


def _fill_array(struct, per_layer):
    arr = (struct * len(per_layer))()
    for i, t in enumerate(per_layer):
        arr[i] = _fill(struct, t)
    return arr


def astl_stack_query_bytes(desc):
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().astl_stack_query_bytes(ctypes.byref(desc), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def astl_stack_forward(desc, x, params, y, saved, ws, stream=None):
    """params: one mapping per layer with the fields of astl_params."""
    p = _fill_array(astl_params, params)
    _check(lib().astl_stack_forward(ctypes.byref(desc), _ptr(x), p, _ptr(y), _ptr(saved), _ptr(ws),
                                    _stream(stream)))


def astl_stack_backward(desc, x, dy, params, saved, dx, grads, ws, stream=None):
    p, g = _fill_array(astl_params, params), _fill_array(astl_grads, grads)
    _check(lib().astl_stack_backward(ctypes.byref(desc), _ptr(x), _ptr(dy), p, _ptr(saved), _ptr(dx), g,
                                     _ptr(ws), _stream(stream)))


def astl_stack_tiled_query_bytes(desc, band_windows):
    a = ctypes.c_size_t()
    _check(lib().astl_stack_tiled_query_bytes(ctypes.byref(desc), band_windows, ctypes.byref(a)))
    return a.value


def astl_stack_forward_tiled(desc, x, params, y, band_windows, ws, stream=None):
    p = _fill_array(astl_params, params)
    _check(lib().astl_stack_forward_tiled(ctypes.byref(desc), _ptr(x), p, _ptr(y), band_windows, _ptr(ws),
                                          _stream(stream)))
