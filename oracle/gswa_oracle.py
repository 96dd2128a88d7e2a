"""ctypes wrapper around the fp64 CPU oracle of Group Shifted Window Attention.

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the CPU-baseline leg
of the benchmark call this; the HIP library never does.  The arithmetic lives
in ``gswa_oracle.c`` (AgileIR, Sec. "Group Shifted Window Attention", Eq. 6-8);
this file only marshals numpy arrays.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gswa_oracle.c")
_SO = os.path.join(_HERE, "libgswa_oracle.so")


def build(force=False):
    """Compile the C oracle with gcc (OpenMP, -O2) next to its source."""
    stale = (not os.path.exists(_SO)) or os.path.getmtime(_SO) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in
                ("B", "H", "W", "C", "heads", "groups", "window", "shift", "cascade", "dqk")]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        lib.gswa_oracle_forward.argtypes = [ctypes.POINTER(_Shape)] + [dp] * 9
        lib.gswa_oracle_forward.restype = ctypes.c_int
        lib.gswa_oracle_backward.argtypes = [ctypes.POINTER(_Shape)] + [dp] * 13
        lib.gswa_oracle_backward.restype = ctypes.c_int
        lib.gswa_oracle_threads.restype = ctypes.c_int
        lib.gswa_oracle_set_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _f64(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _ptr(a):
    if a is None:
        return ctypes.cast(None, ctypes.POINTER(ctypes.c_double))
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def param_shapes(C, heads, groups, window, dqk=0):
    """Shapes of (w_qkv, b_qkv, w_proj, b_proj, bias_table); dqk = channels of q and of k per
    head (0: C // heads, the plain layer)."""
    Cg = C // groups
    Rg = 2 * (heads // groups) * (dqk or C // heads) + Cg
    return ((groups, Rg, Cg), (groups, Rg), (C, C), (C,),
            ((2 * window - 1) ** 2, heads))


def threads():
    return _load().gswa_oracle_threads()


def set_threads(n):
    _load().gswa_oracle_set_threads(int(n))


def forward(x, w_qkv, b_qkv, w_proj, b_proj, table, *, heads, groups, window, shift,
            cascade=True, want_attn=False, want_probs=False, dqk=0):
    """y = GSWA(x); x is [B,H,W,C].  Returns y, or (y, extras dict) if extras are asked for."""
    lib = _load()
    B, H, W, C = x.shape
    shp = _Shape(B, H, W, C, heads, groups, window, shift, int(bool(cascade)), int(dqk))
    ps = param_shapes(C, heads, groups, window, dqk)
    x = _f64(x, (B, H, W, C))
    args = [_f64(a, s) for a, s in zip((w_qkv, b_qkv, w_proj, b_proj, table), ps)]
    y = np.empty_like(x)
    attn = np.empty_like(x) if want_attn else None
    probs = None
    if want_probs:
        N = window * window
        probs = np.empty((B * (H // window) * (W // window), heads, N, N), dtype=np.float64)
    rc = lib.gswa_oracle_forward(ctypes.byref(shp), _ptr(x), *[_ptr(a) for a in args],
                                 _ptr(y), _ptr(attn), _ptr(probs))
    if rc != 0:
        raise ValueError(f"gswa_oracle_forward failed with code {rc}")
    if want_attn or want_probs:
        return y, {"attn": attn, "probs": probs}
    return y


def backward(x, dy, w_qkv, b_qkv, w_proj, b_proj, table, *, heads, groups, window, shift,
             cascade=True, dqk=0):
    """Gradients of sum(dy*y): (dx, dw_qkv, db_qkv, dw_proj, db_proj, dtable)."""
    lib = _load()
    B, H, W, C = x.shape
    shp = _Shape(B, H, W, C, heads, groups, window, shift, int(bool(cascade)), int(dqk))
    ps = param_shapes(C, heads, groups, window, dqk)
    x = _f64(x, (B, H, W, C))
    dy = _f64(dy, (B, H, W, C))
    args = [_f64(a, s) for a, s in zip((w_qkv, b_qkv, w_proj, b_proj, table), ps)]
    dx = np.empty_like(x)
    grads = [np.empty(s, dtype=np.float64) for s in ps]
    rc = lib.gswa_oracle_backward(ctypes.byref(shp), _ptr(x), _ptr(dy),
                                  *[_ptr(a) for a in args], _ptr(dx),
                                  *[_ptr(g) for g in grads])
    if rc != 0:
        raise ValueError(f"gswa_oracle_backward failed with code {rc}")
    return (dx, *grads)
