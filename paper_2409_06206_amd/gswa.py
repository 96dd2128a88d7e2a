"""Thin ctypes binding over libgswa.so (see include/gswa.h for the contract).

Argument marshalling only: every step of the layer runs inside the HIP library.  torch is
used for device memory and for the current stream handle.  The functions carry the names of
the C entry points.  A missing library is an error; there is no fallback path.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgswa.so")

GSWA_OK, GSWA_EINVAL, GSWA_EUNSUPPORTED, GSWA_EHIP, GSWA_ETOOBIG = 0, -1, -2, -3, -4
GSWA_STATIC_SCRATCH_BYTES = 96 * 1024 * 1024
GSWA_F32, GSWA_BF16 = 0, 1
GSWA_NO_CASCADE, GSWA_ACCUM_WGRAD, GSWA_FORCE_STAGED, GSWA_DETERMINISTIC = 1, 2, 4, 8
GSWA_PATH_STAGED, GSWA_PATH_FUSED, GSWA_PATH_WINDOW_FWD = 0, 1, 2

EXPORTS = ("gswa_query_bytes", "gswa_query_path", "gswa_forward", "gswa_backward", "gswa_backward_static", "gswa_strerror",
           "gswa_last_hip_error", "gswa_version", "gswa_profile_enable",
           "gswa_profile_kernel_count", "gswa_profile_kernel_name", "gswa_profile_collect")


class GswaError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"gswa status {status}: {text}")
        self.status = status


class gswa_desc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
                ("C", ctypes.c_int32), ("heads", ctypes.c_int32), ("groups", ctypes.c_int32),
                ("window", ctypes.c_int32), ("shift", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("flags", ctypes.c_uint32), ("dqk", ctypes.c_int32)]


_lib = None


def lib():
    """The loaded library (loads it on first use; raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2409_06206_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        try:
            import torch  # noqa: F401  (its HIP runtime must be the one in the process)
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        vp, sp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_size_t)
        dp = ctypes.POINTER(gswa_desc)
        L.gswa_query_bytes.argtypes = [dp, sp, sp, sp]
        L.gswa_query_bytes.restype = ctypes.c_int
        L.gswa_query_path.argtypes = [dp, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.gswa_query_path.restype = ctypes.c_int
        L.gswa_forward.argtypes = [dp] + [vp] * 10
        L.gswa_forward.restype = ctypes.c_int
        L.gswa_backward.argtypes = [dp] + [vp] * 16
        L.gswa_backward.restype = ctypes.c_int
        L.gswa_backward_static.argtypes = [dp] + [vp] * 15
        L.gswa_backward_static.restype = ctypes.c_int
        L.gswa_strerror.argtypes = [ctypes.c_int]
        L.gswa_strerror.restype = ctypes.c_char_p
        L.gswa_last_hip_error.restype = ctypes.c_char_p
        L.gswa_version.restype = ctypes.c_int
        L.gswa_profile_enable.argtypes = [ctypes.c_int]
        L.gswa_profile_enable.restype = ctypes.c_int
        L.gswa_profile_kernel_count.restype = ctypes.c_int
        L.gswa_profile_kernel_name.argtypes = [ctypes.c_int]
        L.gswa_profile_kernel_name.restype = ctypes.c_char_p
        L.gswa_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double),
                                           ctypes.POINTER(ctypes.c_longlong),
                                           ctypes.POINTER(ctypes.c_longlong)]
        L.gswa_profile_collect.restype = ctypes.c_int
        _lib = L
    return _lib


def make_desc(B, H, W, C, heads, groups, window, shift, dtype, flags=0, dqk=0):
    code = {"f32": GSWA_F32, "bf16": GSWA_BF16}.get(dtype, dtype)
    return gswa_desc(B, H, W, C, heads, groups, window, shift, code, flags, dqk)


def _ptr(t):
    """Device (or null) pointer of a torch tensor, a raw integer address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors passed to the GSWA library must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def _check(status):
    if status != GSWA_OK:
        text = gswa_strerror(status)
        if status == GSWA_EHIP:
            text += ": " + lib().gswa_last_hip_error().decode()
        raise GswaError(status, text)


def gswa_strerror(status):
    return lib().gswa_strerror(int(status)).decode()


def gswa_version():
    return lib().gswa_version()


def gswa_query_bytes(desc):
    """(saved_bytes, fwd_ws_bytes, bwd_ws_bytes) for the layer."""
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().gswa_query_bytes(ctypes.byref(desc), ctypes.byref(a), ctypes.byref(b),
                                  ctypes.byref(c)))
    return a.value, b.value, c.value


def gswa_query_path(desc):
    """(forward_path, backward_path): which organisation of kernels serves the layer (GSWA_PATH_*)."""
    f, b = ctypes.c_int(), ctypes.c_int()
    _check(lib().gswa_query_path(ctypes.byref(desc), ctypes.byref(f), ctypes.byref(b)))
    return f.value, b.value


def gswa_forward(desc, x, w_qkv, b_qkv, w_proj, b_proj, bias_table, y, saved, ws, stream=None):
    _check(lib().gswa_forward(ctypes.byref(desc), _ptr(x), _ptr(w_qkv), _ptr(b_qkv), _ptr(w_proj),
                              _ptr(b_proj), _ptr(bias_table), _ptr(y), _ptr(saved), _ptr(ws),
                              _stream(stream)))


def gswa_backward(desc, x, dy, w_qkv, b_qkv, w_proj, b_proj, bias_table, saved, dx, dw_qkv,
                  db_qkv, dw_proj, db_proj, dbias_table, ws, stream=None):
    _check(lib().gswa_backward(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(w_qkv), _ptr(b_qkv),
                               _ptr(w_proj), _ptr(b_proj), _ptr(bias_table), _ptr(saved), _ptr(dx),
                               _ptr(dw_qkv), _ptr(db_qkv), _ptr(dw_proj), _ptr(db_proj),
                               _ptr(dbias_table), _ptr(ws), _stream(stream)))


def gswa_backward_static(desc, x, dy, w_qkv, b_qkv, w_proj, b_proj, bias_table, saved, dx, dw_qkv,
                         db_qkv, dw_proj, db_proj, dbias_table, stream=None):
    _check(lib().gswa_backward_static(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(w_qkv), _ptr(b_qkv),
                                      _ptr(w_proj), _ptr(b_proj), _ptr(bias_table), _ptr(saved), _ptr(dx),
                                      _ptr(dw_qkv), _ptr(db_qkv), _ptr(dw_proj), _ptr(db_proj),
                                      _ptr(dbias_table), _stream(stream)))


def gswa_profile_enable(on):
    _check(lib().gswa_profile_enable(int(bool(on))))


def gswa_profile_collect():
    """{kernel name: (total_ms, launches)} since the last collect, plus the dropped count."""
    L = lib()
    n = L.gswa_profile_kernel_count()
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_longlong * n)()
    dropped = ctypes.c_longlong()
    _check(L.gswa_profile_collect(ms, cnt, ctypes.byref(dropped)))
    out = {L.gswa_profile_kernel_name(i).decode(): (ms[i], cnt[i]) for i in range(n) if cnt[i]}
    return out, dropped.value
