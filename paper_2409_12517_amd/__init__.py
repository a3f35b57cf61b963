"""Thin Python binding of libssg.so (FP8 Smooth-SwiGLU MLP block for MI355X).

Argument marshalling only: every function below has the name and argument
order of the C entry point in ``include/ssg.h`` and passes device pointers of
``torch`` tensors straight through.  PyTorch is used for device memory and the
current stream, nothing else; there is no fallback path -- if the library has
not been built (``python paper_2409_12517_amd/build.py``) importing fails.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, c_char_p, c_float, c_int, c_int32, c_int64, c_size_t, c_uint8, c_void_p

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libssg.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python paper_2409_12517_amd/build.py` "
        "(hipcc, --offload-arch=gfx950). There is no CPU fallback.")

_lib = ctypes.CDLL(LIB_PATH)

# enums of ssg.h
SSG_OK, SSG_ERR_ARG, SSG_ERR_SHAPE, SSG_ERR_WORKSPACE, SSG_ERR_HIP, SSG_ERR_UNSUPPORTED = 0, -1, -2, -3, -4, -5
SSG_E4M3, SSG_E5M2 = 0, 1
SSG_BF16, SSG_F32 = 0, 1
SSG_SCALE_CURRENT, SSG_SCALE_GIVEN, SSG_SCALE_DELAYED = 0, 1, 2
SSG_ROUND_EXACT_DIV, SSG_ROUND_POW2 = 0, 1

EXPORTS = [
    "ssg_last_error", "ssg_version", "ssg_amax", "ssg_quantize", "ssg_gemm_fp8", "ssg_gemm_fp8_layout", "ssg_swiglu",
    "ssg_smooth_swiglu_quantize", "ssg_fold_w3", "ssg_mlp_saved_bytes", "ssg_mlp_workspace_bytes",
    "ssg_mlp_fwd", "ssg_mlp_bwd", "ssg_mlp_bwd_plan", "ssg_mlp_view_saved", "ssg_mlp_view_workspace",
    "ssg_mlp_scaling_state_bytes", "ssg_mlp_scaling_init",
    "ssg_infer_prepared_bytes", "ssg_infer_workspace_bytes", "ssg_infer_prepare", "ssg_infer_fwd", "ssg_infer_view",
    "ssg_infer_noalloc_max_bytes", "ssg_infer_fwd_noalloc",
    "ssg_adam_state_bytes", "ssg_adam_init", "ssg_adam_step", "ssg_adam_view_state",
    "ssg_profile_enable", "ssg_profile_select", "ssg_profile_read",
]


class ssg_mlp_desc(Structure):
    _fields_ = [("T", c_int64), ("d", c_int64), ("f", c_int64), ("smooth", c_int32), ("rnd", c_int32),
                ("y_dtype", c_int32), ("dw_dtype", c_int32), ("weights_cached", c_int32), ("scale_mode", c_int32),
                ("h_scale_mode", c_int32), ("keep_bf16_grads", c_int32), ("w3_layer_bf16", c_int32), ("reserved", c_int32 * 3),
                ("scaling_state", c_void_p), ("h_scale", c_void_p),
                ("h_counters", c_void_p)]


class ssg_infer_view_t(Structure):
    _fields_ = [(n, c_void_p) for n in ("weight_scales", "w1_q", "w2_q", "w3_q", "x_scale", "x_q", "h_q")]


class ssg_adam_desc(Structure):
    _fields_ = [("n", c_int64), ("lr", c_float), ("beta1", c_float), ("beta2", c_float), ("eps", c_float),
                ("weight_decay", c_float), ("step", c_int32), ("grad_dtype", c_int32), ("rnd", c_int32),
                ("reserved", c_int32 * 3)]


class ssg_adam_state_view(Structure):
    _fields_ = [(n, c_void_p) for n in ("m_q", "v_q", "scales")]


class ssg_mlp_saved_view(Structure):
    _fields_ = [(n, c_void_p) for n in (
        "scales", "s", "sinv", "h_camax", "w3_camax", "x_q", "w1_q", "w2_q", "h_q", "w3_q", "U", "G", "h_b", "h_bT", "w3T")]


class ssg_mlp_workspace_view(Structure):
    _fields_ = [(n, c_void_p) for n in ("scales", "dy_q", "du_q", "dg_q", "dU", "dG", "dyT")]


_lib.ssg_last_error.restype = c_char_p
_lib.ssg_version.restype = c_char_p
_lib.ssg_amax.argtypes = [c_void_p, c_int, c_size_t, c_void_p, c_void_p]
_lib.ssg_quantize.argtypes = [c_void_p, c_int, c_int64, c_int64, c_int, c_int, c_int, c_void_p, c_void_p,
                              c_void_p, c_void_p, c_void_p]
_lib.ssg_gemm_fp8.argtypes = [c_void_p, c_int, c_void_p, c_int, c_int64, c_int64, c_int64, c_void_p, c_void_p,
                              c_void_p, c_int, c_void_p]
_lib.ssg_gemm_fp8_layout.argtypes = [c_void_p, c_int, c_int, c_void_p, c_int, c_int, c_int64, c_int64, c_int64, c_void_p,
                                     c_void_p, c_void_p, c_int, c_void_p]
_lib.ssg_swiglu.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_void_p]
_lib.ssg_smooth_swiglu_quantize.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int, c_void_p, c_void_p,
                                            c_void_p, c_void_p, c_void_p, c_void_p]
_lib.ssg_fold_w3.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_void_p,
                             c_void_p, c_void_p]
_lib.ssg_mlp_saved_bytes.argtypes = [POINTER(ssg_mlp_desc)]
_lib.ssg_mlp_saved_bytes.restype = c_size_t
_lib.ssg_mlp_workspace_bytes.argtypes = [POINTER(ssg_mlp_desc)]
_lib.ssg_mlp_workspace_bytes.restype = c_size_t
_lib.ssg_mlp_fwd.argtypes = [POINTER(ssg_mlp_desc)] + [c_void_p] * 6 + [c_size_t, c_void_p]
_lib.ssg_mlp_bwd.argtypes = [POINTER(ssg_mlp_desc), c_void_p, c_void_p, c_size_t] + [c_void_p] * 5 + [c_size_t, c_void_p]
_lib.ssg_mlp_bwd_plan.argtypes = [POINTER(ssg_mlp_desc), ctypes.c_int32, POINTER(ctypes.c_int32), POINTER(ctypes.c_int32)]
_lib.ssg_mlp_view_saved.argtypes = [POINTER(ssg_mlp_desc), c_void_p, POINTER(ssg_mlp_saved_view)]
_lib.ssg_mlp_view_workspace.argtypes = [POINTER(ssg_mlp_desc), c_void_p, POINTER(ssg_mlp_workspace_view)]
_lib.ssg_profile_enable.argtypes = [c_int]
_lib.ssg_profile_select.argtypes = [c_int]
_lib.ssg_profile_read.argtypes = [POINTER(c_float), POINTER(c_int), POINTER(ctypes.c_double), c_int]
_lib.ssg_mlp_scaling_state_bytes.argtypes = []
_lib.ssg_mlp_scaling_state_bytes.restype = c_size_t
_lib.ssg_mlp_scaling_init.argtypes = [c_void_p, c_void_p]
_lib.ssg_infer_prepared_bytes.argtypes = [POINTER(ssg_mlp_desc)]
_lib.ssg_infer_prepared_bytes.restype = c_size_t
_lib.ssg_infer_workspace_bytes.argtypes = [POINTER(ssg_mlp_desc)]
_lib.ssg_infer_workspace_bytes.restype = c_size_t
_lib.ssg_infer_prepare.argtypes = [POINTER(ssg_mlp_desc)] + [c_void_p] * 6 + [c_size_t, c_void_p]
_lib.ssg_infer_fwd.argtypes = [POINTER(ssg_mlp_desc), c_void_p, c_void_p, c_size_t, c_void_p, c_void_p, c_size_t, c_void_p]
_lib.ssg_infer_noalloc_max_bytes.argtypes = []
_lib.ssg_infer_noalloc_max_bytes.restype = c_size_t
_lib.ssg_infer_fwd_noalloc.argtypes = [POINTER(ssg_mlp_desc), c_void_p, c_void_p, c_size_t, c_void_p, c_void_p]
_lib.ssg_infer_view.argtypes = [POINTER(ssg_mlp_desc), c_void_p, c_void_p, POINTER(ssg_infer_view_t)]
_lib.ssg_adam_state_bytes.argtypes = [c_int64]
_lib.ssg_adam_state_bytes.restype = c_size_t
_lib.ssg_adam_init.argtypes = [c_int64, c_void_p, c_void_p]
_lib.ssg_adam_step.argtypes = [POINTER(ssg_adam_desc), c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
_lib.ssg_adam_view_state.argtypes = [c_int64, c_int32, c_void_p, POINTER(ssg_adam_state_view)]
for _n in EXPORTS[2:]:
    if not _n.endswith("_bytes"):          # the size queries return size_t, everything else a status
        getattr(_lib, _n).restype = c_int


class SsgError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ssg status {status}: {message}")
        self.status = status


def ssg_last_error() -> str:
    return _lib.ssg_last_error().decode()


def ssg_version() -> str:
    return _lib.ssg_version().decode()


def _check(status: int) -> None:
    if status != SSG_OK:
        raise SsgError(status, ssg_last_error())


def _ptr(t):
    """Device pointer of a tensor (None -> NULL); ints pass through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _nbytes(t, given=None) -> int:
    """Size in bytes of a caller-allocated buffer: as given, else that of the tensor backing it."""
    if given is not None:
        return int(given)
    if t is None or isinstance(t, int):
        return 0
    return t.numel() * t.element_size()


def make_desc(T: int, d: int, f: int, smooth: int = 1, rnd: int = SSG_ROUND_EXACT_DIV,
              y_dtype: int = SSG_BF16, dw_dtype: int = SSG_F32, weights_cached: int = 0,
              scale_mode: int = SSG_SCALE_CURRENT, scaling_state=None, h_scale=None, h_counters=None,
              keep_bf16_grads: int = 0, w3_layer_bf16: int = 0) -> ssg_mlp_desc:
    """`scaling_state`: a device byte tensor of ssg_mlp_scaling_state_bytes() bytes; `h_scale`: a device float
    (plain block, given scale of h); `h_counters`: two device int64 words.  All kept alive by the caller."""
    return ssg_mlp_desc(T, d, f, smooth, rnd, y_dtype, dw_dtype, weights_cached, scale_mode,
                        SSG_SCALE_GIVEN if h_scale is not None else SSG_SCALE_CURRENT, keep_bf16_grads, w3_layer_bf16,
                        (c_int32 * 3)(0, 0, 0),
                        _ptr(scaling_state), _ptr(h_scale), _ptr(h_counters))


def ssg_amax(src, src_dtype, n, amax_dev, stream=None):
    _check(_lib.ssg_amax(_ptr(src), src_dtype, n, _ptr(amax_dev), _stream(stream)))


def ssg_quantize(src, src_dtype, rows, cols, fmt, mode, rnd, dst, dst_t, scale_dev, amax_dev, stream=None):
    _check(_lib.ssg_quantize(_ptr(src), src_dtype, rows, cols, fmt, mode, rnd, _ptr(dst), _ptr(dst_t),
                             _ptr(scale_dev), _ptr(amax_dev), _stream(stream)))


def ssg_gemm_fp8(A, a_fmt, B, b_fmt, M, N, K, sa_dev, sb_dev, C, c_dtype, stream=None):
    _check(_lib.ssg_gemm_fp8(_ptr(A), a_fmt, _ptr(B), b_fmt, M, N, K, _ptr(sa_dev), _ptr(sb_dev), _ptr(C),
                             c_dtype, _stream(stream)))


def ssg_gemm_fp8_layout(A, a_fmt, a_kmajor, B, b_fmt, b_kmajor, M, N, K, sa_dev, sb_dev, C, c_dtype, stream=None):
    _check(_lib.ssg_gemm_fp8_layout(_ptr(A), a_fmt, a_kmajor, _ptr(B), b_fmt, b_kmajor, M, N, K, _ptr(sa_dev),
                                    _ptr(sb_dev), _ptr(C), c_dtype, _stream(stream)))


def ssg_swiglu(U, G, T, f, h, stream=None):
    _check(_lib.ssg_swiglu(_ptr(U), _ptr(G), T, f, _ptr(h), _stream(stream)))


def ssg_smooth_swiglu_quantize(U, G, T, f, smooth, h_q, h_qT, s, sinv, camax, stream=None):
    _check(_lib.ssg_smooth_swiglu_quantize(_ptr(U), _ptr(G), T, f, smooth, _ptr(h_q), _ptr(h_qT), _ptr(s),
                                           _ptr(sinv), _ptr(camax), _stream(stream)))


def ssg_fold_w3(W3, sinv, d, f, w3_q, w3_qT, w3_camax, scale_dev, amax_dev, stream=None):
    _check(_lib.ssg_fold_w3(_ptr(W3), _ptr(sinv), d, f, _ptr(w3_q), _ptr(w3_qT), _ptr(w3_camax),
                            _ptr(scale_dev), _ptr(amax_dev), _stream(stream)))


def ssg_mlp_saved_bytes(desc: ssg_mlp_desc) -> int:
    return _lib.ssg_mlp_saved_bytes(ctypes.byref(desc))


def ssg_mlp_workspace_bytes(desc: ssg_mlp_desc) -> int:
    return _lib.ssg_mlp_workspace_bytes(ctypes.byref(desc))


def ssg_mlp_fwd(desc, x, W1, W2, W3, y, saved, stream=None, saved_bytes=None):
    """`saved` (and `workspace`, `prepared` below) are device tensors whose size in bytes is passed along; give
    the *_bytes argument to state a size explicitly (needed when the buffer is a raw pointer)."""
    _check(_lib.ssg_mlp_fwd(ctypes.byref(desc), _ptr(x), _ptr(W1), _ptr(W2), _ptr(W3), _ptr(y), _ptr(saved),
                            _nbytes(saved, saved_bytes), _stream(stream)))


def ssg_mlp_bwd(desc, dy, saved, dx, dW1, dW2, dW3, workspace, stream=None, saved_bytes=None, workspace_bytes=None):
    _check(_lib.ssg_mlp_bwd(ctypes.byref(desc), _ptr(dy), _ptr(saved), _nbytes(saved, saved_bytes), _ptr(dx), _ptr(dW1),
                            _ptr(dW2), _ptr(dW3), _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream)))


def ssg_mlp_bwd_plan(desc, compute_units: int):
    """(sets of dW3 run in the first grouped launch, sets of dW3 in all)"""
    first, total = ctypes.c_int32(), ctypes.c_int32()
    _check(_lib.ssg_mlp_bwd_plan(ctypes.byref(desc), int(compute_units), ctypes.byref(first), ctypes.byref(total)))
    return first.value, total.value


def ssg_mlp_view_saved(desc, saved) -> ssg_mlp_saved_view:
    v = ssg_mlp_saved_view()
    _check(_lib.ssg_mlp_view_saved(ctypes.byref(desc), _ptr(saved), ctypes.byref(v)))
    return v


def ssg_mlp_view_workspace(desc, workspace) -> ssg_mlp_workspace_view:
    v = ssg_mlp_workspace_view()
    _check(_lib.ssg_mlp_view_workspace(ctypes.byref(desc), _ptr(workspace), ctypes.byref(v)))
    return v


def ssg_mlp_scaling_state_bytes() -> int:
    return int(_lib.ssg_mlp_scaling_state_bytes())


def ssg_mlp_scaling_init(state, stream=None) -> None:
    _check(_lib.ssg_mlp_scaling_init(_ptr(state), _stream(stream)))


def ssg_profile_enable(max_records: int) -> None:
    _check(_lib.ssg_profile_enable(max_records))


def ssg_profile_select(tag: int) -> None:
    _check(_lib.ssg_profile_select(tag))


def ssg_profile_read(cap: int, with_bytes: bool = False):
    """Returns (durations_ms, tags) of the launches recorded since the last read; with_bytes = True adds the
    algorithmic bytes of each launch (0 for GEMMs) as a third list."""
    ms = (c_float * cap)()
    tags = (c_int * cap)()
    nbytes = (ctypes.c_double * cap)()
    n = _lib.ssg_profile_read(ms, tags, nbytes, cap)
    if n < 0:
        raise SsgError(n, ssg_last_error())
    if with_bytes:
        return list(ms[:n]), list(tags[:n]), list(nbytes[:n])
    return list(ms[:n]), list(tags[:n])


def ssg_infer_prepared_bytes(desc) -> int:
    return int(_lib.ssg_infer_prepared_bytes(ctypes.byref(desc)))


def ssg_infer_workspace_bytes(desc) -> int:
    return int(_lib.ssg_infer_workspace_bytes(ctypes.byref(desc)))


def ssg_infer_prepare(desc, W1, W2, W3, s, sinv, prepared, stream=None, prepared_bytes=None) -> None:
    _check(_lib.ssg_infer_prepare(ctypes.byref(desc), _ptr(W1), _ptr(W2), _ptr(W3), _ptr(s), _ptr(sinv),
                                  _ptr(prepared), _nbytes(prepared, prepared_bytes), _stream(stream)))


def ssg_infer_fwd(desc, x, prepared, y, workspace, stream=None, prepared_bytes=None, workspace_bytes=None) -> None:
    _check(_lib.ssg_infer_fwd(ctypes.byref(desc), _ptr(x), _ptr(prepared), _nbytes(prepared, prepared_bytes), _ptr(y),
                              _ptr(workspace), _nbytes(workspace, workspace_bytes), _stream(stream)))


def ssg_infer_noalloc_max_bytes() -> int:
    return int(_lib.ssg_infer_noalloc_max_bytes())


def ssg_infer_fwd_noalloc(desc, x, prepared, y, stream=None, prepared_bytes=None) -> None:
    _check(_lib.ssg_infer_fwd_noalloc(ctypes.byref(desc), _ptr(x), _ptr(prepared), _nbytes(prepared, prepared_bytes),
                                      _ptr(y), _stream(stream)))


def ssg_infer_view(desc, prepared, workspace) -> ssg_infer_view_t:
    v = ssg_infer_view_t()
    _check(_lib.ssg_infer_view(ctypes.byref(desc), _ptr(prepared), _ptr(workspace), ctypes.byref(v)))
    return v


def make_adam_desc(n, step, lr, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, grad_dtype=SSG_F32,
                   rnd=SSG_ROUND_EXACT_DIV) -> ssg_adam_desc:
    d = ssg_adam_desc()
    d.n, d.step, d.lr, d.beta1, d.beta2, d.eps, d.weight_decay = n, step, lr, beta1, beta2, eps, weight_decay
    d.grad_dtype, d.rnd = grad_dtype, rnd
    return d


def ssg_adam_state_bytes(n: int) -> int:
    return int(_lib.ssg_adam_state_bytes(n))


def ssg_adam_init(n: int, state, stream=None) -> None:
    _check(_lib.ssg_adam_init(n, _ptr(state), _stream(stream)))


def ssg_adam_step(desc, grad, w, w_bf16, state, stream=None) -> None:
    _check(_lib.ssg_adam_step(ctypes.byref(desc), _ptr(grad), _ptr(w), _ptr(w_bf16), _ptr(state), _stream(stream)))


def ssg_adam_view_state(n: int, step: int, state) -> ssg_adam_state_view:
    v = ssg_adam_state_view()
    _check(_lib.ssg_adam_view_state(n, step, _ptr(state), ctypes.byref(v)))
    return v


def view_tensor(saved, base_ptr: int, field_ptr: int, shape, dtype):
    """A tensor aliasing a region of a caller-owned byte buffer (`saved` or
    `workspace`), located by the pointer a view struct returned."""
    import torch
    off = field_ptr - base_ptr
    n = 1
    for s in shape:
        n *= s
    nbytes = n * torch.empty((), dtype=dtype).element_size()
    return saved[off:off + nbytes].view(dtype).view(*shape)
