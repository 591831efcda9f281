"""ctypes binding of include/svg.h: same names, argument marshalling only.

Device tensors are torch tensors (used for memory and streams only); every step of
the path runs inside the library's kernels.  There is no fallback: if the shared
object is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch  # noqa: F401  -- must come first: the library binds to the HIP runtime torch has loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
# SVG_LIBRARY_PATH selects another build of the same library (e.g. to time two builds side by side)
LIB_PATH = os.environ.get("SVG_LIBRARY_PATH") or os.path.join(_HERE, "libsvg_gfx950.so")

SVG_HEAD_SPATIAL = 0
SVG_HEAD_TEMPORAL = 1
SVG_LIST_TEMPORAL_FRAME_MAJOR = 2   # list pattern only: temporal mask without the layout transformation
SVG_NORM_NONE, SVG_NORM_RMS, SVG_NORM_LAYER = 0, 1, 2           # svg_qk_norm_rope
SVG_ROPE_INTERLEAVED, SVG_ROPE_HALF = 0, 1
SVG_FP8_Q, SVG_FP8_K, SVG_FP8_VT, SVG_FP8_SCALES = 0, 1, 2, 3   # svg_fp8_buffer_bytes
SVG_ATTN_QO_TOKEN_ORDER = 1          # svg_sparse_attn_fwd_ex: q read and o written in token order
SVG_ATTN_ELEMENT_MASK = 2            # svg_sparse_attn_fwd_ex: the pattern's element mask inside every visited tile
SVG_ATTN_KV_TOKEN_ORDER = 4          # svg_sparse_attn_fwd_ex: k, v of temporal heads stay in token order (gathered in the kernel)
SVG_OK = 0

EXPORTS = ("svg_strerror", "svg_version", "svg_last_hip_error", "svg_workspace_bytes", "svg_profile_plan", "svg_tile_counts",
           "svg_tile_list_build", "svg_profile_heads", "svg_profile_heads_static", "svg_layout_fwd", "svg_layout_inv",
           "svg_sparse_attn_fwd", "svg_sparse_attn_fwd_ex", "svg_dense_attn_fwd",
           "svg_layout_kv_temporal", "svg_sparse_attn_fwd_kv2",
           "svg_fp8_buffer_bytes", "svg_fp8_quantize", "svg_sparse_attn_fp8_fwd", "svg_qk_norm_rope",
           "svg_probe_mfma_bf16", "svg_probe_lds")


class SvgShape(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("F", C.c_int32), ("P", C.c_int32),
                ("T", C.c_int32), ("D", C.c_int32), ("text_first", C.c_int32),
                ("w_s", C.c_int32), ("w_t", C.c_int32), ("sink_first_frame", C.c_int32),
                ("block_m", C.c_int32), ("block_n", C.c_int32), ("softmax_scale", C.c_float)]

    @property
    def N(self):
        return self.F * self.P + self.T


class SvgError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        detail = f": {lib().svg_last_hip_error().decode()}" if status == -5 else ""
        super().__init__(f"{where}: {svg_strerror(status)} ({status}){detail}")


_lib = None


def lib():
    """The loaded shared object.  Raises FileNotFoundError if it was never built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2502_01776_amd.build` "
                "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        sp = C.POINTER(SvgShape)
        vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
        L.svg_strerror.restype = C.c_char_p
        L.svg_strerror.argtypes = [C.c_int]
        L.svg_version.restype = C.c_char_p
        L.svg_version.argtypes = []
        L.svg_last_hip_error.restype = C.c_char_p
        L.svg_last_hip_error.argtypes = []
        L.svg_workspace_bytes.restype = C.c_size_t
        L.svg_workspace_bytes.argtypes = [sp, C.c_int32]
        L.svg_profile_plan.restype = C.c_int
        L.svg_profile_plan.argtypes = [sp, C.c_int32, i32p, i32p, i32p]
        L.svg_tile_counts.restype = C.c_int
        L.svg_tile_counts.argtypes = [sp, i32p, i32p]
        L.svg_tile_list_build.restype = C.c_int
        L.svg_tile_list_build.argtypes = [sp, C.c_int, vp, vp, C.c_int64, C.POINTER(C.c_int64)]
        L.svg_profile_heads.restype = C.c_int
        L.svg_profile_heads.argtypes = [sp, vp, vp, vp, vp, C.c_int32, vp, vp, vp, C.c_size_t, vp]
        L.svg_profile_heads_static.restype = C.c_int
        L.svg_profile_heads_static.argtypes = [sp, vp, vp, vp, vp, C.c_int32, vp, vp, vp]
        for name in ("svg_layout_fwd", "svg_layout_inv"):
            f = getattr(L, name)
            f.restype = C.c_int
            f.argtypes = [sp, vp, vp, vp, vp]
        L.svg_sparse_attn_fwd.restype = C.c_int
        L.svg_sparse_attn_fwd.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.svg_sparse_attn_fwd_ex.restype = C.c_int
        L.svg_sparse_attn_fwd_ex.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_uint32, vp, C.c_size_t, vp]
        L.svg_layout_kv_temporal.restype = C.c_int
        L.svg_layout_kv_temporal.argtypes = [sp, vp, vp, vp, vp, vp, vp]
        L.svg_sparse_attn_fwd_kv2.restype = C.c_int
        L.svg_sparse_attn_fwd_kv2.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_uint32, vp]
        L.svg_qk_norm_rope.restype = C.c_int
        L.svg_qk_norm_rope.argtypes = [sp, vp, vp, C.c_int, vp, vp, C.c_float, vp, vp, C.c_int, vp]
        L.svg_fp8_buffer_bytes.restype = C.c_size_t
        L.svg_fp8_buffer_bytes.argtypes = [sp, C.c_int]
        L.svg_fp8_quantize.restype = C.c_int
        L.svg_fp8_quantize.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.svg_sparse_attn_fp8_fwd.restype = C.c_int
        L.svg_sparse_attn_fp8_fwd.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.svg_probe_mfma_bf16.restype = C.c_int
        L.svg_probe_mfma_bf16.argtypes = [C.c_int, C.c_int32, C.c_int32, vp, vp, C.POINTER(C.c_double), vp]
        L.svg_probe_lds.restype = C.c_int
        L.svg_probe_lds.argtypes = [C.c_int, C.c_int32, C.c_int32, vp, C.c_size_t, vp]
        L.svg_dense_attn_fwd.restype = C.c_int
        L.svg_dense_attn_fwd.argtypes = [sp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        _lib = L
    return _lib


def shape_from_config(cfg: dict, **overrides) -> SvgShape:
    keys = ("B", "H", "F", "P", "T", "D", "text_first", "w_s", "w_t", "sink_first_frame",
            "block_m", "block_n")
    vals = {k: int(cfg[k]) for k in keys}
    vals.update(overrides)
    return SvgShape(softmax_scale=float(cfg.get("softmax_scale", 0.0)), **vals)


def _check(status, where):
    if status != SVG_OK:
        raise SvgError(status, where)


def _ptr(x):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def svg_strerror(status: int) -> str:
    return lib().svg_strerror(int(status)).decode()


def svg_version() -> str:
    return lib().svg_version().decode()


def svg_workspace_bytes(shape: SvgShape, t: int) -> int:
    return int(lib().svg_workspace_bytes(C.byref(shape), int(t)))


def svg_profile_plan(shape: SvgShape, t: int):
    """Returns (n_full, n_masked, full_bound[0 .. n_full])."""
    nf, nm = C.c_int32(), C.c_int32()
    bound = (C.c_int32 * 17)()
    _check(lib().svg_profile_plan(C.byref(shape), int(t), C.byref(nf), C.byref(nm), bound), "svg_profile_plan")
    return nf.value, nm.value, list(bound)[:nf.value + 1]


def svg_tile_counts(shape: SvgShape):
    nq, nk = C.c_int32(), C.c_int32()
    _check(lib().svg_tile_counts(C.byref(shape), C.byref(nq), C.byref(nk)), "svg_tile_counts")
    return nq.value, nk.value


def svg_tile_list_build(shape: SvgShape, pattern: int):
    """Host CSR (row_ptr int32[nq+1], col_idx int32[nnz]) as numpy arrays."""
    nq, _ = svg_tile_counts(shape)
    row_ptr = np.zeros(nq + 1, dtype=np.int32)
    nnz = C.c_int64()
    _check(lib().svg_tile_list_build(C.byref(shape), int(pattern), row_ptr.ctypes.data, None, 0,
                                     C.byref(nnz)), "svg_tile_list_build")
    col_idx = np.zeros(max(nnz.value, 1), dtype=np.int32)
    _check(lib().svg_tile_list_build(C.byref(shape), int(pattern), row_ptr.ctypes.data,
                                     col_idx.ctypes.data, nnz.value, C.byref(nnz)),
           "svg_tile_list_build")
    return row_ptr, col_idx[:nnz.value]


def svg_profile_heads(shape, q, k, v, rows, t, labels, mse, workspace, workspace_bytes, stream=None):
    _check(lib().svg_profile_heads(C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(rows), int(t),
                                   _ptr(labels), _ptr(mse), _ptr(workspace), int(workspace_bytes),
                                   _stream(stream)), "svg_profile_heads")


SVG_STATIC_SCRATCH_BYTES = 160 << 20


def svg_profile_heads_static(shape, q, k, v, rows, t, labels, mse, stream=None):
    _check(lib().svg_profile_heads_static(C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(rows), int(t),
                                          _ptr(labels), _ptr(mse), _stream(stream)), "svg_profile_heads_static")


def svg_layout_fwd(shape, x, out, labels=None, stream=None):
    _check(lib().svg_layout_fwd(C.byref(shape), _ptr(x), _ptr(out), _ptr(labels), _stream(stream)),
           "svg_layout_fwd")


def svg_layout_inv(shape, x, out, labels=None, stream=None):
    _check(lib().svg_layout_inv(C.byref(shape), _ptr(x), _ptr(out), _ptr(labels), _stream(stream)),
           "svg_layout_inv")


def svg_sparse_attn_fwd(shape, q, k, v, o, labels, row_ptr_s, col_idx_s, row_ptr_t, col_idx_t,
                        workspace=None, workspace_bytes=0, stream=None):
    _check(lib().svg_sparse_attn_fwd(C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(labels),
                                     _ptr(row_ptr_s), _ptr(col_idx_s), _ptr(row_ptr_t),
                                     _ptr(col_idx_t), _ptr(workspace), int(workspace_bytes),
                                     _stream(stream)), "svg_sparse_attn_fwd")


def svg_sparse_attn_fwd_ex(shape, q, k, v, o, labels, row_ptr_s, col_idx_s, row_ptr_t, col_idx_t,
                           flags=0, workspace=None, workspace_bytes=0, stream=None):
    _check(lib().svg_sparse_attn_fwd_ex(C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(labels),
                                        _ptr(row_ptr_s), _ptr(col_idx_s), _ptr(row_ptr_t),
                                        _ptr(col_idx_t), int(flags), _ptr(workspace),
                                        int(workspace_bytes), _stream(stream)), "svg_sparse_attn_fwd_ex")


def svg_layout_kv_temporal(shape, k, v, k_t, v_t, labels, stream=None):
    _check(lib().svg_layout_kv_temporal(C.byref(shape), _ptr(k), _ptr(v), _ptr(k_t), _ptr(v_t), _ptr(labels),
                                        _stream(stream)), "svg_layout_kv_temporal")


def svg_sparse_attn_fwd_kv2(shape, q, k, v, k_t, v_t, o, labels, row_ptr_s, col_idx_s, row_ptr_t, col_idx_t,
                            flags=0, stream=None):
    _check(lib().svg_sparse_attn_fwd_kv2(C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(k_t), _ptr(v_t), _ptr(o),
                                         _ptr(labels), _ptr(row_ptr_s), _ptr(col_idx_s), _ptr(row_ptr_t),
                                         _ptr(col_idx_t), int(flags), _stream(stream)), "svg_sparse_attn_fwd_kv2")


def svg_dense_attn_fwd(shape, q, k, v, o, workspace=None, workspace_bytes=0, stream=None):
    _check(lib().svg_dense_attn_fwd(C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(o),
                                    _ptr(workspace), int(workspace_bytes), _stream(stream)),
           "svg_dense_attn_fwd")


def svg_fp8_buffer_bytes(shape, which) -> int:
    return int(lib().svg_fp8_buffer_bytes(C.byref(shape), int(which)))


def svg_fp8_quantize(shape, q, k, v, labels, q8, k8, v8t, scales, stream=None):
    _check(lib().svg_fp8_quantize(C.byref(shape), _ptr(q), _ptr(k), _ptr(v), _ptr(labels), _ptr(q8),
                                  _ptr(k8), _ptr(v8t), _ptr(scales), _stream(stream)), "svg_fp8_quantize")


def svg_sparse_attn_fp8_fwd(shape, q8, k8, v8t, scales, o, labels, row_ptr_s, col_idx_s, row_ptr_t,
                            col_idx_t, stream=None):
    _check(lib().svg_sparse_attn_fp8_fwd(C.byref(shape), _ptr(q8), _ptr(k8), _ptr(v8t), _ptr(scales),
                                         _ptr(o), _ptr(labels), _ptr(row_ptr_s), _ptr(col_idx_s),
                                         _ptr(row_ptr_t), _ptr(col_idx_t), _stream(stream)),
           "svg_sparse_attn_fp8_fwd")


def svg_qk_norm_rope(shape, x, y, norm=SVG_NORM_NONE, weight=None, bias=None, eps=1e-6, cos=None, sin=None,
                     pairing=SVG_ROPE_INTERLEAVED, stream=None):
    _check(lib().svg_qk_norm_rope(C.byref(shape), _ptr(x), _ptr(y), int(norm), _ptr(weight), _ptr(bias),
                                  float(eps), _ptr(cos), _ptr(sin), int(pairing), _stream(stream)),
           "svg_qk_norm_rope")


def svg_probe_mfma_bf16(form, workgroups, iterations, operands, sink, stream=None) -> float:
    """Enqueues the matrix-core rate probe; returns the floating point operations of the launch."""
    flop = C.c_double()
    _check(lib().svg_probe_mfma_bf16(int(form), int(workgroups), int(iterations), _ptr(operands), _ptr(sink),
                                     C.byref(flop), _stream(stream)), "svg_probe_mfma_bf16")
    return flop.value


def svg_probe_lds(form, waves, iterations, scratch, stream=None) -> int:
    """Enqueues the LDS rate probe; returns the bytes one wave instruction of this form moves.  Entry w of
    scratch (viewed as int64) receives the shader clocks wavefront w took."""
    _check(lib().svg_probe_lds(int(form), int(waves), int(iterations), _ptr(scratch),
                               scratch.numel() * scratch.element_size(), _stream(stream)), "svg_probe_lds")
    return 1024 if form in (0, 3) else 512
