"""ctypes binding of libagg.so: same names as the C ABI in ``include/agg.h``.

Argument marshalling only -- every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory (``tensor.data_ptr()``) and the HIP
stream.  A missing library is an error: there is no fallback implementation.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# AGG_LIBRARY_PATH points at another build of the same library (kernel development)
LIB_PATH = os.environ.get("AGG_LIBRARY_PATH") or os.path.join(_HERE, "libagg.so")

AGG_DIAG = 1
AGG_MEAN = 2
AGG_OK = 0
AGG_ERR_NULL, AGG_ERR_SHAPE, AGG_ERR_UNSUPPORTED, AGG_ERR_ALIGN = -1, -2, -3, -4
AGG_ERR_WORKSPACE, AGG_ERR_OVERFLOW, AGG_ERR_LAUNCH = -5, -6, -7


class AggError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


class agg_shape(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("N", ctypes.c_int32),
        ("n_h", ctypes.c_int32), ("n_w", ctypes.c_int32),
        ("n_special", ctypes.c_int32),
        ("H", ctypes.c_int32), ("D", ctypes.c_int32),
        ("s_h", ctypes.c_int32), ("s_w", ctypes.c_int32),
        ("keep_first_frame", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
        ("scale", ctypes.c_float),
        ("mean_logit_bias", ctypes.c_float),
    ]

    @property
    def L(self) -> int:
        return self.n_special + self.n_h * self.n_w

    @property
    def NQ(self) -> int:
        return self.N * self.L


def make_shape(B, N, n_h, n_w, n_special, H, D, s_h, s_w, keep_first_frame=1,
               flags=AGG_DIAG | AGG_MEAN, scale=None, mean_logit_bias=0.0) -> agg_shape:
    if scale is None:
        scale = 1.0 / (D ** 0.5)
    return agg_shape(B, N, n_h, n_w, n_special, H, D, s_h, s_w, keep_first_frame, flags, scale,
                     mean_logit_bias)


_lib = None

EXPORTS = [
    "agg_status_string", "agg_sigma_to_strides", "agg_kv_count", "agg_kv_indices_host",
    "agg_dropped_indices_host", "agg_kv_compact_bytes", "agg_kc_offset", "agg_vc_offset", "agg_workspace_bytes",
    "agg_kv_subsample", "agg_global_attn_fwd", "agg_global_attn_fwd_idx",
    "agg_dense_global_attn_fwd", "agg_frame_attn_fwd",
    "agg_block_workspace_bytes", "agg_global_block_fwd",
    "agg_select_kv_indices", "agg_list_compact_bytes", "agg_list_workspace_bytes",
    "agg_kv_subsample_list", "agg_global_attn_fwd_list", "agg_kv_pool",
    "agg_static_scratch_bytes", "agg_kv_subsample_static",
]

AGG_SELECT_FIRST = 0
AGG_SELECT_RANDOM = 1
AGG_SELECT_HIGH = 2
AGG_SELECT_LOW = 3

AGG_BLOCK_SGA = 0
AGG_BLOCK_FRAME = 1
AGG_BLOCK_DENSE = 2


class agg_block_weights(ctypes.Structure):
    _fields_ = [
        ("ln_gamma", ctypes.c_void_p), ("ln_beta", ctypes.c_void_p), ("ln_eps", ctypes.c_float),
        ("w_q", ctypes.c_void_p), ("w_k", ctypes.c_void_p), ("w_v", ctypes.c_void_p),
        ("w_o", ctypes.c_void_p),
        ("b_q", ctypes.c_void_p), ("b_k", ctypes.c_void_p), ("b_v", ctypes.c_void_p),
        ("b_o", ctypes.c_void_p),
    ]


def make_block_weights(ln_gamma, ln_beta, ln_eps, w_q, w_k, w_v, w_o, b_q=None, b_k=None,
                       b_v=None, b_o=None) -> agg_block_weights:
    """Packs device tensors (kept alive by the caller) into the C struct."""
    def p(t):
        return None if t is None else t.data_ptr()
    return agg_block_weights(p(ln_gamma), p(ln_beta), float(ln_eps), p(w_q), p(w_k), p(w_v),
                             p(w_o), p(b_q), p(b_k), p(b_v), p(b_o))


def lib():
    """Opens libagg.so on first use; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "libagg.so is missing at %s -- build it with `python -m paper_2512_02541_amd.build`; "
            "there is no fallback path" % LIB_PATH)
    # PyTorch owns the device memory and streams handed to the library, so the library must
    # bind to the HIP runtime PyTorch ships: load torch (and with it that runtime) first.
    import torch  # noqa: F401

    L = ctypes.CDLL(LIB_PATH)
    vp, i32p, i64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
    shp = ctypes.POINTER(agg_shape)
    L.agg_status_string.restype = ctypes.c_char_p
    L.agg_status_string.argtypes = [ctypes.c_int]
    L.agg_sigma_to_strides.argtypes = [ctypes.c_int, i32p, i32p]
    L.agg_kv_count.argtypes = [shp, i64p, i64p]
    L.agg_kv_indices_host.argtypes = [shp, vp]
    L.agg_dropped_indices_host.argtypes = [shp, vp]
    L.agg_kv_compact_bytes.argtypes = [shp, ctypes.POINTER(ctypes.c_size_t), i64p]
    L.agg_kc_offset.restype = ctypes.c_int64
    L.agg_kc_offset.argtypes = [ctypes.c_int64, ctypes.c_int32]
    L.agg_vc_offset.restype = ctypes.c_int64
    L.agg_vc_offset.argtypes = [ctypes.c_int64, ctypes.c_int32]
    L.agg_workspace_bytes.restype = ctypes.c_size_t
    L.agg_workspace_bytes.argtypes = [shp]
    L.agg_kv_subsample.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.agg_global_attn_fwd.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.agg_global_attn_fwd_idx.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.agg_dense_global_attn_fwd.argtypes = [shp, vp, vp, vp, vp, vp, vp]
    L.agg_frame_attn_fwd.argtypes = [shp, vp, vp, vp, vp, vp, vp]
    L.agg_block_workspace_bytes.restype = ctypes.c_size_t
    L.agg_block_workspace_bytes.argtypes = [shp, ctypes.c_int]
    L.agg_global_block_fwd.argtypes = [shp, ctypes.c_int, ctypes.POINTER(agg_block_weights), vp, vp,
                                       vp, ctypes.c_size_t, vp]
    L.agg_select_kv_indices.argtypes = [shp, ctypes.c_int, ctypes.c_uint64, vp, vp, vp]
    L.agg_list_compact_bytes.argtypes = [shp, ctypes.c_int64, ctypes.POINTER(ctypes.c_size_t), i64p]
    L.agg_list_workspace_bytes.restype = ctypes.c_size_t
    L.agg_list_workspace_bytes.argtypes = [shp]
    L.agg_kv_subsample_list.argtypes = [shp, vp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                        ctypes.c_size_t, vp]
    L.agg_global_attn_fwd_list.argtypes = [shp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                           vp, vp, vp]
    L.agg_kv_pool.argtypes = [shp, vp, vp, vp, vp, vp]
    L.agg_static_scratch_bytes.restype = ctypes.c_size_t
    L.agg_static_scratch_bytes.argtypes = []
    L.agg_kv_subsample_static.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp]
    _lib = L
    return L


def _check(status: int, where: str):
    if status != AGG_OK:
        raise AggError(status, where)


def _ptr(t):
    """Device (or host) address of a torch tensor / numpy array / raw int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    if hasattr(t, "data_ptr"):
        return ctypes.c_void_p(t.data_ptr())
    return ctypes.c_void_p(t.ctypes.data)


def _stream(stream):
    if stream is None:
        import torch

        stream = torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(int(stream))


def status_string(status: int) -> str:
    return lib().agg_status_string(int(status)).decode()


def agg_sigma_to_strides(sigma: int):
    sh, sw = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(lib().agg_sigma_to_strides(int(sigma), ctypes.byref(sh), ctypes.byref(sw)),
           "agg_sigma_to_strides")
    return sh.value, sw.value


def agg_kv_count(shape: agg_shape):
    m, nd = ctypes.c_int64(0), ctypes.c_int64(0)
    _check(lib().agg_kv_count(ctypes.byref(shape), ctypes.byref(m), ctypes.byref(nd)),
           "agg_kv_count")
    return m.value, nd.value


def agg_kv_indices_host(shape: agg_shape):
    import numpy as np

    m, _ = agg_kv_count(shape)
    idx = np.empty(m, dtype=np.int32)
    _check(lib().agg_kv_indices_host(ctypes.byref(shape), _ptr(idx)), "agg_kv_indices_host")
    return idx


def agg_dropped_indices_host(shape: agg_shape):
    import numpy as np

    _, nd = agg_kv_count(shape)
    idx = np.empty(nd, dtype=np.int32)
    _check(lib().agg_dropped_indices_host(ctypes.byref(shape), _ptr(idx)),
           "agg_dropped_indices_host")
    return idx


def agg_kv_compact_bytes(shape: agg_shape):
    nbytes, m_pad = ctypes.c_size_t(0), ctypes.c_int64(0)
    _check(lib().agg_kv_compact_bytes(ctypes.byref(shape), ctypes.byref(nbytes),
                                      ctypes.byref(m_pad)), "agg_kv_compact_bytes")
    return nbytes.value, m_pad.value


def agg_kc_offset(m: int, d: int) -> int:
    return int(lib().agg_kc_offset(int(m), int(d)))


def agg_vc_offset(m: int, d: int) -> int:
    return int(lib().agg_vc_offset(int(m), int(d)))


def agg_workspace_bytes(shape: agg_shape) -> int:
    return int(lib().agg_workspace_bytes(ctypes.byref(shape)))


def agg_kv_subsample(shape, K, V, Kc, Vc, idx, kmean, vmean, workspace, workspace_bytes,
                     stream=None):
    _check(lib().agg_kv_subsample(ctypes.byref(shape), _ptr(K), _ptr(V), _ptr(Kc), _ptr(Vc),
                                  _ptr(idx), _ptr(kmean), _ptr(vmean), _ptr(workspace),
                                  int(workspace_bytes), _stream(stream)), "agg_kv_subsample")


def agg_static_scratch_bytes() -> int:
    return int(lib().agg_static_scratch_bytes())


def agg_kv_subsample_static(shape, K, V, Kc, Vc, idx, kmean, vmean, stream=None):
    _check(lib().agg_kv_subsample_static(ctypes.byref(shape), _ptr(K), _ptr(V), _ptr(Kc), _ptr(Vc),
                                         _ptr(idx), _ptr(kmean), _ptr(vmean), _stream(stream)),
           "agg_kv_subsample_static")


def agg_global_attn_fwd(shape, Q, K, V, Kc, Vc, kmean, vmean, O, lse=None, stream=None):
    _check(lib().agg_global_attn_fwd(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(Kc),
                                     _ptr(Vc), _ptr(kmean), _ptr(vmean), _ptr(O), _ptr(lse),
                                     _stream(stream)), "agg_global_attn_fwd")


def agg_global_attn_fwd_idx(shape, Q, K, V, idx, kmean, vmean, O, lse=None, stream=None):
    _check(lib().agg_global_attn_fwd_idx(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(idx),
                                         _ptr(kmean), _ptr(vmean), _ptr(O), _ptr(lse),
                                         _stream(stream)), "agg_global_attn_fwd_idx")


def agg_dense_global_attn_fwd(shape, Q, K, V, O, lse=None, stream=None):
    _check(lib().agg_dense_global_attn_fwd(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(O),
                                           _ptr(lse), _stream(stream)), "agg_dense_global_attn_fwd")


def agg_frame_attn_fwd(shape, Q, K, V, O, lse=None, stream=None):
    _check(lib().agg_frame_attn_fwd(ctypes.byref(shape), _ptr(Q), _ptr(K), _ptr(V), _ptr(O),
                                    _ptr(lse), _stream(stream)), "agg_frame_attn_fwd")


def agg_block_workspace_bytes(shape: agg_shape, mode: int) -> int:
    return int(lib().agg_block_workspace_bytes(ctypes.byref(shape), int(mode)))


def agg_global_block_fwd(shape, mode, weights, x, y, workspace, workspace_bytes, stream=None):
    _check(lib().agg_global_block_fwd(ctypes.byref(shape), int(mode), ctypes.byref(weights),
                                      _ptr(x), _ptr(y), _ptr(workspace), int(workspace_bytes),
                                      _stream(stream)), "agg_global_block_fwd")


def agg_select_kv_indices(shape, rule, seed, K, list_out, stream=None):
    _check(lib().agg_select_kv_indices(ctypes.byref(shape), int(rule), int(seed), _ptr(K),
                                       _ptr(list_out), _stream(stream)), "agg_select_kv_indices")


def agg_list_compact_bytes(shape: agg_shape, M_list: int):
    nbytes, m_pad = ctypes.c_size_t(0), ctypes.c_int64(0)
    _check(lib().agg_list_compact_bytes(ctypes.byref(shape), int(M_list), ctypes.byref(nbytes),
                                        ctypes.byref(m_pad)), "agg_list_compact_bytes")
    return nbytes.value, m_pad.value


def agg_list_workspace_bytes(shape: agg_shape) -> int:
    return int(lib().agg_list_workspace_bytes(ctypes.byref(shape)))


def agg_kv_subsample_list(shape, list_in, M_list, K, V, Kc, Vc, kmean, vmean, kept_bits, n_dropped,
                          workspace, workspace_bytes, stream=None):
    _check(lib().agg_kv_subsample_list(ctypes.byref(shape), _ptr(list_in), int(M_list), _ptr(K),
                                       _ptr(V), _ptr(Kc), _ptr(Vc), _ptr(kmean), _ptr(vmean),
                                       _ptr(kept_bits), _ptr(n_dropped), _ptr(workspace),
                                       int(workspace_bytes), _stream(stream)),
           "agg_kv_subsample_list")


def agg_global_attn_fwd_list(shape, M_list, Q, K, V, Kc, Vc, kmean, vmean, kept_bits, n_dropped, O,
                             lse=None, stream=None):
    _check(lib().agg_global_attn_fwd_list(ctypes.byref(shape), int(M_list), _ptr(Q), _ptr(K),
                                          _ptr(V), _ptr(Kc), _ptr(Vc), _ptr(kmean), _ptr(vmean),
                                          _ptr(kept_bits), _ptr(n_dropped), _ptr(O), _ptr(lse),
                                          _stream(stream)), "agg_global_attn_fwd_list")


def agg_kv_pool(shape, K, V, Kc, Vc, stream=None):
    _check(lib().agg_kv_pool(ctypes.byref(shape), _ptr(K), _ptr(V), _ptr(Kc), _ptr(Vc),
                             _stream(stream)), "agg_kv_pool")
