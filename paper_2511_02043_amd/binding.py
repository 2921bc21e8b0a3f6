"""ctypes binding of libflattn.so: the same entry points as include/fl_attn.h.

Argument marshalling only.  PyTorch supplies device memory and streams; every step of
the attention path runs in the library's HIP kernels.  There is no fallback: if the
shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FL_ATTN_LIB") or os.path.join(_HERE, "libflattn.so")

# --- enums (include/fl_attn.h) -----------------------------------------------------------
FL_OK, FL_ERR_NULL, FL_ERR_DTYPE, FL_ERR_SHAPE, FL_ERR_STRIDE, FL_ERR_ALIGN = 0, 1, 2, 3, 4, 5
FL_ERR_UNSUPPORTED, FL_ERR_AUX_MISSING, FL_ERR_WORKSPACE, FL_ERR_LAUNCH, FL_ERR_DESC = 6, 7, 8, 9, 10
FL_BF16, FL_F32, FL_I32 = 1, 2, 3
FL_MOD_NONE, FL_MOD_ALIBI, FL_MOD_SOFTCAP = 0, 1, 2
FL_MASK_CAUSAL, FL_MASK_WINDOW, FL_MASK_DOC, FL_MASK_PREFIX = 1, 2, 4, 8
FL_SINGLE, FL_DIFFERENTIAL = 0, 1
FL_EPI_RMSNORM, FL_EPI_GATE_SIGMOID = 1, 2


class fl_tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("dtype", C.c_int32), ("reserved", C.c_int32),
                ("size", C.c_int64 * 5), ("stride", C.c_int64 * 5)]


class fl_variant_desc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("scale", C.c_float), ("score_mod", C.c_uint32),
                ("softcap", C.c_float), ("mask", C.c_uint32), ("window", C.c_int32),
                ("prefix_len", C.c_int32), ("n_bias", C.c_uint32), ("combine", C.c_uint32),
                ("epilogue", C.c_uint32), ("rms_eps", C.c_float), ("q_offset", C.c_int32)]


class fl_aux(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("reserved", C.c_uint32),
                ("alibi_slopes", C.c_void_p), ("q_doc_ids", C.c_void_p), ("kv_doc_ids", C.c_void_p),
                ("bias", fl_tensor * 2), ("gate", fl_tensor), ("q2", fl_tensor), ("k2", fl_tensor),
                ("lambda_", C.c_void_p), ("rms_weight", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


class fl_bwd_extra(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("reserved", C.c_uint32), ("dq2", fl_tensor), ("dk2", fl_tensor),
                ("dbias", fl_tensor * 2), ("dgate", fl_tensor), ("dlambda", C.c_void_p), ("drms_weight", C.c_void_p)]


class fl_paged_kv(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("reserved", C.c_uint32), ("block_table", C.c_void_p),
                ("table_stride", C.c_int32), ("page_size", C.c_int32), ("seq_lens", C.c_void_p),
                ("max_seq_len", C.c_int32), ("reserved2", C.c_int32)]


class FlError(RuntimeError):
    def __init__(self, status: int, text: str, detail: str):
        super().__init__(f"fl_attn status {status} ({text}): {detail}")
        self.status = status
        self.detail = detail


_lib = None


def lib() -> C.CDLL:
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with __graft_entry__.build() "
                "(or make -C paper_2511_02043_amd/csrc); there is no fallback path")
        # PyTorch ships its own HIP runtime; load it first, so that this process has one runtime
        # (the library's launches and torch's allocations must see the same devices and streams)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        TP = C.POINTER(fl_tensor)
        L.fl_attn_fwd.restype = C.c_int
        L.fl_attn_fwd.argtypes = [TP, TP, TP, C.POINTER(fl_variant_desc), C.POINTER(fl_aux), TP, TP,
                                  C.c_void_p]
        L.fl_attn_fwd_noalloc.restype = C.c_int
        L.fl_attn_fwd_noalloc.argtypes = L.fl_attn_fwd.argtypes
        L.fl_attn_fwd_workspace_size.restype = C.c_size_t
        L.fl_attn_fwd_workspace_size.argtypes = [TP, TP, C.POINTER(fl_variant_desc)]
        L.fl_attn_bwd.restype = C.c_int
        L.fl_attn_bwd.argtypes = [TP, TP, TP, TP, TP, TP, C.POINTER(fl_variant_desc), C.POINTER(fl_aux),
                                  TP, TP, TP, C.c_void_p]
        L.fl_attn_bwd_workspace_size.restype = C.c_size_t
        L.fl_attn_bwd_workspace_size.argtypes = [TP, TP, C.POINTER(fl_variant_desc)]
        L.fl_attn_bwd_ex.restype = C.c_int
        L.fl_attn_bwd_ex.argtypes = [TP, TP, TP, TP, TP, TP, C.POINTER(fl_variant_desc), C.POINTER(fl_aux),
                                     TP, TP, TP, C.POINTER(fl_bwd_extra), C.c_void_p]
        L.fl_attn_bwd_ex_workspace_size.restype = C.c_size_t
        L.fl_attn_bwd_ex_workspace_size.argtypes = [TP, TP, TP, C.POINTER(fl_variant_desc)]
        L.fl_bwd_supported.restype = C.c_int
        L.fl_bwd_supported.argtypes = [C.POINTER(fl_variant_desc), C.c_int, C.c_int, C.c_int]
        L.fl_attn_decode.restype = C.c_int
        L.fl_attn_decode.argtypes = [TP, TP, TP, C.POINTER(fl_paged_kv), C.POINTER(fl_variant_desc), C.POINTER(fl_aux),
                                     TP, TP, C.c_void_p]
        L.fl_attn_decode_workspace_size.restype = C.c_size_t
        L.fl_attn_decode_workspace_size.argtypes = [TP, TP, C.POINTER(fl_paged_kv)]
        L.fl_attn_prefill_paged.restype = C.c_int
        L.fl_attn_prefill_paged.argtypes = L.fl_attn_decode.argtypes
        L.fl_attn_prefill_paged_workspace_size.restype = C.c_size_t
        L.fl_attn_prefill_paged_workspace_size.argtypes = [TP, TP, C.POINTER(fl_paged_kv)]
        L.fl_compile_variant.restype = C.c_int
        L.fl_compile_variant.argtypes = [C.c_char_p, C.c_char_p, C.c_uint32, C.c_int, C.POINTER(C.c_void_p)]
        L.fl_attn_fwd_custom.restype = C.c_int
        L.fl_attn_fwd_custom.argtypes = [C.c_void_p, TP, TP, TP, C.c_float, C.c_int32, C.c_int32, TP, TP, C.c_void_p]
        L.fl_compile_variant_aux.restype = C.c_int
        L.fl_compile_variant_aux.argtypes = [C.c_char_p, C.c_char_p, C.c_uint32, C.c_int, C.POINTER(C.c_int32),
                                             C.POINTER(C.c_void_p)]
        L.fl_attn_fwd_custom_aux.restype = C.c_int
        L.fl_attn_fwd_custom_aux.argtypes = [C.c_void_p, TP, TP, TP, C.c_float, C.c_int32, C.c_int32,
                                             C.POINTER(C.c_void_p), TP, TP, C.c_void_p]
        L.fl_attn_fwd_custom_skip.restype = C.c_int
        L.fl_attn_fwd_custom_skip.argtypes = [C.c_void_p, TP, TP, TP, C.c_float, C.c_int32, C.c_int32,
                                              C.POINTER(C.c_void_p), C.c_void_p, C.c_size_t, TP, TP, C.c_void_p]
        L.fl_custom_skip_workspace_size.restype = C.c_size_t
        L.fl_custom_skip_workspace_size.argtypes = [C.c_void_p, TP, TP]
        L.fl_compile_variant_grad.restype = C.c_int
        L.fl_compile_variant_grad.argtypes = [C.c_char_p, C.c_char_p, C.c_char_p, C.c_uint32, C.c_int, C.POINTER(C.c_int32),
                                              C.POINTER(C.c_void_p)]
        L.fl_attn_bwd_custom.restype = C.c_int
        L.fl_attn_bwd_custom.argtypes = [C.c_void_p, TP, TP, TP, TP, TP, TP, C.c_float, C.c_int32, C.c_int32,
                                         C.POINTER(C.c_void_p), C.c_void_p, C.c_size_t, TP, TP, TP, C.c_void_p]
        L.fl_attn_bwd_custom_workspace_size.restype = C.c_size_t
        L.fl_attn_bwd_custom_workspace_size.argtypes = [C.c_void_p, TP, TP]
        L.fl_release_variant.restype = None
        L.fl_release_variant.argtypes = [C.c_void_p]
        L.fl_variant_supported.restype = C.c_int
        L.fl_variant_supported.argtypes = [C.POINTER(fl_variant_desc), C.c_int, C.c_int, C.c_int]
        L.fl_strerror.restype = C.c_char_p
        L.fl_strerror.argtypes = [C.c_int]
        L.fl_last_error_detail.restype = C.c_char_p
        L.fl_last_error_detail.argtypes = []
        L.fl_set_tuning.restype = C.c_int
        L.fl_set_tuning.argtypes = [C.c_char_p, C.c_int]
        L.fl_version.restype = C.c_uint32
        L.fl_version.argtypes = []
        _lib = L
    return _lib


EXPORTS = ["fl_attn_fwd", "fl_attn_fwd_noalloc", "fl_attn_fwd_workspace_size", "fl_attn_bwd", "fl_attn_bwd_workspace_size", "fl_attn_bwd_ex", "fl_attn_bwd_ex_workspace_size",
           "fl_bwd_supported", "fl_attn_decode", "fl_attn_decode_workspace_size", "fl_attn_prefill_paged", "fl_attn_prefill_paged_workspace_size", "fl_compile_variant", "fl_attn_fwd_custom", "fl_compile_variant_aux", "fl_attn_fwd_custom_aux", "fl_attn_fwd_custom_skip", "fl_custom_skip_workspace_size", "fl_compile_variant_grad", "fl_attn_bwd_custom", "fl_attn_bwd_custom_workspace_size",
           "fl_release_variant", "fl_variant_supported", "fl_strerror",
           "fl_last_error_detail", "fl_set_tuning", "fl_version"]


def _dtype_code(t) -> int:
    import torch
    return {torch.bfloat16: FL_BF16, torch.float32: FL_F32, torch.int32: FL_I32}[t.dtype]


def tensor_desc(t, sizes: Optional[Sequence[int]] = None) -> fl_tensor:
    """fl_tensor for a 5-D torch tensor (or None -> a null descriptor)."""
    d = fl_tensor()
    if t is None:
        return d
    if t.dim() != 5:
        raise ValueError(f"expected a 5-D [B,G,H,S,D] view, got {tuple(t.shape)}")
    d.ptr = t.data_ptr()
    d.dtype = _dtype_code(t)
    for a in range(5):
        d.size[a] = t.shape[a] if sizes is None else sizes[a]
        d.stride[a] = t.stride(a)
    return d


def variant_desc(*, scale: float, score_mod: int = FL_MOD_NONE, softcap: float = 0.0, mask: int = 0,
                 window: int = 0, prefix_len: int = 0, n_bias: int = 0, combine: int = FL_SINGLE,
                 epilogue: int = 0, rms_eps: float = 0.0, q_offset: int = 0) -> fl_variant_desc:
    d = fl_variant_desc()
    d.struct_size = C.sizeof(fl_variant_desc)
    d.scale, d.score_mod, d.softcap, d.mask = scale, score_mod, softcap, mask
    d.window, d.prefix_len, d.n_bias, d.combine = window, prefix_len, n_bias, combine
    d.epilogue, d.rms_eps, d.q_offset = epilogue, rms_eps, q_offset
    return d


def aux_desc(*, alibi_slopes=None, q_doc_ids=None, kv_doc_ids=None, biases=(), gate=None, q2=None,
             k2=None, lambda_=None, rms_weight=None, workspace=None) -> fl_aux:
    a = fl_aux()
    a.struct_size = C.sizeof(fl_aux)

    def p(t):
        return None if t is None else t.data_ptr()
    a.alibi_slopes, a.q_doc_ids, a.kv_doc_ids = p(alibi_slopes), p(q_doc_ids), p(kv_doc_ids)
    for n, b in enumerate(biases):
        a.bias[n] = tensor_desc(b)
    a.gate, a.q2, a.k2 = tensor_desc(gate), tensor_desc(q2), tensor_desc(k2)
    a.lambda_, a.rms_weight = p(lambda_), p(rms_weight)
    if workspace is not None:
        a.workspace = workspace.data_ptr()
        a.workspace_bytes = workspace.numel() * workspace.element_size()
    return a


def _ref(x):
    return None if x is None else C.byref(x)


def fl_attn_fwd(q: fl_tensor, k: fl_tensor, v: fl_tensor, desc: fl_variant_desc, aux: Optional[fl_aux],
                out: fl_tensor, lse: Optional[fl_tensor], stream: int = 0) -> int:
    """Raw call; returns the fl_status code."""
    return lib().fl_attn_fwd(_ref(q), _ref(k), _ref(v), _ref(desc), _ref(aux), _ref(out), _ref(lse),
                             C.c_void_p(stream))


def fl_attn_fwd_noalloc(q: fl_tensor, k: fl_tensor, v: fl_tensor, desc: fl_variant_desc, aux: Optional[fl_aux],
                        out: fl_tensor, lse: Optional[fl_tensor], stream: int = 0) -> int:
    """Raw call; returns the fl_status code.  aux.workspace is ignored (the library's built-in scratch is used)."""
    return lib().fl_attn_fwd_noalloc(_ref(q), _ref(k), _ref(v), _ref(desc), _ref(aux), _ref(out), _ref(lse),
                                     C.c_void_p(stream))


def fl_attn_fwd_workspace_size(q: fl_tensor, k: fl_tensor, desc: fl_variant_desc) -> int:
    return lib().fl_attn_fwd_workspace_size(_ref(q), _ref(k), _ref(desc))


def fl_attn_bwd(q: fl_tensor, k: fl_tensor, v: fl_tensor, out: fl_tensor, dout: fl_tensor, lse: fl_tensor,
                desc: fl_variant_desc, aux: Optional[fl_aux], dq: fl_tensor, dk: fl_tensor, dv: fl_tensor,
                stream: int = 0) -> int:
    """Raw call; returns the fl_status code."""
    return lib().fl_attn_bwd(_ref(q), _ref(k), _ref(v), _ref(out), _ref(dout), _ref(lse), _ref(desc), _ref(aux),
                             _ref(dq), _ref(dk), _ref(dv), C.c_void_p(stream))


def bwd_extra(*, dq2=None, dk2=None, dbias=(), dgate=None, dlambda=None, drms_weight=None) -> fl_bwd_extra:
    x = fl_bwd_extra()
    x.struct_size = C.sizeof(fl_bwd_extra)
    x.dq2, x.dk2, x.dgate = tensor_desc(dq2), tensor_desc(dk2), tensor_desc(dgate)
    for n, b in enumerate(dbias):
        x.dbias[n] = tensor_desc(b)
    x.dlambda = None if dlambda is None else dlambda.data_ptr()
    x.drms_weight = None if drms_weight is None else drms_weight.data_ptr()
    return x


def fl_attn_bwd_ex(q: fl_tensor, k: fl_tensor, v: fl_tensor, out: fl_tensor, dout: fl_tensor, lse: fl_tensor,
                   desc: fl_variant_desc, aux: Optional[fl_aux], dq: fl_tensor, dk: fl_tensor, dv: fl_tensor,
                   extra: Optional[fl_bwd_extra], stream: int = 0) -> int:
    """Raw call; returns the fl_status code."""
    return lib().fl_attn_bwd_ex(_ref(q), _ref(k), _ref(v), _ref(out), _ref(dout), _ref(lse), _ref(desc), _ref(aux),
                                _ref(dq), _ref(dk), _ref(dv), _ref(extra), C.c_void_p(stream))


def fl_attn_bwd_ex_workspace_size(q: fl_tensor, k: fl_tensor, v: fl_tensor, desc: fl_variant_desc) -> int:
    return lib().fl_attn_bwd_ex_workspace_size(_ref(q), _ref(k), _ref(v), _ref(desc))


def fl_attn_bwd_workspace_size(q: fl_tensor, k: fl_tensor, desc: fl_variant_desc) -> int:
    return lib().fl_attn_bwd_workspace_size(_ref(q), _ref(k), _ref(desc))


def fl_bwd_supported(desc: fl_variant_desc, dtype: int, D: int, Dv: int) -> bool:
    return bool(lib().fl_bwd_supported(_ref(desc), dtype, D, Dv))


def paged_kv(*, block_table=None, page_size: int, seq_lens, max_seq_len: int) -> fl_paged_kv:
    kv = fl_paged_kv()
    kv.struct_size = C.sizeof(fl_paged_kv)
    kv.block_table = None if block_table is None else block_table.data_ptr()
    kv.table_stride = 0 if block_table is None else block_table.stride(0)
    kv.page_size = page_size
    kv.seq_lens = seq_lens.data_ptr()
    kv.max_seq_len = max_seq_len
    return kv


def fl_attn_decode(q: fl_tensor, k_cache: fl_tensor, v_cache: fl_tensor, kv: fl_paged_kv, desc: fl_variant_desc,
                   aux: Optional[fl_aux], out: fl_tensor, lse: Optional[fl_tensor], stream: int = 0) -> int:
    """Raw call; returns the fl_status code."""
    return lib().fl_attn_decode(_ref(q), _ref(k_cache), _ref(v_cache), _ref(kv), _ref(desc), _ref(aux), _ref(out),
                                _ref(lse), C.c_void_p(stream))


def fl_attn_decode_workspace_size(q: fl_tensor, k_cache: fl_tensor, kv: fl_paged_kv) -> int:
    return lib().fl_attn_decode_workspace_size(_ref(q), _ref(k_cache), _ref(kv))


def fl_attn_prefill_paged(q: fl_tensor, k_cache: fl_tensor, v_cache: fl_tensor, kv: fl_paged_kv, desc: fl_variant_desc,
                          aux: Optional[fl_aux], out: fl_tensor, lse: Optional[fl_tensor], stream: int = 0) -> int:
    """A chunk of query rows per sequence against the paged cache; returns the status code."""
    return lib().fl_attn_prefill_paged(_ref(q), _ref(k_cache), _ref(v_cache), _ref(kv), _ref(desc), _ref(aux), _ref(out),
                                       _ref(lse), C.c_void_p(stream))


def fl_attn_prefill_paged_workspace_size(q: fl_tensor, k_cache: fl_tensor, kv: fl_paged_kv) -> int:
    return lib().fl_attn_prefill_paged_workspace_size(_ref(q), _ref(k_cache), _ref(kv))


def fl_compile_variant(score_mod: Optional[str], mask: Optional[str], D: int, base_mask: int = 0):
    """Returns (status, handle); handle is a ctypes void pointer (NULL on failure)."""
    h = C.c_void_p()
    st = lib().fl_compile_variant(None if score_mod is None else score_mod.encode(),
                                  None if mask is None else mask.encode(), base_mask, D, C.byref(h))
    return st, h


def fl_attn_fwd_custom(handle, q: fl_tensor, k: fl_tensor, v: fl_tensor, scale: float, out: fl_tensor,
                       lse: Optional[fl_tensor] = None, stream: int = 0, window: int = 0, prefix_len: int = 0) -> int:
    """Raw call; returns the fl_status code."""
    return lib().fl_attn_fwd_custom(handle, _ref(q), _ref(k), _ref(v), C.c_float(scale), window, prefix_len, _ref(out),
                                    _ref(lse), C.c_void_p(stream))


def fl_compile_variant_aux(score_mod: Optional[str], mask: Optional[str], D: int, aux=(), base_mask: int = 0):
    """aux: up to four torch tensors (or dtype codes) that the expressions read as aux0 .. aux3.
    Returns (status, handle)."""
    h = C.c_void_p()
    codes = (C.c_int32 * 4)(*([(_dtype_code(a) if hasattr(a, "dtype") else int(a or 0)) for a in aux] + [0] * (4 - len(aux))))
    st = lib().fl_compile_variant_aux(None if score_mod is None else score_mod.encode(),
                                      None if mask is None else mask.encode(), base_mask, D, codes, C.byref(h))
    return st, h


def fl_attn_fwd_custom_aux(handle, q: fl_tensor, k: fl_tensor, v: fl_tensor, scale: float, aux, out: fl_tensor,
                           lse: Optional[fl_tensor] = None, stream: int = 0, window: int = 0, prefix_len: int = 0) -> int:
    """aux: the device tensors for aux0 .. aux3 (None for unused slots).  Returns the fl_status code."""
    ptrs = (C.c_void_p * 4)(*([(None if a is None else a.data_ptr()) for a in aux] + [None] * (4 - len(aux))))
    return lib().fl_attn_fwd_custom_aux(handle, _ref(q), _ref(k), _ref(v), C.c_float(scale), window, prefix_len, ptrs,
                                        _ref(out), _ref(lse), C.c_void_p(stream))


def fl_attn_fwd_custom_skip(handle, q: fl_tensor, k: fl_tensor, v: fl_tensor, scale: float, aux, workspace, out: fl_tensor,
                            lse: Optional[fl_tensor] = None, stream: int = 0, window: int = 0, prefix_len: int = 0) -> int:
    """fl_attn_fwd_custom_aux with the tile-class pre-pass; workspace: a uint8 device tensor (or None).  Returns the status."""
    ptrs = (C.c_void_p * 4)(*([(None if a is None else a.data_ptr()) for a in aux] + [None] * (4 - len(aux))))
    ws_ptr = None if workspace is None else workspace.data_ptr()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return lib().fl_attn_fwd_custom_skip(handle, _ref(q), _ref(k), _ref(v), C.c_float(scale), window, prefix_len, ptrs,
                                         C.c_void_p(ws_ptr), C.c_size_t(ws_bytes), _ref(out), _ref(lse), C.c_void_p(stream))


def fl_custom_skip_workspace_size(handle, q: fl_tensor, k: fl_tensor) -> int:
    return lib().fl_custom_skip_workspace_size(handle, _ref(q), _ref(k))


def fl_compile_variant_grad(score_mod: Optional[str], score_mod_grad: Optional[str], mask: Optional[str], D: int, aux=(),
                            base_mask: int = 0):
    """Compile with a derivative expression for the score_mod (and the backward kernels).  Returns (status, handle)."""
    h = C.c_void_p()
    codes = (C.c_int32 * 4)(*([(_dtype_code(a) if hasattr(a, "dtype") else int(a or 0)) for a in aux] + [0] * (4 - len(aux))))
    enc = lambda x: None if x is None else x.encode()
    st = lib().fl_compile_variant_grad(enc(score_mod), enc(score_mod_grad), enc(mask), base_mask, D, codes, C.byref(h))
    return st, h


def fl_attn_bwd_custom(handle, q: fl_tensor, k: fl_tensor, v: fl_tensor, out: fl_tensor, dout: fl_tensor, lse: fl_tensor,
                       scale: float, aux, workspace, dq: fl_tensor, dk: fl_tensor, dv: fl_tensor, stream: int = 0,
                       window: int = 0, prefix_len: int = 0) -> int:
    """Gradients of a compiled variant; workspace: a uint8 device tensor.  Returns the status code."""
    ptrs = (C.c_void_p * 4)(*([(None if a is None else a.data_ptr()) for a in aux] + [None] * (4 - len(aux))))
    ws_ptr = None if workspace is None else workspace.data_ptr()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    return lib().fl_attn_bwd_custom(handle, _ref(q), _ref(k), _ref(v), _ref(out), _ref(dout), _ref(lse), C.c_float(scale), window,
                                    prefix_len, ptrs, C.c_void_p(ws_ptr), C.c_size_t(ws_bytes), _ref(dq), _ref(dk), _ref(dv),
                                    C.c_void_p(stream))


def fl_attn_bwd_custom_workspace_size(handle, q: fl_tensor, k: fl_tensor) -> int:
    return lib().fl_attn_bwd_custom_workspace_size(handle, _ref(q), _ref(k))


def fl_release_variant(handle) -> None:
    lib().fl_release_variant(handle)


class CustomVariant:
    """A variant compiled at run time from a score_mod and / or a mask expression (C syntax)."""

    def __init__(self, score_mod: Optional[str], mask: Optional[str], D: int, base_mask: int = 0, aux=(),
                 score_mod_grad: Optional[str] = None):
        """aux: up to four device tensors the expressions read as aux0 .. aux3 (kept alive by this object).
        score_mod_grad: derivative of score_mod with respect to s (compiles the backward kernels too)."""
        self.aux = list(aux)
        if score_mod_grad is not None:
            st, h = fl_compile_variant_grad(score_mod, score_mod_grad, mask, D, self.aux, base_mask)
        elif self.aux:
            st, h = fl_compile_variant_aux(score_mod, mask, D, self.aux, base_mask)
        else:
            st, h = fl_compile_variant(score_mod, mask, D, base_mask)
        check(st)
        self.handle = h

    def forward(self, q: fl_tensor, k: fl_tensor, v: fl_tensor, scale: float, out: fl_tensor,
                lse: Optional[fl_tensor] = None, stream: int = 0, window: int = 0, prefix_len: int = 0,
                workspace=None) -> int:
        """workspace (a uint8 device tensor of skip_workspace_size bytes): run with the tile-class pre-pass."""
        if workspace is not None:
            return fl_attn_fwd_custom_skip(self.handle, q, k, v, scale, self.aux, workspace, out, lse, stream, window, prefix_len)
        if self.aux:
            return fl_attn_fwd_custom_aux(self.handle, q, k, v, scale, self.aux, out, lse, stream, window, prefix_len)
        return fl_attn_fwd_custom(self.handle, q, k, v, scale, out, lse, stream, window, prefix_len)

    def backward(self, q: fl_tensor, k: fl_tensor, v: fl_tensor, out: fl_tensor, dout: fl_tensor, lse: fl_tensor, scale: float,
                 workspace, dq: fl_tensor, dk: fl_tensor, dv: fl_tensor, stream: int = 0, window: int = 0, prefix_len: int = 0) -> int:
        return fl_attn_bwd_custom(self.handle, q, k, v, out, dout, lse, scale, self.aux, workspace, dq, dk, dv, stream, window,
                                  prefix_len)

    def backward_workspace_size(self, q: fl_tensor, k: fl_tensor) -> int:
        return fl_attn_bwd_custom_workspace_size(self.handle, q, k)

    def skip_workspace_size(self, q: fl_tensor, k: fl_tensor) -> int:
        return fl_custom_skip_workspace_size(self.handle, q, k)

    def release(self) -> None:
        if self.handle is not None and self.handle.value:
            fl_release_variant(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.release()
        except Exception:
            pass


def fl_variant_supported(desc: fl_variant_desc, dtype: int, D: int, Dv: int) -> bool:
    return bool(lib().fl_variant_supported(_ref(desc), dtype, D, Dv))


def fl_strerror(status: int) -> str:
    return lib().fl_strerror(status).decode()


def fl_last_error_detail() -> str:
    return lib().fl_last_error_detail().decode()


def fl_set_tuning(key: str, value: int) -> int:
    return lib().fl_set_tuning(key.encode(), value)


def fl_version() -> int:
    return lib().fl_version()


def check(status: int) -> None:
    if status != FL_OK:
        raise FlError(status, fl_strerror(status), fl_last_error_detail())
