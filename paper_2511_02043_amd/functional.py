"""PyTorch-facing calls of the library: `attention(q, k, v, ...)` with autograd support and
`decode_attention(...)` for one decode step over a paged cache.

Marshalling only: the forward pass is fl_attn_fwd, the backward pass fl_attn_bwd, both through
the C-ABI binding; no attention arithmetic happens here and there is no fallback path.  Tensors
are [B, H, S, D] (or [B, G, H, S, D] with an extra independent row axis) bf16 CUDA tensors;
strided views are passed as they are.

Differentiable variants: scale, causal / sliding-window / PrefixLM / document masks, ALiBi,
tanh soft-cap, grouped-query heads (the variants fl_attn_bwd covers).  Biases, the sigmoid gate
and differential attention are forward-only here: use runner.upload / fl_attn_fwd for those.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as fb


def _as5(x: torch.Tensor) -> torch.Tensor:
    if x.dim() == 4:
        return x.unsqueeze(1)
    if x.dim() != 5:
        raise ValueError(f"expected [B, H, S, D] or [B, G, H, S, D], got {tuple(x.shape)}")
    return x


def _check_aux(name: str, t: Optional[torch.Tensor], dtype: torch.dtype, shape, device, *, contiguous: bool = True,
               inner_unit: bool = False) -> None:
    """The C ABI reads these arrays as raw int32 / float32 memory of a fixed shape: anything else
    (torch's default int64 ids, a sliced view, a tensor on another device) would be reinterpreted
    silently, so it is refused here."""
    if t is None:
        return
    if not isinstance(t, torch.Tensor):
        raise ValueError(f"{name} must be a torch.Tensor")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if t.device != device:
        raise ValueError(f"{name} is on {t.device}, expected {device}")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    if contiguous and not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if inner_unit and t.dim() >= 2 and t.shape[-1] > 1 and t.stride(-1) != 1:
        raise ValueError(f"{name} must have unit stride along its last axis")


def _desc(scale, causal, window, prefix, softcap, alibi_slopes, q_doc_ids, q_offset=0):
    mask = 0
    if causal:
        mask |= fb.FL_MASK_CAUSAL
    if window is not None:
        mask |= fb.FL_MASK_WINDOW | fb.FL_MASK_CAUSAL
    if prefix is not None:
        mask |= fb.FL_MASK_PREFIX
    if q_doc_ids is not None:
        mask |= fb.FL_MASK_DOC
    if softcap is not None and alibi_slopes is not None:
        raise ValueError("one score_mod at a time")
    mod = fb.FL_MOD_SOFTCAP if softcap is not None else (fb.FL_MOD_ALIBI if alibi_slopes is not None else fb.FL_MOD_NONE)
    return fb.variant_desc(scale=float(scale), score_mod=mod, softcap=float(softcap or 0.0), mask=mask,
                           window=int(window or 0), prefix_len=int(prefix or 0), q_offset=int(q_offset))


class _Attention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, scale, causal, window, prefix, softcap, alibi_slopes, q_doc_ids, kv_doc_ids, q_offset):
        q5, k5, v5 = _as5(q), _as5(k), _as5(v)
        B, G, H, Sq, _ = q5.shape
        desc = _desc(scale, causal, window, prefix, softcap, alibi_slopes, q_doc_ids, q_offset)
        out = torch.empty((B, G, H, Sq, v5.shape[4]), dtype=q.dtype, device=q.device)
        lse = torch.empty((B, G, H, Sq, 1), dtype=torch.float32, device=q.device)
        tq, tk, tv, tout, tlse = (fb.tensor_desc(x) for x in (q5, k5, v5, out, lse))
        ws = None
        nbytes = fb.fl_attn_fwd_workspace_size(tq, tk, desc)
        if nbytes:
            ws = torch.empty(nbytes, dtype=torch.uint8, device=q.device)
        aux = fb.aux_desc(alibi_slopes=alibi_slopes, q_doc_ids=q_doc_ids, kv_doc_ids=kv_doc_ids, workspace=ws)
        stream = torch.cuda.current_stream(q.device).cuda_stream
        fb.check(fb.fl_attn_fwd(tq, tk, tv, desc, aux, tout, tlse, stream))
        ctx.save_for_backward(q, k, v, out, lse)
        ctx.variant = (scale, causal, window, prefix, softcap, q_offset)
        ctx.aux_tensors = (alibi_slopes, q_doc_ids, kv_doc_ids)
        return out if q.dim() == 5 else out.squeeze(1)

    @staticmethod
    def backward(ctx, dout):
        q, k, v, out, lse = ctx.saved_tensors
        scale, causal, window, prefix, softcap, q_offset = ctx.variant
        alibi_slopes, q_doc_ids, kv_doc_ids = ctx.aux_tensors
        q5, k5, v5, d5 = _as5(q), _as5(k), _as5(v), _as5(dout)
        if d5.stride(-1) != 1 or any(st % 8 for st in d5.stride()[:-1]):
            d5 = d5.contiguous()                   # the kernels need unit inner stride and 16-byte aligned rows
        desc = _desc(scale, causal, window, prefix, softcap, alibi_slopes, q_doc_ids, q_offset)
        dq, dk, dv = torch.empty_like(q5), torch.empty_like(k5), torch.empty_like(v5)
        tq, tk, tv, tout, tdo, tlse, tdq, tdk, tdv = (fb.tensor_desc(x) for x in (q5, k5, v5, out, d5, lse, dq, dk, dv))
        nbytes = fb.fl_attn_bwd_workspace_size(tq, tk, desc)
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=q.device)
        aux = fb.aux_desc(alibi_slopes=alibi_slopes, q_doc_ids=q_doc_ids, kv_doc_ids=kv_doc_ids, workspace=ws)
        stream = torch.cuda.current_stream(q.device).cuda_stream
        fb.check(fb.fl_attn_bwd(tq, tk, tv, tout, tdo, tlse, desc, aux, tdq, tdk, tdv, stream))
        if q.dim() == 4:
            dq, dk, dv = dq.squeeze(1), dk.squeeze(1), dv.squeeze(1)
        return (dq, dk, dv) + (None,) * 9


def attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, *, scale: Optional[float] = None,
              causal: bool = False, window: Optional[int] = None, prefix: Optional[int] = None,
              softcap: Optional[float] = None, alibi_slopes: Optional[torch.Tensor] = None,
              q_doc_ids: Optional[torch.Tensor] = None, kv_doc_ids: Optional[torch.Tensor] = None,
              q_offset: int = 0) -> torch.Tensor:
    """softmax(mask(score_mod(scale * q k^T))) v on the library's fused kernels, differentiable in
    q, k and v.  q [B, (G,) H, Sq, D], k and v [B, (G,) Hkv, Sk, D] with Hkv dividing H; bf16.

    alibi_slopes: float32 [H]; q_doc_ids / kv_doc_ids: int32 [B, Sq] / [B, Sk] (kv defaults to q's).
    q_offset: query row i sits at sequence position i + q_offset in the positional masks and ALiBi
    (Sk - Sq aligns a causal mask bottom-right: a chunk of new queries against a longer cache).
    """
    if not q.is_cuda or q.dtype != torch.bfloat16:
        raise ValueError("attention() takes bf16 CUDA tensors (there is no CPU or fallback path)")
    if scale is None:
        scale = q.shape[-1] ** -0.5
    if q_doc_ids is not None and kv_doc_ids is None:
        kv_doc_ids = q_doc_ids
    if kv_doc_ids is not None and q_doc_ids is None:
        raise ValueError("kv_doc_ids needs q_doc_ids")
    q5, k5 = _as5(q), _as5(k)
    _check_aux("alibi_slopes", alibi_slopes, torch.float32, (q5.shape[2],), q.device)
    _check_aux("q_doc_ids", q_doc_ids, torch.int32, (q5.shape[0], q5.shape[3]), q.device)
    _check_aux("kv_doc_ids", kv_doc_ids, torch.int32, (k5.shape[0], k5.shape[3]), q.device)
    if q_offset < 0:
        raise ValueError("q_offset must be >= 0")
    return _Attention.apply(q, k, v, scale, causal, window, prefix, softcap, alibi_slopes, q_doc_ids, kv_doc_ids, int(q_offset))


def decode_attention(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, seq_lens: torch.Tensor,
                     block_table: Optional[torch.Tensor] = None, *, max_seq_len: Optional[int] = None,
                     scale: Optional[float] = None, window: Optional[int] = None, softcap: Optional[float] = None,
                     alibi_slopes: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                     return_lse: bool = False):
    """One decode step (fl_attn_decode): the last token of every sequence against its cached keys.

    q [B, H, D] bf16; k_cache, v_cache [pages, page_size, Hkv, D] bf16 (any strides with unit inner
    stride, e.g. a permuted [pages, Hkv, page_size, D] buffer); seq_lens int32 [B] on the device;
    block_table int32 [B, max_pages] or None for a contiguous cache (sequence b in "page" b).
    max_seq_len is a host-side bound on seq_lens (it fixes the launch shape; default: the capacity
    of the table, so no device value is read back).  workspace: a uint8 tensor of at least
    decode_workspace_size(...) bytes to reuse across steps; allocated here when omitted.
    Returns out [B, H, D] bf16 (and lse [B, H] float32 with return_lse).  Not differentiable.
    """
    if not q.is_cuda or q.dtype != torch.bfloat16 or q.dim() != 3:
        raise ValueError("decode_attention() takes a bf16 CUDA q of shape [B, H, D]")
    B, H, D = q.shape
    page_size = k_cache.shape[1]
    _check_aux("seq_lens", seq_lens, torch.int32, (B,), q.device)
    if block_table is not None:
        if block_table.dim() != 2:
            raise ValueError("block_table must be [B, max_pages]")
        _check_aux("block_table", block_table, torch.int32, (B, block_table.shape[1]), q.device, contiguous=False,
                   inner_unit=True)
    _check_aux("alibi_slopes", alibi_slopes, torch.float32, (H,), q.device)
    if max_seq_len is None:
        max_seq_len = (block_table.shape[1] if block_table is not None else 1) * page_size
    if scale is None:
        scale = D ** -0.5
    if softcap is not None and alibi_slopes is not None:
        raise ValueError("one score_mod at a time")
    mod = fb.FL_MOD_SOFTCAP if softcap is not None else (fb.FL_MOD_ALIBI if alibi_slopes is not None else fb.FL_MOD_NONE)
    desc = fb.variant_desc(scale=float(scale), score_mod=mod, softcap=float(softcap or 0.0),
                           mask=(fb.FL_MASK_WINDOW | fb.FL_MASK_CAUSAL) if window is not None else fb.FL_MASK_CAUSAL,
                           window=int(window or 0))
    q5 = q[:, None, :, None, :]
    k5, v5 = k_cache.permute(0, 2, 1, 3)[:, None], v_cache.permute(0, 2, 1, 3)[:, None]    # [pages, 1, Hkv, page_size, D]
    out = torch.empty((B, 1, H, 1, D), dtype=torch.bfloat16, device=q.device)
    lse = torch.empty((B, 1, H, 1, 1), dtype=torch.float32, device=q.device) if return_lse else None
    kv = fb.paged_kv(block_table=block_table, page_size=page_size, seq_lens=seq_lens, max_seq_len=int(max_seq_len))
    tq, tk, tv, tout = (fb.tensor_desc(x) for x in (q5, k5, v5, out))
    tlse = fb.tensor_desc(lse) if return_lse else None
    need = max(fb.fl_attn_decode_workspace_size(tq, tk, kv), 16)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    elif workspace.numel() * workspace.element_size() < need:
        raise ValueError(f"workspace holds {workspace.numel() * workspace.element_size()} bytes, {need} needed")
    aux = fb.aux_desc(alibi_slopes=alibi_slopes, workspace=workspace)
    fb.check(fb.fl_attn_decode(tq, tk, tv, kv, desc, aux, tout, tlse, torch.cuda.current_stream(q.device).cuda_stream))
    out = out[:, 0, :, 0, :]
    return (out, lse[:, 0, :, 0, 0]) if return_lse else out
