"""PyTorch-facing calls of the library: `attention(q, k, v, ...)` with autograd support and
`decode_attention(...)` for one decode step over a paged cache.

Marshalling only: the forward pass is fl_attn_fwd, the backward pass fl_attn_bwd, both through
the C-ABI binding; no attention arithmetic happens here and there is no fallback path.  Tensors
are [B, H, S, D] (or [B, G, H, S, D] with an extra independent row axis) bf16 CUDA tensors;
strided views are passed as they are.

`attention()`: scale, causal / sliding-window / PrefixLM / document masks, ALiBi, tanh soft-cap,
grouped-query heads, query-position offset (the variants fl_attn_bwd covers).
`variant_attention()`: the same plus additive biases, the sigmoid gate, RMSNorm and the differential
second stream, differentiable in every tensor input (fl_attn_bwd_ex).
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


def _mask_bits(causal, window, prefix, q_doc_ids):
    mask = 0
    if causal:
        mask |= fb.FL_MASK_CAUSAL
    if window is not None:
        mask |= fb.FL_MASK_WINDOW | fb.FL_MASK_CAUSAL
    if prefix is not None:
        mask |= fb.FL_MASK_PREFIX
    if q_doc_ids is not None:
        mask |= fb.FL_MASK_DOC
    return mask


class _VariantAttention(torch.autograd.Function):
    """Forward fl_attn_fwd, backward fl_attn_bwd_ex, for descriptors with biases / gate / RMSNorm / second stream.
    Tensor inputs: q, k, v, q2, k2, lam, gate, bias0, bias1, rms_weight (absent ones are None)."""

    @staticmethod
    def forward(ctx, cfg, q, k, v, q2, k2, lam, gate, bias0, bias1, rms_weight):
        dev = q.device
        q5, k5, v5 = _as5(q), _as5(k), _as5(v)
        B, G, H, Sq, _ = q5.shape
        diff = q2 is not None
        biases = [b for b in (bias0, bias1) if b is not None]
        epi = (fb.FL_EPI_RMSNORM if cfg["rmsnorm"] else 0) | (fb.FL_EPI_GATE_SIGMOID if gate is not None else 0)
        mod = fb.FL_MOD_SOFTCAP if cfg["softcap"] is not None else (fb.FL_MOD_ALIBI if cfg["alibi_slopes"] is not None else fb.FL_MOD_NONE)
        desc = fb.variant_desc(scale=float(cfg["scale"]), score_mod=mod, softcap=float(cfg["softcap"] or 0.0),
                               mask=_mask_bits(cfg["causal"], cfg["window"], cfg["prefix"], cfg["q_doc_ids"]),
                               window=int(cfg["window"] or 0), prefix_len=int(cfg["prefix"] or 0), n_bias=len(biases),
                               combine=fb.FL_DIFFERENTIAL if diff else fb.FL_SINGLE, epilogue=epi,
                               rms_eps=float(cfg["rms_eps"]) if cfg["rmsnorm"] else 0.0, q_offset=int(cfg["q_offset"]))
        out = torch.empty((B, G, H, Sq, v5.shape[4]), dtype=q.dtype, device=dev)
        lse = torch.empty((B, 2 * G if diff else G, H, Sq, 1), dtype=torch.float32, device=dev)
        tq, tk, tv, tout, tlse = (fb.tensor_desc(x) for x in (q5, k5, v5, out, lse))
        ws = None
        nbytes = fb.fl_attn_fwd_workspace_size(tq, tk, desc)
        if nbytes:
            ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        five = lambda x: None if x is None else _as5(x)
        aux = fb.aux_desc(alibi_slopes=cfg["alibi_slopes"], q_doc_ids=cfg["q_doc_ids"], kv_doc_ids=cfg["kv_doc_ids"],
                          biases=biases, gate=five(gate), q2=five(q2), k2=five(k2), lambda_=lam,
                          rms_weight=rms_weight, workspace=ws)
        stream = torch.cuda.current_stream(dev).cuda_stream
        fb.check(fb.fl_attn_fwd(tq, tk, tv, desc, aux, tout, tlse, stream))
        ctx.save_for_backward(q, k, v, q2, k2, lam, gate, bias0, bias1, rms_weight, out, lse)
        ctx.cfg, ctx.desc = cfg, desc
        return out if q.dim() == 5 else out.squeeze(1)

    @staticmethod
    def backward(ctx, dout):
        q, k, v, q2, k2, lam, gate, bias0, bias1, rms_weight, out, lse = ctx.saved_tensors
        cfg, desc = ctx.cfg, ctx.desc
        dev = q.device
        q5, k5, v5, d5 = _as5(q), _as5(k), _as5(v), _as5(dout)
        if d5.stride(-1) != 1 or any(st % 8 for st in d5.stride()[:-1]):
            d5 = d5.contiguous()
        five = lambda x: None if x is None else _as5(x)
        biases = [b for b in (bias0, bias1) if b is not None]
        dq, dk, dv = torch.empty_like(q5), torch.empty_like(k5), torch.empty_like(v5)
        dq2 = None if q2 is None else torch.empty_like(five(q2))
        dk2 = None if k2 is None else torch.empty_like(five(k2))
        dlam = None if lam is None else torch.empty_like(lam)
        dgate = None if gate is None else torch.empty_like(five(gate))
        dbias = [torch.empty(tuple(b.shape), dtype=torch.float32, device=dev) for b in biases]
        tq, tk, tv, tout, tdo, tlse, tdq, tdk, tdv = (fb.tensor_desc(x) for x in (q5, k5, v5, out, d5, lse, dq, dk, dv))
        ws = torch.empty(max(fb.fl_attn_bwd_ex_workspace_size(tq, tk, tv, desc), 16), dtype=torch.uint8, device=dev)
        aux = fb.aux_desc(alibi_slopes=cfg["alibi_slopes"], q_doc_ids=cfg["q_doc_ids"], kv_doc_ids=cfg["kv_doc_ids"],
                          biases=biases, gate=five(gate), q2=five(q2), k2=five(k2), lambda_=lam,
                          rms_weight=rms_weight, workspace=ws)
        drms = torch.empty(v5.shape[4], dtype=torch.float32, device=dev) if (cfg["rmsnorm"] and rms_weight is not None) else None
        extra = fb.bwd_extra(dq2=dq2, dk2=dk2, dbias=dbias, dgate=dgate, dlambda=dlam, drms_weight=drms)
        stream = torch.cuda.current_stream(dev).cuda_stream
        fb.check(fb.fl_attn_bwd_ex(tq, tk, tv, tout, tdo, tlse, desc, aux, tdq, tdk, tdv, extra, stream))
        sq = (lambda x: x) if q.dim() == 5 else (lambda x: None if x is None else x.squeeze(1))
        gb = [g.to(b.dtype) for g, b in zip(dbias, biases)] + [None] * (2 - len(biases))
        if bias0 is None and bias1 is not None:
            gb = [None, gb[0]]
        return (None, sq(dq), sq(dk), sq(dv), sq(dq2), sq(dk2), dlam, sq(dgate), gb[0], gb[1], drms)


def variant_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, *, scale: Optional[float] = None,
                      causal: bool = False, window: Optional[int] = None, prefix: Optional[int] = None,
                      softcap: Optional[float] = None, alibi_slopes: Optional[torch.Tensor] = None,
                      q_doc_ids: Optional[torch.Tensor] = None, kv_doc_ids: Optional[torch.Tensor] = None,
                      q_offset: int = 0, biases=(), gate: Optional[torch.Tensor] = None,
                      q2: Optional[torch.Tensor] = None, k2: Optional[torch.Tensor] = None,
                      lam: Optional[torch.Tensor] = None, rmsnorm: bool = False, rms_eps: float = 1e-6,
                      rms_weight: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Every variant of the forward pass with autograd: attention() plus

    biases    up to two bf16 tensors that broadcast to [B, G, H, Sq, Sk] (5-D, size-1 axes broadcast), added to the
              scaled score; their gradients come back in the biases' own shapes
    gate      pre-sigmoid tensor of the output's shape: out = sigmoid(gate) * (...)
    q2, k2, lam   the second softmax stream of differential attention and its per-head fp32 weights [H]:
              softmax(q k^T) v - lam_h softmax(q2 k2^T) v
    rmsnorm   RMSNorm over the output channels (rms_weight fp32 [Dv] or None for all ones), before the gate
    Tensors are [B, H, S, D] or [B, G, H, S, D], bf16, on the GPU; differentiable in q, k, v, q2, k2, lam, gate, biases
    and rms_weight."""
    if not q.is_cuda or q.dtype != torch.bfloat16:
        raise ValueError("variant_attention() takes bf16 CUDA tensors (there is no CPU or fallback path)")
    if (q2 is None) != (k2 is None) or (q2 is None) != (lam is None):
        raise ValueError("q2, k2 and lam come together")
    if softcap is not None and alibi_slopes is not None:
        raise ValueError("one score_mod at a time")
    if len(biases) > 2:
        raise ValueError("at most two biases")
    q5, k5 = _as5(q), _as5(k)
    if q_doc_ids is not None and kv_doc_ids is None:
        kv_doc_ids = q_doc_ids
    _check_aux("alibi_slopes", alibi_slopes, torch.float32, (q5.shape[2],), q.device)
    _check_aux("q_doc_ids", q_doc_ids, torch.int32, (q5.shape[0], q5.shape[3]), q.device)
    _check_aux("kv_doc_ids", kv_doc_ids, torch.int32, (k5.shape[0], k5.shape[3]), q.device)
    _check_aux("lam", lam, torch.float32, (q5.shape[2],), q.device)
    if rms_weight is not None:
        _check_aux("rms_weight", rms_weight, torch.float32, (_as5(v).shape[4],), q.device)
    for n, b in enumerate(biases):
        if b.dim() != 5 or b.dtype != torch.bfloat16 or b.device != q.device:
            raise ValueError(f"biases[{n}] must be a 5-D bf16 tensor on {q.device}")
    cfg = dict(scale=q.shape[-1] ** -0.5 if scale is None else scale, causal=causal, window=window, prefix=prefix,
               softcap=softcap, alibi_slopes=alibi_slopes, q_doc_ids=q_doc_ids, kv_doc_ids=kv_doc_ids, q_offset=q_offset,
               rmsnorm=rmsnorm, rms_eps=rms_eps)
    b0 = biases[0] if len(biases) > 0 else None
    b1 = biases[1] if len(biases) > 1 else None
    return _VariantAttention.apply(cfg, q, k, v, q2, k2, lam, gate, b0, b1, rms_weight if rmsnorm else None)


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


def paged_prefill_attention(q: torch.Tensor, k_cache: torch.Tensor, v_cache: torch.Tensor, seq_lens: torch.Tensor,
                            block_table: Optional[torch.Tensor] = None, *, max_seq_len: Optional[int] = None,
                            scale: Optional[float] = None, window: Optional[int] = None, softcap: Optional[float] = None,
                            alibi_slopes: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                            return_lse: bool = False):
    """A chunk of query rows per sequence against the paged cache (fl_attn_prefill_paged): the last Sq tokens of every
    sequence, whose keys and values are already cached, attend causally to that sequence's cached keys.

    q [B, H, Sq, D] bf16; caches, seq_lens, block_table, max_seq_len as for decode_attention().  workspace: a uint8
    tensor of at least prefill workspace bytes (two dense copies of the cached rows) to reuse across calls;
    allocated here when omitted.  Returns out [B, H, Sq, D] bf16 (and lse [B, H, Sq] float32 with return_lse);
    rows at negative positions (a sequence shorter than the chunk) are zero.  Not differentiable."""
    if not q.is_cuda or q.dtype != torch.bfloat16 or q.dim() != 4:
        raise ValueError("paged_prefill_attention() takes a bf16 CUDA q of shape [B, H, Sq, D]")
    B, H, Sq, D = q.shape
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
    q5 = q[:, None]
    k5, v5 = k_cache.permute(0, 2, 1, 3)[:, None], v_cache.permute(0, 2, 1, 3)[:, None]    # [pages, 1, Hkv, page_size, D]
    out = torch.empty((B, 1, H, Sq, D), dtype=torch.bfloat16, device=q.device)
    lse = torch.empty((B, 1, H, Sq, 1), dtype=torch.float32, device=q.device) if return_lse else None
    kv = fb.paged_kv(block_table=block_table, page_size=page_size, seq_lens=seq_lens, max_seq_len=int(max_seq_len))
    tq, tk, tv, tout = (fb.tensor_desc(x) for x in (q5, k5, v5, out))
    tlse = fb.tensor_desc(lse) if return_lse else None
    need = max(fb.fl_attn_prefill_paged_workspace_size(tq, tk, kv), 16)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    elif workspace.numel() * workspace.element_size() < need:
        raise ValueError(f"workspace holds {workspace.numel() * workspace.element_size()} bytes, {need} needed")
    aux = fb.aux_desc(alibi_slopes=alibi_slopes, workspace=workspace)
    fb.check(fb.fl_attn_prefill_paged(tq, tk, tv, kv, desc, aux, tout, tlse, torch.cuda.current_stream(q.device).cuda_stream))
    out = out[:, 0]
    return (out, lse[:, 0, :, :, 0]) if return_lse else out
