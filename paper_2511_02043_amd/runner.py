"""Upload an inputs.Workload to the GPU and call fl_attn_fwd / fl_attn_bwd on it (marshalling only).

Used by the GPU tests, the smoke check and the benchmark.  The NumPy layouts of the
workload (including the Evoformer [B, Nseq, Nres, H, D] storage viewed as [B,G,H,S,D])
are reproduced on the device, so the kernels see the strides the workload describes.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np
import torch

from . import binding as fb


def to_device(x: np.ndarray, dtype: torch.dtype, device) -> torch.Tensor:
    """Copy to the device keeping the stride ORDER of `x` (dense in its own axis order)."""
    order = sorted(range(x.ndim), key=lambda a: (-abs(x.strides[a]), a))
    xp = np.ascontiguousarray(np.transpose(x, order))
    t = torch.from_numpy(xp).to(device=device, dtype=dtype)
    inv = [0] * x.ndim
    for pos, a in enumerate(order):
        inv[a] = pos
    return t.permute(inv)


def empty_like_layout(ref: torch.Tensor, last: int, dtype: torch.dtype) -> torch.Tensor:
    """Uninitialised tensor with ref's shape except the last dim, in ref's axis order."""
    shape = list(ref.shape[:-1]) + [last]
    order = sorted(range(ref.dim()), key=lambda a: (-ref.stride(a), a))
    t = torch.empty([shape[a] for a in order], dtype=dtype, device=ref.device)
    inv = [0] * ref.dim()
    for pos, a in enumerate(order):
        inv[a] = pos
    return t.permute(inv)


@dataclasses.dataclass
class DeviceWorkload:
    name: str
    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    out: torch.Tensor
    lse: Optional[torch.Tensor]
    desc: fb.fl_variant_desc
    aux: Optional[fb.fl_aux]
    keep: List[torch.Tensor]            # aux tensors kept alive
    tq: fb.fl_tensor = None
    tk: fb.fl_tensor = None
    tv: fb.fl_tensor = None
    tout: fb.fl_tensor = None
    tlse: Optional[fb.fl_tensor] = None

    def run(self, stream: int = 0) -> int:
        return fb.fl_attn_fwd(self.tq, self.tk, self.tv, self.desc, self.aux, self.tout, self.tlse, stream)

    def run_checked(self, stream: int = 0) -> None:
        fb.check(self.run(stream))


def upload(w, out_dtype: str = "f32", device="cuda:0", want_lse: bool = True) -> DeviceWorkload:
    """Build device tensors, the variant descriptor and aux block for a Workload."""
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    q, k, v = (to_device(x, tdt, device) for x in (w.q, w.k, w.v))
    B, G, H, Sq, D = q.shape
    Dv = v.shape[4]
    odt = torch.float32 if (out_dtype == "f32" or w.dtype == "f32") else tdt
    out = empty_like_layout(q, Dv, odt)
    keep: List[torch.Tensor] = []
    mask = 0
    if w.causal:
        mask |= fb.FL_MASK_CAUSAL
    if w.window is not None:
        mask |= fb.FL_MASK_WINDOW | fb.FL_MASK_CAUSAL
    if w.prefix is not None:
        mask |= fb.FL_MASK_PREFIX
    if w.q_doc is not None:
        mask |= fb.FL_MASK_DOC
    mod = fb.FL_MOD_NONE
    if w.softcap is not None:
        mod = fb.FL_MOD_SOFTCAP
    if w.alibi is not None:
        if mod != fb.FL_MOD_NONE:
            raise ValueError("one score_mod at a time")
        mod = fb.FL_MOD_ALIBI
    diff = w.q2 is not None
    epi = (fb.FL_EPI_RMSNORM if w.rmsnorm else 0) | (fb.FL_EPI_GATE_SIGMOID if w.gate is not None else 0)
    desc = fb.variant_desc(scale=float(w.scale), score_mod=mod, softcap=float(w.softcap or 0.0), mask=mask,
                           window=int(w.window or 0), prefix_len=int(w.prefix or 0), n_bias=len(w.biases),
                           combine=fb.FL_DIFFERENTIAL if diff else fb.FL_SINGLE, epilogue=epi,
                           rms_eps=float(w.rms_eps) if w.rmsnorm else 0.0, q_offset=int(getattr(w, "q_offset", 0) or 0))

    def dev(x, dt):
        t = None if x is None else to_device(np.asarray(x), dt, device)
        if t is not None:
            keep.append(t)
        return t

    slopes = dev(w.alibi, torch.float32)
    qd = dev(w.q_doc, torch.int32)
    kd = qd if (w.kv_doc is w.q_doc) else dev(w.kv_doc, torch.int32)
    biases = [dev(b, tdt) for b in w.biases]
    gate = dev(w.gate, tdt)
    q2, k2 = dev(w.q2, tdt), dev(w.k2, tdt)
    lam = dev(w.lam, torch.float32)
    rmsw = dev(None if w.rms_weight is None else np.asarray(w.rms_weight, np.float32), torch.float32)
    tq, tk, tv, tout = (fb.tensor_desc(x) for x in (q, k, v, out))
    ws = None
    nbytes = fb.fl_attn_fwd_workspace_size(tq, tk, desc)
    if nbytes:
        ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        keep.append(ws)
    need_aux = any(x is not None for x in (slopes, qd, gate, q2, lam, rmsw, ws)) or biases
    aux = fb.aux_desc(alibi_slopes=slopes, q_doc_ids=qd, kv_doc_ids=kd, biases=biases, gate=gate, q2=q2, k2=k2,
                      lambda_=lam, rms_weight=rmsw, workspace=ws) if need_aux else None
    lse = None
    tlse = None
    if want_lse:
        lse = torch.empty((B, 2 * G if diff else G, H, Sq, 1), dtype=torch.float32, device=device)
        tlse = fb.tensor_desc(lse)
    return DeviceWorkload(w.name, q, k, v, out, lse, desc, aux, keep, tq, tk, tv, tout, tlse)


def lse_to_oracle_layout(dw: DeviceWorkload) -> np.ndarray:
    """Device lse [B, G or 2G, H, Sq, 1] -> [B,G,H,Sq] or, for differential, [B,2,G,H,Sq]."""
    l = dw.lse.cpu().numpy()[..., 0]
    if dw.desc.combine == fb.FL_DIFFERENTIAL:
        B, G2, H, Sq = l.shape
        return l.reshape(B, G2 // 2, 2, H, Sq).transpose(0, 2, 1, 3, 4)
    return l


@dataclasses.dataclass
class DeviceBackward:
    """Device tensors of one fl_attn_bwd call on top of a forward DeviceWorkload (bf16 out + lse)."""
    fwd: DeviceWorkload
    dout: torch.Tensor
    dq: torch.Tensor
    dk: torch.Tensor
    dv: torch.Tensor
    aux: fb.fl_aux
    keep: List[torch.Tensor]
    tdout: fb.fl_tensor = None
    tdq: fb.fl_tensor = None
    tdk: fb.fl_tensor = None
    tdv: fb.fl_tensor = None

    def run(self, stream: int = 0) -> int:
        f = self.fwd
        return fb.fl_attn_bwd(f.tq, f.tk, f.tv, f.tout, self.tdout, f.tlse, f.desc, self.aux,
                              self.tdq, self.tdk, self.tdv, stream)

    def run_checked(self, stream: int = 0) -> None:
        fb.check(self.run(stream))


def upload_backward(w, dout: np.ndarray, grad_dtype: str = "f32", device="cuda:0") -> DeviceBackward:
    """Forward tensors (bf16 out, lse) plus dout, the gradient outputs and the backward workspace.
    The forward pass has to be run (fwd.run_checked()) before the backward call."""
    fwd = upload(w, out_dtype="bf16", device=device, want_lse=True)
    tdt = torch.bfloat16
    gdt = torch.float32 if grad_dtype == "f32" else tdt
    d_out = to_device(dout, tdt, device)
    dq = empty_like_layout(fwd.q, fwd.q.shape[4], gdt)
    dk = empty_like_layout(fwd.k, fwd.k.shape[4], gdt)
    dv = empty_like_layout(fwd.v, fwd.v.shape[4], gdt)
    nbytes = fb.fl_attn_bwd_workspace_size(fwd.tq, fwd.tk, fwd.desc)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
    keep = [ws] + list(fwd.keep)
    slopes = qd = kd = None
    # the aux tensors of the forward upload, by the order upload() appended them
    it = iter(fwd.keep)
    if w.alibi is not None:
        slopes = next(it)
    if w.q_doc is not None:
        qd = next(it)
        kd = qd if (w.kv_doc is w.q_doc) else next(it)
    aux = fb.aux_desc(alibi_slopes=slopes, q_doc_ids=qd, kv_doc_ids=kd, workspace=ws)
    return DeviceBackward(fwd, d_out, dq, dk, dv, aux, keep, fb.tensor_desc(d_out), fb.tensor_desc(dq),
                          fb.tensor_desc(dk), fb.tensor_desc(dv))


@dataclasses.dataclass
class DeviceBackwardEx:
    """Device tensors of one fl_attn_bwd_ex call: every gradient the variant has (dq, dk, dv, and dq2 / dk2 /
    dlambda, dbias, dgate, drms_weight where the workload has those inputs)."""
    fwd: DeviceWorkload
    dout: torch.Tensor
    grads: dict                          # name -> tensor (dbias: list)
    aux: fb.fl_aux
    extra: fb.fl_bwd_extra
    keep: List[torch.Tensor]
    tdout: fb.fl_tensor = None
    tdq: fb.fl_tensor = None
    tdk: fb.fl_tensor = None
    tdv: fb.fl_tensor = None

    def run(self, stream: int = 0) -> int:
        f = self.fwd
        return fb.fl_attn_bwd_ex(f.tq, f.tk, f.tv, f.tout, self.tdout, f.tlse, f.desc, self.aux,
                                 self.tdq, self.tdk, self.tdv, self.extra, stream)

    def run_checked(self, stream: int = 0) -> None:
        fb.check(self.run(stream))


def upload_backward_ex(w, dout: np.ndarray, grad_dtype: str = "f32", device="cuda:0") -> DeviceBackwardEx:
    """upload_backward for any variant: the forward upload's aux block (biases, gate, second stream, lambda, ...)
    with the backward workspace, plus every gradient output.  Run fwd.run_checked() first."""
    fwd = upload(w, out_dtype="bf16", device=device, want_lse=True)
    tdt = torch.bfloat16
    gdt = torch.float32 if grad_dtype == "f32" else tdt
    d_out = to_device(dout, tdt, device)
    g = dict(dq=empty_like_layout(fwd.q, fwd.q.shape[4], gdt), dk=empty_like_layout(fwd.k, fwd.k.shape[4], gdt),
             dv=empty_like_layout(fwd.v, fwd.v.shape[4], gdt))
    # the aux tensors of the forward upload, by the order upload() appended them
    it = iter(fwd.keep)
    slopes = next(it) if w.alibi is not None else None
    qd = kd = None
    if w.q_doc is not None:
        qd = next(it)
        kd = qd if (w.kv_doc is w.q_doc) else next(it)
    biases = [next(it) for _ in w.biases]
    gate = next(it) if w.gate is not None else None
    q2 = k2 = lam = None
    if w.q2 is not None:
        q2, k2, lam = next(it), next(it), next(it)
    rmsw = next(it) if w.rms_weight is not None else None
    nbytes = fb.fl_attn_bwd_ex_workspace_size(fwd.tq, fwd.tk, fwd.tv, fwd.desc)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
    aux = fb.aux_desc(alibi_slopes=slopes, q_doc_ids=qd, kv_doc_ids=kd, biases=biases, gate=gate, q2=q2, k2=k2,
                      lambda_=lam, rms_weight=rmsw, workspace=ws)
    if q2 is not None:
        g["dq2"], g["dk2"] = empty_like_layout(q2, q2.shape[4], gdt), empty_like_layout(k2, k2.shape[4], gdt)
        g["dlambda"] = torch.empty(q2.shape[2], dtype=torch.float32, device=device)
    if gate is not None:
        g["dgate"] = empty_like_layout(gate, gate.shape[4], gdt)
    if biases:
        g["dbias"] = [torch.empty(tuple(b.shape), dtype=torch.float32, device=device) for b in biases]
    if w.rmsnorm:
        g["drms_weight"] = torch.empty(w.v.shape[4], dtype=torch.float32, device=device)
    extra = fb.bwd_extra(dq2=g.get("dq2"), dk2=g.get("dk2"), dbias=g.get("dbias", ()), dgate=g.get("dgate"),
                         dlambda=g.get("dlambda"), drms_weight=g.get("drms_weight"))
    return DeviceBackwardEx(fwd, d_out, g, aux, extra, [ws] + list(fwd.keep), fb.tensor_desc(d_out), fb.tensor_desc(g["dq"]),
                            fb.tensor_desc(g["dk"]), fb.tensor_desc(g["dv"]))


@dataclasses.dataclass
class DeviceDecode:
    """Device tensors of one fl_attn_decode call (an inputs.DecodeWorkload)."""
    q: torch.Tensor
    k_cache: torch.Tensor
    v_cache: torch.Tensor
    out: torch.Tensor
    lse: torch.Tensor
    desc: fb.fl_variant_desc
    kv: fb.fl_paged_kv
    aux: fb.fl_aux
    keep: List[torch.Tensor]
    tq: fb.fl_tensor = None
    tk: fb.fl_tensor = None
    tv: fb.fl_tensor = None
    tout: fb.fl_tensor = None
    tlse: fb.fl_tensor = None

    def run(self, stream: int = 0) -> int:
        return fb.fl_attn_decode(self.tq, self.tk, self.tv, self.kv, self.desc, self.aux, self.tout, self.tlse, stream)

    def run_checked(self, stream: int = 0) -> None:
        fb.check(self.run(stream))


def upload_decode(w, out_dtype: str = "f32", device="cuda:0", paged: bool = True) -> DeviceDecode:
    """Cache stored [pages, page_size, Hkv, D] (the serving layout) and viewed [pages, 1, Hkv, page_size, D];
    paged=False passes no block table (the workload's table must then be the identity)."""
    tdt = torch.bfloat16
    q = torch.from_numpy(np.ascontiguousarray(w.q)).to(device, tdt)[:, None, :, None, :]       # [B, 1, H, 1, D]
    kc = torch.from_numpy(np.ascontiguousarray(w.k_cache)).to(device, tdt).permute(0, 2, 1, 3)[:, None]
    vc = torch.from_numpy(np.ascontiguousarray(w.v_cache)).to(device, tdt).permute(0, 2, 1, 3)[:, None]
    B, _, H, _, D = q.shape
    out = torch.empty((B, 1, H, 1, D), dtype=torch.float32 if out_dtype == "f32" else tdt, device=device)
    lse = torch.empty((B, 1, H, 1, 1), dtype=torch.float32, device=device)
    table = torch.from_numpy(w.block_table).to(device) if paged else None
    lens = torch.from_numpy(w.seq_lens).to(device)
    mod = fb.FL_MOD_SOFTCAP if w.softcap is not None else (fb.FL_MOD_ALIBI if w.alibi is not None else fb.FL_MOD_NONE)
    desc = fb.variant_desc(scale=float(w.scale), score_mod=mod, softcap=float(w.softcap or 0.0),
                           mask=(fb.FL_MASK_WINDOW | fb.FL_MASK_CAUSAL) if w.window is not None else fb.FL_MASK_CAUSAL,
                           window=int(w.window or 0))
    kv = fb.paged_kv(block_table=table, page_size=w.k_cache.shape[1], seq_lens=lens,
                     max_seq_len=int(w.seq_lens.max()) if len(w.seq_lens) else 0)
    tq, tk, tv, tout, tlse = (fb.tensor_desc(x) for x in (q, kc, vc, out, lse))
    ws = torch.empty(max(fb.fl_attn_decode_workspace_size(tq, tk, kv), 16), dtype=torch.uint8, device=device)
    slopes = None if w.alibi is None else torch.from_numpy(np.asarray(w.alibi, np.float32)).to(device)
    aux = fb.aux_desc(alibi_slopes=slopes, workspace=ws)
    return DeviceDecode(q, kc, vc, out, lse, desc, kv, aux, [table, lens, ws, slopes], tq, tk, tv, tout, tlse)


@dataclasses.dataclass
class DevicePrefill(DeviceDecode):
    """Device tensors of one fl_attn_prefill_paged call (an inputs.DecodeWorkload whose q is [B, H, Sq, D])."""

    def run(self, stream: int = 0) -> int:
        return fb.fl_attn_prefill_paged(self.tq, self.tk, self.tv, self.kv, self.desc, self.aux, self.tout, self.tlse, stream)


def upload_prefill_paged(w, out_dtype: str = "f32", device="cuda:0", paged: bool = True, max_seq_len=None) -> DevicePrefill:
    """Cache stored and viewed as in upload_decode; q [B, H, Sq, D] viewed [B, 1, H, Sq, D]."""
    tdt = torch.bfloat16
    q = torch.from_numpy(np.ascontiguousarray(w.q)).to(device, tdt)[:, None]                   # [B, 1, H, Sq, D]
    kc = torch.from_numpy(np.ascontiguousarray(w.k_cache)).to(device, tdt).permute(0, 2, 1, 3)[:, None]
    vc = torch.from_numpy(np.ascontiguousarray(w.v_cache)).to(device, tdt).permute(0, 2, 1, 3)[:, None]
    B, _, H, Sq, D = q.shape
    out = torch.empty((B, 1, H, Sq, D), dtype=torch.float32 if out_dtype == "f32" else tdt, device=device)
    lse = torch.empty((B, 1, H, Sq, 1), dtype=torch.float32, device=device)
    table = torch.from_numpy(w.block_table).to(device) if paged else None
    lens = torch.from_numpy(w.seq_lens).to(device)
    mod = fb.FL_MOD_SOFTCAP if w.softcap is not None else (fb.FL_MOD_ALIBI if w.alibi is not None else fb.FL_MOD_NONE)
    desc = fb.variant_desc(scale=float(w.scale), score_mod=mod, softcap=float(w.softcap or 0.0),
                           mask=(fb.FL_MASK_WINDOW | fb.FL_MASK_CAUSAL) if w.window is not None else fb.FL_MASK_CAUSAL,
                           window=int(w.window or 0))
    if max_seq_len is None:
        max_seq_len = int(w.seq_lens.max()) if len(w.seq_lens) else 0
    kv = fb.paged_kv(block_table=table, page_size=w.k_cache.shape[1], seq_lens=lens, max_seq_len=max_seq_len)
    tq, tk, tv, tout, tlse = (fb.tensor_desc(x) for x in (q, kc, vc, out, lse))
    ws = torch.empty(max(fb.fl_attn_prefill_paged_workspace_size(tq, tk, kv), 16), dtype=torch.uint8, device=device)
    slopes = None if w.alibi is None else torch.from_numpy(np.asarray(w.alibi, np.float32)).to(device)
    aux = fb.aux_desc(alibi_slopes=slopes, workspace=ws)
    return DevicePrefill(q, kc, vc, out, lse, desc, kv, aux, [table, lens, ws, slopes], tq, tk, tv, tout, tlse)
