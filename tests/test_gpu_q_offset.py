"""Query-position offset (descriptor field q_offset): query row i sits at sequence position i + q_offset,
so causal / sliding-window / PrefixLM masks and ALiBi are aligned bottom-right when a chunk of new queries
runs against a longer key/value sequence -- the prefill-in-chunks shape of the serving experiment in
Sec. 4.1.  Element by element against the oracle (which takes the same positions), for chunks of 1, 17,
128 and 500 queries against 4k - 8k keys, both head dims, bf16 and fp32 storage, grouped heads."""
import dataclasses

import numpy as np
import pytest

from paper_2511_02043_amd import binding as fb
from paper_2511_02043_amd import inputs, runner
from tests.gpu_util import run_and_compare

pytestmark = pytest.mark.gpu


def chunk(kind, Sq, Sk, D, off=None, Hkv=None, H=4, B=2):
    w = inputs.causal_bf16(B=B, H=H, Hkv=Hkv, S=Sq, Sk=Sk, D=D, causal=kind in ("causal", "alibi_causal", "doc_causal"))
    w.q_offset = Sk - Sq if off is None else off
    w.name = f"{kind}_chunk{Sq}_of_{Sk}_d{D}"
    if kind == "window":
        w.causal, w.window = True, 700
    elif kind == "prefix":
        w.prefix = Sk - Sq // 2 - 100
    elif kind == "alibi_causal":
        w.alibi = inputs.alibi_slopes(H)
    elif kind == "doc_causal":
        ids = inputs.doc_ids(B, Sk, seed=31, lo=200, hi=1500)
        w.kv_doc = ids
        w.q_doc = np.ascontiguousarray(ids[:, w.q_offset:w.q_offset + Sq])
    return w


@pytest.mark.parametrize("Sq", [1, 17, 128, 500])
@pytest.mark.parametrize("kind", ["causal", "window", "prefix", "alibi_causal", "doc_causal"])
def test_chunk_against_longer_cache(kind, Sq):
    D = 128 if Sq in (17, 500) else 64
    Sk = 4096 + 37 if Sq in (1, 128) else 8192 - 91
    run_and_compare(chunk(kind, Sq, Sk, D, Hkv=2 if Sq == 128 else None))


def test_offset_in_the_middle_and_fp32_storage():
    # a chunk that is not the last one: keys beyond its positions are hidden, the tile skipper has to stop early
    run_and_compare(chunk("causal", 300, 5000, 128, off=1234))
    run_and_compare(chunk("window", 300, 5000, 64, off=2222))
    w = chunk("causal", 70, 333, 64, H=2, B=1)
    wf = dataclasses.replace(w, dtype="f32", q=w.q.astype(np.float32), k=w.k.astype(np.float32), v=w.v.astype(np.float32))
    run_and_compare(wf)


def test_chunks_reassemble_the_square_problem():
    """Causal attention over S keys computed in three chunks of query rows equals the one-call result row by row
    (same kernels, same key order per row: bit-equal where the chunk boundaries fall on the q-tile grid)."""
    import torch
    S, D = 1536, 128
    w = inputs.causal_bf16(B=1, H=8, S=S, D=D)
    dw = runner.upload(w, out_dtype="f32")
    dw.run_checked()
    torch.cuda.synchronize()
    whole, whole_lse = dw.out.clone(), dw.lse.clone()
    got = torch.full_like(whole, float("nan"))
    got_lse = torch.full_like(whole_lse, float("nan"))
    for lo, hi in ((0, 512), (512, 1024), (1024, 1536)):
        q = dw.q[:, :, :, lo:hi]
        out = got[:, :, :, lo:hi]
        lse = got_lse[:, :, :, lo:hi]
        desc = fb.variant_desc(scale=w.scale, mask=fb.FL_MASK_CAUSAL, q_offset=lo)
        fb.check(fb.fl_attn_fwd(fb.tensor_desc(q), dw.tk, dw.tv, desc, None, fb.tensor_desc(out), fb.tensor_desc(lse)))
    torch.cuda.synchronize()
    assert torch.equal(got, whole) and torch.equal(got_lse, whole_lse)


def test_offset_is_validated():
    w = inputs.causal_bf16(B=1, H=2, S=64, D=64)
    dw = runner.upload(w)
    bad = fb.variant_desc(scale=w.scale, mask=fb.FL_MASK_CAUSAL, q_offset=-1)
    assert fb.fl_attn_fwd(dw.tq, dw.tk, dw.tv, bad, None, dw.tout, dw.tlse) == fb.FL_ERR_DESC
    off = fb.variant_desc(scale=w.scale, mask=fb.FL_MASK_CAUSAL, q_offset=5)
    assert fb.fl_bwd_supported(off, fb.FL_BF16, 64, 64)
    kv = fb.paged_kv(page_size=64, seq_lens=dw.q.new_zeros(1, dtype=__import__("torch").int32), max_seq_len=64)
    assert fb.fl_attn_decode(dw.tq, dw.tk, dw.tv, kv, off, None, dw.tout, None) == fb.FL_ERR_UNSUPPORTED


@pytest.mark.parametrize("kind,Sq,Sk,D", [("causal", 130, 700, 64), ("window", 300, 4096 + 37, 64), ("prefix", 200, 900, 128),
                                           ("alibi_causal", 77, 500, 64), ("doc_causal", 256, 2000, 128), ("causal", 500, 8192 - 91, 128)])
def test_backward_with_offset(kind, Sq, Sk, D):
    """Gradients of a chunk of queries against a longer key sequence (bottom-right aligned masks): dq, dk, dv against the
    backward oracle with the same positions; keys beyond the chunk's positions get exactly zero."""
    import torch
    from oracle import attention_backward_oracle as bo
    w = chunk(kind, Sq, Sk, D, H=4, Hkv=2 if kind == "causal" else None, B=1)
    if kind == "window":
        w.window = 300
    dout = inputs.dout_for(w)
    db = runner.upload_backward(w, dout, grad_dtype="f32")
    db.fwd.run_checked()
    for t in (db.dq, db.dk, db.dv):
        t.fill_(float("nan"))
    db.run_checked()
    torch.cuda.synchronize()
    ref = bo.run_workload_backward(w, dout)
    for name, t, r in zip(("dq", "dk", "dv"), (db.dq, db.dk, db.dv), ref):
        g = t.float().cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(g)), name
        diff = g - r
        rel = float(np.sqrt(np.sum(diff * diff) / np.sum(r * r)))
        print(f"{w.name} {name}: rel_l2={rel:.3e}", flush=True)
        assert rel <= 5e-3, (name, rel)
        assert np.all(np.abs(diff) <= 1e-2 * float(np.max(np.abs(r))))


def test_backward_ex_with_offset():
    """The composed backward pass (gate + second stream here) takes the offset as well."""
    import torch
    from oracle import attention_backward_oracle as bo
    w = inputs.combination_bf16(D=64, pos_mask="causal", diff=True, gate=True, S=90, Sk=333, B=1, H=2)
    w.q_offset = 333 - 90
    dout = inputs.dout_for(w)
    db = runner.upload_backward_ex(w, dout)
    db.fwd.run_checked()
    db.run_checked()
    torch.cuda.synchronize()
    ref = bo.variant_backward(w, dout)
    for name in ("dq", "dk", "dv", "dq2", "dk2", "dgate", "dlambda"):
        g = db.grads[name].float().cpu().numpy().astype(np.float64)
        diff = g - ref[name]
        rel = float(np.sqrt(np.sum(diff * diff) / np.sum(ref[name] ** 2)))
        print(f"offset + diff + gate {name}: rel_l2={rel:.3e}", flush=True)
        assert rel <= 5e-3, (name, rel)


@pytest.mark.parametrize("kind", ["causal", "window", "alibi_causal", "prefix"])
def test_short_chunks_of_grouped_heads_pack_a_kv_heads_query_heads(kind):
    """Fewer than 128 query rows of grouped heads against 1024 keys or more: the query heads of a kv head share a workgroup
    (kernel shapes instantiated on first use).  Element by element against the oracle, and against the call with packing
    switched off (which may run another tile shape, so equal up to the rounding order: 2e-3); head groups of 2, 4 and 8,
    both head dims."""
    import torch
    for Sq, Sk, D, H, Hkv in ((64, 1500, 128, 8, 2), (20, 2100, 64, 8, 1), (33, 1024, 128, 4, 2), (96, 1300, 128, 8, 2)):
        w = chunk(kind, Sq, Sk, D, H=H, Hkv=Hkv, B=2)
        w.name += f"_h{H}_kv{Hkv}_packed"
        run_and_compare(w)
        outs = []
        for pack_off in (0, 1):
            fb.check(fb.fl_set_tuning("prefill_pack", pack_off))
            try:
                dw = runner.upload(w, out_dtype="f32")
                dw.out.fill_(float("nan"))
                dw.run_checked()
                torch.cuda.synchronize()
                outs.append((dw.out.clone(), dw.lse.clone()))
            finally:
                fb.fl_set_tuning("prefill_pack", 0)
        assert float((outs[0][0] - outs[1][0]).abs().max()) <= 2e-3 and float((outs[0][1] - outs[1][1]).abs().max()) <= 1e-4, w.name
