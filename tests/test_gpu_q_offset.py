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


def test_offset_is_validated_and_refused_where_not_built():
    w = inputs.causal_bf16(B=1, H=2, S=64, D=64)
    dw = runner.upload(w)
    bad = fb.variant_desc(scale=w.scale, mask=fb.FL_MASK_CAUSAL, q_offset=-1)
    assert fb.fl_attn_fwd(dw.tq, dw.tk, dw.tv, bad, None, dw.tout, dw.tlse) == fb.FL_ERR_DESC
    off = fb.variant_desc(scale=w.scale, mask=fb.FL_MASK_CAUSAL, q_offset=5)
    assert not fb.fl_bwd_supported(off, fb.FL_BF16, 64, 64)
