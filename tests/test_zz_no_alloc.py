"""fl_attn_fwd_noalloc (the forward entry point for callers that cannot allocate device memory: the tile
skipper's document-id summaries live in a buffer built into the library) against fl_attn_fwd with a
caller-supplied workspace, through the C-ABI.  Both run the same kernels on the same inputs, so the bar
is bit equality of out and lse; the calls come two in a row, the second on a smaller input, so that
whatever the first call left in the shared buffer has to be harmless."""
import numpy as np
import pytest

from paper_2511_02043_amd import binding as fb
from paper_2511_02043_amd import inputs, runner

pytestmark = pytest.mark.gpu


def both_ways(w):
    import torch
    dw = runner.upload(w, out_dtype="f32")
    assert fb.fl_attn_fwd_workspace_size(dw.tq, dw.tk, dw.desc) > 0
    dw.out.fill_(float("nan"))
    dw.lse.fill_(float("nan"))
    dw.run_checked()
    torch.cuda.synchronize()
    ref, ref_lse = dw.out.clone(), dw.lse.clone()
    dw.out.fill_(float("nan"))
    dw.lse.fill_(float("nan"))
    dw.aux.workspace = None                         # the new entry point must not need it
    dw.aux.workspace_bytes = 0
    fb.check(fb.fl_attn_fwd_noalloc(dw.tq, dw.tk, dw.tv, dw.desc, dw.aux, dw.tout, dw.tlse))
    torch.cuda.synchronize()
    return (ref.cpu().numpy(), ref_lse.cpu().numpy()), (dw.out.cpu().numpy(), dw.lse.cpu().numpy())


def test_two_calls_in_a_row_second_smaller():
    big = inputs.window_doc_bf16(B=2, H=4, S=1500, D=64, window=300, lo=40, hi=400)
    small = inputs.grid_bf16("document_mask", 384, B=1, H=2, n_docs=5)
    for w in (big, small):
        (ref, ref_lse), (got, got_lse) = both_ways(w)
        assert np.all(np.isfinite(got))
        assert np.array_equal(got, ref), w.name
        assert np.array_equal(got_lse, ref_lse), w.name


def test_variant_without_scratch_and_size_limit():
    import torch
    # no document mask: no scratch, same result as fl_attn_fwd
    w = inputs.causal_bf16(B=1, H=2, S=200, D=128)
    dw = runner.upload(w, out_dtype="f32")
    dw.run_checked()
    torch.cuda.synchronize()
    ref = dw.out.clone()
    dw.out.zero_()
    fb.check(fb.fl_attn_fwd_noalloc(dw.tq, dw.tk, dw.tv, dw.desc, dw.aux, dw.tout, dw.tlse))
    torch.cuda.synchronize()
    assert torch.equal(dw.out, ref)
    # beyond the built-in buffer: a clear error, nothing launched (sizes only; the pointers are never used)
    d = fb.variant_desc(scale=0.125, mask=fb.FL_MASK_DOC)
    t = fb.fl_tensor()
    t.ptr = 4096
    t.dtype = fb.FL_BF16
    t.size[:] = [64, 1, 1, 1 << 20, 64]
    t.stride[:] = [1 << 26, 1 << 26, 1 << 26, 64, 1]
    aux = fb.aux_desc()
    assert fb.fl_attn_fwd_noalloc(t, t, t, d, aux, t, None) == fb.FL_ERR_WORKSPACE
    assert "scratch" in fb.fl_last_error_detail()
