"""Host-side validation under random descriptors (CPU only, skipped where a GPU is present: the
pointers are fake, so a case that passed validation would launch on them).  Every call must come back
with a status code and a detail string; a case that passes validation ends in FL_ERR_LAUNCH here."""
import numpy as np
import pytest

from paper_2511_02043_amd import binding as fb


def _gpu_present():
    import torch
    return torch.cuda.is_available()


def _tensor(dtype, sizes):
    t = fb.fl_tensor()
    t.ptr, t.dtype = 0x7f0000001000, dtype
    t.size[:] = sizes
    st, acc = [0] * 5, 1
    for a in range(4, -1, -1):
        st[a] = acc
        acc *= max(int(sizes[a]), 1)
    t.stride[:] = st
    return t


@pytest.mark.skipif(_gpu_present(), reason="fake pointers: host validation only, must not reach a GPU")
def test_random_descriptors_never_crash_the_host():
    """A valid call (causal bf16, grouped heads, ragged sizes) with one to three random fields broken."""
    rng = np.random.Generator(np.random.PCG64(20251102043))
    L = fb.lib()
    seen = set()
    for case in range(600):
        B, G, H, Hkv, Sq, Sk, D = 2, 1, 4, 2, 300, 257, 64
        dt = fb.FL_BF16
        kw = dict(scale=0.125, score_mod=fb.FL_MOD_NONE, softcap=0.0, mask=fb.FL_MASK_CAUSAL, window=0, prefix_len=0,
                  n_bias=0, combine=0, epilogue=0)
        muts = rng.choice(26, size=int(rng.integers(0, 4)), replace=False)
        if 0 in muts: Sq = int(rng.choice([0, 1, 1 << 31]))
        if 1 in muts: Sk = int(rng.choice([0, 1, 1 << 31]))
        if 2 in muts: D = int(rng.choice([0, 16, 96, 128, 256]))
        if 3 in muts: Hkv = int(rng.choice([0, 3, 4]))
        if 4 in muts: dt = int(rng.choice([fb.FL_F32, 7]))
        if 5 in muts: kw["scale"] = float(rng.choice([0.0, -1.0, float("nan")]))
        if 6 in muts: kw["score_mod"] = int(rng.integers(1, 5))
        if 7 in muts: kw["mask"] = int(rng.integers(0, 40))
        if 8 in muts: kw["window"] = -1
        if 9 in muts: kw["n_bias"] = int(rng.integers(1, 4))
        if 10 in muts: kw["combine"] = int(rng.integers(1, 3))
        if 11 in muts: kw["epilogue"] = int(rng.integers(1, 9))
        if 12 in muts: B = 0
        q, k = _tensor(dt, [B, G, H, Sq, D]), _tensor(dt, [B, G, Hkv, Sk, D])
        v, out = _tensor(dt, [B, G, Hkv, Sk, D]), _tensor(dt, [B, G, H, Sq, D])
        lse = _tensor(fb.FL_F32, [B, G, H, Sq, 1])
        if 13 in muts: q.ptr = 0
        if 14 in muts: k.ptr = 0x7f0000001008
        if 15 in muts: v.stride[3] = int(rng.choice([-64, 0, 3, 1 << 24]))
        if 16 in muts: out.stride[4] = 2
        if 17 in muts: out.dtype = fb.FL_F32
        if 18 in muts: v.size[4] = 128
        if 19 in muts: lse.size[3] = Sq + 1
        if 20 in muts: lse.dtype = fb.FL_BF16
        d = fb.variant_desc(**kw)
        a = fb.fl_aux()
        a.struct_size = fb.C.sizeof(fb.fl_aux)
        a.workspace, a.workspace_bytes = 0x7f0000100000, 1 << 30
        a.alibi_slopes = a.q_doc_ids = a.kv_doc_ids = 0x7f0000200000
        if 21 in muts: a.struct_size = 3
        if 22 in muts: a.workspace_bytes = 16
        if 23 in muts: a.workspace = 0
        if 24 in muts: a.alibi_slopes = a.q_doc_ids = 0
        aux = None if 25 in muts else a
        for status in (fb.fl_attn_fwd(q, k, v, d, aux, out, lse), fb.fl_attn_bwd(q, k, v, out, out, lse, d, aux, q, k, v)):
            assert isinstance(status, int) and 0 <= status <= fb.FL_ERR_DESC, status
            assert isinstance(fb.fl_strerror(status), str) and isinstance(fb.fl_last_error_detail(), str)
            seen.add(status)
        assert L.fl_attn_fwd_workspace_size(fb.C.byref(q), fb.C.byref(k), fb.C.byref(d)) >= 0
        assert L.fl_attn_bwd_workspace_size(fb.C.byref(q), fb.C.byref(k), fb.C.byref(d)) >= 0
    # the mutations reach every kind of outcome: a valid call ends in FL_ERR_LAUNCH here (no device), an empty one in FL_OK
    assert seen >= {fb.FL_OK, fb.FL_ERR_NULL, fb.FL_ERR_DTYPE, fb.FL_ERR_SHAPE, fb.FL_ERR_STRIDE, fb.FL_ERR_ALIGN,
                    fb.FL_ERR_UNSUPPORTED, fb.FL_ERR_AUX_MISSING, fb.FL_ERR_WORKSPACE, fb.FL_ERR_LAUNCH, fb.FL_ERR_DESC}, seen


@pytest.mark.skipif(_gpu_present(), reason="fake pointers: host validation only, must not reach a GPU")
def test_random_paged_calls_never_crash_the_host():
    """The two entry points over a paged cache (one query row per sequence, a chunk of rows per sequence): a valid call
    with one to three random fields of the tensors, the page description or the descriptor broken."""
    rng = np.random.Generator(np.random.PCG64(20251102044))
    seen = {"decode": set(), "prefill": set()}
    for case in range(400):
        B, H, Hkv, Sq, D, pages, page_size, max_len, stride = 3, 8, 2, 1100, 128, 50, 16, 200, 13     # (a chunk long enough for the path with a workspace)
        kw = dict(scale=0.0884, score_mod=fb.FL_MOD_NONE, softcap=0.0, mask=fb.FL_MASK_CAUSAL, window=0)
        muts = rng.choice(22, size=int(rng.integers(0, 4)), replace=False)
        if 0 in muts: B = 0
        if 1 in muts: Hkv = int(rng.choice([0, 3, 16]))
        if 2 in muts: D = int(rng.choice([0, 8, 96, 256]))
        if 3 in muts: page_size = int(rng.choice([0, 4, 12, 1 << 20]))
        if 4 in muts: max_len = int(rng.choice([-1, 0, 1 << 30]))
        if 5 in muts: stride = int(rng.choice([0, 1, -5]))
        if 6 in muts: pages = int(rng.choice([0, 1, 1 << 33]))
        if 7 in muts: kw["mask"] = int(rng.integers(0, 40))
        if 8 in muts: kw["score_mod"] = int(rng.integers(1, 5))
        if 9 in muts: kw["scale"] = float(rng.choice([0.0, float("inf")]))
        if 10 in muts: Sq = int(rng.choice([0, 1, 1 << 31]))
        q1, qc = _tensor(fb.FL_BF16, [B, 1, H, 1, D]), _tensor(fb.FL_BF16, [B, 1, H, Sq, D])
        kc, vc = _tensor(fb.FL_BF16, [pages, 1, Hkv, page_size, D]), _tensor(fb.FL_BF16, [pages, 1, Hkv, page_size, D])
        o1, oc = _tensor(fb.FL_BF16, [B, 1, H, 1, D]), _tensor(fb.FL_BF16, [B, 1, H, Sq, D])
        l1, lc = _tensor(fb.FL_F32, [B, 1, H, 1, 1]), _tensor(fb.FL_F32, [B, 1, H, Sq, 1])
        if 11 in muts: kc.ptr = 0
        if 12 in muts: vc.stride[3] = int(rng.choice([-8, 3]))
        if 13 in muts: q1.dtype = qc.dtype = fb.FL_F32
        if 14 in muts: o1.dtype = oc.dtype = 9
        if 15 in muts: l1.size[2] = lc.size[2] = H + 1
        kv = fb.fl_paged_kv()
        kv.struct_size = fb.C.sizeof(fb.fl_paged_kv)
        kv.block_table, kv.seq_lens = 0x7f0000300000, 0x7f0000400000
        kv.table_stride, kv.page_size, kv.max_seq_len = stride, page_size, max_len
        if 16 in muts: kv.struct_size = 5
        if 17 in muts: kv.block_table = 0
        if 18 in muts: kv.seq_lens = 0
        d = fb.variant_desc(**kw)
        a = fb.fl_aux()
        a.struct_size = fb.C.sizeof(fb.fl_aux)
        a.workspace, a.workspace_bytes, a.alibi_slopes = 0x7f0000100000, 1 << 34, 0x7f0000200000
        if 19 in muts: a.workspace_bytes = 64
        if 20 in muts: a.workspace = 0x7f0000100004
        aux = None if 21 in muts else a
        for name, status in (("decode", fb.fl_attn_decode(q1, kc, vc, kv, d, aux, o1, l1)),
                             ("prefill", fb.fl_attn_prefill_paged(qc, kc, vc, kv, d, aux, oc, lc))):
            assert isinstance(status, int) and 0 <= status <= fb.FL_ERR_DESC, (name, status)
            assert isinstance(fb.fl_last_error_detail(), str)
            seen[name].add(status)
        assert fb.fl_attn_decode_workspace_size(q1, kc, kv) >= 0 and fb.fl_attn_prefill_paged_workspace_size(qc, kc, kv) >= 0
    for name in seen:
        assert seen[name] >= {fb.FL_OK, fb.FL_ERR_NULL, fb.FL_ERR_DTYPE, fb.FL_ERR_SHAPE, fb.FL_ERR_UNSUPPORTED, fb.FL_ERR_AUX_MISSING,
                              fb.FL_ERR_WORKSPACE, fb.FL_ERR_LAUNCH, fb.FL_ERR_DESC}, (name, seen[name])
