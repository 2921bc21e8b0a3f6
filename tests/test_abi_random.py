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
