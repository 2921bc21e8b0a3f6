"""GPU parity of fl_attn_decode (through the C-ABI) against the fp64 decode oracle.

Tolerance: the forward pass's (bf16 inputs, bf16 probabilities into an fp32-accumulating
contraction): max-abs <= 1e-2 on fp32 outputs, lse <= 1e-3."""
import numpy as np
import pytest

from oracle import decode_oracle as do
from paper_2511_02043_amd import inputs, runner

pytestmark = pytest.mark.gpu


def run(w, out_dtype="f32", paged=True):
    import torch
    dd = runner.upload_decode(w, out_dtype=out_dtype, paged=paged)
    dd.out.fill_(float("nan"))
    dd.lse.fill_(float("nan"))
    dd.run_checked()
    torch.cuda.synchronize()
    return dd.out.float().cpu().numpy()[:, 0, :, 0], dd.lse.cpu().numpy()[:, 0, :, 0, 0]


def compare(w, label, out_dtype="f32", paged=True):
    got, got_lse = run(w, out_dtype, paged)
    ref, ref_lse = do.decode_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale,
                                       window=w.window, softcap_value=w.softcap, alibi_slopes=w.alibi)
    assert np.all(np.isfinite(got)), label
    err = float(np.max(np.abs(got - ref)))
    dead = np.isneginf(ref_lse)
    assert np.array_equal(np.isneginf(got_lse), dead), label
    le = float(np.max(np.abs(got_lse[~dead] - ref_lse[~dead]))) if np.any(~dead) else 0.0
    print(f"{label}: max_abs={err:.3e} lse={le:.3e}", flush=True)
    slack = 2.0 ** -8 * np.abs(ref) if out_dtype == "bf16" else 0.0
    assert np.all(np.abs(got - ref) <= 1e-2 + slack), (label, err)
    assert le <= 1e-3, (label, le)


CASES = {
    # ragged lengths around tile (32) and page boundaries, several splits' worth of keys, both head dims
    "gqa4_d128_p16": lambda: inputs.decode_bf16(H=8, Hkv=2, D=128, page_size=16, seq_lens=[1, 31, 32, 33, 500, 1027]),
    "gqa8_d64_p32": lambda: inputs.decode_bf16(H=16, Hkv=2, D=64, page_size=32, seq_lens=[7, 64, 65, 900, 2049]),
    "mha_d128_p8": lambda: inputs.decode_bf16(H=4, Hkv=4, D=128, page_size=8, seq_lens=[15, 16, 17, 300]),
    "gqa32_d64_p128": lambda: inputs.decode_bf16(H=32, Hkv=1, D=64, page_size=128, seq_lens=[129, 1000, 3]),
    "long_many_splits": lambda: inputs.decode_bf16(H=8, Hkv=1, D=128, page_size=16, seq_lens=[8191, 4097]),
    "empty_and_one": lambda: inputs.decode_bf16(H=4, Hkv=2, D=64, page_size=16, seq_lens=[0, 1, 0, 40]),
}


@pytest.mark.parametrize("name", list(CASES))
def test_decode_matches_oracle(name):
    compare(CASES[name](), name)


def test_decode_variants():
    w = inputs.decode_bf16(H=8, Hkv=2, D=128, page_size=16, seq_lens=[5, 100, 700, 1500], salt=1)
    w.window = 255
    compare(w, "window_255")
    w.window = 0
    compare(w, "window_0")
    w.window = None
    w.softcap = 2.0
    compare(w, "softcap")
    w.softcap = None
    w.alibi = inputs.alibi_slopes(8)
    compare(w, "alibi")
    w.window = 300
    compare(w, "alibi_window")


def test_decode_bf16_output_and_contiguous_cache():
    w = inputs.decode_bf16(H=8, Hkv=2, D=64, page_size=16, seq_lens=[33, 500, 77], salt=2)
    compare(w, "bf16_out", out_dtype="bf16")
    # no block table: sequence b is page b of a cache whose pages hold a whole sequence
    c = inputs.decode_bf16(H=8, Hkv=4, D=128, page_size=1024, seq_lens=[1000, 17, 513], salt=3, shuffle_pages=False,
                           spare_pages=0)
    assert np.array_equal(c.block_table[:, 0], np.arange(3))
    compare(c, "contiguous", paged=False)


def test_decode_is_reproducible_and_page_placement_does_not_matter():
    w = inputs.decode_bf16(H=8, Hkv=2, D=128, page_size=16, seq_lens=[100, 900, 2500], salt=4)
    a, la = run(w)
    b, lb = run(w)
    assert np.array_equal(a, b) and np.array_equal(la, lb)
    perm = np.random.Generator(np.random.PCG64(5)).permutation(w.k_cache.shape[0])
    inv = np.argsort(perm)
    import dataclasses
    w2 = dataclasses.replace(w, k_cache=w.k_cache[perm], v_cache=w.v_cache[perm], block_table=inv[w.block_table].astype(np.int32))
    c, lc = run(w2)
    assert np.array_equal(a, c) and np.array_equal(la, lc)


def test_decode_error_paths():
    from paper_2511_02043_amd import binding as fb
    w = inputs.decode_bf16(H=8, Hkv=2, D=128, page_size=16, seq_lens=[40, 50])
    dd = runner.upload_decode(w)
    bad = fb.variant_desc(scale=0.1, mask=fb.FL_MASK_DOC)
    assert fb.fl_attn_decode(dd.tq, dd.tk, dd.tv, dd.kv, bad, dd.aux, dd.tout, dd.tlse) == fb.FL_ERR_UNSUPPORTED
    assert fb.fl_attn_decode(dd.tq, dd.tk, dd.tv, dd.kv, dd.desc, None, dd.tout, dd.tlse) == fb.FL_ERR_AUX_MISSING
    small = fb.aux_desc(workspace=dd.keep[2][:16])
    assert fb.fl_attn_decode(dd.tq, dd.tk, dd.tv, dd.kv, dd.desc, small, dd.tout, dd.tlse) == fb.FL_ERR_WORKSPACE
    kv = fb.paged_kv(block_table=dd.keep[0], page_size=32, seq_lens=dd.keep[1], max_seq_len=50)
    assert fb.fl_attn_decode(dd.tq, dd.tk, dd.tv, kv, dd.desc, dd.aux, dd.tout, dd.tlse) == fb.FL_ERR_SHAPE


def test_decode_full_size_sampled():
    """The benchmark's decode workload (64 sequences of 4k-8k cached tokens, 32 query / 8 kv heads,
    D = 128, 16-token pages, shuffled placement) in the launch configuration bench.py times; three
    sequences (the shortest, the longest, one in between) are checked against the oracle on the
    cache contents read back from the device, and every output has to be finite."""
    import torch
    from paper_2511_02043_amd import binding as fb
    B, H, Hkv, D, ctx, ps = 64, 32, 8, 128, 8192, 16
    g = torch.Generator(device="cuda").manual_seed(7)
    rng = np.random.Generator(np.random.PCG64(7))
    lens = rng.integers(ctx // 2, ctx + 1, size=B).astype(np.int32)
    npg = (lens + ps - 1) // ps
    pool = rng.permutation(int(npg.sum())).astype(np.int32)
    table = np.zeros((B, int(npg.max())), dtype=np.int32)
    pos = 0
    for b in range(B):
        table[b, :npg[b]] = pool[pos:pos + npg[b]]
        pos += npg[b]
    dev = "cuda:0"
    kc = torch.randn((int(npg.sum()), ps, Hkv, D), generator=g, device=dev).to(torch.bfloat16)
    vc = torch.randn((int(npg.sum()), ps, Hkv, D), generator=g, device=dev).to(torch.bfloat16)
    q = torch.randn((B, H, D), generator=g, device=dev).to(torch.bfloat16)
    out = torch.full((B, 1, H, 1, D), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((B, 1, H, 1, 1), float("nan"), dtype=torch.float32, device=dev)
    t_table, t_lens = torch.from_numpy(table).to(dev), torch.from_numpy(lens).to(dev)
    tq, tout, tlse = fb.tensor_desc(q[:, None, :, None, :]), fb.tensor_desc(out), fb.tensor_desc(lse)
    tk, tv = fb.tensor_desc(kc.permute(0, 2, 1, 3)[:, None]), fb.tensor_desc(vc.permute(0, 2, 1, 3)[:, None])
    kv = fb.paged_kv(block_table=t_table, page_size=ps, seq_lens=t_lens, max_seq_len=int(lens.max()))
    desc = fb.variant_desc(scale=D ** -0.5, mask=fb.FL_MASK_CAUSAL)
    ws = torch.empty(fb.fl_attn_decode_workspace_size(tq, tk, kv), dtype=torch.uint8, device=dev)
    fb.check(fb.fl_attn_decode(tq, tk, tv, kv, desc, fb.aux_desc(workspace=ws), tout, tlse))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(lse).all())
    picks = [int(np.argmin(lens)), int(np.argmax(lens)), 17]
    for b in picks:
        pages = torch.from_numpy(table[b, :npg[b]].astype(np.int64)).to(dev)
        k_b = kc[pages].float().cpu().numpy()            # this sequence's pages, in logical order
        v_b = vc[pages].float().cpu().numpy()
        ident = np.arange(npg[b], dtype=np.int32)[None]
        ref, ref_lse = do.decode_attention(q[b:b + 1].float().cpu().numpy(), k_b, v_b, ident, lens[b:b + 1], scale=D ** -0.5)
        err = float(np.max(np.abs(out[b, 0, :, 0].cpu().numpy() - ref[0])))
        le = float(np.max(np.abs(lse[b, 0, :, 0, 0].cpu().numpy() - ref_lse[0])))
        print(f"decode full size, sequence {b} (len {lens[b]}): max_abs={err:.3e} lse={le:.3e}", flush=True)
        assert err <= 1e-2 and le <= 1e-3


def test_lengths_outside_the_host_bound_are_cut_to_it():
    """seq_lens is device data the host cannot check; a value beyond max_seq_len (or negative) must not
    walk past the block table: the kernel cuts it to [0, max_seq_len]."""
    import torch
    w = inputs.decode_bf16(H=8, Hkv=2, D=128, page_size=16, seq_lens=[100, 500, 37])
    dd = runner.upload_decode(w)                    # max_seq_len = 500, table 32 pages wide
    lens = dd.keep[1]
    lens.copy_(torch.tensor([100, 1 << 30, -5], dtype=torch.int32))
    dd.run_checked()
    torch.cuda.synchronize()
    got, got_lse = dd.out.float().cpu().numpy()[:, 0, :, 0], dd.lse.cpu().numpy()[:, 0, :, 0, 0]
    cut = np.array([100, 500, 0], dtype=np.int32)
    # sequence 1 owns 32 pages (500 tokens -> 32 pages of 16): all 500 positions of the cut length are its own
    ref, ref_lse = do.decode_attention(w.q, w.k_cache, w.v_cache, w.block_table, cut, scale=w.scale)
    assert np.max(np.abs(got - ref)) <= 1e-2
    assert np.all(np.isneginf(got_lse[2])) and np.all(got[2] == 0.0)
    assert np.max(np.abs(got_lse[:2] - ref_lse[:2])) <= 1e-3


def test_table_entries_outside_the_cache_are_cut_to_it():
    """A corrupt block table must not turn into a wild address: entries are cut to [0, pages)."""
    import torch
    w = inputs.decode_bf16(H=4, Hkv=2, D=64, page_size=16, seq_lens=[40, 90], shuffle_pages=False)
    n_pages = w.k_cache.shape[0]
    bad = w.block_table.copy()
    bad[0, 1], bad[1, 2] = 1 << 30, -7               # read as pages n_pages - 1 and 0
    cut = np.clip(bad, 0, n_pages - 1)
    dd = runner.upload_decode(w)
    dd.keep[0].copy_(torch.from_numpy(bad))
    dd.run_checked()
    torch.cuda.synchronize()
    got = dd.out.float().cpu().numpy()[:, 0, :, 0]
    ref, _ = do.decode_attention(w.q, w.k_cache, w.v_cache, cut, w.seq_lens, scale=w.scale)
    assert np.max(np.abs(got - ref)) <= 1e-2


def test_all_sequences_empty_without_table_columns():
    """max_seq_len = 0 with a block table that has no columns (table_stride = 0): no workgroup owns a
    tile, so nothing may be looked up in the table; every output is 0 and every lse is -inf."""
    import torch
    from paper_2511_02043_amd import binding as fb
    w = inputs.decode_bf16(H=4, Hkv=2, D=64, page_size=16, seq_lens=[0, 0, 0])
    dd = runner.upload_decode(w)
    empty_table = torch.empty((3, 0), dtype=torch.int32, device="cuda:0")
    kv = fb.paged_kv(block_table=dd.keep[0], page_size=16, seq_lens=dd.keep[1], max_seq_len=0)
    kv.block_table = empty_table.data_ptr() or dd.keep[0].data_ptr()   # a zero-size tensor may have no storage
    kv.table_stride = 0
    dd.out.fill_(float("nan"))
    dd.lse.fill_(float("nan"))
    fb.check(fb.fl_attn_decode(dd.tq, dd.tk, dd.tv, kv, dd.desc, dd.aux, dd.tout, dd.tlse))
    torch.cuda.synchronize()
    assert bool((dd.out == 0).all()) and bool(torch.isneginf(dd.lse).all())


def test_decode_of_several_rows():
    """fl_attn_decode on q [B, 1, H, T, D]: the T newest tokens of every sequence, causal among themselves (a speculative
    step's verification), against the oracle of a chunk of rows over the paged cache; more than 64 (row, head) pairs
    per kv head are refused."""
    import torch
    from paper_2511_02043_amd import binding as fb
    for H, Hkv, D, T in ((8, 2, 128, 4), (8, 2, 64, 16), (8, 8, 128, 33)):
        w = inputs.prefill_paged_bf16(H=H, Hkv=Hkv, D=D, Sq=T, page_size=16, seq_lens=[2, T, T + 1, 95, 1300, 4000], salt=50 + T)
        dd = runner.upload_prefill_paged(w)
        ws = torch.empty(fb.fl_attn_decode_workspace_size(dd.tq, dd.tk, dd.kv), dtype=torch.uint8, device="cuda:0")
        dd.out.fill_(float("nan"))
        dd.lse.fill_(float("nan"))
        fb.check(fb.fl_attn_decode(dd.tq, dd.tk, dd.tv, dd.kv, dd.desc, fb.aux_desc(workspace=ws), dd.tout, dd.tlse))
        torch.cuda.synchronize()
        got, got_lse = dd.out.cpu().numpy()[:, 0], dd.lse.cpu().numpy()[:, 0, :, :, 0]
        ref, ref_lse = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale)
        dead = np.isneginf(ref_lse)
        assert np.array_equal(np.isneginf(got_lse), dead) and np.all(got[dead] == 0.0)
        err = float(np.max(np.abs(got - ref)))
        le = float(np.max(np.abs(got_lse[~dead] - ref_lse[~dead])))
        print(f"decode H={H}/{Hkv} D={D} T={T}: max_abs={err:.3e} lse={le:.3e}", flush=True)
        assert err <= 1e-2 and le <= 1e-3
    w = inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=17, page_size=16, seq_lens=[100, 200], salt=60)
    dd = runner.upload_prefill_paged(w)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    assert fb.fl_attn_decode(dd.tq, dd.tk, dd.tv, dd.kv, dd.desc, fb.aux_desc(workspace=ws), dd.tout, dd.tlse) == fb.FL_ERR_SHAPE


@pytest.mark.parametrize("T", [8, 16])
def test_decode_of_several_rows_full_size_sampled(T):
    """The decode workload at full size (64 sequences of 4k-8k cached tokens, 32 / 8 heads, D = 128, 16-token pages) with
    the T newest rows of every sequence, through fl_attn_prefill_paged as `bench.py --prefill-chunk T --decode-batch 64`
    launches it (8 rows: the decode kernels; 16 rows: the in-place forward kernel with the four heads of a kv head
    packed into a workgroup, which such a launch fills the chip with); two sequences against the oracle, everything
    finite.  (fl_attn_decode itself with two column blocks: test_decode_of_several_rows, ..._random_shapes.)"""
    import torch
    from paper_2511_02043_amd import binding as fb
    B, H, Hkv, D, ctx, ps = 64, 32, 8, 128, 8192, 16
    g = torch.Generator(device="cuda").manual_seed(11 + T)
    rng = np.random.Generator(np.random.PCG64(11 + T))
    lens = rng.integers(ctx // 2, ctx + 1, size=B).astype(np.int32)
    npg = (lens + ps - 1) // ps
    pool = rng.permutation(int(npg.sum())).astype(np.int32)
    table = np.zeros((B, int(npg.max())), dtype=np.int32)
    pos = 0
    for b in range(B):
        table[b, :npg[b]] = pool[pos:pos + npg[b]]
        pos += npg[b]
    dev = "cuda:0"
    kc = torch.randn((int(npg.sum()), ps, Hkv, D), generator=g, device=dev).to(torch.bfloat16)
    vc = torch.randn((int(npg.sum()), ps, Hkv, D), generator=g, device=dev).to(torch.bfloat16)
    q = torch.randn((B, 1, H, T, D), generator=g, device=dev).to(torch.bfloat16)
    out = torch.full((B, 1, H, T, D), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((B, 1, H, T, 1), float("nan"), dtype=torch.float32, device=dev)
    t_table, t_lens = torch.from_numpy(table).to(dev), torch.from_numpy(lens).to(dev)
    tq, tout, tlse = fb.tensor_desc(q), fb.tensor_desc(out), fb.tensor_desc(lse)
    tk, tv = fb.tensor_desc(kc.permute(0, 2, 1, 3)[:, None]), fb.tensor_desc(vc.permute(0, 2, 1, 3)[:, None])
    kv = fb.paged_kv(block_table=t_table, page_size=ps, seq_lens=t_lens, max_seq_len=int(lens.max()))
    desc = fb.variant_desc(scale=D ** -0.5, mask=fb.FL_MASK_CAUSAL)
    need = fb.fl_attn_prefill_paged_workspace_size(tq, tk, kv)
    if T * (H // Hkv) <= 32:
        assert need == fb.fl_attn_decode_workspace_size(tq, tk, kv) > 0  # one column block: the decode kernels' route
    else:
        assert need == 0                                                 # two: this launch fills the chip with packed heads, in place
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    fb.check(fb.fl_attn_prefill_paged(tq, tk, tv, kv, desc, fb.aux_desc(workspace=ws), tout, tlse))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(lse).all())
    for b in (int(np.argmax(lens)), 23):
        pages = torch.from_numpy(table[b, :npg[b]].astype(np.int64)).to(dev)
        k_b = kc[pages].float().cpu().numpy()
        v_b = vc[pages].float().cpu().numpy()
        ident = np.arange(npg[b], dtype=np.int32)[None]
        ref, ref_lse = do.prefill_attention(q[b:b + 1, 0].float().cpu().numpy(), k_b, v_b, ident, lens[b:b + 1], scale=D ** -0.5)
        err = float(np.max(np.abs(out[b, 0].cpu().numpy() - ref[0])))
        le = float(np.max(np.abs(lse[b, 0, :, :, 0].cpu().numpy() - ref_lse[0])))
        print(f"decode of {T} rows at full size, sequence {b} (len {lens[b]}): max_abs={err:.3e} lse={le:.3e}", flush=True)
        assert err <= 1e-2 and le <= 1e-3


def test_decode_of_several_rows_random_shapes():
    """Thirty seeded random shapes of the several-row decode step: head groups of 1 ... 16, 1 ... 64 (row, head) pairs per
    kv head (one and two column blocks, partly filled), both head dims, page sizes 8 ... 64, windows, soft-cap, ALiBi,
    lengths from below the row count to a few key-range splits; every output against the oracle."""
    import torch
    from paper_2511_02043_amd import binding as fb
    rng = np.random.Generator(np.random.PCG64(20251102043))
    for case in range(30):
        group = int(rng.choice([1, 2, 4, 8, 16]))
        T = int(rng.integers(1, 64 // group + 1))
        Hkv = int(rng.choice([1, 2, 3]))
        D = int(rng.choice([64, 128]))
        ps = int(rng.choice([8, 16, 32, 64]))
        B = int(rng.integers(1, 5))
        hi = int(rng.choice([40, 300, 2500]))
        lens = [int(x) for x in rng.integers(0, hi + 1, size=B)]
        w = inputs.prefill_paged_bf16(H=group * Hkv, Hkv=Hkv, D=D, Sq=T, page_size=ps, seq_lens=lens, salt=100 + case)
        kind = int(rng.integers(0, 4))
        if kind == 1:
            w.softcap = 3.0
        elif kind == 2:
            w.alibi = inputs.alibi_slopes(group * Hkv)
        if rng.integers(0, 2):
            w.window = int(rng.choice([0, 1, T, 33, 500]))
        label = f"case {case}: group={group} T={T} Hkv={Hkv} D={D} page={ps} lens={lens} kind={kind} window={w.window}"
        print(label, flush=True)
        dd = runner.upload_prefill_paged(w)
        ws = torch.empty(max(fb.fl_attn_decode_workspace_size(dd.tq, dd.tk, dd.kv), 16), dtype=torch.uint8, device="cuda:0")
        slopes = dd.keep[3]
        dd.out.fill_(float("nan"))
        dd.lse.fill_(float("nan"))
        fb.check(fb.fl_attn_decode(dd.tq, dd.tk, dd.tv, dd.kv, dd.desc, fb.aux_desc(alibi_slopes=slopes, workspace=ws), dd.tout, dd.tlse))
        torch.cuda.synchronize()
        got, got_lse = dd.out.cpu().numpy()[:, 0], dd.lse.cpu().numpy()[:, 0, :, :, 0]
        ref, ref_lse = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale, window=w.window,
                                            softcap_value=w.softcap, alibi_slopes=w.alibi)
        dead = np.isneginf(ref_lse)
        assert np.array_equal(np.isneginf(got_lse), dead), label
        assert np.all(got[dead] == 0.0) and np.all(np.isfinite(got)), label
        assert float(np.max(np.abs(got - ref))) <= 1e-2, label
        if np.any(~dead):
            assert float(np.max(np.abs(got_lse[~dead] - ref_lse[~dead]))) <= 1e-3, label
