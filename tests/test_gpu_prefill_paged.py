"""GPU parity of fl_attn_prefill_paged (through the C-ABI) against the fp64 oracle of a chunk of query rows over
a paged key/value cache.

Tolerance: the forward pass's (bf16 inputs, bf16 probabilities into an fp32-accumulating contraction):
max-abs <= 1e-2 on fp32 outputs, lse <= 1e-3."""
import numpy as np
import pytest

from oracle import decode_oracle as do
from paper_2511_02043_amd import binding as fb
from paper_2511_02043_amd import inputs, runner

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["auto", "in_place", "gather"], autouse=True)
def prefill_mode(request):
    """Every test runs three times: with the library's own choice (the decode kernels for chunks whose (row, head) pairs
    per kv head number at most 64, else as follows), with the forward kernel reading the pages in place (its choice for
    chunks of up to 1024 rows), and with the pages copied into dense tensors first (its choice for longer chunks and for
    page sizes below a load instruction's rows)."""
    fb.check(fb.fl_set_tuning("prefill_gather", {"auto": 0, "gather": 1, "in_place": 2}[request.param]))
    yield request.param
    fb.fl_set_tuning("prefill_gather", 0)


def run(w, out_dtype="f32", paged=True, max_seq_len=None):
    import torch
    dd = runner.upload_prefill_paged(w, out_dtype=out_dtype, paged=paged, max_seq_len=max_seq_len)
    dd.out.fill_(float("nan"))
    dd.lse.fill_(float("nan"))
    dd.run_checked()
    torch.cuda.synchronize()
    return dd.out.float().cpu().numpy()[:, 0], dd.lse.cpu().numpy()[:, 0, :, :, 0]


def check(got, got_lse, ref, ref_lse, label, out_dtype="f32"):
    assert np.all(np.isfinite(got)), label
    err = float(np.max(np.abs(got - ref)))
    dead = np.isneginf(ref_lse)
    assert np.array_equal(np.isneginf(got_lse), dead), label
    assert np.all(got[dead] == 0.0), label
    le = float(np.max(np.abs(got_lse[~dead] - ref_lse[~dead]))) if np.any(~dead) else 0.0
    print(f"{label}: max_abs={err:.3e} lse={le:.3e}", flush=True)
    slack = 2.0 ** -8 * np.abs(ref) if out_dtype == "bf16" else 0.0
    assert np.all(np.abs(got - ref) <= 1e-2 + slack), (label, err)
    assert le <= 1e-3, (label, le)


def compare(w, label, out_dtype="f32", paged=True, max_seq_len=None):
    got, got_lse = run(w, out_dtype, paged, max_seq_len)
    ref, ref_lse = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale,
                                        window=w.window, softcap_value=w.softcap, alibi_slopes=w.alibi)
    check(got, got_lse, ref, ref_lse, label, out_dtype)


CASES = {
    # lengths below, at and above the chunk, around the key tile (64) and page boundaries, several q tiles
    "gqa4_d128_p16_q96": lambda: inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=96, page_size=16,
                                                           seq_lens=[0, 1, 95, 96, 97, 500, 1027]),
    "gqa8_d64_p32_q300": lambda: inputs.prefill_paged_bf16(H=16, Hkv=2, D=64, Sq=300, page_size=32,
                                                           seq_lens=[7, 300, 301, 900, 2049]),
    "mha_d128_p8_q17": lambda: inputs.prefill_paged_bf16(H=4, Hkv=4, D=128, Sq=17, page_size=8, seq_lens=[15, 16, 17, 18, 333]),
    "mqa_d64_p128_q64": lambda: inputs.prefill_paged_bf16(H=8, Hkv=1, D=64, Sq=64, page_size=128, seq_lens=[129, 1000, 3]),
    # few rows: all (row, head) pairs of a kv head are columns of one or two MFMA tiles of the decode kernels; lengths
    # below the chunk (rows at negative positions), around the 32-key tile and the pages
    "few_gqa4_d128_q8": lambda: inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=8, page_size=16,
                                                          seq_lens=[0, 1, 7, 8, 9, 31, 32, 33, 64, 500, 1027], salt=11),
    "few_gqa4_d128_q16": lambda: inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=16, page_size=16,
                                                           seq_lens=[3, 15, 16, 17, 40, 65, 900], salt=12),
    "few_gqa8_d64_q5": lambda: inputs.prefill_paged_bf16(H=16, Hkv=2, D=64, Sq=5, page_size=8,
                                                         seq_lens=[4, 5, 6, 32, 36, 37, 777], salt=13),
    "few_mha_d64_q40": lambda: inputs.prefill_paged_bf16(H=2, Hkv=2, D=64, Sq=40, page_size=32,
                                                         seq_lens=[39, 40, 41, 100, 1500], salt=14),
    "few_gqa4_d128_q3": lambda: inputs.prefill_paged_bf16(H=4, Hkv=1, D=128, Sq=3, page_size=64, seq_lens=[2, 3, 4, 64, 66, 2100], salt=15),
    "d32_p16_q40": lambda: inputs.prefill_paged_bf16(H=4, Hkv=2, D=32, Sq=40, page_size=16, seq_lens=[40, 41, 200]),
}


@pytest.mark.parametrize("name", list(CASES))
def test_prefill_matches_oracle(name):
    compare(CASES[name](), name)


@pytest.mark.parametrize("Sq", [1, 4, 16, 17, 128, 500])
def test_chunks_against_a_long_cache(Sq):
    """Chunks of 1, 4, 16 (the decode kernels' range, several splits of the key range), 17, 128 and 500 rows against 4k - 8k cached tokens per sequence (the serving shape of Sec. 4.1:
    32 query heads on 8 kv heads would take the oracle minutes, so 8 on 2), every row checked."""
    w = inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=Sq, page_size=16, seq_lens=[4096, 5000, 8191], salt=20 + Sq)
    compare(w, f"long_cache_q{Sq}")
    w.window = 1000
    compare(w, f"long_cache_q{Sq}_window")


def test_prefill_variants():
    w = inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=80, page_size=16, seq_lens=[5, 100, 700, 1500], salt=1)
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


def test_few_row_variants():
    """Window, soft-cap and ALiBi on chunks of a few rows, windows shorter than the chunk included (the rows' windows
    then differ inside one key tile)."""
    for D, Sq in ((128, 6), (64, 13)):
        w = inputs.prefill_paged_bf16(H=8, Hkv=2, D=D, Sq=Sq, page_size=16, seq_lens=[5, 33, 100, 700, 1500], salt=30 + Sq)
        for window in (255, 3, 0):
            w.window = window
            compare(w, f"few_d{D}_window_{window}")
        w.window = None
        w.softcap = 2.0
        compare(w, f"few_d{D}_softcap")
        w.softcap = None
        w.alibi = inputs.alibi_slopes(8)
        compare(w, f"few_d{D}_alibi")
        w.window = 40
        compare(w, f"few_d{D}_alibi_window")
    w = inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=7, page_size=16, seq_lens=[33, 500, 77], salt=31)
    compare(w, "few_bf16_out", out_dtype="bf16")
    compare(w, "few_max_seq_len_512", max_seq_len=512)
    c = inputs.prefill_paged_bf16(H=8, Hkv=4, D=128, Sq=9, page_size=1024, seq_lens=[1000, 7, 513], salt=32, shuffle_pages=False)
    compare(c, "few_contiguous", paged=False)


def test_prefill_bf16_output_contiguous_cache_and_loose_bound():
    w = inputs.prefill_paged_bf16(H=8, Hkv=2, D=64, Sq=50, page_size=16, seq_lens=[33, 500, 77], salt=2)
    compare(w, "bf16_out", out_dtype="bf16")
    # the host-side bound on the lengths may exceed every length: only the rows before each sequence grow
    compare(w, "max_seq_len_512", max_seq_len=512)
    # no block table: sequence b is page b of a cache whose pages hold a whole sequence
    c = inputs.prefill_paged_bf16(H=8, Hkv=4, D=128, Sq=70, page_size=1024, seq_lens=[1000, 17, 513], salt=3,
                                  shuffle_pages=False)
    assert np.array_equal(c.block_table[:, 0], np.arange(3))
    compare(c, "contiguous", paged=False)


def test_one_row_chunk_is_the_decode_step():
    """Sq = 1 against fl_attn_decode on the same cache (two different kernels, one definition)."""
    import torch
    w = inputs.decode_bf16(H=8, Hkv=2, D=128, page_size=16, seq_lens=[0, 1, 64, 65, 700], salt=4)
    dd = runner.upload_decode(w)
    dd.run_checked()
    torch.cuda.synchronize()
    dec, dec_lse = dd.out.cpu().numpy()[:, 0, :, 0], dd.lse.cpu().numpy()[:, 0, :, 0, 0]
    w.q = w.q[:, :, None, :]
    got, got_lse = run(w)
    assert np.array_equal(np.isneginf(got_lse[:, :, 0]), np.isneginf(dec_lse))
    live = ~np.isneginf(dec_lse)
    assert float(np.max(np.abs(got[:, :, 0] - dec))) <= 1e-2
    assert float(np.max(np.abs(got_lse[:, :, 0][live] - dec_lse[live]))) <= 1e-3


def test_chunks_of_a_prompt_give_the_rows_of_the_whole_prompt():
    """The prompt in chunks of 100, 28 and 172 rows (each call sees the cache up to the end of its chunk) against the
    one-shot oracle over all 300 rows."""
    n = 300
    w = inputs.prefill_paged_bf16(B=2, H=4, Hkv=2, D=128, Sq=n, page_size=16, seq_lens=[n, n], salt=5)
    ref, ref_lse = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale)
    q_all, start = w.q, 0
    for size in (100, 28, 172):
        end = start + size
        w.q = np.ascontiguousarray(q_all[:, :, start:end])
        w.seq_lens = np.array([end, end], dtype=np.int32)
        got, got_lse = run(w, max_seq_len=n)
        check(got, got_lse, ref[:, :, start:end], ref_lse[:, :, start:end], f"chunk_{start}_{end}")
        start = end


def test_lengths_and_table_entries_out_of_range_are_cut_not_followed():
    """A device length above max_seq_len is cut to it, a table entry outside the cache to the cache: wrong data by the
    caller's own mistake, never a wild address."""
    import torch
    w = inputs.prefill_paged_bf16(H=4, Hkv=2, D=64, Sq=33, page_size=16, seq_lens=[100, 60], salt=6)
    dd = runner.upload_prefill_paged(w, max_seq_len=100)
    dd.keep[1].copy_(torch.tensor([5000, -7], dtype=torch.int32))                    # seq_lens on the device
    dd.run_checked()
    torch.cuda.synchronize()
    got_lse = dd.lse.cpu().numpy()[:, 0, :, :, 0]
    assert np.all(np.isfinite(got_lse[0])) and np.all(np.isneginf(got_lse[1]))      # cut to 100 and to 0
    w2 = inputs.prefill_paged_bf16(H=4, Hkv=2, D=64, Sq=33, page_size=16, seq_lens=[100, 60], salt=6)
    w2.seq_lens = np.array([100, 0], dtype=np.int32)
    ref, ref_lse = do.prefill_attention(w2.q, w2.k_cache, w2.v_cache, w2.block_table, w2.seq_lens, scale=w2.scale)
    check(dd.out.cpu().numpy()[:, 0], got_lse, ref, ref_lse, "lengths_cut")
    dd.keep[1].copy_(torch.tensor([100, 60], dtype=torch.int32))
    dd.keep[0].fill_(2 ** 30)                                                        # every table entry far outside
    dd.run_checked()
    torch.cuda.synchronize()
    assert np.all(np.isfinite(dd.out.cpu().numpy()))


def test_errors(prefill_mode):
    w = inputs.prefill_paged_bf16(H=4, Hkv=2, D=64, Sq=16, page_size=16, seq_lens=[40, 60], salt=7)
    dd = runner.upload_prefill_paged(w)
    need = fb.fl_attn_prefill_paged_workspace_size(dd.tq, dd.tk, dd.kv)
    if prefill_mode == "auto":                      # 16 rows x 2 heads per kv head: the decode kernels and their workspace
        assert need == fb.fl_attn_decode_workspace_size(dd.tq, dd.tk, dd.kv) > 0
        small = fb.aux_desc(workspace=dd.keep[2][: need - 16])
        assert fb.fl_attn_prefill_paged(dd.tq, dd.tk, dd.tv, dd.kv, dd.desc, small, dd.tout, dd.tlse) == fb.FL_ERR_WORKSPACE
        assert fb.fl_attn_prefill_paged(dd.tq, dd.tk, dd.tv, dd.kv, dd.desc, None, dd.tout, dd.tlse) == fb.FL_ERR_AUX_MISSING
    elif prefill_mode == "gather":
        assert need >= 2 * 2 * 2 * 60 * 64 * 2
        small = fb.aux_desc(workspace=dd.keep[2][: need - 256])
        assert fb.fl_attn_prefill_paged(dd.tq, dd.tk, dd.tv, dd.kv, dd.desc, small, dd.tout, dd.tlse) == fb.FL_ERR_WORKSPACE
        assert fb.fl_attn_prefill_paged(dd.tq, dd.tk, dd.tv, dd.kv, dd.desc, None, dd.tout, dd.tlse) == fb.FL_ERR_AUX_MISSING
    else:                                           # in place: no workspace, and no aux unless the variant needs slopes
        assert need == 0
        assert fb.fl_attn_prefill_paged(dd.tq, dd.tk, dd.tv, dd.kv, dd.desc, None, dd.tout, dd.tlse) == fb.FL_OK
    for bad in (fb.variant_desc(scale=1.0, mask=fb.FL_MASK_DOC), fb.variant_desc(scale=1.0, mask=fb.FL_MASK_PREFIX, prefix_len=4),
                fb.variant_desc(scale=1.0, q_offset=3), fb.variant_desc(scale=1.0, epilogue=fb.FL_EPI_GATE_SIGMOID)):
        assert fb.fl_attn_prefill_paged(dd.tq, dd.tk, dd.tv, dd.kv, bad, dd.aux, dd.tout, dd.tlse) == fb.FL_ERR_UNSUPPORTED
    alibi = fb.variant_desc(scale=1.0, score_mod=fb.FL_MOD_ALIBI)
    assert fb.fl_attn_prefill_paged(dd.tq, dd.tk, dd.tv, dd.kv, alibi, dd.aux, dd.tout, dd.tlse) == fb.FL_ERR_AUX_MISSING
    kv = fb.paged_kv(block_table=dd.keep[0], page_size=8, seq_lens=dd.keep[1], max_seq_len=60)
    assert fb.fl_attn_prefill_paged(dd.tq, dd.tk, dd.tv, kv, dd.desc, dd.aux, dd.tout, dd.tlse) == fb.FL_ERR_SHAPE


def test_wide_in_place_shape_at_serving_size():
    """32 query heads on 8 kv heads, 8 sequences, 512-row chunks: the launch for which the in-place kernel takes its
    eight-wave shape.  Both ways must agree bit for bit (same arithmetic on the same keys), and the first query-head group
    of one sequence is checked against the oracle."""
    import torch
    w = inputs.prefill_paged_bf16(B=8, H=32, Hkv=8, D=128, Sq=512, page_size=16,
                                  seq_lens=[512, 700, 1500, 1023, 1024, 1025, 600, 2000], salt=40)
    outs = []
    for mode in (2, 1):
        fb.check(fb.fl_set_tuning("prefill_gather", mode))
        dd = runner.upload_prefill_paged(w)
        dd.out.fill_(float("nan"))
        dd.run_checked()
        torch.cuda.synchronize()
        outs.append((dd.out.clone(), dd.lse.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    b = 2
    ref, ref_lse = do.prefill_attention(w.q[b:b + 1, :4], w.k_cache[:, :, :1], w.v_cache[:, :, :1], w.block_table[b:b + 1],
                                        w.seq_lens[b:b + 1], scale=w.scale)
    got = outs[0][0].float().cpu().numpy()[b:b + 1, 0, :4]
    got_lse = outs[0][1].cpu().numpy()[b:b + 1, 0, :4, :, 0]
    check(got, got_lse, ref, ref_lse, "wide_in_place")
