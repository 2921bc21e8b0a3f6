"""Pins for the decode oracle: checked against things other than itself."""
import math

import numpy as np
import pytest

from oracle import attention_oracle as ao
from oracle import decode_oracle as do
from paper_2511_02043_amd import inputs


def contiguous(w, b):
    """Keys / values of sequence b as [1, 1, Hkv, len, D] arrays, gathered by plain indexing."""
    n, ps = int(w.seq_lens[b]), w.k_cache.shape[1]
    idx = [(w.block_table[b, j // ps], j % ps) for j in range(n)]
    k = np.stack([w.k_cache[p, o] for p, o in idx], axis=1)[None, None].astype(np.float64)   # [1,1,Hkv,n,D]
    v = np.stack([w.v_cache[p, o] for p, o in idx], axis=1)[None, None].astype(np.float64)
    return k, v


@pytest.mark.parametrize("variant", ["plain", "window", "softcap", "alibi"])
def test_last_row_of_the_forward_oracle(variant):
    """The decode step is the last query row of causal attention over the gathered keys: the pinned
    forward oracle, evaluated for that single row through its q_pos argument."""
    w = inputs.decode_bf16(B=3, H=8, Hkv=2, D=32, page_size=4, seq_lens=[1, 13, 40])
    kw, fkw = {}, {}
    if variant == "window":
        kw["window"], fkw["window"] = 5, 5
    if variant == "softcap":
        kw["softcap_value"], fkw["softcap_value"] = 0.7, 0.7
    if variant == "alibi":
        sl = inputs.alibi_slopes(8).astype(np.float64)
        kw["alibi_slopes"], fkw["alibi_slopes"] = sl, sl
    out, lse = do.decode_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale, **kw)
    for b in range(3):
        n = int(w.seq_lens[b])
        k, v = contiguous(w, b)
        q = w.q[b][None, None, :, None, :].astype(np.float64)                 # [1,1,H,1,D]
        ref, ref_lse = ao.attention(q, k, v, scale=w.scale, causal=True, q_pos=np.array([n - 1]), **fkw)
        np.testing.assert_allclose(out[b], ref[0, 0, :, 0], rtol=0, atol=1e-13)
        np.testing.assert_allclose(lse[b], ref_lse[0, 0, :, 0], rtol=0, atol=1e-13)


def test_brute_force_scalar_loops():
    w = inputs.decode_bf16(B=2, H=4, Hkv=2, D=8, page_size=2, seq_lens=[5, 9], salt=1)
    slopes = inputs.alibi_slopes(4).astype(np.float64)
    out, lse = do.decode_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=0.3, window=6,
                                   alibi_slopes=slopes)
    for b in range(2):
        n = int(w.seq_lens[b])
        for h in range(4):
            hk = h // 2
            scores = []
            for j in range(n):
                page, off = w.block_table[b, j // 2], j % 2
                s = 0.3 * sum(float(w.q[b, h, d]) * float(w.k_cache[page, off, hk, d]) for d in range(8))
                s -= slopes[h] * (n - 1 - j)
                scores.append(s if (n - 1 - j) <= 6 else None)
            m = max(s for s in scores if s is not None)
            den = sum(math.exp(s - m) for s in scores if s is not None)
            for d in range(8):
                acc = 0.0
                for j, s in enumerate(scores):
                    if s is not None:
                        acc += math.exp(s - m) / den * float(w.v_cache[w.block_table[b, j // 2], j % 2, hk, d])
                assert abs(acc - out[b, h, d]) < 1e-12
            assert abs(m + math.log(den) - lse[b, h]) < 1e-12


def test_page_permutation_invariance():
    """Moving a sequence's pages to other physical slots (and updating its block table) changes nothing."""
    w = inputs.decode_bf16(B=3, H=4, Hkv=1, D=16, page_size=4, seq_lens=[7, 16, 30], salt=2)
    out, lse = do.decode_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale)
    perm = np.random.Generator(np.random.PCG64(3)).permutation(w.k_cache.shape[0])
    inv = np.argsort(perm)
    k2, v2 = w.k_cache[perm], w.v_cache[perm]                 # new slot s holds old page perm[s]
    table2 = inv[w.block_table].astype(np.int32)              # old page p now lives in slot inv[p]
    out2, lse2 = do.decode_attention(w.q, k2, v2, table2, w.seq_lens, scale=w.scale)
    np.testing.assert_array_equal(out, out2)
    np.testing.assert_array_equal(lse, lse2)


def test_closed_forms():
    w = inputs.decode_bf16(B=3, H=4, Hkv=2, D=16, page_size=4, seq_lens=[0, 1, 21], salt=4)
    out, lse = do.decode_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale)
    assert np.all(out[0] == 0) and np.all(np.isneginf(lse[0]))                 # empty sequence
    page = w.block_table[1, 0]
    for h in range(4):                                                          # one key: out = v_0, lse = s_0
        np.testing.assert_allclose(out[1, h], w.v_cache[page, 0, h // 2], atol=1e-15)
        s0 = w.scale * float(np.dot(w.q[1, h].astype(np.float64), w.k_cache[page, 0, h // 2].astype(np.float64)))
        assert abs(lse[1, h] - s0) < 1e-13
    # q = 0 with a window: uniform weights over the window + 1 visible keys, lse = ln(count)
    q0 = np.zeros_like(w.q)
    out0, lse0 = do.decode_attention(q0, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale, window=4)
    np.testing.assert_allclose(lse0[2], math.log(5), atol=1e-14)
    vals = do.gather_sequence(w.v_cache, w.block_table, 2, 21)
    np.testing.assert_allclose(out0[2, 3], vals[-5:, 1].mean(axis=0), atol=1e-14)


# --- a chunk of query rows per sequence (prefill over the paged cache) -------------------------------------

def chunk_variant(variant, H):
    kw, fkw = {}, {}
    if variant == "window":
        kw["window"], fkw["window"] = 5, 5
    if variant == "softcap":
        kw["softcap_value"], fkw["softcap_value"] = 0.7, 0.7
    if variant == "alibi":
        sl = inputs.alibi_slopes(H).astype(np.float64)
        kw["alibi_slopes"], fkw["alibi_slopes"] = sl, sl
    return kw, fkw


@pytest.mark.parametrize("variant", ["plain", "window", "softcap", "alibi"])
def test_chunk_rows_of_the_forward_oracle(variant):
    """Row i of the chunk is row len - Sq + i of causal attention over the gathered keys (the pinned forward
    oracle, rows placed through q_pos); rows before position 0 are empty."""
    Sq = 7
    w = inputs.prefill_paged_bf16(B=4, H=8, Hkv=2, D=32, Sq=Sq, page_size=4, seq_lens=[1, 7, 13, 40])
    kw, fkw = chunk_variant(variant, 8)
    out, lse = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale, **kw)
    for b in range(4):
        n = int(w.seq_lens[b])
        k, v = contiguous(w, b)
        first = max(0, Sq - n)                                               # rows before it sit at negative positions
        assert np.all(out[b, :, :first] == 0.0) and np.all(np.isneginf(lse[b, :, :first]))
        q = w.q[b][None, None, :, first:, :].astype(np.float64)
        ref, ref_lse = ao.attention(q, k, v, scale=w.scale, causal=True, q_pos=np.arange(n - Sq + first, n), **fkw)
        np.testing.assert_allclose(out[b, :, first:], ref[0, 0], rtol=0, atol=1e-13)
        np.testing.assert_allclose(lse[b, :, first:], ref_lse[0, 0], rtol=0, atol=1e-13)


def test_chunk_against_sdpa_bottom_right_causal():
    """PyTorch's fp64 scaled_dot_product_attention with an explicit bottom-right aligned causal mask."""
    import torch
    Sq = 6
    w = inputs.prefill_paged_bf16(B=2, H=4, Hkv=2, D=16, Sq=Sq, page_size=8, seq_lens=[19, 33], salt=2)
    out, _ = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale)
    for b in range(2):
        n = int(w.seq_lens[b])
        k, v = contiguous(w, b)
        kt = torch.from_numpy(k[0, 0]).repeat_interleave(2, dim=0)           # [H, n, D]
        vt = torch.from_numpy(v[0, 0]).repeat_interleave(2, dim=0)
        qt = torch.from_numpy(w.q[b].astype(np.float64))                     # [H, Sq, D]
        allowed = torch.arange(n)[None, :] <= (torch.arange(Sq)[:, None] + n - Sq)
        ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=allowed, scale=w.scale)
        np.testing.assert_allclose(out[b], ref.numpy(), rtol=0, atol=1e-12)


def test_chunk_of_one_row_is_the_decode_step():
    w = inputs.prefill_paged_bf16(B=3, H=8, Hkv=4, D=16, Sq=1, page_size=4, seq_lens=[0, 9, 22], salt=3)
    sl = inputs.alibi_slopes(8).astype(np.float64)
    a, la = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale, window=6,
                                 alibi_slopes=sl)
    b_, lb = do.decode_attention(w.q[:, :, 0], w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale, window=6,
                                 alibi_slopes=sl)
    np.testing.assert_array_equal(a[:, :, 0], b_)
    np.testing.assert_array_equal(la[:, :, 0], lb)


def test_any_chunking_of_a_prompt_gives_the_same_rows():
    """Processing a prompt in chunks (each against the cache filled up to the end of that chunk) gives the rows of
    the one-shot pass: the defining property of chunked prefill."""
    n, ps = 29, 4
    w = inputs.prefill_paged_bf16(B=1, H=4, Hkv=2, D=16, Sq=n, page_size=ps, seq_lens=[n], salt=4)
    whole, whole_lse = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale,
                                            softcap_value=1.3)
    start = 0
    for size in (5, 1, 16, 7):
        end = start + size
        part, part_lse = do.prefill_attention(w.q[:, :, start:end], w.k_cache, w.v_cache, w.block_table, np.array([end]),
                                              scale=w.scale, softcap_value=1.3)
        np.testing.assert_allclose(part, whole[:, :, start:end], rtol=0, atol=1e-13)
        np.testing.assert_allclose(part_lse, whole_lse[:, :, start:end], rtol=0, atol=1e-13)
        start = end
    assert start == n
