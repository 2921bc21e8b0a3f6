"""Pins for the CPU oracle: it is checked against things other than itself.

Each test names the definition, closed form, invariant or independent routine it
uses.  Citations are to the paper's sections / equations / algorithms.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attention_oracle as ao
from oracle import brute_force as bf
from paper_2511_02043_amd import inputs


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def rand(shape, seed):
    return rng(seed).standard_normal(shape)


# ---------------------------------------------------------------------------------------
# 1. Independent library routine: PyTorch's fp64 CPU scaled_dot_product_attention
# ---------------------------------------------------------------------------------------

def sdpa(q, k, v, scale, allowed=None, bias=None):
    """q,k,v [B,G,H,S,D] -> out via torch SDPA in fp64 with a float attn_mask."""
    B, G, H, Sq, D = q.shape
    Sk = k.shape[3]
    mask = torch.zeros(B, G, H, Sq, Sk, dtype=torch.float64)
    if bias is not None:
        mask = mask + torch.from_numpy(np.broadcast_to(bias, mask.shape).copy())
    if allowed is not None:
        mask = mask.masked_fill(~torch.from_numpy(np.broadcast_to(allowed, mask.shape).copy()),
                                float("-inf"))
    tq, tk, tv = (torch.from_numpy(np.ascontiguousarray(x)).reshape(B * G, *x.shape[2:])
                  for x in (q, k, v))
    o = torch.nn.functional.scaled_dot_product_attention(
        tq, tk, tv, attn_mask=mask.reshape(B * G, H, Sq, Sk), scale=scale)
    return o.reshape(B, G, H, Sq, -1).numpy()


@pytest.mark.parametrize("Sq,Sk", [(37, 37), (16, 53), (53, 16)])
def test_plain_matches_sdpa(Sq, Sk):
    q, k, v = rand((2, 1, 3, Sq, 8), 1), rand((2, 1, 3, Sk, 8), 2), rand((2, 1, 3, Sk, 5), 3)
    out, _ = ao.attention(q, k, v, scale=0.31)
    np.testing.assert_allclose(out, sdpa(q, k, v, 0.31), rtol=0, atol=1e-12)


def test_causal_window_doc_prefix_match_sdpa():
    S = 41
    q, k, v = rand((2, 1, 2, S, 8), 4), rand((2, 1, 2, S, 8), 5), rand((2, 1, 2, S, 6), 6)
    i = np.arange(S)[:, None]
    j = np.arange(S)[None, :]
    doc = inputs.doc_ids(2, S, seed=7, lo=3, hi=9)
    cases = {
        "causal": (dict(causal=True), j <= i),
        "window": (dict(causal=True, window=5), (j <= i) & (i - j <= 5)),
        "prefix": (dict(prefix=7), (j <= i) | (j < 7)),
    }
    for name, (kw, allowed) in cases.items():
        out, _ = ao.attention(q, k, v, scale=0.4, **kw)
        ref = sdpa(q, k, v, 0.4, allowed=allowed[None, None, None])
        np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12, err_msg=name)
    same = (doc[:, :, None] == doc[:, None, :])[:, None, None]          # [B,1,1,S,S]
    out, _ = ao.attention(q, k, v, scale=0.4, causal=True, window=5, q_doc=doc, kv_doc=doc)
    ref = sdpa(q, k, v, 0.4, allowed=same & ((j <= i) & (i - j <= 5))[None, None, None])
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    out, _ = ao.attention(q, k, v, scale=0.4, q_doc=doc, kv_doc=doc)
    np.testing.assert_allclose(out, sdpa(q, k, v, 0.4, allowed=same), rtol=0, atol=1e-12)


def test_alibi_and_bias_match_sdpa_float_mask():
    B, G, H, S, D = 1, 3, 4, 29, 8
    q, k, v = rand((B, G, H, S, D), 8), rand((B, G, H, S, D), 9), rand((B, G, H, S, D), 10)
    slopes = inputs.alibi_slopes(H).astype(np.float64)
    dist = np.abs(np.arange(S)[:, None] - np.arange(S)[None, :])
    alibi_bias = -slopes[None, None, :, None, None] * dist[None, None, None]
    out, _ = ao.attention(q, k, v, scale=0.35, alibi_slopes=slopes)
    np.testing.assert_allclose(out, sdpa(q, k, v, 0.35, bias=alibi_bias), rtol=0, atol=1e-12)
    pair = rand((B, 1, H, S, S), 11)          # broadcast over G (Evoformer pair bias)
    rowmask = rand((B, G, 1, 1, S), 12)       # broadcast over heads and queries
    out, _ = ao.attention(q, k, v, scale=0.35, biases=(pair, rowmask))
    np.testing.assert_allclose(out, sdpa(q, k, v, 0.35, bias=pair + rowmask), rtol=0, atol=1e-12)


def test_gqa_matches_sdpa_with_repeated_heads():
    q, k, v = rand((1, 1, 8, 19, 4), 13), rand((1, 1, 2, 23, 4), 14), rand((1, 1, 2, 23, 4), 15)
    out, _ = ao.attention(q, k, v, scale=0.5)
    kr, vr = np.repeat(k, 4, axis=2), np.repeat(v, 4, axis=2)
    np.testing.assert_allclose(out, sdpa(q, kr, vr, 0.5), rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------------------
# 2. Brute force on tiny shapes (separately written, online recurrence of Alg. 2)
# ---------------------------------------------------------------------------------------

TINY = [(1, 1, 1, 5, 5, 3, 3), (1, 2, 2, 7, 9, 4, 2), (2, 1, 3, 6, 4, 2, 5)]


@pytest.mark.parametrize("B,G,H,Sq,Sk,D,Dv", TINY)
@pytest.mark.parametrize("variant", ["plain", "causal", "window", "prefix", "softcap", "alibi",
                                     "bias", "doc", "all"])
def test_matches_brute_force(B, G, H, Sq, Sk, D, Dv, variant):
    q, k, v = rand((B, G, H, Sq, D), 20), rand((B, G, H, Sk, D), 21), rand((B, G, H, Sk, Dv), 22)
    kw, bkw = {}, {}
    bias = None
    qd = kd = None
    slopes = None
    if variant in ("causal", "all"):
        kw["causal"] = bkw["causal"] = True
    if variant in ("window", "all"):
        kw.update(causal=True, window=2)
        bkw.update(causal=True, window=2)
    if variant == "prefix":
        kw["prefix"] = bkw["prefix"] = 2
    if variant in ("softcap", "all"):
        kw["softcap_value"] = bkw["cap"] = 0.7
    if variant in ("alibi", "all"):
        slopes = np.linspace(0.1, 0.9, H)
        kw["alibi_slopes"] = slopes
    if variant in ("bias", "all"):
        bias = rand((B, 1, H, Sq, Sk), 23)
        kw["biases"] = (bias,)
    if variant in ("doc", "all"):
        qd = rng(24).integers(0, 2, (B, Sq)).astype(np.int32)
        kd = rng(25).integers(0, 2, (B, Sk)).astype(np.int32)
        kw.update(q_doc=qd, kv_doc=kd)
    out, lse, probs = ao.attention(q, k, v, scale=0.6, return_probs=True, **kw)
    for b in range(B):
        for g in range(G):
            for h in range(H):
                for i in range(Sq):
                    o, l, p = bf.attention_row(
                        q[b, g, h, i].tolist(), k[b, g, h].tolist(), v[b, g, h].tolist(),
                        scale=0.6, i=i, slope=None if slopes is None else float(slopes[h]),
                        bias_row=None if bias is None else bias[b, 0, h, i].tolist(),
                        q_doc=None if qd is None else int(qd[b, i]),
                        kv_doc=None if kd is None else kd[b].tolist(), **bkw)
                    np.testing.assert_allclose(out[b, g, h, i], o, rtol=0, atol=1e-13)
                    np.testing.assert_allclose(probs[b, g, h, i], p, rtol=0, atol=1e-13)
                    if l == -math.inf:
                        assert lse[b, g, h, i] == -np.inf
                    else:
                        assert abs(lse[b, g, h, i] - l) < 1e-13


def test_differential_rmsnorm_gate_match_brute_force():
    B, H, S, D, Dv = 1, 2, 6, 3, 4
    w = inputs.differential_bf16(B=B, H=H, S=S, D=D, Dv=Dv, lam=0.8)
    w.rms_weight = np.linspace(0.5, 1.5, Dv)
    w.gate = rand((B, 1, H, S, Dv), 30)
    out, lse = ao.run_workload(w)
    for h in range(H):
        for i in range(S):
            o1, l1, _ = bf.attention_row(w.q[0, 0, h, i].tolist(), w.k[0, 0, h].tolist(),
                                         w.v[0, 0, h].tolist(), scale=w.scale, i=i, causal=True)
            o2, l2, _ = bf.attention_row(w.q2[0, 0, h, i].tolist(), w.k2[0, 0, h].tolist(),
                                         w.v[0, 0, h].tolist(), scale=w.scale, i=i, causal=True)
            d = [a - float(w.lam[h]) * b for a, b in zip(o1, o2)]
            y = bf.rmsnorm_row(d, 1e-6, w.rms_weight.tolist())
            y = [bf.sigmoid(float(w.gate[0, 0, h, i, c])) * y[c] for c in range(Dv)]
            np.testing.assert_allclose(out[0, 0, h, i], y, rtol=0, atol=1e-12)
            assert abs(lse[0, 0, 0, h, i] - l1) < 1e-12 and abs(lse[0, 1, 0, h, i] - l2) < 1e-12


# ---------------------------------------------------------------------------------------
# 3. Closed forms
# ---------------------------------------------------------------------------------------

def test_zero_query_gives_uniform_weights_over_allowed_keys():
    """Q = 0: all allowed scores are equal, so out_i is the mean of the allowed V rows
    and lse_i = ln(number of allowed keys)."""
    S, D = 33, 4
    q = np.zeros((1, 1, 1, S, D))
    k, v = rand((1, 1, 1, S, D), 40), rand((1, 1, 1, S, D), 41)
    csum = np.cumsum(v[0, 0, 0], axis=0)
    out, lse = ao.attention(q, k, v, scale=1.0, causal=True)
    for i in range(S):
        np.testing.assert_allclose(out[0, 0, 0, i], csum[i] / (i + 1), atol=1e-13)
        assert abs(lse[0, 0, 0, i] - math.log(i + 1)) < 1e-13
    W = 4
    out, lse = ao.attention(q, k, v, scale=1.0, causal=True, window=W)
    for i in range(S):
        lo = max(0, i - W)
        np.testing.assert_allclose(out[0, 0, 0, i], v[0, 0, 0, lo:i + 1].mean(axis=0), atol=1e-13)
        assert abs(lse[0, 0, 0, i] - math.log(min(i, W) + 1)) < 1e-13   # W + 1 keys incl. self
    doc = inputs.doc_ids(1, S, seed=42, lo=3, hi=8)
    out, lse = ao.attention(q, k, v, scale=1.0, q_doc=doc, kv_doc=doc)
    for i in range(S):
        sel = doc[0] == doc[0, i]
        np.testing.assert_allclose(out[0, 0, 0, i], v[0, 0, 0, sel].mean(axis=0), atol=1e-13)
        assert abs(lse[0, 0, 0, i] - math.log(sel.sum())) < 1e-13
    P = 5
    out, lse = ao.attention(q, k, v, scale=1.0, prefix=P)
    for i in range(S):
        n = max(i + 1, P)
        np.testing.assert_allclose(out[0, 0, 0, i], csum[n - 1] / n, atol=1e-13)


def test_zero_query_alibi_is_two_geometric_sums():
    """Q = 0 with ALiBi: weights are r^|i-j| with r = e^{-slope}; the normaliser is
    (1 - r^{i+1})/(1 - r) + (r - r^{S-i})/(1 - r)."""
    S, H = 25, 3
    slopes = np.array([0.05, 0.3, 1.1])
    q = np.zeros((1, 1, H, S, 2))
    k, v = rand((1, 1, H, S, 2), 43), rand((1, 1, H, S, 2), 44)
    _, lse = ao.attention(q, k, v, scale=1.0, alibi_slopes=slopes)
    for h in range(H):
        r = math.exp(-slopes[h])
        for i in range(S):
            z = (1 - r ** (i + 1)) / (1 - r) + (r - r ** (S - i)) / (1 - r)
            assert abs(lse[0, 0, h, i] - math.log(z)) < 1e-12


def test_single_visible_key_returns_that_value_row_and_score():
    """A row masked everywhere but one key returns that V row; lse is that score."""
    S, D = 9, 3
    q, k, v = rand((1, 1, 1, S, D), 45), rand((1, 1, 1, S, D), 46), rand((1, 1, 1, S, D), 47)
    out, lse = ao.attention(q, k, v, scale=0.5, causal=True, window=0)   # only j = i visible
    np.testing.assert_allclose(out[0, 0, 0], v[0, 0, 0], atol=1e-14)
    diag = 0.5 * np.einsum("id,id->i", q[0, 0, 0], k[0, 0, 0])
    np.testing.assert_allclose(lse[0, 0, 0], diag, atol=1e-14)
    qd = np.arange(S, dtype=np.int32)[None]
    kd = np.arange(S, dtype=np.int32)[::-1].copy()[None]                 # i sees only S-1-i
    out, _ = ao.attention(q, k, v, scale=0.5, q_doc=qd, kv_doc=kd)
    np.testing.assert_allclose(out[0, 0, 0], v[0, 0, 0, ::-1], atol=1e-14)


def test_fully_masked_row_is_zero_with_minus_inf_lse():
    q, k, v = rand((1, 1, 1, 4, 2), 48), rand((1, 1, 1, 4, 2), 49), rand((1, 1, 1, 4, 2), 50)
    qd = np.array([[0, 1, 0, 7]], dtype=np.int32)
    kd = np.array([[0, 0, 1, 1]], dtype=np.int32)
    out, lse = ao.attention(q, k, v, scale=1.0, q_doc=qd, kv_doc=kd)
    assert np.all(out[0, 0, 0, 3] == 0.0) and lse[0, 0, 0, 3] == -np.inf
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse[0, 0, 0, :3]))


def test_constant_value_rows_are_returned_unchanged():
    """Rows of P sum to 1 (Eq. 1), so V with identical rows comes back for any variant."""
    S = 17
    q, k = rand((1, 2, 2, S, 4), 51), rand((1, 2, 2, S, 4), 52)
    row = rand((5,), 53)
    v = np.broadcast_to(row, (1, 2, 2, S, 5))
    bias = rand((1, 1, 2, S, S), 54)
    for kw in (dict(), dict(causal=True), dict(causal=True, window=3), dict(softcap_value=2.0),
               dict(alibi_slopes=np.array([0.2, 0.7])), dict(biases=(bias,))):
        out, _ = ao.attention(q, k, v, scale=0.9, **kw)
        np.testing.assert_allclose(out, np.broadcast_to(row, out.shape), atol=1e-13)


def test_rows_of_p_are_positive_and_sum_to_one_and_lse_reproduces_p():
    S = 23
    q, k, v = rand((1, 1, 2, S, 4), 55), rand((1, 1, 2, S, 4), 56), rand((1, 1, 2, S, 4), 57)
    out, lse, p = ao.attention(q, k, v, scale=0.7, causal=True, return_probs=True)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-14)
    allowed = np.tril(np.ones((S, S), dtype=bool))
    assert np.all(p[..., allowed] > 0) and np.all(p[..., ~allowed] == 0)
    s = 0.7 * np.einsum("bghid,bghjd->bghij", q, k)
    np.testing.assert_allclose(np.exp(s - lse[..., None])[..., allowed], p[..., allowed], atol=1e-13)


def test_stable_softmax_state_equals_online_recurrence():
    """Post-condition shared by Alg. 1 and Alg. 2, any order, with -inf entries."""
    x = rand((6, 50), 58) * 5
    x[2, :7] = -np.inf
    x[4, ::3] = -np.inf
    p, lse = ao.stable_softmax(x)
    for r in range(6):
        m, d = bf.online_softmax_state(x[r].tolist())
        assert abs(lse[r] - (m + math.log(d))) < 1e-12
        m2, d2 = bf.online_softmax_state(x[r, ::-1].tolist())
        assert m2 == m and abs(d2 - d) < 1e-12 * d


# ---------------------------------------------------------------------------------------
# 4. Invariances
# ---------------------------------------------------------------------------------------

def test_key_permutation_invariance():
    S = 21
    q, k, v = rand((1, 1, 2, S, 4), 60), rand((1, 1, 2, S, 4), 61), rand((1, 1, 2, S, 3), 62)
    bias = rand((1, 1, 2, S, S), 63)
    qd = rng(64).integers(0, 3, (1, S)).astype(np.int32)
    kd = rng(65).integers(0, 3, (1, S)).astype(np.int32)
    perm = rng(66).permutation(S)
    o1, l1 = ao.attention(q, k, v, scale=0.5, biases=(bias,), q_doc=qd, kv_doc=kd,
                          softcap_value=1.5)
    o2, l2 = ao.attention(q, k[..., perm, :], v[..., perm, :], scale=0.5,
                          biases=(bias[..., perm],), q_doc=qd, kv_doc=kd[:, perm],
                          softcap_value=1.5)
    np.testing.assert_allclose(o1, o2, atol=1e-13)
    np.testing.assert_allclose(l1, l2, atol=1e-13)


def test_row_constant_bias_shifts_lse_only():
    S = 14
    q, k, v = rand((1, 1, 1, S, 4), 67), rand((1, 1, 1, S, 4), 68), rand((1, 1, 1, S, 4), 69)
    c = rand((1, 1, 1, S, 1), 70)
    o1, l1 = ao.attention(q, k, v, scale=0.5, causal=True)
    o2, l2 = ao.attention(q, k, v, scale=0.5, causal=True, biases=(np.broadcast_to(c, (1, 1, 1, S, S)),))
    np.testing.assert_allclose(o1, o2, atol=1e-13)
    np.testing.assert_allclose(l2 - l1, c[0, 0, 0, :, 0][None, None, None], atol=1e-13)


def test_softcap_limits():
    S = 12
    q, k, v = rand((1, 1, 1, S, 4), 71) * 6, rand((1, 1, 1, S, 4), 72), rand((1, 1, 1, S, 4), 73)
    o_big, l_big = ao.attention(q, k, v, scale=0.5, softcap_value=1e9)
    o_none, l_none = ao.attention(q, k, v, scale=0.5)
    np.testing.assert_allclose(o_big, o_none, atol=1e-9)
    s = rand((5, 7), 74) * 100
    assert np.all(np.abs(ao.softcap(s, 30.0)) <= 30.0)
    np.testing.assert_allclose(ao.softcap(-s, 30.0), -ao.softcap(s, 30.0), atol=0)
    # small-argument expansion cap*tanh(s/cap) = s - s^3/(3 cap^2) + O(s^5)
    t = np.array([0.1, -0.2, 0.3])
    np.testing.assert_allclose(ao.softcap(t, 30.0), t - t ** 3 / 2700.0, atol=1e-9)


# ---------------------------------------------------------------------------------------
# 5. Differential, RMSNorm, gate
# ---------------------------------------------------------------------------------------

def test_differential_reductions():
    w = inputs.differential_bf16(B=1, H=2, S=19, D=4, Dv=6, lam=0.8)
    std, lse_std = ao.attention(w.q, w.k, w.v, scale=w.scale, causal=True)
    o, lse = ao.differential_attention(w.q, w.k, w.q2, w.k2, w.v, np.zeros(2), scale=w.scale,
                                       causal=True)
    np.testing.assert_allclose(o, std, atol=0)                  # lambda = 0 -> stream 1 alone
    np.testing.assert_allclose(lse[:, 0], lse_std, atol=0)
    o, _ = ao.differential_attention(w.q, w.k, w.q, w.k, w.v, w.lam, scale=w.scale, causal=True)
    np.testing.assert_allclose(o, (1 - np.float64(np.float32(0.8))) * std, atol=1e-14)


def test_rmsnorm_unit_mean_square_and_scale_invariance():
    x = rand((3, 5, 128), 80)
    y = ao.rmsnorm(x, 0.0)
    np.testing.assert_allclose((y * y).mean(-1), 1.0, atol=1e-13)
    np.testing.assert_allclose(ao.rmsnorm(7.5 * x, 0.0), y, atol=1e-13)
    wgt = rand((128,), 81)
    np.testing.assert_allclose(ao.rmsnorm(x, 1e-6, wgt), ao.rmsnorm(x, 1e-6) * wgt, atol=1e-15)
    # eps enters under the square root, added to the mean square
    one = np.full((1, 4), 2.0)
    np.testing.assert_allclose(ao.rmsnorm(one, 5.0), 2.0 / 3.0, atol=1e-15)


def test_gate_limits_and_commutation():
    w = inputs.evoformer_bf16(B=1, Nseq=3, Nres=11, H=2, D=4)
    base, _ = ao.attention(w.q, w.k, w.v, scale=w.scale, biases=w.biases)
    np.testing.assert_allclose(ao.sigmoid_gate(base, np.full(base.shape, 40.0)), base, rtol=1e-15)
    np.testing.assert_allclose(ao.sigmoid_gate(base, np.full(base.shape, -40.0)), 0, atol=1e-16)
    np.testing.assert_allclose(ao.sigmoid_gate(base, np.zeros(base.shape)), 0.5 * base, atol=0)
    full, _ = ao.run_workload(w)
    np.testing.assert_allclose(full, base * torch.sigmoid(torch.from_numpy(
        np.ascontiguousarray(w.gate).astype(np.float64))).numpy(), atol=1e-15)


def test_evoformer_view_layout_and_bias_broadcast():
    """The [B,G,H,S,D] views alias [B,Nseq,Nres,H,D] storage; the pair bias is shared
    by all Nseq rows, so each row g equals ordinary attention with that bias."""
    w = inputs.evoformer_bf16(B=1, Nseq=4, Nres=9, H=2, D=4, two_biases=True)
    assert w.q.strides[3] == 2 * 4 * 4 and w.q.strides[2] == 4 * 4   # S stride H*D, head stride D
    out, _ = ao.attention(w.q, w.k, w.v, scale=w.scale, biases=w.biases)
    for g in range(4):
        b = w.biases[0][:, 0:1] + w.biases[1][:, g:g + 1]
        ref = sdpa(np.ascontiguousarray(w.q[:, g:g + 1]).astype(np.float64),
                   np.ascontiguousarray(w.k[:, g:g + 1]).astype(np.float64),
                   np.ascontiguousarray(w.v[:, g:g + 1]).astype(np.float64), w.scale,
                   bias=b.astype(np.float64))
        np.testing.assert_allclose(out[:, g:g + 1], ref, atol=1e-12)


def test_row_sampling_agrees_with_full_evaluation():
    for w in (inputs.window_doc_bf16(B=2, H=2, S=50, D=8, window=7, lo=3, hi=12),
              inputs.differential_bf16(B=1, H=2, S=21, D=4, Dv=8),
              inputs.evoformer_bf16(B=1, Nseq=3, Nres=10, H=2, D=4, two_biases=True),
              inputs.alibi_bf16(B=1, H=4, S=20, D=8),
              inputs.causal_bf16(B=1, H=4, S=20, D=8, Hkv=2)):
        out, lse = ao.run_workload(w)
        d = w.dims
        picks = [(d["B"] - 1, d["G"] - 1, d["H"] - 1, d["Sq"] - 1), (0, 0, 1, 3), (0, 0, 0, 0)]
        for (b, g, h, i), (o, l) in zip(picks, ao.run_workload_rows(w, picks)):
            np.testing.assert_allclose(o, out[b, g, h, i], atol=1e-13)
            full = lse[b, :, g, h, i] if w.q2 is not None else lse[b, g, h, i]
            np.testing.assert_allclose(l, full, atol=1e-13)


# ---------------------------------------------------------------------------------------
# attention_custom: callables for score_mod and mask
# ---------------------------------------------------------------------------------------

def test_custom_callables_reproduce_the_named_variants():
    q, k, v = rand((2, 1, 4, 29, 8), 91), rand((2, 1, 2, 29, 8), 92), rand((2, 1, 2, 29, 6), 93)
    slopes = inputs.alibi_slopes(4).astype(np.float64)
    ref, ref_lse = ao.attention(q, k, v, scale=0.3, window=6, alibi_slopes=slopes)
    out, lse = ao.attention_custom(q, k, v, scale=0.3,
                                   score_mod=lambda s, b, g, h, i, j: s - slopes[h] * np.abs(i - j),
                                   mask=lambda b, g, h, i, j: (j > i) | (i - j > 6))
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, ref_lse, rtol=0, atol=1e-13)
    ref, _ = ao.attention(q, k, v, scale=0.3, softcap_value=0.8, causal=True)
    out, _ = ao.attention_custom(q, k, v, scale=0.3, score_mod=lambda s, b, g, h, i, j: 0.8 * np.tanh(s / 0.8),
                                 mask=lambda b, g, h, i, j: j > i)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)


def test_custom_predicate_matches_sdpa():
    q, k, v = rand((1, 1, 2, 21, 8), 94), rand((1, 1, 2, 21, 8), 95), rand((1, 1, 2, 21, 8), 96)
    i = np.arange(21)[:, None]
    j = np.arange(21)[None, :]
    hidden = (j > i) | (((i ^ j) & 4) != 0)
    bias = 0.05 * ((i - j) % 5)
    out, _ = ao.attention_custom(q, k, v, scale=0.4, score_mod=lambda s, b, g, h, ii, jj: s + 0.05 * ((ii - jj) % 5),
                                 mask=lambda b, g, h, ii, jj: (jj > ii) | (((ii ^ jj) & 4) != 0))
    np.testing.assert_allclose(out, sdpa(q, k, v, 0.4, allowed=~hidden, bias=bias.astype(np.float64)), rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------------------
# Query-position offset (chunked prefill / bottom-right aligned masks: query row i sits at
# position i + q_offset): run_workload against SDPA with the mask written out explicitly,
# and against the rows of the square problem the chunk is cut from.
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("kind", ["causal", "window", "prefix", "alibi_causal"])
def test_query_offset_matches_sdpa_explicit_mask(kind):
    Sq, Sk, off = 13, 40, 27
    w = inputs.causal_bf16(B=2, H=2, S=Sq, Sk=Sk, D=64, causal=kind in ("causal", "alibi_causal"))
    w.q_offset = off
    i = np.arange(Sq)[:, None] + off
    j = np.arange(Sk)[None, :]
    bias = None
    if kind == "causal":
        allowed = j <= i
    elif kind == "window":
        w.causal, w.window = True, 9
        allowed = (j <= i) & (i - j <= 9)
    elif kind == "prefix":
        w.prefix = 31
        allowed = (j <= i) | (j < 31)
    else:
        w.alibi = inputs.alibi_slopes(2)
        allowed = j <= i
        bias = -w.alibi.astype(np.float64)[None, None, :, None, None] * np.abs(i - j)[None, None, None]
    out, lse = ao.run_workload(w)
    ref = sdpa(w.q.astype(np.float64), w.k.astype(np.float64), w.v.astype(np.float64), w.scale,
               allowed=np.broadcast_to(allowed, (2, 1, 2, Sq, Sk)), bias=bias)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    # the last Sq rows of the square causal problem over the same keys are these rows
    if kind == "causal":
        full = inputs.causal_bf16(B=2, H=2, S=Sk, D=64)
        full.k, full.v = w.k, w.v
        full.q = np.concatenate([np.zeros((2, 1, 2, off, 64), w.q.dtype), w.q], axis=3)
        out_full, lse_full = ao.run_workload(full)
        np.testing.assert_allclose(out, out_full[:, :, :, off:], rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse, lse_full[:, :, :, off:], rtol=0, atol=1e-12)
        rows = ao.run_workload_rows(w, [(1, 0, 1, 5), (0, 0, 0, 12)])
        np.testing.assert_allclose(rows[0][0], out[1, 0, 1, 5], rtol=0, atol=1e-12)
        np.testing.assert_allclose(rows[1][1], lse[0, 0, 0, 12], rtol=0, atol=1e-12)
