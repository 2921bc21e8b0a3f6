"""Pins for the backward oracle: it is checked against things other than itself.

The gradient is pinned by (1) central finite differences of the FORWARD oracle, which is pinned
on its own, (2) autograd through PyTorch's fp64 CPU scaled_dot_product_attention, (3) closed
forms and identities of the softmax Jacobian.  Citations are to the paper's equations.
"""
import numpy as np
import pytest
import torch

from oracle import attention_backward_oracle as bo
from oracle import attention_oracle as ao
from paper_2511_02043_amd import inputs


def rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def variants(S):
    doc = inputs.doc_ids(2, S, seed=11, lo=3, hi=9)
    slopes = inputs.alibi_slopes(4).astype(np.float64)
    return {
        "plain": {},
        "causal": dict(causal=True),
        "window": dict(window=5),
        "prefix": dict(prefix=7),
        "doc": dict(q_doc=doc, kv_doc=doc),
        "window_doc": dict(window=6, q_doc=doc, kv_doc=doc),
        "softcap": dict(softcap_value=1.7),
        "softcap_causal": dict(softcap_value=0.9, causal=True),
        "alibi": dict(alibi_slopes=slopes),
        "alibi_causal": dict(alibi_slopes=slopes, causal=True),
    }


# ---------------------------------------------------------------------------------------
# 1. Central finite differences of the forward oracle (Eq. 3 / Eq. 4 / attention listing)
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("name", list(variants(19)))
@pytest.mark.parametrize("hkv", [4, 2])
def test_finite_differences_of_forward(name, hkv):
    S, D, Dv = 19, 6, 5
    var = variants(S)[name]
    q, k, v = rand((2, 1, 4, S, D), 1), rand((2, 1, hkv, S, D), 2), rand((2, 1, hkv, S, Dv), 3)
    dout = rand((2, 1, 4, S, Dv), 4)
    dq, dk, dv = bo.attention_backward(q, k, v, dout, scale=0.41, **var)

    def loss(q_, k_, v_):
        out, _ = ao.attention(q_, k_, v_, scale=0.41, **var)
        return float(np.sum(out * dout))

    eps = 1e-6
    r = np.random.Generator(np.random.PCG64(5))
    for grad, which in ((dq, 0), (dk, 1), (dv, 2)):
        base = (q, k, v)[which]
        for _ in range(12):
            idx = tuple(int(r.integers(0, n)) for n in base.shape)
            plus, minus = base.copy(), base.copy()
            plus[idx] += eps
            minus[idx] -= eps
            args_p = [q, k, v]
            args_m = [q, k, v]
            args_p[which], args_m[which] = plus, minus
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - grad[idx]) < 2e-8 * max(1.0, abs(fd)), (name, which, idx, fd, grad[idx])


def test_rectangular_shapes_finite_differences():
    q, k, v = rand((1, 2, 2, 7, 4), 6), rand((1, 2, 1, 23, 4), 7), rand((1, 2, 1, 23, 3), 8)
    dout = rand((1, 2, 2, 7, 3), 9)
    dq, dk, dv = bo.attention_backward(q, k, v, dout, scale=0.5, causal=True)
    eps = 1e-6
    for grad, which in ((dq, 0), (dk, 1), (dv, 2)):
        base = (q, k, v)[which]
        for idx in np.ndindex(*base.shape):
            if sum(idx) % 5:
                continue
            args_p, args_m = [q, k, v], [q, k, v]
            p_, m_ = base.copy(), base.copy()
            p_[idx] += eps
            m_[idx] -= eps
            args_p[which], args_m[which] = p_, m_
            fp = np.sum(ao.attention(*args_p, scale=0.5, causal=True)[0] * dout)
            fm = np.sum(ao.attention(*args_m, scale=0.5, causal=True)[0] * dout)
            assert abs((fp - fm) / (2 * eps) - grad[idx]) < 2e-8


# ---------------------------------------------------------------------------------------
# 2. Independent library routine: autograd through torch SDPA (fp64, CPU)
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["plain", "causal", "window", "prefix", "doc", "alibi_causal"])
def test_autograd_of_sdpa(name):
    S, D, Dv, H = 23, 8, 8, 4
    var = variants(S)[name]
    q, k, v = rand((2, 1, H, S, D), 21), rand((2, 1, H, S, D), 22), rand((2, 1, H, S, Dv), 23)
    dout = rand((2, 1, H, S, Dv), 24)
    i = np.arange(S)[:, None]
    j = np.arange(S)[None, :]
    allowed = np.ones((2, 1, H, S, S), dtype=bool)
    if var.get("causal"):
        allowed &= j <= i
    if "window" in var:
        allowed &= (j <= i) & (i - j <= var["window"])
    if "prefix" in var:
        allowed &= (j <= i) | (j < var["prefix"])
    if "q_doc" in var:
        d = var["q_doc"]
        allowed &= (d[:, :, None] == d[:, None, :])[:, None, None]
    bias = np.zeros((2, 1, H, S, S))
    if "alibi_slopes" in var:
        bias = bias - var["alibi_slopes"][None, None, :, None, None] * np.abs(i - j)
    mask = torch.from_numpy(np.where(allowed, bias, -np.inf)).reshape(2, H, S, S)
    tq, tk, tv = (torch.from_numpy(x.reshape(2, H, S, -1).copy()).requires_grad_(True) for x in (q, k, v))
    out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=0.37)
    out.backward(torch.from_numpy(dout.reshape(2, H, S, Dv).copy()))
    dq, dk, dv = bo.attention_backward(q, k, v, dout, scale=0.37, **var)
    for mine, ref in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        np.testing.assert_allclose(mine.reshape(ref.shape), ref.numpy(), rtol=0, atol=1e-12)


def test_softcap_autograd_of_plain_torch_ops():
    """Soft-cap is not expressible as an SDPA mask: autograd through matmul / tanh / softmax."""
    S, D, H = 17, 6, 2
    q, k, v = rand((1, 1, H, S, D), 31), rand((1, 1, H, S, D), 32), rand((1, 1, H, S, D), 33)
    dout = rand((1, 1, H, S, D), 34)
    tq, tk, tv = (torch.from_numpy(x[0, 0].copy()).requires_grad_(True) for x in (q, k, v))
    z = tq @ tk.transpose(-1, -2) * 0.6
    s = 1.3 * torch.tanh(z / 1.3)
    causal = torch.ones(S, S, dtype=torch.bool).tril()
    s = s.masked_fill(~causal, float("-inf"))
    o = torch.softmax(s, dim=-1) @ tv
    o.backward(torch.from_numpy(dout[0, 0].copy()))
    dq, dk, dv = bo.attention_backward(q, k, v, dout, scale=0.6, softcap_value=1.3, causal=True)
    np.testing.assert_allclose(dq[0, 0], tq.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dk[0, 0], tk.grad.numpy(), rtol=0, atol=1e-12)
    np.testing.assert_allclose(dv[0, 0], tv.grad.numpy(), rtol=0, atol=1e-12)


# ---------------------------------------------------------------------------------------
# 3. Closed forms and identities
# ---------------------------------------------------------------------------------------

def test_zero_queries_closed_form():
    """Q = 0, no mask: P = 1/Sk everywhere, so dV_j = mean-weight sum of dO rows, dK = 0 (it is
    multiplied by Q), and dQ_i = scale/Sk * sum_j (c_ij - mean_j c_ij) k_j with c = dO V^T."""
    Sq, Sk, D, Dv = 9, 13, 5, 4
    q = np.zeros((1, 1, 1, Sq, D))
    k, v, dout = rand((1, 1, 1, Sk, D), 41), rand((1, 1, 1, Sk, Dv), 42), rand((1, 1, 1, Sq, Dv), 43)
    dq, dk, dv = bo.attention_backward(q, k, v, dout, scale=0.7)
    np.testing.assert_allclose(dv[0, 0, 0], np.tile(dout[0, 0, 0].sum(0) / Sk, (Sk, 1)), atol=1e-13)
    np.testing.assert_allclose(dk, 0.0, atol=1e-15)
    c = dout[0, 0, 0] @ v[0, 0, 0].T
    want = 0.7 / Sk * (c - c.mean(axis=1, keepdims=True)) @ k[0, 0, 0]
    np.testing.assert_allclose(dq[0, 0, 0], want, atol=1e-13)


def test_identities():
    """Rows of P sum to one: sum_j dV_j = sum_i dO_i over rows with a visible key; the softmax
    Jacobian annihilates constants: sum_j dS_ij = 0, so dQ vanishes when every key is the same
    vector; delta equals rowsum(dO * O)."""
    S, D = 21, 4
    q, v, dout = rand((1, 1, 2, S, D), 51), rand((1, 1, 2, S, D), 52), rand((1, 1, 2, S, D), 53)
    k = rand((1, 1, 2, S, D), 54)
    dq, dk, dv, delta = bo.attention_backward(q, k, v, dout, scale=0.3, window=4, return_delta=True)
    np.testing.assert_allclose(dv.sum(axis=3), dout.sum(axis=3), atol=1e-12)
    # delta equals rowsum(dO * O), the form the fused kernels use
    out, _ = ao.attention(q, k, v, scale=0.3, window=4)
    np.testing.assert_allclose(delta, np.sum(out * dout, axis=-1), atol=1e-13)
    # with all keys equal to a constant vector c, dQ_i = scale * (sum_j dS_ij) c = 0
    kc = np.broadcast_to(rand((1, 1, 2, 1, D), 55), k.shape).copy()
    dq_c, _, _ = bo.attention_backward(q, kc, v, dout, scale=0.3, window=4)
    np.testing.assert_allclose(dq_c, 0.0, atol=1e-13)


def test_dead_rows_and_unseen_keys_get_no_gradient():
    """Document ids that never match: query rows of document 7 see no key -> dQ = 0 there, and
    keys of document 9 are seen by no row -> dK = dV = 0 there."""
    S, D = 12, 4
    q, k, v, dout = (rand((1, 1, 1, S, D), s) for s in (61, 62, 63, 64))
    q_doc = np.array([[0] * 6 + [7] * 6], dtype=np.int32)
    kv_doc = np.array([[0] * 8 + [9] * 4], dtype=np.int32)
    dq, dk, dv = bo.attention_backward(q, k, v, dout, scale=0.5, q_doc=q_doc, kv_doc=kv_doc)
    assert np.all(dq[0, 0, 0, 6:] == 0) and np.any(dq[0, 0, 0, :6] != 0)
    assert np.all(dk[0, 0, 0, 8:] == 0) and np.all(dv[0, 0, 0, 8:] == 0)
    assert np.any(dk[0, 0, 0, :8] != 0)


def test_single_visible_key_rows():
    """Causal row 0 sees only key 0: P = 1, dS = 0, so it adds dO_0 to dV_0 and nothing else."""
    S, D = 6, 4
    q, k, v = (rand((1, 1, 1, S, D), s) for s in (71, 72, 73))
    dout = np.zeros((1, 1, 1, S, D))
    dout[0, 0, 0, 0] = rand((D,), 74)
    dq, dk, dv = bo.attention_backward(q, k, v, dout, scale=0.5, causal=True)
    np.testing.assert_allclose(dq, 0.0, atol=1e-15)
    np.testing.assert_allclose(dk, 0.0, atol=1e-15)
    np.testing.assert_allclose(dv[0, 0, 0, 0], dout[0, 0, 0, 0], atol=1e-15)
    np.testing.assert_allclose(dv[0, 0, 0, 1:], 0.0, atol=1e-15)


def test_gqa_sums_over_the_group():
    """dK / dV of a shared head = sum of the per-head gradients with the head replicated."""
    S, D = 11, 4
    q, dout = rand((1, 1, 4, S, D), 81), rand((1, 1, 4, S, D), 82)
    k, v = rand((1, 1, 2, S, D), 83), rand((1, 1, 2, S, D), 84)
    dq, dk, dv = bo.attention_backward(q, k, v, dout, scale=0.5, causal=True)
    kr, vr = np.repeat(k, 2, axis=2), np.repeat(v, 2, axis=2)
    dq_r, dk_r, dv_r = bo.attention_backward(q, kr, vr, dout, scale=0.5, causal=True)
    np.testing.assert_allclose(dq, dq_r, atol=1e-14)
    np.testing.assert_allclose(dk, dk_r.reshape(1, 1, 2, 2, S, D).sum(axis=3), atol=1e-14)
    np.testing.assert_allclose(dv, dv_r.reshape(1, 1, 2, 2, S, D).sum(axis=3), atol=1e-14)
