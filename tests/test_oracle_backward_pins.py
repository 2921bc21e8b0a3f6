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


# ---------------------------------------------------------------------------------------
# 6. Biases, gate, differential streams and RMSNorm (variant_backward): central finite differences of
#    the pinned forward oracle in every input, and autograd through an fp64 torch program built from
#    the library routine scaled_dot_product_attention (float mask = bias), sigmoid and elementwise ops.
# ---------------------------------------------------------------------------------------

def small_combo(diff, rms, gate, n_bias, mods, seed):
    w = inputs.combination_bf16(D=8, Dv=6, score_mod=mods[0], pos_mask=mods[1], doc=mods[2], n_bias=n_bias, diff=diff,
                                rmsnorm=rms, gate=gate, B=2, G=2, H=2, S=11, window=4, prefix=5, cap=1.3, salt=seed)
    # full-precision random values instead of bf16-rounded ones: the finite differences need smooth inputs
    for n, f in enumerate(("q", "k", "v", "q2", "k2", "gate")):
        x = getattr(w, f)
        if x is not None:
            setattr(w, f, rand(x.shape, seed * 31 + n))
    w.biases = tuple(rand(b.shape, seed * 7 + n) for n, b in enumerate(w.biases))
    if w.lam is not None:
        w.lam = np.array([0.35, 0.8])
    return w


COMBOS = {
    "bias1": dict(diff=False, rms=False, gate=False, n_bias=1, mods=("none", "none", False)),
    "bias2_gate_causal": dict(diff=False, rms=False, gate=True, n_bias=2, mods=("none", "causal", False)),
    "gate_softcap_window": dict(diff=False, rms=False, gate=True, n_bias=0, mods=("softcap", "window", False)),
    "rms_alone_prefix": dict(diff=False, rms=True, gate=False, n_bias=0, mods=("none", "prefix", False)),
    "diff_causal": dict(diff=True, rms=False, gate=False, n_bias=0, mods=("none", "causal", False)),
    "diff_rms_causal": dict(diff=True, rms=True, gate=False, n_bias=0, mods=("none", "causal", False)),
    "diff_rms_gate_bias_alibi_doc": dict(diff=True, rms=True, gate=True, n_bias=1, mods=("alibi", "causal", True)),
}


@pytest.mark.parametrize("name", list(COMBOS))
def test_variant_backward_finite_differences(name):
    w = small_combo(seed=3, **COMBOS[name])
    dout = rand(w.q.shape[:4] + (w.v.shape[4],), 99)
    g = bo.variant_backward(w, dout)

    def loss():
        out, _ = ao.run_workload(w)
        return float(np.sum(out * dout))

    fields = [("q", "dq"), ("k", "dk"), ("v", "dv")]
    if w.q2 is not None:
        fields += [("q2", "dq2"), ("k2", "dk2"), ("lam", "dlambda")]
    if w.gate is not None:
        fields.append(("gate", "dgate"))
    if w.rmsnorm:
        fields.append(("rms_weight", "drms_weight"))
    r = np.random.Generator(np.random.PCG64(17))
    eps = 1e-6

    def check(arr, grad, label):
        assert grad.shape == arr.shape, (label, grad.shape, arr.shape)
        for _ in range(8):
            idx = tuple(int(r.integers(0, n)) for n in arr.shape)
            keep = arr[idx]
            arr[idx] = keep + eps
            lp = loss()
            arr[idx] = keep - eps
            lm = loss()
            arr[idx] = keep
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - grad[idx]) <= 2e-6 * max(1.0, abs(fd)), (label, idx, fd, grad[idx])

    for field, gname in fields:
        arr = np.array(getattr(w, field), dtype=np.float64)
        setattr(w, field, arr)
        check(arr, g[gname], gname)
    biases = [np.array(b, dtype=np.float64) for b in w.biases]
    w.biases = tuple(biases)
    for n, b in enumerate(biases):
        check(b, g["dbias"][n], f"dbias[{n}]")


@pytest.mark.parametrize("name", ["bias2_gate_causal", "diff_rms_causal", "diff_rms_gate_bias_alibi_doc"])
def test_variant_backward_matches_torch_autograd(name):
    w = small_combo(seed=5, **COMBOS[name])
    dout = rand(w.q.shape[:4] + (w.v.shape[4],), 98)
    g = bo.variant_backward(w, dout)
    B, G, H, S, D = w.q.shape
    t = lambda x: torch.tensor(np.asarray(x, dtype=np.float64), requires_grad=True)
    q, k, v = t(w.q), t(w.k), t(w.v)
    biases = [t(b) for b in w.biases]
    i = np.arange(S)[:, None]
    j = np.arange(S)[None, :]
    hidden = np.zeros((B, 1, 1, S, S), dtype=bool)
    if w.causal:
        hidden |= (j > i)
    if w.q_doc is not None:
        hidden |= (w.q_doc[:, None, None, :, None] != w.kv_doc[:, None, None, None, :])
    mask = torch.zeros(B, G, H, S, S, dtype=torch.float64)
    if w.alibi is not None:
        mask = mask - torch.tensor(w.alibi.astype(np.float64))[None, None, :, None, None] * torch.tensor(np.abs(i - j).astype(np.float64))
    for b in biases:
        mask = mask + b
    mask = mask.masked_fill(torch.tensor(np.broadcast_to(hidden, (B, G, H, S, S)).copy()), float("-inf"))

    def sdpa(q_, k_):
        f = lambda x: x.reshape(B * G, H, S, -1)
        return torch.nn.functional.scaled_dot_product_attention(f(q_), f(k_), f(v), attn_mask=mask.reshape(B * G, H, S, S),
                                                                scale=w.scale).reshape(B, G, H, S, -1)
    x = sdpa(q, k)
    extra = {}
    if w.q2 is not None:
        q2, k2, lam = t(w.q2), t(w.k2), t(w.lam)
        x = x - lam[None, None, :, None, None] * sdpa(q2, k2)
        extra = dict(dq2=q2, dk2=k2, dlambda=lam)
    if w.rmsnorm:
        wt = t(w.rms_weight)
        x = wt * x / torch.sqrt(torch.mean(x * x, dim=-1, keepdim=True) + w.rms_eps)
        extra["drms_weight"] = wt
    if w.gate is not None:
        gt = t(w.gate)
        x = torch.sigmoid(gt) * x
        extra["dgate"] = gt
    (x * torch.tensor(dout)).sum().backward()
    for name_, leaf in dict(dq=q, dk=k, dv=v, **extra).items():
        np.testing.assert_allclose(g[name_], leaf.grad.numpy(), rtol=0, atol=1e-10, err_msg=name_)
    for n, b in enumerate(biases):
        np.testing.assert_allclose(g["dbias"][n], b.grad.numpy(), rtol=0, atol=1e-10, err_msg=f"dbias[{n}]")


def test_variant_backward_reduces_to_the_plain_one_and_identities():
    w = small_combo(seed=8, diff=False, rms=False, gate=False, n_bias=0, mods=("none", "causal", False))
    dout = rand(w.q.shape[:4] + (w.v.shape[4],), 97)
    g = bo.variant_backward(w, dout)
    ref = bo.attention_backward(w.q, w.k, w.v, dout, scale=w.scale, causal=True)
    for a, b in zip((g["dq"], g["dk"], g["dv"]), ref):
        np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)
    # a bias row-constant shift does not change the output, so the gradient of a [.., Sq, 1]-shaped bias is 0;
    # dbias of a full bias sums to zero over keys (rowsum(dS) = 0)
    wb = small_combo(seed=8, diff=False, rms=False, gate=True, n_bias=1, mods=("none", "none", False))
    gb = bo.variant_backward(wb, dout)
    np.testing.assert_allclose(np.sum(gb["dbias"][0], axis=-1), 0.0, atol=1e-12)
    # lambda = 0: the second stream gets no gradient; identical streams: dq2 = -lambda dq / (1 - lambda) ... checked by FD above
    wd = small_combo(seed=8, diff=True, rms=False, gate=False, n_bias=0, mods=("none", "none", False))
    wd.lam = np.zeros(2)
    gd = bo.variant_backward(wd, dout)
    assert np.all(gd["dq2"] == 0) and np.all(gd["dk2"] == 0)
    single = bo.attention_backward(wd.q, wd.k, wd.v, dout, scale=wd.scale)
    np.testing.assert_allclose(gd["dq"], single[0], rtol=0, atol=1e-13)
    np.testing.assert_allclose(gd["dv"], single[2], rtol=0, atol=1e-13)


# ---------------------------------------------------------------------------------------
# 7. Query-position offset: finite differences of the forward oracle (whose offset handling is pinned
#    against SDPA with the mask written out), and equality with the rows of the square problem.
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("kind", ["causal", "window", "prefix", "alibi_causal"])
def test_query_offset_backward(kind):
    Sq, Sk, off, D = 7, 19, 12, 6
    q, k, v = rand((1, 1, 2, Sq, D), 71), rand((1, 1, 2, Sk, D), 72), rand((1, 1, 2, Sk, D), 73)
    dout = rand((1, 1, 2, Sq, D), 74)
    var = dict(causal=dict(causal=True), window=dict(window=4), prefix=dict(prefix=15),
               alibi_causal=dict(causal=True, alibi_slopes=np.array([0.3, 0.7])))[kind]
    dq, dk, dv = bo.attention_backward(q, k, v, dout, scale=0.37, q_offset=off, **var)
    pos = np.arange(Sq) + off

    def loss(q_, k_, v_):
        out, _ = ao.attention(q_, k_, v_, scale=0.37, q_pos=pos, **var)
        return float(np.sum(out * dout))

    r = np.random.Generator(np.random.PCG64(75))
    eps = 1e-6
    for grad, which in ((dq, 0), (dk, 1), (dv, 2)):
        base = (q, k, v)[which]
        for _ in range(10):
            idx = tuple(int(r.integers(0, n)) for n in base.shape)
            plus, minus = base.copy(), base.copy()
            plus[idx] += eps
            minus[idx] -= eps
            args_p = [q, k, v]
            args_m = [q, k, v]
            args_p[which], args_m[which] = plus, minus
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - grad[idx]) <= 2e-6 * max(1.0, abs(fd)), (kind, which, idx)
    if kind == "causal":                            # the chunk's rows inside the square problem over the same keys
        qf = np.concatenate([np.zeros((1, 1, 2, off, D)), q], axis=3)
        df = np.concatenate([np.zeros((1, 1, 2, off, D)), dout], axis=3)
        dqf, dkf, dvf = bo.attention_backward(qf, k, v, df, scale=0.37, causal=True)
        np.testing.assert_allclose(dq, dqf[:, :, :, off:], rtol=0, atol=1e-13)
        np.testing.assert_allclose(dk, dkf, rtol=0, atol=1e-13)
        np.testing.assert_allclose(dv, dvf, rtol=0, atol=1e-13)


# --- arbitrary score_mod / mask callables -------------------------------------------------------------------------------

def test_custom_backward_equals_the_named_variants_written_as_callables():
    """Soft-cap + causal and ALiBi + window as callables against attention_backward's own branches."""
    from paper_2511_02043_amd import inputs
    w = inputs.causal_bf16(B=1, H=4, Hkv=2, S=37, Sk=53, D=16, causal=False, salt=31)
    dout = inputs.dout_for(w)
    cap = 1.7
    a = bo.attention_custom_backward(w.q, w.k, w.v, dout, scale=w.scale,
                                     score_mod=lambda s, b, g, h, i, j: cap * np.tanh(s / cap),
                                     score_mod_grad=lambda s, b, g, h, i, j: 1.0 - np.tanh(s / cap) ** 2,
                                     mask=lambda b, g, h, i, j: j > i)
    r = bo.attention_backward(w.q, w.k, w.v, dout, scale=w.scale, causal=True, softcap_value=cap)
    for x, y in zip(a, r):
        np.testing.assert_allclose(x, y, rtol=0, atol=1e-13)
    slopes = inputs.alibi_slopes(4).astype(np.float64)
    a = bo.attention_custom_backward(w.q, w.k, w.v, dout, scale=w.scale,
                                     score_mod=lambda s, b, g, h, i, j: s - slopes[h] * np.abs(i - j),
                                     mask=lambda b, g, h, i, j: (j > i) | (i - j > 9))
    r = bo.attention_backward(w.q, w.k, w.v, dout, scale=w.scale, causal=True, window=9, alibi_slopes=slopes)
    for x, y in zip(a, r):
        np.testing.assert_allclose(x, y, rtol=0, atol=1e-13)


def test_custom_backward_against_finite_differences_of_the_forward_oracle():
    """A score_mod that is neither additive nor monotone in a simple way, a mask that reads h, grouped heads."""
    from oracle import attention_oracle as ao
    rng = np.random.Generator(np.random.PCG64(77))
    B, G, H, Hkv, Sq, Sk, D = 1, 1, 2, 1, 5, 7, 4
    q, k, v = rng.normal(size=(B, G, H, Sq, D)), rng.normal(size=(B, G, Hkv, Sk, D)), rng.normal(size=(B, G, Hkv, Sk, D))
    dout = rng.normal(size=(B, G, H, Sq, D))
    mod = lambda s, b, g, h, i, j: 2.0 * np.sin(0.7 * s) + 0.1 * s * s - 0.05 * (h + 1) * np.abs(i - j)
    grad = lambda s, b, g, h, i, j: 1.4 * np.cos(0.7 * s) + 0.2 * s
    msk = lambda b, g, h, i, j: ((i + j + h) % 3 == 0) & (j > 0)
    dq, dk, dv = bo.attention_custom_backward(q, k, v, dout, scale=0.5, score_mod=mod, score_mod_grad=grad, mask=msk)

    def loss(q_, k_, v_):
        o, _ = ao.attention_custom(q_, k_, v_, scale=0.5, score_mod=mod, mask=msk)
        return float(np.sum(o * dout))

    eps = 1e-6
    for name, x, gx in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        flat = x.reshape(-1)
        for idx in rng.choice(flat.size, size=12, replace=False):
            old = flat[idx]
            flat[idx] = old + eps
            up = loss(q, k, v)
            flat[idx] = old - eps
            dn = loss(q, k, v)
            flat[idx] = old
            np.testing.assert_allclose(gx.reshape(-1)[idx], (up - dn) / (2 * eps), rtol=2e-6, atol=2e-8, err_msg=name)
