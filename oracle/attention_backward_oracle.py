"""CPU oracle for the gradient of the attention-variant forward pass.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this file; the
product path never does, and it shares no code with the HIP kernels.

The paper's conclusion names training as an extension it leaves open and prints no backward
algorithm, so this oracle is the plain derivative of the forward definition (Eq. 3, Eq. 4,
the attention listing), written out in NumPy float64 with every [Sq, Sk] matrix
materialised.  For one (b, g, h), with dO the gradient that arrives at the output:

    z  = scale * Q K^T                          Eq. 3
    t  = tanh(z / cap),  s = cap * t            soft-cap score_mod (Eq. 4), else s = z
    s  = s - slope_h |i - j|                    ALiBi score_mod (no dependence on Q, K)
    s  = -inf where masked
    P  = softmax_j(s)                           Eq. 2
    O  = P V

    dV = P^T dO
    dP = dO V^T
    dS = P * (dP - rowsum(P * dP))              Jacobian of the row softmax
    dZ = dS * (1 - t^2)                         soft-cap only; dZ = dS otherwise
    dQ = scale * dZ K
    dK = scale * dZ^T Q

With grouped-query attention the dK / dV of a key/value head are the sums over the query
heads that read it.  Masked positions have P = 0 and therefore dS = 0; a row whose keys are
all masked contributes nothing.

Additive biases enter s after the score_mod and before the mask, so dBias = dS summed over the
axes the bias broadcasts along.  The epilogues and the second softmax stream (variant_backward):

    x  = O1 - lambda_h O2                       differential listing (x = O for one stream)
    y  = w * x / r,  r = sqrt(mean_c x_c^2 + eps)        RMSNorm (benchmark configuration)
    out = sigmoid(g) * y                        gate

    dy = dout * sigmoid(g),   dg = dout * y * sigmoid(g) (1 - sigmoid(g))
    dx = w dy / r - x (sum_c w_c dy_c x_c) / (Dv r^3)
    dO1 = dx,  dO2 = -lambda_h dx,  dlambda_h = - sum_{rows, c} dx * O2
    then the softmax / contraction derivative above per stream; dV is the sum of both streams'.

Pins (tests/test_oracle_backward_pins.py): central finite differences of the forward oracle
on every variant; autograd through PyTorch's fp64 CPU scaled_dot_product_attention;
closed forms for Q = 0; the identities sum_j dV_j = sum_i dO_i and rowsum(dS) = 0;
zero gradient for fully masked rows and for keys no row can see.  attention_custom_backward (callable score_mod with
its derivative, callable mask) is pinned by finite differences of the forward oracle's attention_custom and by
attention_backward on named variants written as callables.
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def softmax_rows(s: np.ndarray):
    """Row softmax of s [Sq, Sk] with -inf entries; all -inf rows give zeros (Eq. 2)."""
    m = np.max(s, axis=1)
    dead = np.isneginf(m)
    e = np.exp(s - np.where(dead, 0.0, m)[:, None])
    l = np.sum(e, axis=1)
    return np.where(dead[:, None], 0.0, e / np.where(dead, 1.0, l)[:, None])


def mask_matrix(Sq: int, Sk: int, *, causal: bool, window: Optional[int], prefix: Optional[int],
                q_doc: Optional[np.ndarray], kv_doc: Optional[np.ndarray], q_offset: int = 0) -> np.ndarray:
    """True where score (i, j) is masked; the same four mask kinds as the forward pass.  Query row i sits
    at sequence position i + q_offset (the positional masks compare positions, document ids are per row)."""
    i = np.arange(Sq)[:, None] + q_offset
    j = np.arange(Sk)[None, :]
    masked = np.zeros((Sq, Sk), dtype=bool)
    if prefix is not None:
        masked |= (j > i) & (j >= prefix)
    elif causal or window is not None:
        masked |= j > i
    if window is not None:
        masked |= (i - j) > window
    if q_doc is not None:
        masked |= np.asarray(q_doc)[:, None] != np.asarray(kv_doc)[None, :]
    return masked


def attention_backward(q: np.ndarray, k: np.ndarray, v: np.ndarray, dout: np.ndarray, *,
                       scale: float, causal: bool = False, window: Optional[int] = None,
                       prefix: Optional[int] = None, softcap_value: Optional[float] = None,
                       alibi_slopes: Optional[np.ndarray] = None,
                       q_doc: Optional[np.ndarray] = None, kv_doc: Optional[np.ndarray] = None,
                       return_delta: bool = False, biases=(), return_dbias: bool = False, q_offset: int = 0):
    """Gradients of sum(out * dout) with respect to q, k, v.

    q [B,G,H,Sq,D], k [B,G,Hkv,Sk,D], v [B,G,Hkv,Sk,Dv], dout [B,G,H,Sq,Dv]; biases: arrays that
    broadcast to [B,G,H,Sq,Sk], added to the score after the score_mod (forward pipeline order).
    Returns dq, dk, dv (float64, shapes of q, k, v); with return_delta also
    delta [B,G,H,Sq] = rowsum(P * dP); with return_dbias also a list with the gradient of each
    bias in the bias's own shape (dS summed over the axes it broadcasts along).
    """
    B, G, H, Sq, D = q.shape
    Hkv, Sk, Dv = k.shape[2], k.shape[3], v.shape[4]
    assert H % Hkv == 0 and dout.shape == (B, G, H, Sq, Dv)
    group = H // Hkv
    dq = np.zeros((B, G, H, Sq, D))
    dk = np.zeros((B, G, Hkv, Sk, D))
    dv = np.zeros((B, G, Hkv, Sk, Dv))
    delta = np.zeros((B, G, H, Sq))
    full_biases = [np.broadcast_to(np.asarray(bb, dtype=np.float64), (B, G, H, Sq, Sk)) for bb in biases]
    ds_all = np.zeros((B, G, H, Sq, Sk)) if (return_dbias and biases) else None
    dist = np.abs(np.arange(Sq)[:, None] + q_offset - np.arange(Sk)[None, :]).astype(np.float64)
    for b in range(B):
        masked = mask_matrix(Sq, Sk, causal=causal, window=window, prefix=prefix,
                             q_doc=None if q_doc is None else q_doc[b],
                             kv_doc=None if kv_doc is None else kv_doc[b], q_offset=q_offset)
        for g in range(G):
            for h in range(H):
                hk = h // group
                qh = np.asarray(q[b, g, h], dtype=np.float64)
                kh = np.asarray(k[b, g, hk], dtype=np.float64)
                vh = np.asarray(v[b, g, hk], dtype=np.float64)
                do = np.asarray(dout[b, g, h], dtype=np.float64)
                z = (qh @ kh.T) * scale
                if softcap_value is not None:
                    t = np.tanh(z / softcap_value)
                    s = softcap_value * t
                else:
                    s = z
                if alibi_slopes is not None:
                    s = s - float(alibi_slopes[h]) * dist
                for fb_ in full_biases:
                    s = s + fb_[b, g, h]
                s = np.where(masked, -np.inf, s)
                p = softmax_rows(s)
                dv[b, g, hk] += p.T @ do
                dp = do @ vh.T
                row = np.sum(p * dp, axis=1)
                ds = p * (dp - row[:, None])
                if ds_all is not None:
                    ds_all[b, g, h] = ds               # gradient of the score after the score_mod
                if softcap_value is not None:
                    ds = ds * (1.0 - t * t)
                dq[b, g, h] = scale * (ds @ kh)
                dk[b, g, hk] += scale * (ds.T @ qh)
                delta[b, g, h] = row
    res = (dq, dk, dv)
    if return_delta:
        res = res + (delta,)
    if return_dbias:
        dbs = []
        for bb in biases:
            axes = tuple(a for a in range(5) if np.asarray(bb).shape[a] == 1 and (B, G, H, Sq, Sk)[a] != 1)
            dbs.append(np.sum(ds_all, axis=axes, keepdims=True) if axes else ds_all.copy())
        res = res + (dbs,)
    return res


def variant_backward(w, dout):
    """Gradients of sum(out * dout) for every part of an inputs.Workload (duck-typed): biases, the second
    softmax stream with lambda, RMSNorm and the sigmoid gate included.  Returns a dict with dq, dk, dv and,
    where the workload has them, dq2, dk2, dlambda [H], dbias (list), dgate, drms_weight [Dv]."""
    from oracle import attention_oracle as ao            # the pinned forward oracle gives the intermediates
    variant = dict(scale=w.scale, causal=w.causal, window=w.window, prefix=w.prefix, softcap_value=w.softcap,
                   alibi_slopes=w.alibi, q_doc=w.q_doc, kv_doc=w.kv_doc)
    fwd = dict(variant)
    fwd["biases"] = w.biases
    off = int(getattr(w, "q_offset", 0) or 0)
    if off:
        variant["q_offset"] = off
        fwd["q_pos"] = np.arange(w.q.shape[3], dtype=np.int64) + off
    dout = np.asarray(dout, dtype=np.float64)
    B, G, H, Sq, _ = w.q.shape
    Dv = w.v.shape[4]
    o1, _ = ao.attention(w.q, w.k, w.v, **fwd)
    diff = w.q2 is not None
    if diff:
        o2, _ = ao.attention(w.q2, w.k2, w.v, **fwd)
        lam = np.asarray(w.lam, dtype=np.float64)[None, None, :, None, None]
        x = o1 - lam * o2
    else:
        x = o1
    y = x
    if w.rmsnorm:
        wt = np.ones(Dv) if w.rms_weight is None else np.asarray(w.rms_weight, dtype=np.float64)
        r = np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + w.rms_eps)
        y = wt * x / r
    out = {}
    dy = dout
    if w.gate is not None:
        sg = 1.0 / (1.0 + np.exp(-np.asarray(w.gate, dtype=np.float64)))
        out["dgate"] = dout * y * sg * (1.0 - sg)
        dy = dout * sg
    dx = dy
    if w.rmsnorm:
        out["drms_weight"] = np.sum(dy * x / r, axis=(0, 1, 2, 3))
        dot = np.sum(wt * dy * x, axis=-1, keepdims=True)
        dx = wt * dy / r - x * dot / (Dv * r ** 3)
    do1 = dx
    if diff:
        out["dlambda"] = -np.sum(dx * o2, axis=(0, 1, 3, 4))
        do2 = -lam * dx
    need_db = len(w.biases) > 0
    r1 = attention_backward(w.q, w.k, w.v, do1, biases=w.biases, return_dbias=need_db, **variant)
    out["dq"], out["dk"], out["dv"] = r1[0], r1[1], r1[2]
    if need_db:
        out["dbias"] = r1[3]
    if diff:
        r2 = attention_backward(w.q2, w.k2, w.v, do2, biases=w.biases, return_dbias=need_db, **variant)
        out["dq2"], out["dk2"] = r2[0], r2[1]
        out["dv"] = out["dv"] + r2[2]
        if need_db:
            out["dbias"] = [a + b for a, b in zip(out["dbias"], r2[3])]
    return out


def run_workload_backward(w, dout):
    """Gradients for an inputs.Workload (duck-typed) that has no bias, gate, second stream or
    RMSNorm: the variants the backward kernels cover."""
    assert not w.biases and w.gate is None and w.q2 is None and not w.rmsnorm
    return attention_backward(w.q, w.k, w.v, dout, scale=w.scale, causal=w.causal, window=w.window,
                              prefix=w.prefix, softcap_value=w.softcap, alibi_slopes=w.alibi,
                              q_doc=w.q_doc, kv_doc=w.kv_doc, q_offset=int(getattr(w, "q_offset", 0) or 0))


def attention_custom_backward(q: np.ndarray, k: np.ndarray, v: np.ndarray, dout: np.ndarray, *, scale: float,
                              score_mod=None, score_mod_grad=None, mask=None):
    """Gradients of sum(out * dout) for the forward oracle's attention_custom(): an arbitrary score_mod (Eq. 4) and mask
    predicate (the mask_mod of Sec. 2.2, inverted), given as callables on NumPy arrays, plus the derivative of the
    score_mod with respect to the scaled score:

        score_mod(s, b, g, h, i, j) -> new scores          s [Sq, Sk], i [Sq, 1], j [1, Sk]
        score_mod_grad(s, b, g, h, i, j) -> d new / d s    (None: ones, right for s + f(b, g, h, i, j))
        mask(b, g, h, i, j) -> bool [Sq, Sk], True = hidden

    The same chain as attention_backward(): dV = P^T dO, dS = P * (dO V^T - rowsum), dZ = dS * score_mod_grad(z),
    dQ = scale dZ K, dK = scale dZ^T Q.  Returns dq, dk, dv (float64)."""
    B, G, H, Sq, D = q.shape
    Hkv, Sk = k.shape[2], k.shape[3]
    group = H // Hkv
    i = np.arange(Sq, dtype=np.int64)[:, None]
    j = np.arange(Sk, dtype=np.int64)[None, :]
    dq, dk, dv = np.zeros(q.shape), np.zeros(k.shape), np.zeros(v.shape)
    for b in range(B):
        for g in range(G):
            for h in range(H):
                hk = h // group
                qh = np.asarray(q[b, g, h], dtype=np.float64)
                kh = np.asarray(k[b, g, hk], dtype=np.float64)
                vh = np.asarray(v[b, g, hk], dtype=np.float64)
                do = np.asarray(dout[b, g, h], dtype=np.float64)
                z = (qh @ kh.T) * scale
                s = z if score_mod is None else np.asarray(score_mod(z, b, g, h, i, j), dtype=np.float64)
                slope = np.ones_like(z) if score_mod_grad is None else \
                    np.broadcast_to(np.asarray(score_mod_grad(z, b, g, h, i, j), dtype=np.float64), z.shape)
                if mask is not None:
                    s = np.where(np.broadcast_to(mask(b, g, h, i, j), z.shape), -np.inf, s)
                p = softmax_rows(s)
                dv[b, g, hk] += p.T @ do
                dp = do @ vh.T
                ds = p * (dp - np.sum(p * dp, axis=1)[:, None])
                dz = ds * slope
                dq[b, g, h] = scale * (dz @ kh)
                dk[b, g, hk] += scale * (dz.T @ qh)
    return dq, dk, dv
