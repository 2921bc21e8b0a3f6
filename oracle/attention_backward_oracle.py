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

Pins (tests/test_oracle_backward_pins.py): central finite differences of the forward oracle
on every variant; autograd through PyTorch's fp64 CPU scaled_dot_product_attention;
closed forms for Q = 0; the identities sum_j dV_j = sum_i dO_i and rowsum(dS) = 0;
zero gradient for fully masked rows and for keys no row can see.
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
                q_doc: Optional[np.ndarray], kv_doc: Optional[np.ndarray]) -> np.ndarray:
    """True where score (i, j) is masked; the same four mask kinds as the forward pass."""
    i = np.arange(Sq)[:, None]
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
                       return_delta: bool = False):
    """Gradients of sum(out * dout) with respect to q, k, v.

    q [B,G,H,Sq,D], k [B,G,Hkv,Sk,D], v [B,G,Hkv,Sk,Dv], dout [B,G,H,Sq,Dv].
    Returns dq, dk, dv (float64, shapes of q, k, v); with return_delta also
    delta [B,G,H,Sq] = rowsum(P * dP).
    """
    B, G, H, Sq, D = q.shape
    Hkv, Sk, Dv = k.shape[2], k.shape[3], v.shape[4]
    assert H % Hkv == 0 and dout.shape == (B, G, H, Sq, Dv)
    group = H // Hkv
    dq = np.zeros((B, G, H, Sq, D))
    dk = np.zeros((B, G, Hkv, Sk, D))
    dv = np.zeros((B, G, Hkv, Sk, Dv))
    delta = np.zeros((B, G, H, Sq))
    dist = np.abs(np.arange(Sq)[:, None] - np.arange(Sk)[None, :]).astype(np.float64)
    for b in range(B):
        masked = mask_matrix(Sq, Sk, causal=causal, window=window, prefix=prefix,
                             q_doc=None if q_doc is None else q_doc[b],
                             kv_doc=None if kv_doc is None else kv_doc[b])
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
                s = np.where(masked, -np.inf, s)
                p = softmax_rows(s)
                dv[b, g, hk] += p.T @ do
                dp = do @ vh.T
                row = np.sum(p * dp, axis=1)
                ds = p * (dp - row[:, None])
                if softcap_value is not None:
                    ds = ds * (1.0 - t * t)
                dq[b, g, h] = scale * (ds @ kh)
                dk[b, g, hk] += scale * (ds.T @ qh)
                delta[b, g, h] = row
    if return_delta:
        return dq, dk, dv, delta
    return dq, dk, dv


def run_workload_backward(w, dout):
    """Gradients for an inputs.Workload (duck-typed) that has no bias, gate, second stream or
    RMSNorm: the variants the backward kernels cover."""
    assert not w.biases and w.gate is None and w.q2 is None and not w.rmsnorm
    return attention_backward(w.q, w.k, w.v, dout, scale=w.scale, causal=w.causal, window=w.window,
                              prefix=w.prefix, softcap_value=w.softcap, alibi_slopes=w.alibi,
                              q_doc=w.q_doc, kv_doc=w.kv_doc)
