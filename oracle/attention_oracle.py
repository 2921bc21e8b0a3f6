"""CPU oracle for the attention-variant forward pass.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition that the GPU kernels are checked against.
Only tests, the smoke check and the benchmark's cpu_baseline leg may import it; the
product path never does, and it shares no code with the HIP kernels.

Everything is NumPy float64.  For every (batch b, row-axis g, head h) the full
[Sq, Sk] score matrix is materialised, the variant is applied to it, a stable
softmax is taken per row and the result is multiplied by V -- exactly the unfused
program of the paper's attention listing (Sec. 2.2, Eq. 3, Listing "Attention in
PyTorch"), which the fused kernel reproduces exactly in real arithmetic (Sec. 2.2,
FlashAttention paragraph; Sec. 3.3, ds[N] = do[N]).

Order of the per-score pipeline (the paper fixes scale -> score_mod -> softmax in
Eq. 4 and scale -> mask -> softmax in the attention listing; the relative order of
the mods when several are combined is this build's reading):

    s = scale * <q_i, k_j>                      Eq. 3
    s = cap * tanh(s / cap)                     score_mod on the scaled score, Eq. 4
    s = s - slope_h * |i - j|                   score_mod (ALiBi), Eq. 4
    s = s + sum_k bias_k[b, g, h, i, j]         Evoformer biases, Sec. 4.1 "Benchmarks"
    s = -inf where masked                       attention listing, masked_fill(mask, -INF)
    P = stable softmax over j                   Eq. 2, Alg. 1
    o_i = sum_j P_ij v_j                        Eq. 3

Masks (True = masked) combine by OR:
    causal : j > i
    window : j > i  or  i - j > W               sliding-window listings (both agree)
    prefix : j > i  and  j >= prefix_len        PrefixLM (named in Sec. 4.1)
    doc    : doc_q[b, i] != doc_kv[b, j]        Document mask (named in Sec. 4.1)

A row whose keys are all masked has out = 0 and lse = -inf (the unfused listing would
produce NaN there; the paper does not discuss it).

lse_i = m_i + ln(l_i) with m_i, l_i the post-conditions of Alg. 1 / Alg. 2.

Pins (tests/test_oracle_*.py): the fp64 CPU scaled_dot_product_attention routine of
PyTorch on every mask / bias kind; a pure-Python brute force written separately
(oracle/brute_force.py); closed forms for Q = 0 (prefix means, ln(count), geometric
ALiBi sums); single-visible-key rows; constant-V rows; row sums of P; a scalar run
of Alg. 2; key-permutation and bias-shift invariances; differential with lambda = 0
and with identical streams; gate = +40 / -40; attention_custom against attention() with
ALiBi / window written as callables and against SDPA with an arbitrary predicate.  RMSNorm (not in the paper; defined by
the benchmark configuration) is pinned only by its definition written out in the
brute force, unit mean square, and scale invariance: parity unpinned beyond that.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import numpy as np

NEG_INF = -np.inf


def scaled_scores(q: np.ndarray, k: np.ndarray, scale: float) -> np.ndarray:
    """s_ij = scale * sum_d q_id k_jd  (Eq. 3).  q [Sq, D], k [Sk, D] -> [Sq, Sk]."""
    return (q @ k.T) * scale


def softcap(s: np.ndarray, cap: float) -> np.ndarray:
    """Soft-capping score_mod: cap * tanh(s / cap), applied to the scaled score (Eq. 4)."""
    return cap * np.tanh(s / cap)


def alibi(s: np.ndarray, slope: float, q_pos: np.ndarray, k_pos: np.ndarray) -> np.ndarray:
    """ALiBi score_mod: s - slope * |i - j|  (Eq. 4; symmetric, no mask implied)."""
    dist = np.abs(q_pos[:, None] - k_pos[None, :]).astype(np.float64)
    return s - slope * dist


def masked_positions(q_pos: np.ndarray, k_pos: np.ndarray, *, causal: bool = False,
                     window: Optional[int] = None, prefix: Optional[int] = None,
                     q_doc: Optional[np.ndarray] = None,
                     kv_doc: Optional[np.ndarray] = None) -> np.ndarray:
    """Boolean [Sq, Sk], True where the score is to be replaced by -inf."""
    i = q_pos[:, None]
    j = k_pos[None, :]
    masked = np.zeros((q_pos.shape[0], k_pos.shape[0]), dtype=bool)
    if prefix is not None:
        masked |= (j > i) & (j >= prefix)
    elif causal or window is not None:
        masked |= j > i
    if window is not None:
        masked |= (i - j) > window
    if q_doc is not None:
        masked |= q_doc[:, None] != kv_doc[None, :]
    return masked


def stable_softmax(s: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Row-wise stable softmax (Eq. 2 / Alg. 1) and its log-sum-exp.

    Returns P [Sq, Sk] and lse [Sq] = m + ln(l).  Rows that are entirely -inf give
    P = 0 and lse = -inf.
    """
    m = np.max(s, axis=1)                                  # first loop of Alg. 1
    dead = np.isneginf(m)
    m_safe = np.where(dead, 0.0, m)
    e = np.exp(s - m_safe[:, None])                        # e^{x_j - m_N}; exp(-inf) = 0
    l = np.sum(e, axis=1)                                  # second loop of Alg. 1
    with np.errstate(divide="ignore", invalid="ignore"):
        p = np.where(dead[:, None], 0.0, e / np.where(dead, 1.0, l)[:, None])
        lse = np.where(dead, NEG_INF, m_safe + np.log(np.where(dead, 1.0, l)))
    return p, lse


def _bias_slice(bias: np.ndarray, b: int, g: int, h: int) -> np.ndarray:
    """[.., .., .., Sq|1, Sk|1] slice of a bias broadcastable to [B, G, H, Sq, Sk]."""
    bb = b if bias.shape[0] > 1 else 0
    gg = g if bias.shape[1] > 1 else 0
    hh = h if bias.shape[2] > 1 else 0
    return np.asarray(bias[bb, gg, hh], dtype=np.float64)


def attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, *, scale: float,
              causal: bool = False, window: Optional[int] = None,
              prefix: Optional[int] = None, softcap_value: Optional[float] = None,
              alibi_slopes: Optional[np.ndarray] = None,
              biases: Sequence[np.ndarray] = (),
              q_doc: Optional[np.ndarray] = None, kv_doc: Optional[np.ndarray] = None,
              q_pos: Optional[np.ndarray] = None,
              return_probs: bool = False):
    """Attention variant forward on q [B,G,H,Sq,D], k [B,G,Hkv,Sk,D], v [B,G,Hkv,Sk,Dv].

    Hkv divides H: query head h reads key/value head h // (H // Hkv) (grouped-query
    attention, Sec. 4.1).  q_pos gives the absolute sequence position of each query
    row (default 0..Sq-1); it lets a caller evaluate a sample of rows of a large
    problem.  Returns out [B,G,H,Sq,Dv] and lse [B,G,H,Sq] (float64), and the
    probabilities [B,G,H,Sq,Sk] too if return_probs.
    """
    B, G, H, Sq, D = q.shape
    Hkv, Sk, Dv = k.shape[2], k.shape[3], v.shape[4]
    assert H % Hkv == 0
    group = H // Hkv
    q_pos = np.arange(Sq, dtype=np.int64) if q_pos is None else np.asarray(q_pos, np.int64)
    k_pos = np.arange(Sk, dtype=np.int64)
    out = np.zeros((B, G, H, Sq, Dv), dtype=np.float64)
    lse = np.zeros((B, G, H, Sq), dtype=np.float64)
    probs = np.zeros((B, G, H, Sq, Sk), dtype=np.float64) if return_probs else None
    any_mask = causal or window is not None or prefix is not None or q_doc is not None
    for b in range(B):
        masked = None
        if any_mask:
            masked = masked_positions(
                q_pos, k_pos, causal=causal, window=window, prefix=prefix,
                q_doc=None if q_doc is None else np.asarray(q_doc[b]),
                kv_doc=None if kv_doc is None else np.asarray(kv_doc[b]))
        for g in range(G):
            for h in range(H):
                qh = np.asarray(q[b, g, h], dtype=np.float64)
                kh = np.asarray(k[b, g, h // group], dtype=np.float64)
                vh = np.asarray(v[b, g, h // group], dtype=np.float64)
                s = scaled_scores(qh, kh, scale)
                if softcap_value is not None:
                    s = softcap(s, float(softcap_value))
                if alibi_slopes is not None:
                    s = alibi(s, float(alibi_slopes[h]), q_pos, k_pos)
                for bias in biases:
                    s = s + _bias_slice(bias, b, g, h)
                if masked is not None:
                    s = np.where(masked, NEG_INF, s)
                p, row_lse = stable_softmax(s)
                out[b, g, h] = p @ vh
                lse[b, g, h] = row_lse
                if return_probs:
                    probs[b, g, h] = p
    if return_probs:
        return out, lse, probs
    return out, lse


def attention_custom(q: np.ndarray, k: np.ndarray, v: np.ndarray, *, scale: float, score_mod=None, mask=None):
    """Attention with an arbitrary score_mod (Eq. 4) and mask predicate (the mask_mod of Sec. 2.2,
    inverted: True = hidden), given as callables on NumPy arrays:

        score_mod(s, b, g, h, i, j) -> new scores     s [Sq, Sk] scaled scores, i [Sq, 1], j [1, Sk]
        mask(b, g, h, i, j)         -> bool [Sq, Sk]

    Same unfused program as attention(): scores, score_mod, mask -> -inf, stable softmax, P V.
    Returns out [B,G,H,Sq,Dv] and lse [B,G,H,Sq] (float64)."""
    B, G, H, Sq, D = q.shape
    Hkv, Sk = k.shape[2], k.shape[3]
    group = H // Hkv
    i = np.arange(Sq, dtype=np.int64)[:, None]
    j = np.arange(Sk, dtype=np.int64)[None, :]
    out = np.zeros((B, G, H, Sq, v.shape[4]))
    lse = np.zeros((B, G, H, Sq))
    for b in range(B):
        for g in range(G):
            for h in range(H):
                s = scaled_scores(np.asarray(q[b, g, h], np.float64), np.asarray(k[b, g, h // group], np.float64), scale)
                if score_mod is not None:
                    s = np.asarray(score_mod(s, b, g, h, i, j), dtype=np.float64)
                if mask is not None:
                    s = np.where(np.broadcast_to(mask(b, g, h, i, j), s.shape), NEG_INF, s)
                p, row_lse = stable_softmax(s)
                out[b, g, h] = p @ np.asarray(v[b, g, h // group], np.float64)
                lse[b, g, h] = row_lse
    return out, lse


def rmsnorm(x: np.ndarray, eps: float, weight: Optional[np.ndarray] = None) -> np.ndarray:
    """x * w / sqrt(mean(x^2 over the last axis) + eps).  Defined by the benchmark
    configuration for differential attention, not by the paper."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    y = x / np.sqrt(ms + eps)
    if weight is not None:
        y = y * np.asarray(weight, dtype=np.float64)
    return y


def differential_attention(q1, k1, q2, k2, v, lam, *, scale: float,
                           rms: bool = False, rms_eps: float = 1e-6,
                           rms_weight: Optional[np.ndarray] = None, **variant):
    """Differential attention (differential-attention listing, Sec. 3):
    attention(q1, k1, v) - lambda_h * attention(q2, k2, v), same V and mask for both
    streams, optionally followed by per-head RMSNorm over the Dv channels.

    Returns out [B,G,H,Sq,Dv] and lse [B,2,G,H,Sq] (stream index in axis 1).
    """
    o1, lse1 = attention(q1, k1, v, scale=scale, **variant)
    o2, lse2 = attention(q2, k2, v, scale=scale, **variant)
    lam = np.asarray(lam, dtype=np.float64).reshape(1, 1, -1, 1, 1)
    out = o1 - lam * o2
    if rms:
        out = rmsnorm(out, rms_eps, rms_weight)
    return out, np.stack([lse1, lse2], axis=1)


def sigmoid_gate(out: np.ndarray, gate: np.ndarray) -> np.ndarray:
    """Evoformer output gating: sigmoid(g) * out, elementwise (Sec. 1 / Sec. 4.1 name
    the gated variant; the gate tensor has the output's shape)."""
    g = np.asarray(gate, dtype=np.float64)
    return out / (1.0 + np.exp(-g))


def run_workload(w, q_rows=None):
    """Evaluate an inputs.Workload (duck-typed: only its fields are read).

    Returns out [B,G,H,Sq,Dv] and lse ([B,G,H,Sq], or [B,2,G,H,Sq] for differential).
    """
    variant = dict(causal=w.causal, window=w.window, prefix=w.prefix,
                   softcap_value=w.softcap, alibi_slopes=w.alibi, biases=w.biases,
                   q_doc=w.q_doc, kv_doc=w.kv_doc)
    off = int(getattr(w, "q_offset", 0) or 0)
    if off:                                                # query row i sits at position i + q_offset
        variant["q_pos"] = np.arange(w.q.shape[3], dtype=np.int64) + off
    if w.q2 is not None:
        out, lse = differential_attention(w.q, w.k, w.q2, w.k2, w.v, w.lam, scale=w.scale,
                                          rms=w.rmsnorm, rms_eps=w.rms_eps,
                                          rms_weight=w.rms_weight, **variant)
    else:
        out, lse = attention(w.q, w.k, w.v, scale=w.scale, **variant)
        if w.rmsnorm:
            out = rmsnorm(out, w.rms_eps, w.rms_weight)
    if w.gate is not None:
        out = sigmoid_gate(out, w.gate)
    return out, lse


def run_workload_rows(w, picks):
    """Oracle values for single output rows of a (possibly very large) workload.

    picks: iterable of (b, g, h, i).  Each row is computed from the plain definition
    against all keys of its head.  Returns a list of (out_row [Dv], lse) where lse is
    a float (or a length-2 array for differential).
    """
    results = []
    H = w.q.shape[2]
    group = H // w.k.shape[2]

    def one(x, b, g, h):
        return np.asarray(x[b:b + 1, g:g + 1, h:h + 1], dtype=np.float64)

    def sl(n, idx):
        return 0 if n == 1 else idx

    for (b, g, h, i) in picks:
        hk = h // group
        biases = []
        for bias in w.biases:
            bb, gg, hh = sl(bias.shape[0], b), sl(bias.shape[1], g), sl(bias.shape[2], h)
            ii = sl(bias.shape[3], i)
            biases.append(np.asarray(bias[bb:bb + 1, gg:gg + 1, hh:hh + 1, ii:ii + 1],
                                     dtype=np.float64))
        variant = dict(causal=w.causal, window=w.window, prefix=w.prefix,
                       softcap_value=w.softcap,
                       alibi_slopes=None if w.alibi is None else w.alibi[h:h + 1],
                       biases=biases,
                       q_doc=None if w.q_doc is None else w.q_doc[b:b + 1, i:i + 1],
                       kv_doc=None if w.kv_doc is None else w.kv_doc[b:b + 1],
                       q_pos=np.array([i + int(getattr(w, "q_offset", 0) or 0)]))
        q = one(w.q, b, g, h)[:, :, :, i:i + 1]
        k, v = one(w.k, b, g, hk), one(w.v, b, g, hk)
        if w.q2 is not None:
            q2 = one(w.q2, b, g, h)[:, :, :, i:i + 1]
            k2 = one(w.k2, b, g, hk)
            out, lse = differential_attention(q, k, q2, k2, v, w.lam[h:h + 1], scale=w.scale,
                                              rms=w.rmsnorm, rms_eps=w.rms_eps,
                                              rms_weight=w.rms_weight, **variant)
            lse_val = lse[0, :, 0, 0, 0]
        else:
            out, lse = attention(q, k, v, scale=w.scale, **variant)
            if w.rmsnorm:
                out = rmsnorm(out, w.rms_eps, w.rms_weight)
            lse_val = float(lse[0, 0, 0, 0])
        if w.gate is not None:
            out = sigmoid_gate(out, np.asarray(w.gate[b:b + 1, g:g + 1, h:h + 1, i:i + 1]))
        results.append((out[0, 0, 0, 0], lse_val))
    return results
