"""CPU oracle for single-query (decode-step) attention over a paged key/value cache.
TEST INFRASTRUCTURE ONLY: only tests, the smoke check and the benchmark's cpu_baseline leg may
import this file; the product path never does, and it shares no code with the HIP kernels.

The paper evaluates its kernels inside a serving system (Sec. 4.1, the LLaMa / vLLM experiment:
time to first token and inter-token latency), where every generated token runs attention with
one query row per sequence against that sequence's cached keys and values.  The arithmetic is the
forward definition (Eq. 3 with the score_mod of Eq. 4) for the single query at position
len_b - 1; what is new is only where the keys live: in fixed-size pages of a shared cache,
addressed through a per-sequence block table.

    k_cache, v_cache  [num_pages, page_size, Hkv, D]
    block_table       [B, max_pages]   page of the p-th block of sequence b
    seq_lens          [B]              number of cached tokens (the query is the last of them)

For sequence b and query head h (kv head h // (H // Hkv)), with keys j = 0 .. len_b - 1:

    s_j = scale * <q, k_j>;  s_j = cap * tanh(s_j / cap);  s_j -= slope_h * (len_b - 1 - j)
    visible iff len_b - 1 - j <= window (when a window is given)
    out = sum_j softmax(s)_j v_j,   lse = log sum_j exp(s_j)

A sequence of length 0 has out = 0 and lse = -inf.  Everything is float64.

Pins (tests/test_oracle_decode_pins.py): the last row of the pinned forward oracle on the
gathered contiguous keys (causal), a pure-Python brute force, invariance under a permutation of
the physical pages, len = 1 (out = v_0), constant values, and the window's visible count.
prefill_attention (a chunk of query rows per sequence) is pinned to the forward oracle on the gathered
keys with the rows placed at their positions, to PyTorch's fp64 scaled_dot_product_attention with a
bottom-right causal mask, to decode_attention at Sq = 1, to chunk-by-chunk consistency (any split of
a prompt into chunks gives the rows of the one-shot result), and to the empty rows of len < Sq.
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def gather_sequence(cache: np.ndarray, block_table: np.ndarray, b: int, length: int) -> np.ndarray:
    """[length, Hkv, D] rows of sequence b, token by token through its block table."""
    page_size = cache.shape[1]
    rows = np.empty((length,) + cache.shape[2:], dtype=np.float64)
    for j in range(length):
        rows[j] = cache[block_table[b, j // page_size], j % page_size]
    return rows


def decode_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, block_table: np.ndarray,
                     seq_lens: np.ndarray, *, scale: float, window: Optional[int] = None,
                     softcap_value: Optional[float] = None, alibi_slopes: Optional[np.ndarray] = None):
    """q [B, H, D] -> out [B, H, Dv], lse [B, H] (float64)."""
    B, H, D = q.shape
    Hkv = k_cache.shape[2]
    assert H % Hkv == 0
    group = H // Hkv
    out = np.zeros((B, H, v_cache.shape[3]))
    lse = np.full((B, H), -np.inf)
    for b in range(B):
        n = int(seq_lens[b])
        if n == 0:
            continue
        keys = gather_sequence(k_cache, block_table, b, n)
        vals = gather_sequence(v_cache, block_table, b, n)
        dist = (n - 1 - np.arange(n)).astype(np.float64)          # query position minus key position
        for h in range(H):
            hk = h // group
            s = scale * (keys[:, hk] @ np.asarray(q[b, h], dtype=np.float64))
            if softcap_value is not None:
                s = softcap_value * np.tanh(s / softcap_value)
            if alibi_slopes is not None:
                s = s - float(alibi_slopes[h]) * dist
            if window is not None:
                s = np.where(dist > window, -np.inf, s)
            m = np.max(s)
            e = np.exp(s - m)
            l = np.sum(e)
            out[b, h] = (e / l) @ vals[:, hk]
            lse[b, h] = m + np.log(l)
    return out, lse


def prefill_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, block_table: np.ndarray,
                      seq_lens: np.ndarray, *, scale: float, window: Optional[int] = None,
                      softcap_value: Optional[float] = None, alibi_slopes: Optional[np.ndarray] = None):
    """A chunk of Sq query rows per sequence against that sequence's paged cache -- the prompt phase of
    the serving experiment (Sec. 4.1, time to first token) when the prompt is processed in chunks, or a
    prompt that continues a cached prefix.  The chunk's own keys are already in the cache: row i of
    sequence b is the token at position len_b - Sq + i and sees keys 0 .. that position (causal; with a
    window, the last window + 1 of them).  Rows whose position is negative (len_b < Sq) see nothing:
    out = 0, lse = -inf.  Same score pipeline as decode_attention, which is the case Sq = 1.

    q [B, H, Sq, D] -> out [B, H, Sq, Dv], lse [B, H, Sq] (float64)."""
    B, H, Sq, D = q.shape
    Hkv = k_cache.shape[2]
    assert H % Hkv == 0
    group = H // Hkv
    out = np.zeros((B, H, Sq, v_cache.shape[3]))
    lse = np.full((B, H, Sq), -np.inf)
    for b in range(B):
        n = int(seq_lens[b])
        if n == 0:
            continue
        keys = gather_sequence(k_cache, block_table, b, n)
        vals = gather_sequence(v_cache, block_table, b, n)
        for i in range(Sq):
            pos = n - Sq + i
            if pos < 0:
                continue
            dist = (pos - np.arange(pos + 1)).astype(np.float64)
            for h in range(H):
                hk = h // group
                s = scale * (keys[:pos + 1, hk] @ np.asarray(q[b, h, i], dtype=np.float64))
                if softcap_value is not None:
                    s = softcap_value * np.tanh(s / softcap_value)
                if alibi_slopes is not None:
                    s = s - float(alibi_slopes[h]) * dist
                if window is not None:
                    s = np.where(dist > window, -np.inf, s)
                m = np.max(s)
                e = np.exp(s - m)
                l = np.sum(e)
                out[b, h, i] = (e / l) @ vals[:pos + 1, hk]
                lse[b, h, i] = m + np.log(l)
    return out, lse
