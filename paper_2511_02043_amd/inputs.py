"""Seeded synthetic inputs for the attention-variant forward path.

This module is the one piece shared by the CPU oracle's tests and the HIP path's
tests / benchmark.  It holds no attention arithmetic: it only draws random tensors,
rounds them to the storage precision, and names the workload shapes.

Every tensor is returned as a float32 NumPy array whose values are exactly
representable in the storage dtype (bf16 or fp32), so that the oracle (which
upcasts to fp64) and the GPU (which receives the same bits) see identical inputs.

The paper's own kernel benchmarks run on randomly generated tensors (artifact
appendix, "Data sets"), so synthetic N(0,1) data *is* the paper's workload.

Logical layout used everywhere: q [B, G, H, Sq, D], k [B, G, Hkv, Sk, D],
v [B, G, Hkv, Sk, Dv], where G is an extra independent row axis (1 for ordinary
attention, the MSA-sequence axis for Evoformer row-wise attention).
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np

SEED_BASE = 251102043 * 1000


def tensor_seed(config: int, tensor_index: int, salt: int = 0) -> int:
    """One independent PCG64 stream per (config, tensor)."""
    return SEED_BASE + 10 * config + tensor_index + 100000 * salt


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even), in integer arithmetic.

    Returns float32 holding bf16-representable values.  NaN is not expected in inputs.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = bits + np.uint32(0x7FFF) + lsb
    rounded &= np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    if np.any(bits & np.uint32(0xFFFF)):
        raise ValueError("values are not bf16-representable")
    return (bits >> np.uint32(16)).astype(np.uint16)


def normal(shape, seed: int, dtype: str = "bf16", scale: float = 1.0) -> np.ndarray:
    """N(0, scale^2) tensor from its own PCG64 stream, rounded to `dtype`."""
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        x = x * np.float32(scale)
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return x
    raise ValueError(f"unknown dtype {dtype!r}")


def alibi_slopes(n_heads: int) -> np.ndarray:
    """Geometric slope sequence 2^(-8 (h+1) / H) for zero-based head h (float32)."""
    h = np.arange(1, n_heads + 1, dtype=np.float64)
    return np.exp2(-8.0 * h / n_heads).astype(np.float32)


def doc_ids(batch: int, seq: int, seed: int, lo: int = 64, hi: int = 1024) -> np.ndarray:
    """Per-token document ids [batch, seq] (int32).

    For each batch element independently: integer run lengths uniform on [lo, hi]
    inclusive, concatenated until the sequence is covered, last run truncated;
    the id of a token is the index of its run.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    out = np.empty((batch, seq), dtype=np.int32)
    for b in range(batch):
        pos, doc = 0, 0
        while pos < seq:
            run = int(rng.integers(lo, hi + 1))
            out[b, pos:pos + run] = doc
            pos += run
            doc += 1
    return out


@dataclasses.dataclass
class Workload:
    """A named problem instance: tensors plus the variant's parameters."""
    name: str
    dtype: str                      # storage dtype of q/k/v: "bf16" | "f32"
    q: np.ndarray                   # [B, G, H, Sq, D]
    k: np.ndarray                   # [B, G, Hkv, Sk, D]
    v: np.ndarray                   # [B, G, Hkv, Sk, Dv]
    scale: float
    causal: bool = False
    window: Optional[int] = None    # allowed iff 0 <= i - j <= window (with causal)
    prefix: Optional[int] = None    # prefix-LM: keys j < prefix are visible to every query
    softcap: Optional[float] = None
    alibi: Optional[np.ndarray] = None      # [H] float32 slopes
    q_doc: Optional[np.ndarray] = None      # [B, Sq] int32
    kv_doc: Optional[np.ndarray] = None     # [B, Sk] int32
    biases: tuple = ()                      # each broadcastable to [B, G, H, Sq, Sk]
    gate: Optional[np.ndarray] = None       # [B, G, H, Sq, Dv] pre-sigmoid
    q2: Optional[np.ndarray] = None         # differential: second stream
    k2: Optional[np.ndarray] = None
    lam: Optional[np.ndarray] = None        # [H] float32
    rmsnorm: bool = False
    rms_eps: float = 1e-6
    rms_weight: Optional[np.ndarray] = None  # [Dv] float32
    q_offset: int = 0               # query row i sits at sequence position i + q_offset (keys: j at j)

    @property
    def dims(self) -> Dict[str, int]:
        B, G, H, Sq, D = self.q.shape
        return dict(B=B, G=G, H=H, Hkv=self.k.shape[2], Sq=Sq, Sk=self.k.shape[3],
                    D=D, Dv=self.v.shape[4])


def _qkv(cfg, B, G, H, Sq, Sk, D, Dv, dtype, Hkv=None, salt=0, qscale=1.0):
    Hkv = H if Hkv is None else Hkv
    q = normal((B, G, H, Sq, D), tensor_seed(cfg, 0, salt), dtype, qscale)
    k = normal((B, G, Hkv, Sk, D), tensor_seed(cfg, 1, salt), dtype)
    v = normal((B, G, Hkv, Sk, Dv), tensor_seed(cfg, 2, salt), dtype)
    return q, k, v


def dout_for(w: "Workload", salt: int = 0) -> np.ndarray:
    """Seeded N(0,1) gradient arriving at the output of `w` ([B, G, H, Sq, Dv], rounded to the
    storage dtype), for the backward pass.  Tensor index 9 of configuration 7 in the seed recipe."""
    B, G, H, Sq, _ = w.q.shape
    return normal((B, G, H, Sq, w.v.shape[4]), tensor_seed(7, 9, salt), w.dtype)


# --- the five benchmark configurations, each shrinkable for parity tests -----------------

def plain_f32(B=1, H=2, S=128, D=64, Sk=None, salt=0) -> Workload:
    """Config 1: plain softmax attention, fp32 storage, no mask."""
    Sk = S if Sk is None else Sk
    q, k, v = _qkv(1, B, 1, H, S, Sk, D, D, "f32", salt=salt)
    return Workload("plain_f32", "f32", q, k, v, scale=D ** -0.5)


def causal_bf16(B=4, H=16, S=8192, D=128, Hkv=None, Sk=None, salt=0, causal=True) -> Workload:
    """Config 2: causal attention, bf16 storage (D=128, repeated at D=64)."""
    Sk = S if Sk is None else Sk
    q, k, v = _qkv(2, B, 1, H, S, Sk, D, D, "bf16", Hkv=Hkv, salt=salt)
    return Workload(f"causal_bf16_d{D}" if causal else f"plain_bf16_d{D}", "bf16", q, k, v,
                    scale=D ** -0.5, causal=causal)


def alibi_bf16(B=8, H=16, S=2048, D=64, salt=0) -> Workload:
    """Config 3a: ALiBi bias -slope_h |i-j| on the scaled score, no mask."""
    q, k, v = _qkv(3, B, 1, H, S, S, D, D, "bf16", salt=salt)
    return Workload("alibi_bf16", "bf16", q, k, v, scale=D ** -0.5, alibi=alibi_slopes(H))


def softcap_bf16(B=8, H=16, S=2048, D=64, cap=30.0, qscale=1.0, salt=0) -> Workload:
    """Config 3b: tanh soft-capping of the scaled score at `cap`.

    qscale > 1 widens the score distribution so that tanh actually saturates.
    """
    q, k, v = _qkv(3, B, 1, H, S, S, D, D, "bf16", salt=salt, qscale=qscale)
    return Workload("softcap_bf16", "bf16", q, k, v, scale=D ** -0.5, softcap=cap)


def window_doc_bf16(B=8, H=16, S=2048, D=64, window=512, lo=64, hi=1024, salt=0) -> Workload:
    """Config 3c: sliding-window causal mask AND a document mask from per-token ids."""
    q, k, v = _qkv(3, B, 1, H, S, S, D, D, "bf16", salt=salt)
    ids = doc_ids(B, S, tensor_seed(3, 3, salt), lo, hi)
    return Workload("window_doc_bf16", "bf16", q, k, v, scale=D ** -0.5, causal=True,
                    window=window, q_doc=ids, kv_doc=ids)


def differential_bf16(B=2, H=16, S=4096, D=64, Dv=128, lam=0.8, salt=0, dtype="bf16", causal=True,
                      rmsnorm=True) -> Workload:
    """Config 4: differential attention (two softmax streams sharing V), causal, RMSNorm.

    One allocation of 2H heads for q and for k; pair h is (head h, head H + h),
    as in the paper's differential-attention listing (chunk along the head axis).
    """
    q_all = normal((B, 1, 2 * H, S, D), tensor_seed(4, 0, salt), dtype)
    k_all = normal((B, 1, 2 * H, S, D), tensor_seed(4, 1, salt), dtype)
    v = normal((B, 1, H, S, Dv), tensor_seed(4, 2, salt), dtype)
    return Workload("differential_" + dtype, dtype, q_all[:, :, :H], k_all[:, :, :H], v,
                    scale=D ** -0.5, causal=causal, q2=q_all[:, :, H:], k2=k_all[:, :, H:],
                    lam=np.full((H,), lam, dtype=np.float32), rmsnorm=rmsnorm, rms_eps=1e-6)


def evoformer_bf16(B=1, Nseq=128, Nres=384, H=8, D=32, two_biases=False, salt=0,
                   dtype="bf16") -> Workload:
    """Config 5: Evoformer row-wise gated self-attention with pair bias.

    Activations are stored [B, Nseq, Nres, H, D]; the returned arrays are the
    [B, G=Nseq, H, S=Nres, D] *views* of that storage (non-contiguous), which is the
    layout the kernel must consume.  The pair bias [B, 1, H, Nres, Nres] broadcasts
    over the Nseq axis; the optional second bias [B, Nseq, 1, 1, Nres] is the
    per-row key mask bias of the MSA stack, broadcast over heads and queries.
    """
    def act(idx):
        x = normal((B, Nseq, Nres, H, D), tensor_seed(5, idx, salt), dtype)
        return x.transpose(0, 1, 3, 2, 4)
    q, k, v, gate = act(0), act(1), act(2), act(4)
    biases = [normal((B, 1, H, Nres, Nres), tensor_seed(5, 3, salt), dtype)]
    if two_biases:
        biases.append(normal((B, Nseq, 1, 1, Nres), tensor_seed(5, 5, salt), dtype))
    return Workload("evoformer_" + dtype, dtype, q, k, v, scale=D ** -0.5,
                    biases=tuple(biases), gate=gate)


# --- the paper's benchmark grid (Sec. 4.1, "Benchmarks") -----------------------------------

GRID_VARIANTS = ("vanilla", "alibi", "softcap", "causal", "sliding_window", "prefix_lm", "document_mask")
GRID_SEQ_LENS = (512, 1024, 2048, 4096, 8192, 16384)


def doc_ids_fixed_count(batch: int, seq: int, n_docs: int, seed: int) -> np.ndarray:
    """Per-token document ids [batch, seq] (int32) with exactly n_docs documents per batch
    element: n_docs - 1 distinct cut points drawn uniformly from 1..seq-1, sorted."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = np.empty((batch, seq), dtype=np.int32)
    for b in range(batch):
        cuts = np.sort(rng.choice(np.arange(1, seq), size=n_docs - 1, replace=False))
        out[b] = np.searchsorted(cuts, np.arange(seq), side="right").astype(np.int32)
    return out


def grid_bf16(variant: str, S: int, gqa: bool = False, B: Optional[int] = None, tokens: int = 16384,
              H: int = 16, D: int = 64, window: int = 256, prefix: int = 256, n_docs: int = 12,
              cap: float = 30.0, salt: int = 0) -> Workload:
    """One cell of the paper's grid: sequence length S with batch * S = 16k tokens, head dim 64,
    16 query heads and 16 (MHA) or 2 (GQA) key/value heads; window and prefix length 256,
    12 documents (Sec. 4.1).  Config number 6 in the seed recipe."""
    if variant not in GRID_VARIANTS:
        raise ValueError(f"unknown grid variant {variant!r}")
    B = max(1, tokens // S) if B is None else B
    q, k, v = _qkv(6, B, 1, H, S, S, D, D, "bf16", Hkv=2 if gqa else H, salt=salt + 100 * GRID_VARIANTS.index(variant))
    w = Workload(f"grid_{variant}_{'gqa' if gqa else 'mha'}_s{S}", "bf16", q, k, v, scale=D ** -0.5)
    if variant == "alibi":
        w.alibi = alibi_slopes(H)
    elif variant == "softcap":
        w.softcap = cap
    elif variant == "causal":
        w.causal = True
    elif variant == "sliding_window":
        w.causal, w.window = True, window
    elif variant == "prefix_lm":
        w.prefix = min(prefix, S)
    elif variant == "document_mask":
        ids = doc_ids_fixed_count(B, S, min(n_docs, S), tensor_seed(6, 3, salt))
        w.q_doc = w.kv_doc = ids
    return w


def columnwise_gated_bf16(B=1, Nseq=128, Nres=256, H=8, D=32, salt=0, dtype="bf16") -> Workload:
    """Column-wise gated self-attention of the MSA stack (named in Sec. 1): attention runs over the
    sequence axis independently for each residue column, no bias, sigmoid gate.  Activations are
    stored [B, Nseq, Nres, H, D] as for the row-wise case; the arrays returned are the
    [B, G=Nres, H, S=Nseq, D] views of that storage."""
    def act(idx):
        x = normal((B, Nseq, Nres, H, D), tensor_seed(5, idx, salt + 7), dtype)
        return x.transpose(0, 2, 3, 1, 4)
    q, k, v, gate = act(0), act(1), act(2), act(4)
    return Workload("columnwise_gated_" + dtype, dtype, q, k, v, scale=D ** -0.5, gate=gate)


def evoformer_paper_bf16(B=1, N=256, H=4, D=64, salt=0) -> Workload:
    """The paper's Evoformer benchmark shape (Sec. 4.1): both sequence dimensions 256, 4 heads,
    head dim 64 or 128, batch 1..32, two biases (one broadcast over the extra dimension), gate."""
    w = evoformer_bf16(B=B, Nseq=N, Nres=N, H=H, D=D, two_biases=True, salt=salt + 11)
    w.name = f"evoformer_paper_b{B}_d{D}"
    return w


def diffattn_paper_bf16(S=2048, D=64, B=None, H=16, tokens=16384, salt=0) -> Workload:
    """The paper's DiffAttn benchmark shape (Sec. 4.1): the MHA grid (16 heads, head dim 64, batch * S =
    16k tokens) and 16 heads with head dim 128; no mask, no normalisation, as in the listing."""
    B = max(1, tokens // S) if B is None else B
    w = differential_bf16(B=B, H=H, S=S, D=D, Dv=D, salt=salt + 13, causal=False, rmsnorm=False)
    w.name = f"diffattn_paper_s{S}_d{D}"
    return w


def combination_bf16(D=64, Dv=None, score_mod="none", pos_mask="none", doc=False, n_bias=0, diff=False, rmsnorm=False,
                     gate=False, B=2, G=1, H=4, Hkv=None, S=200, Sk=None, window=37, prefix=45, cap=4.0, qscale=2.0,
                     salt=0) -> Workload:
    """Any combination of the descriptor's independent parts (Eq. 4 score_mod x positional mask x
    document mask x additive biases x differential streams x epilogues), small enough for the oracle:
    score_mod in {"none", "alibi", "softcap"}, pos_mask in {"none", "causal", "window", "prefix"}.
    Bias 0 is a per-query pair bias [B, 1, H, Sq, Sk] (broadcast over G), bias 1 a per-row key bias
    [B, G, 1, 1, Sk].  Configuration 7 in the seed recipe."""
    Dv = D if Dv is None else Dv
    Sk = S if Sk is None else Sk
    Hkv = H if Hkv is None else Hkv
    nq = 2 * H if diff else H
    nk = 2 * Hkv if diff else Hkv
    q_all = normal((B, G, nq, S, D), tensor_seed(7, 0, salt), "bf16", qscale if score_mod == "softcap" else 1.0)
    k_all = normal((B, G, nk, Sk, D), tensor_seed(7, 1, salt), "bf16")
    v = normal((B, G, Hkv, Sk, Dv), tensor_seed(7, 2, salt), "bf16")
    w = Workload(f"combo_d{D}_{Dv}_{score_mod}_{pos_mask}{'_doc' if doc else ''}_b{n_bias}{'_diff' if diff else ''}"
                 f"{'_rms' if rmsnorm else ''}{'_gate' if gate else ''}", "bf16", q_all[:, :, :H], k_all[:, :, :Hkv], v,
                 scale=D ** -0.5)
    if diff:
        w.q2, w.k2 = q_all[:, :, H:], k_all[:, :, Hkv:]
        w.lam = np.linspace(0.3, 0.9, H).astype(np.float32)
    if score_mod == "alibi":
        w.alibi = alibi_slopes(H)
    elif score_mod == "softcap":
        w.softcap = cap
    if pos_mask == "causal":
        w.causal = True
    elif pos_mask == "window":
        w.causal, w.window = True, window
    elif pos_mask == "prefix":
        w.prefix = prefix
    if doc:
        ids = doc_ids(B, max(S, Sk), tensor_seed(7, 3, salt), 20, 90)
        w.q_doc, w.kv_doc = np.ascontiguousarray(ids[:, :S]), np.ascontiguousarray(ids[:, :Sk])
    biases = []
    if n_bias >= 1:
        biases.append(normal((B, 1, H, S, Sk), tensor_seed(7, 4, salt), "bf16"))
    if n_bias >= 2:
        biases.append(normal((B, G, 1, 1, Sk), tensor_seed(7, 5, salt), "bf16"))
    w.biases = tuple(biases)
    if gate:
        w.gate = normal((B, G, H, S, Dv), tensor_seed(7, 6, salt), "bf16")
    if rmsnorm:
        w.rmsnorm = True
        w.rms_weight = (1.0 + 0.1 * np.cos(np.arange(Dv))).astype(np.float32)
    return w


# --- decode step over a paged key/value cache (the serving experiment of Sec. 4.1) -----------

@dataclasses.dataclass
class DecodeWorkload:
    """One decode step: a query per sequence against that sequence's cached keys / values."""
    name: str
    q: np.ndarray                   # [B, H, D]
    k_cache: np.ndarray             # [num_pages, page_size, Hkv, D]
    v_cache: np.ndarray             # [num_pages, page_size, Hkv, D]
    block_table: np.ndarray         # [B, max_pages] int32
    seq_lens: np.ndarray            # [B] int32
    scale: float
    window: Optional[int] = None
    softcap: Optional[float] = None
    alibi: Optional[np.ndarray] = None


def decode_bf16(B=4, H=8, Hkv=2, D=128, page_size=16, seq_lens=None, max_len=512, salt=0, shuffle_pages=True,
                spare_pages=3) -> DecodeWorkload:
    """Paged-cache decode step.  Sequence lengths (if not given) are uniform on [1, max_len]; every
    sequence owns ceil(len / page_size) pages drawn from one shuffled pool, so the physical order
    of a sequence's pages is arbitrary (as in a serving system's allocator).  Configuration 8 in
    the seed recipe.  Unused slots of the cache hold NaN-free random values like the used ones."""
    rng = np.random.Generator(np.random.PCG64(tensor_seed(8, 5, salt)))
    if seq_lens is None:
        seq_lens = rng.integers(1, max_len + 1, size=B)
    seq_lens = np.asarray(seq_lens, dtype=np.int32)
    B = len(seq_lens)
    pages_per_seq = [(int(n) + page_size - 1) // page_size for n in seq_lens]
    max_pages = max(1, max(pages_per_seq))
    n_pages = sum(pages_per_seq) + spare_pages
    pool = np.arange(n_pages, dtype=np.int32)
    if shuffle_pages:
        rng.shuffle(pool)
    table = np.zeros((B, max_pages), dtype=np.int32)
    pos = 0
    for b, npg in enumerate(pages_per_seq):
        table[b, :npg] = pool[pos:pos + npg]
        pos += npg
    q = normal((B, H, D), tensor_seed(8, 0, salt))
    k_cache = normal((n_pages, page_size, Hkv, D), tensor_seed(8, 1, salt))
    v_cache = normal((n_pages, page_size, Hkv, D), tensor_seed(8, 2, salt))
    return DecodeWorkload(f"decode_bf16_d{D}_p{page_size}", q, k_cache, v_cache, table, seq_lens, scale=D ** -0.5)


def prefill_paged_bf16(B=3, H=8, Hkv=2, D=128, Sq=64, page_size=16, seq_lens=None, max_len=512, salt=0,
                       shuffle_pages=True) -> DecodeWorkload:
    """A chunk of Sq query rows per sequence against the same kind of paged cache as decode_bf16 (the
    prompt phase of the serving experiment of Sec. 4.1, processed in chunks): q is [B, H, Sq, D], row i
    of sequence b being the token at position len_b - Sq + i.  Lengths (if not given) are uniform on
    [1, max_len], so some may be shorter than the chunk."""
    w = decode_bf16(B=B, H=H, Hkv=Hkv, D=D, page_size=page_size, seq_lens=seq_lens, max_len=max_len, salt=salt,
                    shuffle_pages=shuffle_pages)
    w.q = normal((len(w.seq_lens), H, Sq, D), tensor_seed(8, 6, salt))
    w.name = f"prefill_paged_bf16_d{D}_p{page_size}_q{Sq}"
    return w
