"""Every part of the variant descriptor combines with every other (Eq. 4's score_mod x the mask_mod kinds
x additive biases x the differential streams x the epilogues, Sec. 2.2 / 4.1), at every head dim: a
pairwise-covering sample of the whole product is run through fl_attn_fwd and compared with the oracle
element by element.  Combinations outside the compiled table are instantiated from the same kernel
template on first use, so fl_variant_supported has to say yes to all of them."""
import itertools

import numpy as np
import pytest

from paper_2511_02043_amd import binding as fb
from paper_2511_02043_amd import inputs
from tests.gpu_util import run_and_compare

FACTORS = dict(D=[32, 64, 128], score_mod=["none", "alibi", "softcap"], pos_mask=["none", "causal", "window", "prefix"],
               doc=[False, True], n_bias=[0, 1, 2], diff=[False, True], rmsnorm=[False, True], gate=[False, True])


def pairwise_sample():
    """Greedy pairwise cover of FACTORS (deterministic): every pair of values of every two factors occurs in a case."""
    names = list(FACTORS)
    need = set()
    for a, b in itertools.combinations(range(len(names)), 2):
        for va in FACTORS[names[a]]:
            for vb in FACTORS[names[b]]:
                need.add((a, va, b, vb))
    rng = np.random.Generator(np.random.PCG64(2511))
    cases = []
    while need:
        best, gain = None, -1
        for _ in range(60):
            cand = tuple(FACTORS[n][int(rng.integers(len(FACTORS[n])))] for n in names)
            g = sum((a, cand[a], b, cand[b]) in need for a, b in itertools.combinations(range(len(names)), 2))
            if g > gain:
                best, gain = cand, g
        cases.append(dict(zip(names, best)))
        for a, b in itertools.combinations(range(len(names)), 2):
            need.discard((a, best[a], b, best[b]))
    return cases


CASES = pairwise_sample()


def case_id(c):
    return "-".join(f"{k}={v}" for k, v in c.items())


def test_sample_covers_every_pair_of_parts():
    assert 12 <= len(CASES) <= 60
    names = list(FACTORS)
    for a, b in itertools.combinations(names, 2):
        for va in FACTORS[a]:
            for vb in FACTORS[b]:
                assert any(c[a] == va and c[b] == vb for c in CASES), (a, va, b, vb)


def test_every_combination_is_reported_as_supported():
    for D, Dv in itertools.product((32, 64, 128), repeat=2):
        for mod in (fb.FL_MOD_NONE, fb.FL_MOD_ALIBI, fb.FL_MOD_SOFTCAP):
            for mask in (0, fb.FL_MASK_CAUSAL, fb.FL_MASK_WINDOW, fb.FL_MASK_PREFIX, fb.FL_MASK_DOC,
                         fb.FL_MASK_WINDOW | fb.FL_MASK_DOC, fb.FL_MASK_PREFIX | fb.FL_MASK_DOC):
                for nb, comb, epi in itertools.product((0, 1, 2), (fb.FL_SINGLE, fb.FL_DIFFERENTIAL), (0, 1, 2, 3)):
                    d = fb.variant_desc(scale=0.1, score_mod=mod, softcap=5.0, mask=mask, window=3, prefix_len=3, n_bias=nb,
                                        combine=comb, epilogue=epi, rms_eps=1e-6)
                    assert fb.fl_variant_supported(d, fb.FL_BF16, D, Dv), (D, Dv, mod, mask, nb, comb, epi)
    contradictory = fb.variant_desc(scale=0.1, mask=fb.FL_MASK_PREFIX | fb.FL_MASK_CAUSAL)
    assert not fb.fl_variant_supported(contradictory, fb.FL_BF16, 64, 64)
    assert not fb.fl_variant_supported(fb.variant_desc(scale=0.1), fb.FL_BF16, 96, 96)


@pytest.mark.gpu
@pytest.mark.parametrize("case", CASES, ids=case_id)
def test_combination_matches_oracle(case):
    w = inputs.combination_bf16(S=200, B=2, H=4, **case)
    run_and_compare(w, label=w.name)


@pytest.mark.gpu
def test_combinations_with_different_head_dims_grouped_heads_and_row_axis():
    """D != Dv, grouped-query heads, an extra row axis and a ragged rectangular problem on combinations
    that only exist as run-time instantiations."""
    run_and_compare(inputs.combination_bf16(D=32, Dv=128, score_mod="alibi", pos_mask="causal", gate=True, S=150, H=4, Hkv=2))
    run_and_compare(inputs.combination_bf16(D=128, Dv=64, score_mod="softcap", pos_mask="window", doc=True, n_bias=1, G=3, S=130))
    run_and_compare(inputs.combination_bf16(D=64, Dv=32, pos_mask="prefix", diff=True, rmsnorm=True, gate=True, S=97, Sk=230))
