"""GPU parity of the backward pass for variants outside the compiled table of backward kernels: the kernel templates
are instantiated at run time for the descriptor (score_mod x positional mask x document mask x biases), both through
fl_attn_bwd and as the core of the composed pass (fl_attn_bwd_ex), against the fp64 backward oracle.

Every descriptor the forward pass takes has a backward pass; the product is sampled here (each new variant costs a
few seconds of compilation): every score_mod, every positional mask, the document mask and both bias counts occur,
at both head dims of the kernels.  Tolerance: as for fl_attn_bwd_ex."""
import itertools

import pytest

from paper_2511_02043_amd import binding as fb
from paper_2511_02043_amd import inputs
from tests.test_gpu_backward_ex import compare

pytestmark = pytest.mark.gpu

C = inputs.combination_bf16
CASES = {
    # no bias: fl_attn_bwd
    "softcap_window_d64": lambda: C(D=64, score_mod="softcap", pos_mask="window", S=300),
    "alibi_prefix_d64": lambda: C(D=64, score_mod="alibi", pos_mask="prefix", S=260),
    "softcap_causal_doc_d64_gqa": lambda: C(D=64, score_mod="softcap", pos_mask="causal", doc=True, S=280, H=4, Hkv=2),
    "alibi_window_doc_d64": lambda: C(D=64, score_mod="alibi", pos_mask="window", doc=True, S=230, window=70),
    "alibi_causal_d128": lambda: C(D=128, score_mod="alibi", pos_mask="causal", S=300),
    "softcap_window_d128_gqa": lambda: C(D=128, score_mod="softcap", pos_mask="window", S=270, H=4, Hkv=1),
    "prefix_doc_d128": lambda: C(D=128, pos_mask="prefix", doc=True, S=200),
    "alibi_prefix_doc_d128": lambda: C(D=128, score_mod="alibi", pos_mask="prefix", doc=True, S=190),
    # biases: the composed pass around a run-time core
    "bias1_window_d64": lambda: C(D=64, n_bias=1, pos_mask="window", S=260),
    "bias2_softcap_causal_d64": lambda: C(D=64, n_bias=2, score_mod="softcap", pos_mask="causal", S=200, G=2),
    "bias1_alibi_doc_d64": lambda: C(D=64, n_bias=1, score_mod="alibi", doc=True, S=220),
    "bias1_prefix_d128": lambda: C(D=128, n_bias=1, pos_mask="prefix", S=180),
    "bias2_softcap_d128": lambda: C(D=128, n_bias=2, score_mod="softcap", S=150, G=2),
    # epilogues, the second stream and a padded head dim around a run-time core
    "gate_softcap_window_d32": lambda: C(D=32, score_mod="softcap", pos_mask="window", gate=True, S=240),
    "diff_alibi_causal_d64": lambda: C(D=64, score_mod="alibi", pos_mask="causal", diff=True, S=220),
    "rms_gate_bias1_softcap_prefix_doc_d64_dv128": lambda: C(D=64, Dv=128, n_bias=1, score_mod="softcap", pos_mask="prefix", doc=True,
                                                              rmsnorm=True, gate=True, S=170),
}


@pytest.mark.parametrize("name", list(CASES))
def test_backward_of_a_variant_outside_the_table(name):
    compare(CASES[name](), "f32", label=name)


def test_every_forward_descriptor_has_a_backward_pass():
    mods = (fb.FL_MOD_NONE, fb.FL_MOD_SOFTCAP, fb.FL_MOD_ALIBI)
    Cm, W, P, Dm = fb.FL_MASK_CAUSAL, fb.FL_MASK_WINDOW, fb.FL_MASK_PREFIX, fb.FL_MASK_DOC
    masks = (0, Cm, W | Cm, P, Dm, Cm | Dm, W | Cm | Dm, P | Dm)
    epis = (0, fb.FL_EPI_RMSNORM, fb.FL_EPI_GATE_SIGMOID, fb.FL_EPI_RMSNORM | fb.FL_EPI_GATE_SIGMOID)
    checked = 0
    for D, Dv in ((32, 32), (64, 64), (128, 128), (64, 128), (32, 64)):
        for mod, mask, nb, epi, comb in itertools.product(mods, masks, (0, 1, 2), epis, (fb.FL_SINGLE, fb.FL_DIFFERENTIAL)):
            d = fb.variant_desc(scale=0.1, score_mod=mod, softcap=2.0, mask=mask, window=5, prefix_len=5, n_bias=nb, epilogue=epi,
                                combine=comb, rms_eps=1e-5)
            if fb.fl_variant_supported(d, fb.FL_BF16, D, Dv):
                assert fb.fl_bwd_supported(d, fb.FL_BF16, D, Dv), (D, Dv, mod, mask, nb, epi, comb)
                checked += 1
    assert checked >= 1000
