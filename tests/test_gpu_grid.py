"""GPU parity on cells of the paper's benchmark grid (Sec. 4.1): seven variants, MHA and GQA
(16 query heads, 2 key/value heads), head dim 64, window and prefix length 256, 12 documents."""
import pytest

from paper_2511_02043_amd import inputs
from gpu_util import run_and_compare

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("variant", inputs.GRID_VARIANTS)
@pytest.mark.parametrize("gqa", [False, True])
def test_grid_cell_s512(variant, gqa):
    run_and_compare(inputs.grid_bf16(variant, 512, gqa=gqa, B=2), label=f"grid {variant} gqa={gqa} S=512")


@pytest.mark.parametrize("variant", ["vanilla", "causal", "softcap", "prefix_lm", "sliding_window", "document_mask"])
def test_grid_cell_s512_both_tile_shapes(variant):
    """Short key loops run the 32-key-tile shape by default; the 64-key-tile shape of the same variant
    (the default of long sequences) is forced here on the same cell."""
    from paper_2511_02043_amd import binding as fb
    try:
        for bn, wpe in ((64, 2), (32, 3 if variant == "document_mask" else 4)):
            fb.check(fb.fl_set_tuning("bn", bn))
            fb.check(fb.fl_set_tuning("wpe", wpe))
            run_and_compare(inputs.grid_bf16(variant, 512, B=2), label=f"grid {variant} S=512 bn={bn} wpe={wpe}")
            if variant == "document_mask":          # the same two shapes under window + document and causal + document masks
                run_and_compare(inputs.window_doc_bf16(B=2, H=2, S=700, D=64, window=100, lo=20, hi=300),
                                label=f"window + document bn={bn} wpe={wpe}")
                w = inputs.causal_bf16(B=2, H=2, S=600, D=64)
                w.q_doc = w.kv_doc = inputs.doc_ids(2, 600, seed=5, lo=20, hi=300)
                run_and_compare(w, label=f"causal + document bn={bn} wpe={wpe}")
    finally:
        fb.fl_set_tuning("bn", 0)
        fb.fl_set_tuning("wpe", 0)


@pytest.mark.parametrize("variant", ["sliding_window", "prefix_lm", "document_mask", "causal"])
def test_grid_cell_s2048_gqa(variant):
    """Longer rows: several key tiles inside and outside the window / prefix / documents."""
    run_and_compare(inputs.grid_bf16(variant, 2048, gqa=True, B=1), label=f"grid {variant} gqa S=2048")


@pytest.mark.parametrize("D", [32, 64, 128])
def test_columnwise_gated(D):
    """Attention over the sequence axis of [B, Nseq, Nres, H, D] storage (strided views), gate only."""
    run_and_compare(inputs.columnwise_gated_bf16(B=1, Nseq=200, Nres=6, H=2, D=D), label=f"column-wise gated D={D}")


@pytest.mark.parametrize("D", [64, 128])
def test_evoformer_paper_shape(D):
    run_and_compare(inputs.evoformer_paper_bf16(B=1, N=256, H=4, D=D), label=f"Evoformer 256x256 H=4 D={D}")


@pytest.mark.parametrize("S,D", [(512, 64), (1024, 128)])
def test_diffattn_paper_shape(S, D):
    run_and_compare(inputs.diffattn_paper_bf16(S=S, D=D, B=1, H=4), label=f"DiffAttn S={S} D={D}")


def test_diffattn_s512_both_tile_shapes():
    from paper_2511_02043_amd import binding as fb
    try:
        for bn, wpe in ((64, 2), (32, 4)):
            fb.check(fb.fl_set_tuning("bn", bn))
            fb.check(fb.fl_set_tuning("wpe", wpe))
            run_and_compare(inputs.diffattn_paper_bf16(S=512, D=64, B=1, H=4), label=f"DiffAttn S=512 D=64 bn={bn} wpe={wpe}")
    finally:
        fb.fl_set_tuning("bn", 0)
        fb.fl_set_tuning("wpe", 0)


def test_evoformer_d64_both_tile_shapes():
    from paper_2511_02043_amd import binding as fb
    try:
        for bn, wpe in ((64, 2), (32, 3)):
            fb.check(fb.fl_set_tuning("bn", bn))
            fb.check(fb.fl_set_tuning("wpe", wpe))
            run_and_compare(inputs.evoformer_paper_bf16(B=1, N=256, H=4, D=64), label=f"Evoformer 256x256 D=64 bn={bn} wpe={wpe}")
    finally:
        fb.fl_set_tuning("bn", 0)
        fb.fl_set_tuning("wpe", 0)


@pytest.mark.parametrize("variant", ["vanilla", "causal", "prefix_lm"])
def test_grid_cell_s4160_default_long_loop_shape(variant):
    """The two-row-block shape at head dim 64, the host's choice for long key loops on large launches (forced here:
    this launch is small), at a ragged length (4160 = 16 * 256 + 64); then the host's own choice for this launch."""
    from paper_2511_02043_amd import binding as fb
    w = inputs.grid_bf16(variant, 4160, B=1, H=2)
    try:
        fb.check(fb.fl_set_tuning("rb", 2))
        fb.check(fb.fl_set_tuning("bn", 32))
        run_and_compare(w, label=f"grid {variant} S=4160 H=2 two row blocks")
    finally:
        fb.fl_set_tuning("rb", 0)
        fb.fl_set_tuning("bn", 0)
    run_and_compare(w, label=f"grid {variant} S=4160 H=2")
