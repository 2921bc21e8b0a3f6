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


@pytest.mark.parametrize("variant", ["sliding_window", "prefix_lm", "document_mask", "causal"])
def test_grid_cell_s2048_gqa(variant):
    """Longer rows: several key tiles inside and outside the window / prefix / documents."""
    run_and_compare(inputs.grid_bf16(variant, 2048, gqa=True, B=1), label=f"grid {variant} gqa S=2048")
