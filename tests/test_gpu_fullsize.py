"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

C3 (three score-mod / mask variants), C4 and C5 are compared element by element against the
full oracle (it finishes in tens of seconds on the host).  C2 (S = 8192, 64 heads) is checked
on sampled output rows that the oracle computes one by one from the plain definition, chosen to
cover the first rows, tile and workgroup boundaries, the diagonal tiles and the last row."""
import numpy as np
import pytest

from oracle import attention_oracle as ao
from paper_2511_02043_amd import inputs, runner
from tests.gpu_util import TOL, compare_whole_heads, errors, run_and_compare

pytestmark = pytest.mark.gpu


def sample_rows(S, rng, n_random=24):
    fixed = [0, 1, 2, 3, 31, 32, 33, 63, 64, 127, 128, 255, 256, 257, 511, 512, S // 2 - 1, S // 2, S - 257, S - 256,
             S - 2, S - 1]
    rows = sorted(set(r for r in fixed if 0 <= r < S) | set(int(x) for x in rng.integers(0, S, n_random)))
    return rows


@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("out_dtype", ["same", "f32"])
def test_c2_full_size_sampled_rows(D, out_dtype):
    import torch
    w = inputs.causal_bf16(D=D)
    dw = runner.upload(w, out_dtype=out_dtype)
    dw.run_checked()
    torch.cuda.synchronize()
    rng = np.random.Generator(np.random.PCG64(99 + D))
    picks = []
    for (b, h) in [(0, 0), (1, 5), (3, 15), (2, 8)]:
        picks += [(b, 0, h, i) for i in sample_rows(8192, rng)]
    out = dw.out.float().cpu().numpy()
    lse = dw.lse.cpu().numpy()[..., 0]
    ref = ao.run_workload_rows(w, picks)
    got = np.stack([out[b, g, h, i] for (b, g, h, i) in picks]).astype(np.float64)
    want = np.stack([o for (o, _) in ref])
    max_abs, rel_l2 = errors(got, want)
    lse_err = max(abs(float(lse[b, g, h, i]) - l) for (b, g, h, i), (_, l) in zip(picks, ref))
    print(f"c2 D={D} out={out_dtype}: {len(picks)} rows max_abs={max_abs:.3e} rel_l2={rel_l2:.3e} lse={lse_err:.3e}", flush=True)
    tol = TOL["bf16"]
    if out_dtype == "f32":
        assert max_abs <= tol["max_abs"]
    else:
        assert np.all(np.abs(got - want) <= tol["max_abs"] + 2.0 ** -8 * np.abs(want))
    assert rel_l2 <= tol["rel_l2"] and lse_err <= tol["lse"]
    # properties that hold at any size: causal row 0 returns V row 0; every lse is finite
    np.testing.assert_allclose(out[:, 0, :, 0], w.v[:, 0, :, 0], atol=2.0 ** -8 * 4)
    assert np.all(np.isfinite(lse)) and np.all(np.isfinite(out))


@pytest.mark.parametrize("D", [128, 64])
def test_c2_full_size_whole_heads(D):
    """The benchmark launch, eight whole (batch, head) problems element by element: every row of every q-tile
    (the long and the short tile of each workgroup's pair, the diagonal tiles, the ragged-free last tile), one
    problem on each of the eight XCDs of the XCD-aware workgroup order (problem index b * H + h mod 8 = 0 .. 7),
    spread over the four batch elements."""
    heads = [(0, 0), (0, 9), (1, 2), (1, 11), (2, 4), (2, 13), (3, 6), (3, 15)]
    assert sorted((b * 16 + h) % 8 for b, h in heads) == list(range(8))
    compare_whole_heads(inputs.causal_bf16(D=D), heads, out_dtype="f32", label=f"c2 D={D} whole heads")


@pytest.mark.parametrize("variant", inputs.GRID_VARIANTS)
def test_grid_cell_s16384_whole_head(variant):
    """The longest cell of the paper's grid (S = 16384, one batch element, 16 heads, D = 64): two whole heads
    per variant against the oracle, grouped-query heads for every second variant."""
    gqa = inputs.GRID_VARIANTS.index(variant) % 2 == 1
    compare_whole_heads(inputs.grid_bf16(variant, 16384, gqa=gqa), [(0, 3), (0, 12)], out_dtype="f32",
                        label=f"grid {variant} S=16384 gqa={gqa}")


def test_c3a_alibi_full_size():
    run_and_compare(inputs.alibi_bf16())


def test_c3b_softcap_full_size():
    run_and_compare(inputs.softcap_bf16())


def test_c3c_window_doc_full_size():
    run_and_compare(inputs.window_doc_bf16())


def test_c4_differential_full_size():
    run_and_compare(inputs.differential_bf16())


def test_c5_evoformer_full_size():
    run_and_compare(inputs.evoformer_bf16())
    run_and_compare(inputs.evoformer_bf16(), out_dtype="same")
