"""Seeded input generators: rounding, reproducibility and the stated recipes."""
import numpy as np
import torch

from paper_2511_02043_amd import inputs


def test_bf16_rounding_is_round_to_nearest_even():
    x = np.random.Generator(np.random.PCG64(1)).standard_normal(100000).astype(np.float32) * 37
    ours = inputs.round_to_bf16(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours, ref)
    # exact ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even mantissa (1.0)
    ties = np.array([1 + 2 ** -8, 1 + 3 * 2 ** -8], dtype=np.float32)
    assert np.array_equal(inputs.round_to_bf16(ties), np.array([1.0, 1 + 2 ** -6], np.float32))
    bits = inputs.bf16_bits(ours)
    assert np.array_equal(torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
                          .to(torch.float32).numpy(), ours)


def test_streams_are_reproducible_and_independent():
    a = inputs.causal_bf16(B=1, H=2, S=16, D=8)
    b = inputs.causal_bf16(B=1, H=2, S=16, D=8)
    assert np.array_equal(a.q, b.q) and np.array_equal(a.v, b.v)
    assert not np.array_equal(a.q, a.k)
    c = inputs.causal_bf16(B=1, H=2, S=16, D=8, salt=1)
    assert not np.array_equal(a.q, c.q)


def test_doc_ids_recipe():
    ids = inputs.doc_ids(8, 2048, inputs.tensor_seed(3, 3))
    assert ids.shape == (8, 2048) and ids.dtype == np.int32
    for b in range(8):
        assert ids[b, 0] == 0 and np.all(np.diff(ids[b]) >= 0) and np.all(np.diff(ids[b]) <= 1)
        runs = np.diff(np.flatnonzero(np.diff(ids[b])))       # interior run lengths
        assert runs.min() >= 64 and runs.max() <= 1024


def test_alibi_slopes_geometric():
    s = inputs.alibi_slopes(16)
    assert np.isclose(s[0], 2 ** -0.5) and np.isclose(s[-1], 2 ** -8)
    np.testing.assert_allclose(s[1:] / s[:-1], 2 ** -0.5, rtol=1e-6)


def test_config_shapes():
    d = inputs.evoformer_bf16(B=1, Nseq=4, Nres=6, H=2, D=8).dims
    assert d == dict(B=1, G=4, H=2, Hkv=2, Sq=6, Sk=6, D=8, Dv=8)
    w = inputs.differential_bf16(B=1, H=2, S=8, D=4, Dv=8)
    assert w.q2.shape == w.q.shape == (1, 1, 2, 8, 4) and w.v.shape == (1, 1, 2, 8, 8)
    assert np.all(w.lam == np.float32(0.8))
