"""GPU parity of fl_attn_bwd_ex (through the C-ABI) against the fp64 backward oracle of the variants with
additive biases, the sigmoid gate, RMSNorm and the differential second stream, and of the head dims the
plain backward kernels do not take (D = 32, D != Dv).

Tolerance: as for fl_attn_bwd (P and dS are rounded to bf16 before the fp32-accumulating contractions:
relative L2 <= 5e-3 per gradient tensor, no element off by more than 1e-2 of the tensor's largest
magnitude).  With RMSNorm the per-element bound is 2e-2 of the largest magnitude: the normalisation divides
by the rms of a difference of two nearly cancelling stream outputs, which are recomputed here with bf16
probabilities, so single elements of rows with a small rms carry a larger error (measured 1.5e-2; the
relative L2 error stays at 3e-3).  dlambda is a sum over all rows of a head and comes out far tighter."""
import numpy as np
import pytest

from oracle import attention_backward_oracle as bo
from paper_2511_02043_amd import binding as fb
from paper_2511_02043_amd import inputs, runner

pytestmark = pytest.mark.gpu

REL_L2 = 5e-3
MAX_REL = 1e-2


def compare(w, grad_dtype="f32", label=None, rel_l2=REL_L2, tweak=None):
    max_rel = 2 * MAX_REL if w.rmsnorm else MAX_REL
    import torch
    dout = inputs.dout_for(w)
    db = runner.upload_backward_ex(w, dout, grad_dtype=grad_dtype)
    if tweak is not None:
        tweak(db)
    db.fwd.run_checked()
    for t in db.grads.values():
        for x in (t if isinstance(t, list) else [t]):
            x.fill_(float("nan"))
    db.run_checked()
    torch.cuda.synchronize()
    ref = bo.variant_backward(w, dout)
    names = [n for n in ("dq", "dk", "dv", "dq2", "dk2", "dlambda", "dgate", "drms_weight") if n in db.grads]
    pairs = [(n, db.grads[n], ref[n]) for n in names]
    for n, t in enumerate(db.grads.get("dbias", [])):
        pairs.append((f"dbias[{n}]", t, ref["dbias"][n]))
    for name, t, r in pairs:
        g = t.float().cpu().numpy().astype(np.float64)
        assert g.shape == r.shape, (name, g.shape, r.shape)
        assert np.all(np.isfinite(g)), f"{label or w.name} {name}: non-finite gradient"
        diff = g - r
        scale = max(float(np.max(np.abs(r))), 1e-3)
        rel = float(np.sqrt(np.sum(diff * diff)) / max(np.sqrt(np.sum(r * r)), 1e-3 * np.sqrt(r.size)))
        print(f"{label or w.name} {name}: rel_l2={rel:.3e} max_abs={np.max(np.abs(diff)):.3e} (max |ref| {scale:.3e})", flush=True)
        slack = 2.0 ** -8 * np.abs(r) if (grad_dtype == "bf16" and name in ("dq", "dk", "dv", "dq2", "dk2", "dgate")) else 0.0
        assert rel <= rel_l2, (name, rel)
        assert np.all(np.abs(diff) <= max_rel * scale + slack), (name, float(np.max(np.abs(diff))), scale)


C = inputs.combination_bf16
CASES = {
    "gate_causal_d64": lambda: C(D=64, pos_mask="causal", gate=True, S=300),
    "gate_window_doc_d128": lambda: C(D=128, pos_mask="window", doc=True, gate=True, S=260, window=60),
    "gate_alibi_causal_d64": lambda: C(D=64, score_mod="alibi", pos_mask="causal", gate=True, S=260),
    "bias1_d64": lambda: C(D=64, n_bias=1, S=300),
    "bias2_causal_d64_rows_axis": lambda: C(D=64, n_bias=2, pos_mask="causal", G=3, S=170),
    "bias1_gate_d32_evoformer_like": lambda: inputs.evoformer_bf16(B=1, Nseq=5, Nres=200, H=4, D=32),
    "bias2_gate_d128": lambda: C(D=128, n_bias=2, gate=True, S=140, G=2),
    "plain_d32": lambda: C(D=32, S=300),
    "causal_d64_dv128": lambda: C(D=64, Dv=128, pos_mask="causal", S=200),
    "softcap_causal_d32_dv64_gqa": lambda: C(D=32, Dv=64, score_mod="softcap", pos_mask="causal", S=230, H=4, Hkv=2),
    "rms_prefix_d64": lambda: C(D=64, pos_mask="prefix", rmsnorm=True, S=200),
    "diff_causal_d64": lambda: C(D=64, pos_mask="causal", diff=True, S=300),
    "diff_d128_gqa": lambda: C(D=128, diff=True, S=200, H=4, Hkv=2),
    "diff_rms_causal_d64_dv128": lambda: inputs.differential_bf16(B=1, H=3, S=333),
    "diff_rms_gate_bias_causal_d64": lambda: C(D=64, pos_mask="causal", n_bias=1, diff=True, rmsnorm=True, gate=True, S=180),
    "diff_doc_window_d32": lambda: C(D=32, pos_mask="window", doc=True, diff=True, S=210, window=50),
}


@pytest.mark.parametrize("name", list(CASES))
def test_backward_ex_matches_oracle(name):
    compare(CASES[name](), "f32", label=name)


def test_bf16_gradient_outputs():
    compare(C(D=64, pos_mask="causal", n_bias=1, gate=True, S=200), "bf16", label="bias_gate_bf16_grads")
    compare(inputs.differential_bf16(B=1, H=2, S=200), "bf16", label="diff_rms_bf16_grads")


def test_rms_weight_without_16_byte_alignment():
    """The derivative of the epilogue reads eight channels per lane when every row it touches is 16-byte aligned; an
    rms_weight that is only 4-byte aligned (the header asks for no more) takes the one-row-per-wave kernel instead."""
    import torch
    w = C(D=64, pos_mask="causal", n_bias=1, diff=True, rmsnorm=True, gate=True, S=180)

    def shift(db):
        buf = torch.empty(len(w.rms_weight) + 1, dtype=torch.float32, device="cuda:0")
        buf[1:].copy_(torch.from_numpy(np.asarray(w.rms_weight, np.float32)))
        db.keep.append(buf)
        assert buf[1:].data_ptr() % 16 == 4
        db.aux.rms_weight = buf[1:].data_ptr()
        db.fwd.aux.rms_weight = buf[1:].data_ptr()

    compare(w, "f32", label="rms_weight_4_byte_aligned", tweak=shift)


def test_benchmark_shapes_reduced_batch():
    """The differential + RMSNorm configuration at its full sequence length (S = 4096, D = 64, Dv = 128, two head
    pairs of one batch element) and the Evoformer configuration at its full residue count (384 residues, 8 heads,
    D = 32, eight of the 128 sequence rows), element by element."""
    compare(inputs.differential_bf16(B=1, H=2, S=4096), "f32", label="c4_b1_h2")
    compare(inputs.evoformer_bf16(Nseq=8), "f32", label="c5_nseq8")


def test_supported_and_error_paths():
    import torch
    d = fb.variant_desc(scale=0.1, n_bias=1, epilogue=fb.FL_EPI_GATE_SIGMOID)
    assert fb.fl_bwd_supported(d, fb.FL_BF16, 32, 32) and fb.fl_bwd_supported(d, fb.FL_BF16, 128, 128)
    d4 = fb.variant_desc(scale=0.1, mask=fb.FL_MASK_CAUSAL, combine=fb.FL_DIFFERENTIAL, epilogue=fb.FL_EPI_RMSNORM, rms_eps=1e-6)
    assert fb.fl_bwd_supported(d4, fb.FL_BF16, 64, 128)
    assert fb.fl_bwd_supported(fb.variant_desc(scale=0.1, n_bias=1, score_mod=fb.FL_MOD_SOFTCAP, softcap=2.0), fb.FL_BF16, 64, 64)
    assert fb.fl_bwd_supported(fb.variant_desc(scale=0.1, n_bias=1, mask=fb.FL_MASK_DOC), fb.FL_BF16, 64, 64)
    assert not fb.fl_bwd_supported(d, fb.FL_BF16, 96, 96)
    w = inputs.differential_bf16(B=1, H=2, S=100)
    db = runner.upload_backward_ex(w, inputs.dout_for(w))
    db.fwd.run_checked()
    f = db.fwd
    # the differential variant needs dq2 / dk2
    assert fb.fl_attn_bwd_ex(f.tq, f.tk, f.tv, f.tout, db.tdout, f.tlse, f.desc, db.aux, db.tdq, db.tdk, db.tdv, None) == fb.FL_ERR_AUX_MISSING
    small = fb.aux_desc(q2=db.keep[1], k2=db.keep[2], lambda_=db.keep[3], workspace=db.keep[0][:64])
    assert fb.fl_attn_bwd_ex(f.tq, f.tk, f.tv, f.tout, db.tdout, f.tlse, f.desc, small, db.tdq, db.tdk, db.tdv, db.extra) == fb.FL_ERR_WORKSPACE
    torch.cuda.synchronize()
