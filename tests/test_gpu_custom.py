"""Variants compiled at run time (fl_compile_variant / fl_attn_fwd_custom) against the oracle's
callable form of the same score_mod and mask."""
import numpy as np
import pytest

from oracle import attention_oracle as ao
from paper_2511_02043_amd import binding as fb
from paper_2511_02043_amd import inputs, runner

pytestmark = pytest.mark.gpu

CASES = {
    # (C score_mod, C mask, numpy score_mod, numpy mask)
    "relative_bucket_bias": ("s + 0.05f * (float)((i - j + 4096) % 7)", None,
                             lambda s, b, g, h, i, j: s + np.float32(0.05) * ((i - j + 4096) % 7), None),
    "dilated_causal_window": (None, "j > i || (i - j) % 3 != 0 || i - j > 90",
                              None, lambda b, g, h, i, j: (j > i) | ((i - j) % 3 != 0) | (i - j > 90)),
    "head_dependent_decay_and_checker": ("s - 0.03125f * (float)(h + 1) * sqrtf(fabsf((float)(i - j)))",
                                         "((i >> 4) + (j >> 4) + h) % 2 != 0 && j > i",
                                         lambda s, b, g, h, i, j: s - 0.03125 * (h + 1) * np.sqrt(np.abs(i - j)),
                                         lambda b, g, h, i, j: ((((i >> 4) + (j >> 4) + h) % 2) != 0) & (j > i)),
    "softcap_then_alibi": ("8.0f * tanhf(s / 8.0f) - 0.1f * fabsf((float)(i - j))", "j > i",
                           lambda s, b, g, h, i, j: 8.0 * np.tanh(s / 8.0) - 0.1 * np.abs(i - j),
                           lambda b, g, h, i, j: j > i),
}


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("D", [64, 128])
def test_custom_variant_matches_oracle(name, D):
    import torch
    c_mod, c_mask, np_mod, np_mask = CASES[name]
    w = inputs.causal_bf16(B=2, H=4, Hkv=2, S=300, D=D, causal=False, salt=3)
    var = fb.CustomVariant(c_mod, c_mask, D)
    dw = runner.upload(w, out_dtype="f32")
    dw.out.fill_(float("nan"))
    dw.lse.fill_(float("nan"))
    fb.check(var.forward(dw.tq, dw.tk, dw.tv, float(w.scale), dw.tout, dw.tlse))
    torch.cuda.synchronize()
    ref, ref_lse = ao.attention_custom(w.q, w.k, w.v, scale=w.scale, score_mod=np_mod, mask=np_mask)
    got, got_lse = dw.out.cpu().numpy(), dw.lse.cpu().numpy()[..., 0]
    err = float(np.max(np.abs(got - ref)))
    dead = np.isneginf(ref_lse)
    assert np.array_equal(np.isneginf(got_lse), dead)
    le = float(np.max(np.abs(got_lse[~dead] - ref_lse[~dead])))
    print(f"{name} D={D}: max_abs={err:.3e} lse={le:.3e}", flush=True)
    assert err <= 1e-2 and le <= 1e-3
    var.release()


def test_custom_variant_equals_the_built_in_kernel_on_a_named_variant():
    """ALiBi written as an expression runs the same kernel template as the compiled ALiBi variant."""
    import torch
    w = inputs.alibi_bf16(B=1, H=8, S=400, D=64)
    w.causal = True
    ref, _ = ao.run_workload(w)
    var = fb.CustomVariant("s - exp2f(-(float)(h + 1)) * fabsf((float)(i - j))", "j > i", 64)
    dw = runner.upload(w, out_dtype="f32")
    fb.check(var.forward(dw.tq, dw.tk, dw.tv, float(w.scale), dw.tout, dw.tlse))
    torch.cuda.synchronize()
    assert float(np.max(np.abs(dw.out.cpu().numpy() - ref))) <= 1e-2


def test_base_mask_with_expressions():
    """Structural masks the kernel knows (tile skipping) combined with an expression mask and score_mod."""
    import torch
    w = inputs.causal_bf16(B=1, H=8, Hkv=2, S=700, D=64, causal=False, salt=5)
    dw = runner.upload(w, out_dtype="f32")
    # causal base, score_mod only: full tiles skip the mask arithmetic
    var = fb.CustomVariant("s + 0.05f * (float)((i - j) % 7)", None, 64, base_mask=fb.FL_MASK_CAUSAL)
    fb.check(var.forward(dw.tq, dw.tk, dw.tv, float(w.scale), dw.tout, dw.tlse))
    torch.cuda.synchronize()
    ref, ref_lse = ao.attention_custom(w.q, w.k, w.v, scale=w.scale, score_mod=lambda s, b, g, h, i, j: s + np.float32(0.05) * ((i - j) % 7),
                                       mask=lambda b, g, h, i, j: j > i)
    assert float(np.max(np.abs(dw.out.cpu().numpy() - ref))) <= 1e-2
    assert float(np.max(np.abs(dw.lse.cpu().numpy()[..., 0] - ref_lse))) <= 1e-3
    # window base + dilation expression
    var2 = fb.CustomVariant(None, "(i - j) % 3 != 0", 64, base_mask=fb.FL_MASK_WINDOW)
    fb.check(var2.forward(dw.tq, dw.tk, dw.tv, float(w.scale), dw.tout, dw.tlse, window=200))
    torch.cuda.synchronize()
    ref, ref_lse = ao.attention_custom(w.q, w.k, w.v, scale=w.scale,
                                       mask=lambda b, g, h, i, j: (j > i) | (i - j > 200) | ((i - j) % 3 != 0))
    assert float(np.max(np.abs(dw.out.cpu().numpy() - ref))) <= 1e-2
    assert float(np.max(np.abs(dw.lse.cpu().numpy()[..., 0] - ref_lse))) <= 1e-3


def test_compile_errors_are_reported():
    with pytest.raises(fb.FlError) as e:
        fb.CustomVariant("s + no_such_name", None, 64)
    assert e.value.status == fb.FL_ERR_DESC and "no_such_name" in e.value.detail
    with pytest.raises(fb.FlError) as e:
        fb.CustomVariant("s; while (1)", None, 64)
    assert e.value.status == fb.FL_ERR_DESC
    with pytest.raises(fb.FlError) as e:
        fb.CustomVariant("s", None, 96)
    assert e.value.status == fb.FL_ERR_UNSUPPORTED


@pytest.mark.parametrize("D", [64, 128])
def test_chunked_prefill_offset_as_a_custom_mask(D):
    """Sq new tokens against a longer cache (bottom-right causal alignment: query row i sits at position
    i + Sk - Sq), with ALiBi measured from those positions: the offset is a literal in the expressions."""
    import torch
    Sq, Sk = 200, 1000
    off = Sk - Sq
    w = inputs.causal_bf16(B=2, H=4, Hkv=2, S=Sq, Sk=Sk, D=D, causal=False, salt=9)
    var = fb.CustomVariant(f"s - 0.0625f * (float)(i + {off} - j)", f"j > i + {off}", D)
    dw = runner.upload(w, out_dtype="f32")
    fb.check(var.forward(dw.tq, dw.tk, dw.tv, float(w.scale), dw.tout, dw.tlse))
    torch.cuda.synchronize()
    ref, ref_lse = ao.attention_custom(w.q, w.k, w.v, scale=w.scale, score_mod=lambda s, b, g, h, i, j: s - 0.0625 * (i + off - j),
                                       mask=lambda b, g, h, i, j: j > i + off)
    assert float(np.max(np.abs(dw.out.cpu().numpy() - ref))) <= 1e-2
    assert float(np.max(np.abs(dw.lse.cpu().numpy()[..., 0] - ref_lse))) <= 1e-3
    var.release()


@pytest.mark.parametrize("D", [64, 128])
def test_expressions_that_capture_tensors(D):
    """The closures of Sec. 2.2 capture tensors: a document mask written as an expression over the per-token
    id arrays (Sec. 4.1), on top of a causal base mask, and a learned relative-position bias read from a
    bf16 table per head plus per-head fp32 slopes; against the oracle's callable form with the same arrays."""
    import torch
    dev = "cuda:0"
    B, H, S = 2, 4, 333
    w = inputs.causal_bf16(B=B, H=H, Hkv=2, S=S, D=D, causal=False, salt=9)
    ids = inputs.doc_ids(B, S, seed=77, lo=20, hi=120)
    table = inputs.normal((H, 64), inputs.tensor_seed(9, 7), "bf16")          # bias by clipped distance, per head
    slopes = (0.01 * (1 + np.arange(H))).astype(np.float32)
    t_ids = torch.from_numpy(ids).to(dev)
    t_table = torch.from_numpy(table.astype(np.float32)).to(dev, torch.bfloat16)
    t_slopes = torch.from_numpy(slopes).to(dev)
    var = fb.CustomVariant("s + aux2[h * 64 + min(abs(i - j), 63)] - aux3[h] * (float)(i - j)",
                           "aux0[b * Sq + i] != aux1[b * Sk + j]", D, base_mask=fb.FL_MASK_CAUSAL,
                           aux=[t_ids, t_ids, t_table, t_slopes])
    dw = runner.upload(w, out_dtype="f32")
    dw.out.fill_(float("nan"))
    fb.check(var.forward(dw.tq, dw.tk, dw.tv, float(w.scale), dw.tout, dw.tlse))
    torch.cuda.synchronize()
    tab64 = table.astype(np.float64)
    ref, ref_lse = ao.attention_custom(
        w.q, w.k, w.v, scale=w.scale,
        score_mod=lambda s, b, g, h, i, j: s + tab64[h][np.minimum(np.abs(i - j), 63)] - np.float64(slopes[h]) * (i - j),
        mask=lambda b, g, h, i, j: (j > i) | (ids[b][:, None] != ids[b][None, :]))
    got, got_lse = dw.out.cpu().numpy(), dw.lse.cpu().numpy()[..., 0]
    err = float(np.max(np.abs(got - ref)))
    le = float(np.max(np.abs(got_lse - ref_lse)))
    print(f"captured tensors D={D}: max_abs={err:.3e} lse={le:.3e}", flush=True)
    assert err <= 1e-2 and le <= 1e-3
    # the same document mask through the descriptor (ids in aux, tile skipping): the same result up to the
    # bf16 rounding of the probabilities (the two kernels differ in tile shape and running-max reference)
    wd = inputs.causal_bf16(B=B, H=H, Hkv=2, S=S, D=D, causal=True, salt=9)
    wd.q_doc = wd.kv_doc = ids
    var2 = fb.CustomVariant(None, "aux0[b * Sq + i] != aux1[b * Sk + j]", D, base_mask=fb.FL_MASK_CAUSAL, aux=[t_ids, t_ids])
    dd = runner.upload(wd, out_dtype="f32")
    dd.run_checked()
    fb.check(var2.forward(dw.tq, dw.tk, dw.tv, float(w.scale), dw.tout, dw.tlse))
    torch.cuda.synchronize()
    assert float((dd.out - dw.out).abs().max()) <= 1e-2
    # a variant that reads an array refuses a call without it
    assert fb.fl_attn_fwd_custom(var2.handle, dw.tq, dw.tk, dw.tv, float(w.scale), dw.tout, dw.tlse) == fb.FL_ERR_AUX_MISSING


# --- tile skipping for mask expressions (fl_attn_fwd_custom_skip) ---------------------------------------------------

def run_both_ways(var, dw, scale, **kw):
    """The variant without and with the tile-class pre-pass; returns (out, lse) of both as numpy arrays."""
    import torch
    res = []
    need = var.skip_workspace_size(dw.tq, dw.tk)
    for ws in (None, torch.empty(max(need, 16), dtype=torch.uint8, device="cuda:0")):
        dw.out.fill_(float("nan"))
        dw.lse.fill_(float("nan"))
        fb.check(var.forward(dw.tq, dw.tk, dw.tv, scale, dw.tout, dw.tlse, workspace=ws, **kw))
        torch.cuda.synchronize()
        res.append((dw.out.cpu().numpy().copy(), dw.lse.cpu().numpy()[..., 0].copy()))
    return res, need


@pytest.mark.parametrize("name", ["dilated_causal_window", "head_dependent_decay_and_checker", "softcap_then_alibi"])
@pytest.mark.parametrize("D", [64, 128])
def test_tile_skipping_changes_nothing(name, D):
    """Tiles the pre-pass classifies as hidden contribute exact zeros and tiles classified as fully visible lose only a
    mask evaluation that hid nothing, so the result is bit-equal to the run that evaluates the mask everywhere -- and
    within tolerance of the oracle.  Ragged sizes (Sq and Sk multiples of neither 32 nor 64), a mask that reads h."""
    c_mod, c_mask, np_mod, np_mask = CASES[name]
    w = inputs.causal_bf16(B=2, H=4, Hkv=2, S=333, Sk=715, D=D, causal=False, salt=5)
    var = fb.CustomVariant(c_mod, c_mask, D)
    dw = runner.upload(w, out_dtype="f32")
    (plain, skip), need = run_both_ways(var, dw, float(w.scale))
    nqb8, nkt = ((333 + 31) // 32 + 7) // 8 * 8, (715 + 63) // 64
    blocks = (2 * 4 if name.startswith("head") else 2) * nkt * nqb8            # per (b, g, h) only when the mask reads h
    assert need == (blocks + 255) // 256 * 256 + blocks * 256                   # class bytes, then 64 words per block
    assert np.array_equal(plain[0], skip[0]) and np.array_equal(plain[1], skip[1])
    ref, ref_lse = ao.attention_custom(w.q, w.k, w.v, scale=w.scale, score_mod=np_mod, mask=np_mask)
    dead = np.isneginf(ref_lse)
    assert np.array_equal(np.isneginf(skip[1]), dead)
    assert float(np.max(np.abs(skip[0] - ref))) <= 1e-2
    assert float(np.max(np.abs(skip[1][~dead] - ref_lse[~dead]))) <= 1e-3
    var.release()


@pytest.mark.parametrize("D", [64, 128])
def test_document_mask_expression_with_tile_skipping(D):
    """The document mask of Sec. 4.1 as an expression over captured id arrays, on a causal base mask, long enough that
    most tiles are hidden (runs of hidden tiles between a row's document and the diagonal do not occur under causal +
    document, so a second variant without the causal base covers those runs)."""
    import torch
    B, H, S = 2, 4, 2100
    w = inputs.causal_bf16(B=B, H=H, Hkv=2, S=S, D=D, causal=False, salt=11)
    ids = inputs.doc_ids(B, S, seed=5, lo=100, hi=400)
    t_ids = torch.from_numpy(ids).to("cuda:0")
    dw = runner.upload(w, out_dtype="f32")
    for base, np_mask in ((fb.FL_MASK_CAUSAL, lambda b, g, h, i, j: (j > i) | (ids[b][:, None] != ids[b][None, :])),
                          (0, lambda b, g, h, i, j: (ids[b][:, None] != ids[b][None, :]) & ((i - j) % 5 != 0))):
        expr = "aux0[b * Sq + i] != aux1[b * Sk + j]" + ("" if base else " && (i - j) % 5 != 0")
        var = fb.CustomVariant(None, expr, D, base_mask=base, aux=[t_ids, t_ids])
        (plain, skip), need = run_both_ways(var, dw, float(w.scale))
        blocks = B * ((S + 63) // 64) * (((S + 31) // 32 + 7) // 8 * 8)              # the expression reads neither g nor h
        assert need == (blocks + 255) // 256 * 256 + blocks * 256
        assert np.array_equal(plain[0], skip[0]) and np.array_equal(plain[1], skip[1])
        ref, ref_lse = ao.attention_custom(w.q, w.k, w.v, scale=w.scale, score_mod=None, mask=np_mask)
        assert float(np.max(np.abs(skip[0] - ref))) <= 1e-2
        assert float(np.max(np.abs(skip[1] - ref_lse))) <= 1e-3
        var.release()


def test_tile_skipping_with_a_window_base_mask_and_errors():
    import torch
    w = inputs.causal_bf16(B=1, H=8, Hkv=8, S=900, D=64, causal=False, salt=12)
    dw = runner.upload(w, out_dtype="f32")
    var = fb.CustomVariant(None, "(i >> 6) % 2 == 1 && (j >> 6) % 2 == 0", 64, base_mask=fb.FL_MASK_WINDOW)
    (plain, skip), need = run_both_ways(var, dw, float(w.scale), window=300)
    assert np.array_equal(plain[0], skip[0]) and np.array_equal(plain[1], skip[1])
    ref, ref_lse = ao.attention_custom(w.q, w.k, w.v, scale=w.scale, score_mod=None,
                                       mask=lambda b, g, h, i, j: (j > i) | (i - j > 300) | (((i >> 6) % 2 == 1) & ((j >> 6) % 2 == 0)))
    assert float(np.max(np.abs(skip[0] - ref))) <= 1e-2
    small = torch.empty(need - 8, dtype=torch.uint8, device="cuda:0")
    assert var.forward(dw.tq, dw.tk, dw.tv, float(w.scale), dw.tout, dw.tlse, workspace=small, window=300) == fb.FL_ERR_WORKSPACE
    var.release()
    # a variant without a mask expression has nothing to classify: no workspace needed, same call
    mod_only = fb.CustomVariant("s * 0.5f", None, 64)
    assert mod_only.skip_workspace_size(dw.tq, dw.tk) == 0
    assert fb.fl_attn_fwd_custom_skip(mod_only.handle, dw.tq, dw.tk, dw.tv, float(w.scale), [], None, dw.tout, dw.tlse) == fb.FL_OK
    torch.cuda.synchronize()
    mod_only.release()
