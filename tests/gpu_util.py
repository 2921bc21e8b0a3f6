"""Helpers for the GPU parity tests: run a workload through the C-ABI and compare with the oracle."""
import numpy as np

from oracle import attention_oracle as ao
from paper_2511_02043_amd import runner

# Tolerances stated by the benchmark definition: bf16 inputs with fp32 accumulation and fp32 inputs.
TOL = {"bf16": dict(max_abs=1e-2, rel_l2=5e-3, lse=1e-3),
       "f32": dict(max_abs=1e-5, rel_l2=1e-5, lse=1e-3)}


def errors(got, ref):
    got = np.asarray(got, dtype=np.float64)
    diff = got - ref
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    denom = float(np.sqrt(np.sum(ref * ref)))
    rel_l2 = float(np.sqrt(np.sum(diff * diff)) / denom) if denom > 0 else float(np.sqrt(np.sum(diff * diff)))
    return max_abs, rel_l2


def lse_error(got, ref):
    got = np.asarray(got, dtype=np.float64)
    inf = np.isneginf(ref)
    assert np.array_equal(np.isneginf(got), inf), "-inf pattern of lse differs"
    if np.all(inf):
        return 0.0
    return float(np.max(np.abs(got[~inf] - ref[~inf])))


def run_and_compare(w, out_dtype="f32", label=None):
    """Full element-by-element comparison against the oracle.  Returns the error dict."""
    import torch
    dw = runner.upload(w, out_dtype=out_dtype)
    dw.out.fill_(float("nan"))
    dw.lse.fill_(float("nan"))
    dw.run_checked()
    torch.cuda.synchronize()
    got = dw.out.float().cpu().numpy()
    got_lse = runner.lse_to_oracle_layout(dw)
    ref, ref_lse = ao.run_workload(w)
    tol = TOL[w.dtype]
    max_abs, rel_l2 = errors(got, ref)
    le = lse_error(got_lse, ref_lse)
    msg = f"{label or w.name}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e} lse={le:.3e}"
    print(msg, flush=True)
    assert np.all(np.isfinite(got)), msg + " (non-finite output)"
    if out_dtype == "f32" or w.dtype == "f32":
        assert max_abs <= tol["max_abs"], msg
    else:
        # bf16 storage of the result: half an ulp of the value on top of the arithmetic tolerance
        assert np.all(np.abs(got - ref) <= tol["max_abs"] + 2.0 ** -8 * np.abs(ref)), msg
    assert rel_l2 <= tol["rel_l2"], msg
    assert le <= tol["lse"], msg
    return dict(max_abs=max_abs, rel_l2=rel_l2, lse=le)


def head_slice(w, b, h):
    """The (b, h) problem of a workload as a workload of its own (B = H = 1; all rows of the G axis)."""
    import dataclasses
    d = w.dims
    group = d["H"] // d["Hkv"]
    sub = dataclasses.replace(w)
    for f in ("q", "k", "v", "q2", "k2", "gate"):
        x = getattr(w, f)
        if x is not None:
            hh = h if x.shape[2] == d["H"] else h // group
            setattr(sub, f, x[b:b + 1, :, hh:hh + 1])
    sub.biases = tuple(bb[(b if bb.shape[0] > 1 else 0):(b if bb.shape[0] > 1 else 0) + 1, :,
                          (h if bb.shape[2] > 1 else 0):(h if bb.shape[2] > 1 else 0) + 1] for bb in w.biases)
    if w.alibi is not None:
        sub.alibi = w.alibi[h:h + 1]
    if w.lam is not None:
        sub.lam = w.lam[h:h + 1]
    if w.q_doc is not None:
        sub.q_doc, sub.kv_doc = w.q_doc[b:b + 1], w.kv_doc[b:b + 1]
    return sub


def compare_whole_heads(w, heads, out_dtype="f32", label=None):
    """One launch of the whole workload; the listed (b, h) problems are compared element by element with
    the oracle (which evaluates one head at a time), and everything else has to be finite."""
    import torch
    dw = runner.upload(w, out_dtype=out_dtype)
    dw.out.fill_(float("nan"))
    dw.lse.fill_(float("nan"))
    dw.run_checked()
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dw.out).all()), f"{label or w.name}: non-finite output"
    tol = TOL[w.dtype]
    worst = dict(max_abs=0.0, rel_l2=0.0, lse=0.0)
    for (b, h) in heads:
        got = dw.out[b, :, h].float().cpu().numpy()[None, :, None]
        got_lse = dw.lse[b, :, h, :, 0].cpu().numpy()[None, :, None]
        ref, ref_lse = ao.run_workload(head_slice(w, b, h))
        max_abs, rel_l2 = errors(got, ref)
        le = lse_error(got_lse, ref_lse)
        msg = f"{label or w.name} head ({b}, {h}): max_abs={max_abs:.3e} rel_l2={rel_l2:.3e} lse={le:.3e}"
        print(msg, flush=True)
        if out_dtype == "f32":
            assert max_abs <= tol["max_abs"], msg
        else:
            assert np.all(np.abs(got - ref) <= tol["max_abs"] + 2.0 ** -8 * np.abs(ref)), msg
        assert rel_l2 <= tol["rel_l2"] and le <= tol["lse"], msg
        worst = dict(max_abs=max(worst["max_abs"], max_abs), rel_l2=max(worst["rel_l2"], rel_l2), lse=max(worst["lse"], le))
    return worst
