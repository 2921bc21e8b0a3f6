"""Long sequences (S = 131072: 2048 key tiles, 1024 query tiles per head).

Causal forward on sampled rows that the oracle computes one by one; causal + document mask forward and
backward on whole documents: under that mask a document's rows and keys see nothing outside of it, so
the oracle's result on the document alone (causal) is the result of the full problem for those rows.
The query tiles near the end of the sequence skip runs of thousands of hidden key tiles."""
import numpy as np
import pytest

from oracle import attention_backward_oracle as bo
from oracle import attention_oracle as ao
from paper_2511_02043_amd import inputs, runner
from tests.gpu_util import TOL, errors

pytestmark = pytest.mark.gpu

S_LONG = 131072


def test_long_causal_forward_sampled_rows():
    import torch
    w = inputs.causal_bf16(B=1, H=2, S=S_LONG, D=128)
    dw = runner.upload(w, out_dtype="f32")
    dw.run_checked()
    torch.cuda.synchronize()
    rng = np.random.Generator(np.random.PCG64(131))
    rows = sorted({0, 1, 63, 64, 255, 256, S_LONG // 2 - 1, S_LONG // 2, S_LONG - 257, S_LONG - 256, S_LONG - 1}
                  | set(int(x) for x in rng.integers(0, S_LONG, 10)))
    picks = [(0, 0, h, i) for h in (0, 1) for i in rows]
    out = dw.out.float().cpu().numpy()
    lse = dw.lse.cpu().numpy()[..., 0]
    ref = ao.run_workload_rows(w, picks)
    got = np.stack([out[b, g, h, i] for (b, g, h, i) in picks]).astype(np.float64)
    want = np.stack([o for (o, _) in ref])
    max_abs, rel_l2 = errors(got, want)
    lse_err = max(abs(float(lse[b, g, h, i]) - l) for (b, g, h, i), (_, l) in zip(picks, ref))
    print(f"causal S={S_LONG}: {len(picks)} rows max_abs={max_abs:.3e} rel_l2={rel_l2:.3e} lse={lse_err:.3e}", flush=True)
    tol = TOL["bf16"]
    assert max_abs <= tol["max_abs"] and rel_l2 <= tol["rel_l2"] and lse_err <= tol["lse"]
    assert np.all(np.isfinite(lse)) and np.all(np.isfinite(out))


@pytest.mark.parametrize("D,H,Hkv", [(128, 2, 2), (64, 4, 2)])
def test_long_document_causal_forward_backward(D, H, Hkv):
    import torch
    w = inputs.causal_bf16(B=1, H=H, Hkv=Hkv, S=S_LONG, D=D)
    ids = inputs.doc_ids(1, S_LONG, seed=1310 + D, lo=64, hi=6000)
    w.q_doc, w.kv_doc = ids, ids
    w.name = f"causal_document_long_d{D}"
    dout = inputs.dout_for(w)
    db = runner.upload_backward(w, dout, grad_dtype="f32")
    db.fwd.run_checked()
    for t in (db.dq, db.dk, db.dv):
        t.fill_(float("nan"))
    db.run_checked()
    torch.cuda.synchronize()
    out = db.fwd.out.float().cpu().numpy()
    lse = db.fwd.lse.cpu().numpy()[..., 0]
    dq, dk, dv = (t.float().cpu().numpy() for t in (db.dq, db.dk, db.dv))
    assert all(np.all(np.isfinite(x)) for x in (out, lse, dq, dk, dv))

    starts = np.flatnonzero(np.diff(ids[0], prepend=-1))
    ends = np.append(starts[1:], S_LONG)
    n_docs = len(starts)
    longest = int(np.argmax(ends - starts))
    tol = TOL["bf16"]
    for d in sorted({0, n_docs // 2, longest, n_docs - 2, n_docs - 1}):
        a, b = int(starts[d]), int(ends[d])
        sub = inputs.Workload(f"document_{d}", "bf16", w.q[:, :, :, a:b], w.k[:, :, :, a:b], w.v[:, :, :, a:b],
                              scale=w.scale, causal=True)
        ref_out, ref_lse = ao.run_workload(sub)
        max_abs, rel_l2 = errors(out[:, :, :, a:b].astype(np.float64), ref_out)
        lse_err = float(np.max(np.abs(lse[:, :, :, a:b] - ref_lse)))
        print(f"D={D} document {d} rows [{a}, {b}): out max_abs={max_abs:.3e} rel_l2={rel_l2:.3e} lse={lse_err:.3e}", flush=True)
        assert np.all(np.abs(out[:, :, :, a:b] - ref_out) <= tol["max_abs"] + 2.0 ** -8 * np.abs(ref_out))
        assert rel_l2 <= tol["rel_l2"] and lse_err <= tol["lse"]
        ref = bo.run_workload_backward(sub, dout[:, :, :, a:b])
        for name, g, r in zip(("dq", "dk", "dv"), (dq, dk, dv), ref):
            diff = g[:, :, :, a:b] - r
            rel = float(np.sqrt(np.sum(diff * diff)) / max(np.sqrt(np.sum(r * r)), 1e-3 * np.sqrt(r.size)))
            print(f"D={D} document {d} {name}: rel_l2={rel:.3e}", flush=True)
            assert rel <= 5e-3, (d, name, rel)


@pytest.mark.parametrize("D", [128, 64])
def test_long_decode(D):
    """One query against 131072 cached tokens (8192 pages of 16, shuffled; the key axis is cut into the
    maximum number of splits), next to a shorter and a tiny sequence in the same call."""
    from tests.test_gpu_decode import compare
    w = inputs.decode_bf16(H=8, Hkv=2, D=D, page_size=16, seq_lens=[S_LONG, 100001, 5])
    compare(w, f"decode_long_d{D}")
