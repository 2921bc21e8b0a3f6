"""attention() (autograd wrapper over fl_attn_fwd / fl_attn_bwd) against the oracles."""
import numpy as np
import pytest

from oracle import attention_backward_oracle as bo
from oracle import attention_oracle as ao
from paper_2511_02043_amd import inputs

pytestmark = pytest.mark.gpu


def rel_l2(got, ref):
    d = got - ref
    return float(np.sqrt(np.sum(d * d) / np.sum(ref * ref)))


@pytest.mark.parametrize("case", ["causal_gqa", "window_doc", "alibi", "softcap_strided"])
def test_autograd_matches_oracles(case):
    import torch
    from paper_2511_02043_amd.functional import attention
    if case == "causal_gqa":
        w = inputs.causal_bf16(B=2, H=4, Hkv=2, S=200, D=64)
    elif case == "window_doc":
        w = inputs.window_doc_bf16(B=2, H=2, S=300, D=128, window=64, lo=20, hi=120)
    elif case == "alibi":
        w = inputs.alibi_bf16(B=1, H=4, S=260, D=64)
    else:
        w = inputs.softcap_bf16(B=1, H=2, S=260, D=128, cap=10.0, qscale=2.0)
    dout = inputs.dout_for(w)
    dev = "cuda:0"

    def leaf(x, strided=False):
        t = torch.from_numpy(np.ascontiguousarray(x[:, 0])).to(dev, torch.bfloat16)      # [B, H, S, D]
        if strided:                                 # stored [B, S, H, D], viewed [B, H, S, D]
            t = t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        return t.requires_grad_(True)

    strided = case == "softcap_strided"
    q, k, v = leaf(w.q, strided), leaf(w.k, strided), leaf(w.v, strided)
    kw = dict(scale=w.scale, causal=w.causal, window=w.window, prefix=w.prefix, softcap=w.softcap)
    if w.alibi is not None:
        kw["alibi_slopes"] = torch.from_numpy(w.alibi).to(dev)
    if w.q_doc is not None:
        kw["q_doc_ids"] = torch.from_numpy(w.q_doc).to(dev)
    out = attention(q, k, v, **kw)
    out.backward(torch.from_numpy(np.ascontiguousarray(dout[:, 0])).to(dev, torch.bfloat16))
    torch.cuda.synchronize()
    ref_out, _ = ao.run_workload(w)
    ref = bo.run_workload_backward(w, dout)
    got_out = out.detach().float().cpu().numpy()[:, None]
    assert np.all(np.abs(got_out - ref_out) <= 1e-2 + 2.0 ** -8 * np.abs(ref_out))
    for name, t, r in zip(("dq", "dk", "dv"), (q.grad, k.grad, v.grad), ref):
        g = t.float().cpu().numpy()[:, None]
        e = rel_l2(g, r)
        print(f"{case} {name}: rel_l2={e:.3e}", flush=True)
        assert e <= 5e-3, (name, e)          # bf16 gradients: P and dS rounding plus half an ulp of the stored value


def test_rejects_what_it_cannot_run():
    import torch
    from paper_2511_02043_amd.functional import attention
    x = torch.zeros(1, 2, 16, 64)
    with pytest.raises(ValueError):
        attention(x, x, x)                          # CPU tensors: there is no fallback
    y = torch.zeros(1, 2, 16, 64, device="cuda:0", dtype=torch.float32)
    with pytest.raises(ValueError):
        attention(y, y, y)


def test_decode_wrapper_matches_oracle():
    import torch
    from oracle import decode_oracle as do
    from paper_2511_02043_amd.functional import decode_attention
    w = inputs.decode_bf16(H=8, Hkv=2, D=128, page_size=16, seq_lens=[1, 47, 600, 1025])
    dev = "cuda:0"
    q = torch.from_numpy(w.q).to(dev, torch.bfloat16)
    kc = torch.from_numpy(w.k_cache).to(dev, torch.bfloat16)
    vc = torch.from_numpy(w.v_cache).to(dev, torch.bfloat16)
    table, lens = torch.from_numpy(w.block_table).to(dev), torch.from_numpy(w.seq_lens).to(dev)
    ref, ref_lse = do.decode_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale, window=300)
    out, lse = decode_attention(q, kc, vc, lens, table, window=300, return_lse=True)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    assert np.all(np.abs(got - ref) <= 1e-2 + 2.0 ** -8 * np.abs(ref))
    assert np.max(np.abs(lse.cpu().numpy() - ref_lse)) <= 1e-3
    # a reused workspace and a tight length bound give the same result
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=dev)
    out2 = decode_attention(q, kc, vc, lens, table, window=300, max_seq_len=1025, workspace=ws)
    torch.cuda.synchronize()
    assert np.all(np.abs(out2.float().cpu().numpy() - ref) <= 1e-2 + 2.0 ** -8 * np.abs(ref))
    with pytest.raises(ValueError):
        decode_attention(q, kc, vc, lens, table, workspace=torch.empty(8, dtype=torch.uint8, device=dev))


def test_paged_prefill_wrapper_matches_oracle():
    import torch
    from oracle import decode_oracle as do
    from paper_2511_02043_amd.functional import paged_prefill_attention
    w = inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=70, page_size=16, seq_lens=[30, 70, 600, 1025])
    dev = "cuda:0"
    q = torch.from_numpy(w.q).to(dev, torch.bfloat16)
    kc = torch.from_numpy(w.k_cache).to(dev, torch.bfloat16)
    vc = torch.from_numpy(w.v_cache).to(dev, torch.bfloat16)
    table, lens = torch.from_numpy(w.block_table).to(dev), torch.from_numpy(w.seq_lens).to(dev)
    ref, ref_lse = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale, softcap_value=3.0)
    out, lse = paged_prefill_attention(q, kc, vc, lens, table, softcap=3.0, return_lse=True)
    torch.cuda.synchronize()
    got, got_lse = out.float().cpu().numpy(), lse.cpu().numpy()
    dead = np.isneginf(ref_lse)
    assert np.array_equal(np.isneginf(got_lse), dead) and dead[0, :, :40].all()      # the 30-token sequence: 40 rows before position 0
    assert np.all(np.abs(got - ref) <= 1e-2 + 2.0 ** -8 * np.abs(ref))
    assert np.max(np.abs(got_lse[~dead] - ref_lse[~dead])) <= 1e-3
    with pytest.raises(ValueError):
        paged_prefill_attention(q, kc, vc, lens.long(), table)
    with pytest.raises(ValueError):
        paged_prefill_attention(q, kc, vc, lens, table, workspace=torch.empty(8, dtype=torch.uint8, device=dev))


def test_wrapper_refuses_arrays_the_abi_would_misread():
    """int64 document ids (torch's default integer type), sliced id views, slopes on the CPU and
    int64 lengths would be reinterpreted as int32 / float32 memory by the C ABI: the wrapper raises."""
    import torch
    from paper_2511_02043_amd.functional import attention, decode_attention
    dev = "cuda:0"
    q = torch.zeros(2, 4, 64, 64, dtype=torch.bfloat16, device=dev)
    ids = torch.zeros(2, 64, dtype=torch.int64, device=dev)
    with pytest.raises(ValueError):
        attention(q, q, q, q_doc_ids=ids)
    with pytest.raises(ValueError):
        attention(q, q, q, q_doc_ids=torch.zeros(2, 128, dtype=torch.int32, device=dev)[:, ::2])
    with pytest.raises(ValueError):
        attention(q, q, q, alibi_slopes=torch.ones(4))
    with pytest.raises(ValueError):
        attention(q, q, q, alibi_slopes=torch.ones(3, device=dev))
    kc = torch.zeros(8, 16, 2, 64, dtype=torch.bfloat16, device=dev)
    with pytest.raises(ValueError):
        decode_attention(q[:, :, 0], kc, kc, torch.tensor([3, 4], device=dev),
                         torch.zeros(2, 4, dtype=torch.int32, device=dev))
    with pytest.raises(ValueError):
        decode_attention(q[:, :, 0], kc, kc, torch.tensor([3, 4], dtype=torch.int32, device=dev),
                         torch.zeros(2, 4, dtype=torch.int64, device=dev))
    # the accepted forms still run
    out = attention(q, q, q, q_doc_ids=ids.to(torch.int32))
    assert out.shape == q.shape


def test_autograd_with_query_offset():
    """attention(..., q_offset=Sk - Sq): a chunk of queries against a longer key sequence, output and gradients."""
    import torch
    from paper_2511_02043_amd.functional import attention
    w = inputs.causal_bf16(B=1, H=4, Hkv=2, S=100, Sk=420, D=64)
    w.q_offset = 320
    dout = inputs.dout_for(w)
    dev = "cuda:0"
    q, k, v = (torch.from_numpy(np.ascontiguousarray(x[:, 0])).to(dev, torch.bfloat16).requires_grad_(True) for x in (w.q, w.k, w.v))
    out = attention(q, k, v, scale=w.scale, causal=True, q_offset=320)
    out.backward(torch.from_numpy(np.ascontiguousarray(dout[:, 0])).to(dev, torch.bfloat16))
    torch.cuda.synchronize()
    ref_out, _ = ao.run_workload(w)
    ref = bo.run_workload_backward(w, dout)
    got = out.detach().float().cpu().numpy()[:, None]
    assert np.all(np.abs(got - ref_out) <= 1e-2 + 2.0 ** -8 * np.abs(ref_out))
    for name, t, r in zip(("dq", "dk", "dv"), (q.grad, k.grad, v.grad), ref):
        e = rel_l2(t.float().cpu().numpy()[:, None], r)
        print(f"offset {name}: rel_l2={e:.3e}", flush=True)
        assert e <= 5e-3, (name, e)


@pytest.mark.parametrize("case", ["evoformer", "differential_rms", "bias_gate_causal"])
def test_variant_attention_autograd(case):
    """variant_attention(): forward fl_attn_fwd, backward fl_attn_bwd_ex, gradients of every tensor input."""
    import torch
    from paper_2511_02043_amd.functional import variant_attention
    dev = "cuda:0"
    if case == "evoformer":
        w = inputs.evoformer_bf16(B=1, Nseq=4, Nres=150, H=4, D=32)
    elif case == "differential_rms":
        w = inputs.differential_bf16(B=1, H=3, S=260)
    else:
        w = inputs.combination_bf16(D=64, pos_mask="causal", n_bias=2, gate=True, S=200, G=2)
    dout = inputs.dout_for(w)

    def leaf(x, dt=torch.bfloat16):
        return None if x is None else torch.from_numpy(np.ascontiguousarray(x)).to(dev, dt).requires_grad_(True)

    q, k, v, gate, q2, k2 = (leaf(x) for x in (w.q, w.k, w.v, w.gate, w.q2, w.k2))
    lam = leaf(w.lam, torch.float32)
    biases = [leaf(b) for b in w.biases]
    rw = leaf(None if w.rms_weight is None else np.asarray(w.rms_weight, np.float32), torch.float32)
    out = variant_attention(q, k, v, scale=w.scale, causal=w.causal, biases=biases, gate=gate, q2=q2, k2=k2, lam=lam,
                            rmsnorm=w.rmsnorm, rms_eps=w.rms_eps, rms_weight=rw)
    out.backward(torch.from_numpy(np.ascontiguousarray(dout)).to(dev, torch.bfloat16))
    torch.cuda.synchronize()
    ref_out, _ = ao.run_workload(w)
    got = out.detach().float().cpu().numpy()
    assert np.all(np.abs(got - ref_out) <= 1e-2 + 2.0 ** -8 * np.abs(ref_out))
    ref = bo.variant_backward(w, dout)
    pairs = [("dq", q), ("dk", k), ("dv", v), ("dq2", q2), ("dk2", k2), ("dlambda", lam), ("dgate", gate), ("drms_weight", rw)]
    pairs += [(("dbias", n), b) for n, b in enumerate(biases)]
    for name, t in pairs:
        if t is None:
            continue
        r = ref[name[0]][name[1]] if isinstance(name, tuple) else ref[name]
        e = rel_l2(t.grad.float().cpu().numpy(), r)
        print(f"{case} {name}: rel_l2={e:.3e}", flush=True)
        assert e <= 6e-3, (name, e)          # bf16 gradient storage on top of the 5e-3 of the fp32 outputs
