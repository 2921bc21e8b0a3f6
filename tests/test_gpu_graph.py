"""The library under HIP graph capture: fl_attn_fwd, fl_attn_bwd and fl_attn_decode allocate nothing, never
synchronise and launch only on the caller's stream, so a captured call sequence can be replayed.
Every replay is compared bit for bit with the eager result, with eager work and synchronisations
between the replays."""
import numpy as np
import pytest

from paper_2511_02043_amd import inputs, runner

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", ["causal_gqa_d128", "window_doc_d64"])
def test_forward_and_backward_replay_from_a_graph(case):
    import torch
    if case == "causal_gqa_d128":
        w = inputs.causal_bf16(B=2, H=4, Hkv=2, S=300, D=128)
    else:
        w = inputs.window_doc_bf16(B=2, H=2, S=400, D=64, window=100, lo=20, hi=150)
    db = runner.upload_backward(w, inputs.dout_for(w), grad_dtype="bf16")
    outs = (db.fwd.out, db.fwd.lse, db.dq, db.dk, db.dv)
    # eager reference (also the warm-up that sets the kernels' LDS limits before any capture)
    db.fwd.run_checked()
    db.run_checked()
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        s = torch.cuda.current_stream().cuda_stream
        db.fwd.run_checked(s)
        db.run_checked(s)
        graph.capture_end()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outs:
            t.fill_(float("nan"))                   # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t, r in zip(("out", "lse", "dq", "dk", "dv"), outs, ref):
            assert torch.equal(t, r), f"{case}: replay {rep} differs in {name}"


def test_decode_replays_from_a_graph_while_sequences_grow():
    """A serving loop captures one decode step and replays it as the sequences grow: seq_lens and the
    block table are device data, the launch shape depends on the host-side bound max_seq_len only."""
    import torch
    from oracle import decode_oracle as do
    final = np.array([131, 741, 53, 1], dtype=np.int32)
    w = inputs.decode_bf16(H=8, Hkv=2, D=128, page_size=16, seq_lens=final)
    dd = runner.upload_decode(w)                    # pages, table and max_seq_len sized for the final lengths
    lens = dd.keep[1]
    outs = (dd.out, dd.lse)

    def eager(cur):
        lens.copy_(torch.from_numpy(cur))
        dd.run_checked()
        torch.cuda.synchronize()
        return [t.clone() for t in outs]

    steps = [np.maximum(final - 20, 0).astype(np.int32), np.maximum(final - 7, 0).astype(np.int32), final]
    refs = [eager(cur) for cur in steps]
    ref_out, ref_lse = do.decode_attention(w.q, w.k_cache, w.v_cache, w.block_table, final, scale=w.scale)
    got_out, got_lse = refs[-1][0].float().cpu().numpy()[:, 0, :, 0], refs[-1][1].cpu().numpy()[:, 0, :, 0, 0]
    assert np.max(np.abs(got_out - ref_out)) <= 1e-2 and np.max(np.abs(got_lse - ref_lse)) <= 1e-3

    lens.copy_(torch.from_numpy(steps[0]))
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        dd.run_checked(torch.cuda.current_stream().cuda_stream)
        graph.capture_end()
    torch.cuda.synchronize()
    for rep, (cur, ref) in enumerate(zip(steps, refs)):
        lens.copy_(torch.from_numpy(cur))           # eager work between the replays
        for t in outs:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t, r in zip(("out", "lse"), outs, ref):
            assert torch.equal(t, r), f"decode replay {rep} differs in {name}"


@pytest.mark.parametrize("case", ["evoformer_bias_gate_d32", "differential_rms_d64_dv128"])
def test_composed_backward_replays_from_a_graph(case):
    """fl_attn_bwd_ex (recomputed stream outputs, elementwise kernels, padded copies, staged bias gradients; no
    memset nodes, no atomics): captured after one eager call, every replay bit-equal to the eager result."""
    import torch
    if case == "evoformer_bias_gate_d32":
        w = inputs.evoformer_bf16(B=1, Nseq=3, Nres=150, H=4, D=32)
    else:
        w = inputs.differential_bf16(B=1, H=2, S=300)
    db = runner.upload_backward_ex(w, inputs.dout_for(w), grad_dtype="f32")
    outs = [db.fwd.out, db.fwd.lse] + [x for t in db.grads.values() for x in (t if isinstance(t, list) else [t])]
    db.fwd.run_checked()
    db.run_checked()                                # eager: also compiles / loads whatever the composed pass instantiates
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        s = torch.cuda.current_stream().cuda_stream
        db.fwd.run_checked(s)
        db.run_checked(s)
        graph.capture_end()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outs:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, (t, r) in enumerate(zip(outs, ref)):
            assert torch.equal(t, r), f"{case}: replay {rep} differs in output {n}"


def test_noalloc_forward_replays_from_a_graph():
    """fl_attn_fwd_noalloc under capture: the document-id summaries live in the library's own buffer."""
    import torch
    from paper_2511_02043_amd import binding as fb
    w = inputs.window_doc_bf16(B=2, H=2, S=500, D=64, window=120, lo=20, hi=150)
    dw = runner.upload(w, out_dtype="f32")
    dw.run_checked()
    torch.cuda.synchronize()
    ref, ref_lse = dw.out.clone(), dw.lse.clone()
    dw.aux.workspace = None
    dw.aux.workspace_bytes = 0
    fb.check(fb.fl_attn_fwd_noalloc(dw.tq, dw.tk, dw.tv, dw.desc, dw.aux, dw.tout, dw.tlse))     # looks the buffer's address up
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        fb.check(fb.fl_attn_fwd_noalloc(dw.tq, dw.tk, dw.tv, dw.desc, dw.aux, dw.tout, dw.tlse, torch.cuda.current_stream().cuda_stream))
        graph.capture_end()
    torch.cuda.synchronize()
    for rep in range(3):
        dw.out.fill_(float("nan"))
        dw.lse.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(dw.out, ref) and torch.equal(dw.lse, ref_lse), rep


def test_paged_prefill_replays_from_a_graph_while_sequences_grow():
    """Chunked prefill in a serving loop: one captured fl_attn_prefill_paged call (page gather + forward kernel, lengths
    read on the device) replayed as the sequences grow by a chunk per step, with new query rows each time."""
    import torch
    from oracle import decode_oracle as do
    Sq = 48
    final = np.array([4 * Sq, 3 * Sq + 5, Sq, 7], dtype=np.int32)          # the last one stays shorter than a chunk
    w = inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=Sq, page_size=16, seq_lens=final)
    dd = runner.upload_prefill_paged(w)             # pages, table and max_seq_len sized for the final lengths
    lens = dd.keep[1]
    outs = (dd.out, dd.lse)
    q_steps = [torch.randn(dd.q.shape, device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(s)).to(torch.bfloat16)
               for s in (1, 2)] + [dd.q.clone()]
    steps = [np.maximum(final - 2 * Sq, 0).astype(np.int32), np.maximum(final - Sq, 0).astype(np.int32), final]

    def eager(cur, qs):
        lens.copy_(torch.from_numpy(cur))
        dd.q.copy_(qs)
        dd.run_checked()
        torch.cuda.synchronize()
        return [t.clone() for t in outs]

    refs = [eager(cur, qs) for cur, qs in zip(steps, q_steps)]
    ref_out, ref_lse = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, final, scale=w.scale)
    got_out, got_lse = refs[-1][0].float().cpu().numpy()[:, 0], refs[-1][1].cpu().numpy()[:, 0, :, :, 0]
    dead = np.isneginf(ref_lse)
    assert np.array_equal(np.isneginf(got_lse), dead)
    assert np.max(np.abs(got_out - ref_out)) <= 1e-2 and np.max(np.abs(got_lse[~dead] - ref_lse[~dead])) <= 1e-3

    lens.copy_(torch.from_numpy(steps[0]))
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        dd.run_checked(torch.cuda.current_stream().cuda_stream)
        graph.capture_end()
    torch.cuda.synchronize()
    for rep, (cur, qs, ref) in enumerate(zip(steps, q_steps, refs)):
        lens.copy_(torch.from_numpy(cur))           # eager work between the replays
        dd.q.copy_(qs)
        for t in outs:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, t, r in zip(("out", "lse"), outs, ref):
            assert torch.equal(t, r), f"prefill replay {rep} differs in {name}"
