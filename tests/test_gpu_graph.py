"""The library under HIP graph capture: fl_attn_fwd and fl_attn_bwd allocate nothing, never
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
