"""Concurrent callers: several host threads, each with its own stream and buffers, call the forward,
backward and decode entry points at the same time (ctypes releases the interpreter lock around the
calls); every result must equal the one the same call gives alone.  The library keeps no per-call
state outside its arguments (the error detail is per thread)."""
import threading

import pytest

from paper_2511_02043_amd import inputs, runner

pytestmark = pytest.mark.gpu


def test_concurrent_calls_from_several_threads():
    import torch
    jobs = []
    for n, w in enumerate([inputs.causal_bf16(B=2, H=4, Hkv=2, S=400, D=128), inputs.alibi_bf16(B=1, H=4, S=500, D=64),
                           inputs.window_doc_bf16(B=2, H=2, S=600, D=64, window=100, lo=20, hi=200),
                           inputs.softcap_bf16(B=1, H=4, S=300, D=64, cap=10.0, qscale=2.0)]):
        db = runner.upload_backward(w, inputs.dout_for(w), grad_dtype="bf16")
        jobs.append(("bwd", db, (db.fwd.out, db.fwd.lse, db.dq, db.dk, db.dv)))
    for D in (64, 128):
        dd = runner.upload_decode(inputs.decode_bf16(H=8, Hkv=2, D=D, page_size=16, seq_lens=[5, 300, 1000]))
        jobs.append(("dec", dd, (dd.out, dd.lse)))

    def run(kind, obj, stream):
        if kind == "bwd":
            obj.fwd.run_checked(stream)
        obj.run_checked(stream)

    refs = []
    for kind, obj, outs in jobs:                    # alone, on the default stream
        run(kind, obj, 0)
        torch.cuda.synchronize()
        refs.append([t.clone() for t in outs])
        for t in outs:
            t.fill_(float("nan"))
    torch.cuda.synchronize()

    errors = []

    def worker(kind, obj):
        try:
            s = torch.cuda.Stream()
            for _ in range(10):
                run(kind, obj, s.cuda_stream)
            s.synchronize()
        except Exception as e:                      # noqa: BLE001 - reported below
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(kind, obj)) for kind, obj, _ in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for (kind, _, outs), ref in zip(jobs, refs):
        for t, r in zip(outs, ref):
            assert torch.equal(t, r), f"{kind}: a concurrent call changed the result"
