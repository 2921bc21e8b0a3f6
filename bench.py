#!/usr/bin/env python3
"""Benchmark of the fused attention-variant forward path on one MI355X.

    python bench.py --gpus 1 --steps 20 --warmup 10

A step is one fl_attn_fwd call (all steps of the hot path: grid decode + tile skipper, Q load,
K/V tiles through LDS, score tile, variant transform, online softmax, P.V, epilogue) on one
batch of synthetic inputs that are already resident in HBM.  The default workload is the
configuration the metric is quoted on: causal bf16, B=4 H=16 S=8192 D=128.  One JSON line is
printed on stdout.  `--config NAME` times another benchmark configuration, `--all` times every
configuration and writes bench_all.json into --out-dir as well.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
OUT_DIR = os.path.join(ROOT, "bench_out")          # --out-dir: where --all / --grid / --backward leave their tables
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


WINDOW_OVERRIDE = None           # --window: replaces the window of a windowed configuration (0: a row sees its own key only)


def make_workload(name):
    w = _make_workload(name)
    if WINDOW_OVERRIDE is not None and w.window is not None:
        w.window = WINDOW_OVERRIDE
    return w


def _make_workload(name):
    from paper_2511_02043_amd import inputs
    if name == "c2_d128":
        return inputs.causal_bf16(D=128)
    if name == "c2_d64":
        return inputs.causal_bf16(D=64)
    if name == "c3a_alibi":
        return inputs.alibi_bf16()
    if name == "c3b_softcap":
        return inputs.softcap_bf16()
    if name == "c3c_window_doc":
        return inputs.window_doc_bf16()
    if name == "c4_differential":
        return inputs.differential_bf16()
    if name == "c5_evoformer":
        return inputs.evoformer_bf16()
    raise SystemExit(f"unknown config {name!r}")


HBM_BOUND = ("c3c_window_doc", "c5_evoformer")    # configurations whose roofline is HBM bandwidth (algorithmic bytes)
CONFIGS = ["c2_d128", "c2_d64", "c3a_alibi", "c3b_softcap", "c3c_window_doc", "c4_differential", "c5_evoformer"]


def unmasked_pairs(w):
    """Number of (i, j) pairs per (b, g, h) problem that are not masked, summed over the batch."""
    d = w.dims
    Sq, Sk, B = d["Sq"], d["Sk"], d["B"]
    if w.q_doc is None:
        i = np.arange(Sq, dtype=np.int64)
        if w.prefix is not None:
            cnt = np.minimum(np.maximum(i + 1, w.prefix), Sk)
        elif w.causal or w.window is not None:
            cnt = np.minimum(i + 1, Sk)
            if w.window is not None:
                cnt = cnt - np.maximum(0, i - w.window)
        else:
            cnt = np.full(Sq, Sk, dtype=np.int64)
        return int(cnt.sum()) * B
    total = 0
    i = np.arange(Sq)[:, None]
    j = np.arange(Sk)[None, :]
    for b in range(B):
        ok = w.q_doc[b][:, None] == w.kv_doc[b][None, :]
        if w.causal or w.window is not None:
            ok &= j <= i
        if w.window is not None:
            ok &= (i - j) <= w.window
        total += int(ok.sum())
    return total


def flops_and_bytes(w):
    d = w.dims
    streams = 2 if w.q2 is not None else 1
    pairs = unmasked_pairs(w) * d["G"] * d["H"]            # pairs already summed over the batch
    flops = pairs * streams * (2 * d["D"] + 2 * d["Dv"])
    es = 2 if w.dtype == "bf16" else 4
    nq = d["B"] * d["G"] * d["H"] * d["Sq"]
    nk = d["B"] * d["G"] * d["Hkv"] * d["Sk"]
    byt = es * (streams * nq * d["D"] + streams * nk * d["D"] + nk * d["Dv"] + nq * d["Dv"]) + 4 * nq * streams
    if w.gate is not None:
        byt += es * nq * d["Dv"]
    for b in w.biases:
        byt += es * b.size
    return flops, byt


def time_config(name, steps, warmup, out_dtype="same", rotate=1, before=None):
    """rotate > 1: cycle over that many independent copies of every buffer, so that a workload
    smaller than the 256 MB Infinity Cache is timed from HBM ("cold") rather than from cache.
    before: called once the inputs are resident, right before the warm-up steps (the reference
    measurements of the default run: no idle gap between them and the timed region)."""
    import torch
    from paper_2511_02043_amd import runner
    w = make_workload(name)
    flops, byt = flops_and_bytes(w)
    dws = [runner.upload(w, out_dtype=out_dtype) for _ in range(rotate)]
    stream = torch.cuda.current_stream().cuda_stream
    if before is not None:
        before()
    for n in range(warmup):
        dws[n % rotate].run_checked(stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for n in range(steps):
        dws[n % rotate].run_checked(stream)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    ev_ms = e0.elapsed_time(e1) / steps
    # spread of single launches (the paper's protocol, Sec. 4.1: 20 timed launches), each between
    # its own pair of events; the clock cannot be pinned here, so min and std-dev go with the median
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(20)]
    for n, (a, b) in enumerate(evs):
        a.record()
        dws[n % rotate].run_checked(stream)
        b.record()
    torch.cuda.synchronize()
    one = np.array([a.elapsed_time(b) * 1e3 for a, b in evs])
    launch_us = dict(n=len(one), median=float(np.median(one)), mean=float(one.mean()), min=float(one.min()),
                     std=float(one.std()))
    return dict(config=name, flops=flops, bytes=byt, ms_per_step=wall_ms, kernel_ms=ev_ms, launch_us=launch_us,
                tflops=flops / (wall_ms * 1e-3) / 1e12, kernel_tflops=flops / (ev_ms * 1e-3) / 1e12,
                gbs=byt / (ev_ms * 1e-3) / 1e9, dims=w.dims, device_workload=dws[0]), w


BWD_CONFIGS = ["c2_d128", "c2_d64", "c3a_alibi", "c3b_softcap", "c3c_window_doc", "c4_differential", "c5_evoformer"]


def time_backward(name, steps, warmup):
    """One fl_attn_bwd call (pre-pass + dQ kernel + dK/dV kernel) per step on the configuration's
    inputs, bf16 gradients; out and lse come from one untimed forward call.  FLOPs are the five
    contractions of the backward pass on unmasked pairs (2.5 x the forward count); the kernels
    recompute the score and dP tiles in both passes, which is not counted."""
    import torch
    from paper_2511_02043_amd import inputs, runner
    w = make_workload(name)
    flops, _ = flops_and_bytes(w)
    flops = flops * 5 // 2
    composed = bool(w.biases) or w.gate is not None or w.q2 is not None or w.rmsnorm or w.dims["D"] != w.dims["Dv"] \
        or w.dims["D"] not in (64, 128)
    # biases, gate, RMSNorm, second stream, other head dims: fl_attn_bwd_ex (every gradient the variant has)
    db = (runner.upload_backward_ex if composed else runner.upload_backward)(w, inputs.dout_for(w), grad_dtype="bf16")
    stream = torch.cuda.current_stream().cuda_stream
    db.fwd.run_checked(stream)
    for _ in range(warmup):
        db.run_checked(stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        db.run_checked(stream)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    return dict(config=name, flops=flops, ms_per_step=ms, tflops=flops / (ms * 1e-3) / 1e12, dims=w.dims)


def run_grid_backward(steps, warmup):
    """fl_attn_bwd on the paper's benchmark grid (Sec. 4.1 shapes; the paper itself times no backward pass)."""
    import torch
    from paper_2511_02043_amd import inputs, runner
    rows = []
    for variant in inputs.GRID_VARIANTS:
        for gqa in (False, True):
            for S in inputs.GRID_SEQ_LENS:
                w = inputs.grid_bf16(variant, S, gqa=gqa)
                flops = flops_and_bytes(w)[0] * 5 // 2
                db = runner.upload_backward(w, inputs.dout_for(w), grad_dtype="bf16")
                stream = torch.cuda.current_stream().cuda_stream
                db.fwd.run_checked(stream)
                for _ in range(warmup):
                    db.run_checked(stream)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(steps):
                    db.run_checked(stream)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / steps
                rows.append(dict(variant=variant, heads="gqa" if gqa else "mha", S=S, B=w.dims["B"], ms=ms,
                                 tflops=flops / (ms * 1e-3) / 1e12))
                print(f"# bwd {variant:15s} {'gqa' if gqa else 'mha'} S={S:5d} B={w.dims['B']:2d}: {ms:.4f} ms  "
                      f"{rows[-1]['tflops']:.1f} TFLOP/s", file=sys.stderr, flush=True)
                del db
    os.makedirs(OUT_DIR, exist_ok=True)
    with open(os.path.join(OUT_DIR, "bench_grid_bwd.json"), "w") as f:
        json.dump(rows, f, indent=1)
    print(json.dumps({"grid_cells": len(rows), "file": os.path.join(OUT_DIR, "bench_grid_bwd.json")}), flush=True)


def time_decode(steps, warmup, B=64, H=32, Hkv=8, D=128, ctx=8192, page_size=16, layout="NHD"):
    """One fl_attn_decode call per step: B sequences with lengths uniform on [ctx / 2, ctx], a paged cache in the
    serving layout [pages, page_size, Hkv, D] with shuffled page placement, bf16.  The cache is drawn on the
    device (seeded N(0,1)); the algorithmic bytes are the visible keys and values read once plus q and out."""
    import torch
    from paper_2511_02043_amd import binding as fb
    g = torch.Generator(device="cuda").manual_seed(251102043)
    rng = np.random.Generator(np.random.PCG64(251102043))
    lens = rng.integers(ctx // 2, ctx + 1, size=B).astype(np.int32)
    pages_per_seq = (lens + page_size - 1) // page_size
    n_pages = int(pages_per_seq.sum())
    pool = rng.permutation(n_pages).astype(np.int32)
    table = np.zeros((B, int(pages_per_seq.max())), dtype=np.int32)
    pos = 0
    for b in range(B):
        table[b, :pages_per_seq[b]] = pool[pos:pos + pages_per_seq[b]]
        pos += pages_per_seq[b]
    dev = "cuda:0"
    # NHD: [pages, page_size, Hkv, D] (a token's heads are adjacent); HND: [pages, Hkv, page_size, D] (a head's page is one block)
    shape = (n_pages, page_size, Hkv, D) if layout == "NHD" else (n_pages, Hkv, page_size, D)
    kc = torch.randn(shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    vc = torch.randn(shape, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((B, H, D), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty((B, 1, H, 1, D), dtype=torch.bfloat16, device=dev)
    t_table, t_lens = torch.from_numpy(table).to(dev), torch.from_numpy(lens).to(dev)
    tq = fb.tensor_desc(q[:, None, :, None, :])
    tk = fb.tensor_desc((kc.permute(0, 2, 1, 3) if layout == "NHD" else kc)[:, None])
    tv = fb.tensor_desc((vc.permute(0, 2, 1, 3) if layout == "NHD" else vc)[:, None])
    tout = fb.tensor_desc(out)
    kv = fb.paged_kv(block_table=t_table, page_size=page_size, seq_lens=t_lens, max_seq_len=int(lens.max()))
    desc = fb.variant_desc(scale=D ** -0.5, mask=fb.FL_MASK_CAUSAL)
    ws = torch.empty(max(fb.fl_attn_decode_workspace_size(tq, tk, kv), 16), dtype=torch.uint8, device=dev)
    aux = fb.aux_desc(workspace=ws)
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(warmup):
        fb.check(fb.fl_attn_decode(tq, tk, tv, kv, desc, aux, tout, None, stream))
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        fb.check(fb.fl_attn_decode(tq, tk, tv, kv, desc, aux, tout, None, stream))
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    byt = int(lens.sum()) * Hkv * D * 2 * 2 + 2 * B * H * D * 2
    return dict(ms_per_step=ms, bytes=byt, gbs=byt / (ms * 1e-3) / 1e9, tokens=int(lens.sum()),
                dims=dict(B=B, H=H, Hkv=Hkv, D=D, ctx=ctx, page_size=page_size, cache_layout=layout))


def time_prefill_paged(steps, warmup, B=8, H=32, Hkv=8, D=128, ctx=8192, chunk=512, page_size=16):
    """One fl_attn_prefill_paged call per step: the last `chunk` rows of B sequences of ctx cached tokens each (a
    paged cache in the serving layout with shuffled page placement, bf16), and beside it fl_attn_fwd on the same
    keys held densely (causal, query offset ctx - chunk): the difference is the cost of reading through the pages."""
    import torch
    from paper_2511_02043_amd import binding as fb
    g = torch.Generator(device="cuda").manual_seed(251102043)
    rng = np.random.Generator(np.random.PCG64(251102043))
    per_seq = (ctx + page_size - 1) // page_size
    n_pages = B * per_seq
    table = rng.permutation(n_pages).astype(np.int32).reshape(B, per_seq)
    lens = np.full(B, ctx, dtype=np.int32)
    dev = "cuda:0"
    kc = torch.randn((n_pages, page_size, Hkv, D), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    vc = torch.randn((n_pages, page_size, Hkv, D), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((B, 1, H, chunk, D), generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(q)
    t_table, t_lens = torch.from_numpy(table).to(dev), torch.from_numpy(lens).to(dev)
    tq, tout = fb.tensor_desc(q), fb.tensor_desc(out)
    tk, tv = fb.tensor_desc(kc.permute(0, 2, 1, 3)[:, None]), fb.tensor_desc(vc.permute(0, 2, 1, 3)[:, None])
    kv = fb.paged_kv(block_table=t_table, page_size=page_size, seq_lens=t_lens, max_seq_len=ctx)
    desc = fb.variant_desc(scale=D ** -0.5, mask=fb.FL_MASK_CAUSAL)
    ws = torch.empty(max(fb.fl_attn_prefill_paged_workspace_size(tq, tk, kv), 16), dtype=torch.uint8, device=dev)
    aux = fb.aux_desc(workspace=ws)
    # the same keys and values held densely, [B, 1, Hkv, ctx, D]
    idx = t_table.long()
    kd = kc[idx].reshape(B, per_seq * page_size, Hkv, D)[:, :ctx].permute(0, 2, 1, 3)[:, None].contiguous()
    vd = vc[idx].reshape(B, per_seq * page_size, Hkv, D)[:, :ctx].permute(0, 2, 1, 3)[:, None].contiguous()
    out_d = torch.empty_like(q)
    tkd, tvd, tout_d = fb.tensor_desc(kd), fb.tensor_desc(vd), fb.tensor_desc(out_d)
    desc_d = fb.variant_desc(scale=D ** -0.5, mask=fb.FL_MASK_CAUSAL, q_offset=ctx - chunk)
    stream = torch.cuda.current_stream().cuda_stream
    calls = {"paged": lambda: fb.check(fb.fl_attn_prefill_paged(tq, tk, tv, kv, desc, aux, tout, None, stream)),
             "dense": lambda: fb.check(fb.fl_attn_fwd(tq, tkd, tvd, desc_d, None, tout_d, None, stream))}
    ms = {}
    for name, call in calls.items():
        for _ in range(warmup):
            call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms[name] = e0.elapsed_time(e1) / steps
    same = bool(torch.equal(out, out_d))
    pairs = B * H * sum(ctx - chunk + i + 1 for i in range(chunk))
    flops = 4 * D * pairs
    return dict(ms_per_step=ms["paged"], ms_dense=ms["dense"], flops=flops, tflops=flops / (ms["paged"] * 1e-3) / 1e12,
                tflops_dense=flops / (ms["dense"] * 1e-3) / 1e12, identical_to_dense=same,
                dims=dict(B=B, H=H, Hkv=Hkv, D=D, ctx=ctx, chunk=chunk, page_size=page_size))


def time_custom(steps, warmup):
    """Variants compiled at run time, on the shapes of the ALiBi configuration (B=8 H=16 S=2048 D=64): the ALiBi
    score_mod as an expression (same arithmetic as the built-in variant, for comparison), and two variants no
    descriptor names.  FLOPs on unmasked pairs, as everywhere."""
    import torch
    from paper_2511_02043_amd import binding as fb, inputs, runner
    w = inputs.alibi_bf16()
    d = w.dims
    dw = runner.upload(w, out_dtype="same")
    stream = torch.cuda.current_stream().cuda_stream
    S = d["Sq"]
    i = np.arange(S, dtype=np.int64)[:, None]
    j = np.arange(S, dtype=np.int64)[None, :]
    cases = [
        ("built-in ALiBi (descriptor)", None, None, 0, S * S, False),
        ("ALiBi as an expression", "s - exp2f(-0.5f * (float)(h + 1)) * fabsf((float)(i - j))", None, 0, S * S, False),
        ("bucketed relative bias, causal as an expression (every tile computed)", "s + 0.05f * (float)((i - j) % 7)", "j > i", 0,
         int((j <= i).sum()), False),
        ("bucketed relative bias, causal as an expression, tile classes from a pre-pass", "s + 0.05f * (float)((i - j) % 7)", "j > i", 0,
         int((j <= i).sum()), True),
        ("bucketed relative bias, causal as base mask", "s + 0.05f * (float)((i - j) % 7)", None, fb.FL_MASK_CAUSAL,
         int((j <= i).sum()), False),
        ("dilated window 768: base window + expression", None, "(i - j) % 3 != 0", fb.FL_MASK_WINDOW,
         int(((j <= i) & ((i - j) % 3 == 0) & (i - j <= 768)).sum()), False),
    ]
    res = []
    for name, mod, mask, base, pairs, skip in cases:
        t0 = time.perf_counter()
        var = None if (mod is None and mask is None) else fb.CustomVariant(mod, mask, d["D"], base_mask=base)
        compile_s = time.perf_counter() - t0
        ws = torch.empty(max(var.skip_workspace_size(dw.tq, dw.tk), 16), dtype=torch.uint8, device="cuda:0") if skip else None
        call = (lambda: dw.run_checked(stream)) if var is None else \
            (lambda: fb.check(var.forward(dw.tq, dw.tk, dw.tv, float(w.scale), dw.tout, dw.tlse, stream, window=768, workspace=ws)))
        for _ in range(warmup):
            call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        flops = pairs * d["B"] * d["H"] * 4 * d["D"]
        res.append(dict(variant=name, ms=ms, tflops=flops / (ms * 1e-3) / 1e12, compile_s=compile_s))
        print(f"# {name}: {ms:.4f} ms  {res[-1]['tflops']:.1f} TFLOP/s  (compiled in {compile_s:.1f} s)", file=sys.stderr, flush=True)
    # the document mask of the paper's grid (12 documents, S = 4096, B = 4, 16 heads, D = 64): through the
    # descriptor (per-token ids in aux, tiles of other documents skipped) and as an expression over the same
    # id arrays captured by the variant (every tile computed, the paper's own behaviour)
    wd = inputs.grid_bf16("document_mask", 4096)
    dd = runner.upload(wd, out_dtype="same")
    ids = dd.keep[0]
    pairs = unmasked_pairs(wd)
    doc_var = fb.CustomVariant(None, "aux0[b * Sq + i] != aux1[b * Sk + j]", wd.dims["D"], aux=[ids, ids])
    map_ws = torch.empty(max(doc_var.skip_workspace_size(dd.tq, dd.tk), 16), dtype=torch.uint8, device="cuda:0")
    for name, var, ws in (("document mask (descriptor, tile skipper)", None, None),
                          ("document mask as an expression over captured id arrays (every tile computed)", doc_var, None),
                          ("document mask as an expression, tile classes from a pre-pass (fl_attn_fwd_custom_skip)", doc_var, map_ws)):
        call = (lambda: dd.run_checked(stream)) if var is None else \
            (lambda: fb.check(var.forward(dd.tq, dd.tk, dd.tv, float(wd.scale), dd.tout, dd.tlse, stream, workspace=ws)))
        for _ in range(warmup):
            call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            call()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        flops = pairs * wd.dims["H"] * 4 * wd.dims["D"]
        res.append(dict(variant=name, ms=ms, tflops=flops / (ms * 1e-3) / 1e12, compile_s=0.0))
        print(f"# {name}: {ms:.4f} ms  {res[-1]['tflops']:.1f} TFLOP/s", file=sys.stderr, flush=True)
    return res


def gemm_reference(n=8192, reps=50):
    """TFLOP/s of torch.matmul on random bf16 data of size n^3: what the matrix cores sustain under the
    board's power limit with nothing but a contraction to run (context for roofline.frac, not a target)."""
    import torch
    a = torch.randn(n, n, device="cuda", dtype=torch.bfloat16)
    b = torch.randn(n, n, device="cuda", dtype=torch.bfloat16)
    for _ in range(10):
        a @ b
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        a @ b
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * n ** 3 * reps / (e0.elapsed_time(e1) * 1e-3) / 1e12


def _bench_lib():
    """libflbench.so: the two measurement kernels of csrc/fl_bench_kernels.hip (no attention code)."""
    import ctypes as C
    path = os.path.join(ROOT, "paper_2511_02043_amd", "libflbench.so")
    L = C.CDLL(path)
    L.flb_mfma_peak.restype = C.c_double
    L.flb_mfma_peak.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
    L.flb_copy.restype = C.c_int
    L.flb_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.flb_read.restype = C.c_int
    L.flb_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    return L


def mfma_peak_reference(zero_data=False, blocks=2048, iters=4000, reps=10):
    """TFLOP/s of a pure chain of v_mfma_f32_32x32x16_bf16 (two waves per SIMD, no memory traffic) on
    pseudo-random operands: the peak the matrix cores reach on this board at the clock its power limit allows."""
    import torch
    L = _bench_lib()
    sink = torch.empty(blocks * 512, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(3):
        L.flb_mfma_peak(sink.data_ptr(), blocks, iters, int(zero_data), stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    flops = 0.0
    for _ in range(reps):
        f = L.flb_mfma_peak(sink.data_ptr(), blocks, iters, int(zero_data), stream)
        if f < 0:
            raise RuntimeError("flb_mfma_peak failed")
        flops += f
    e1.record()
    torch.cuda.synchronize()
    return flops / (e0.elapsed_time(e1) * 1e-3) / 1e12


def copy_reference(mib=1024, reps=10):
    """GB/s (bytes read + bytes written) of a plain device copy kernel of `mib` MiB: the HBM reference."""
    import torch
    L = _bench_lib()
    n = mib << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(3):
        L.flb_copy(dst.data_ptr(), src.data_ptr(), n, stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        if L.flb_copy(dst.data_ptr(), src.data_ptr(), n, stream) != 0:
            raise RuntimeError("flb_copy failed")
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def read_reference(mib=2048, reps=10):
    """GB/s of a plain read-only kernel over `mib` MiB (more than the 256 MB Infinity Cache holds): what a stream that
    only reads, like the decode step, can reach on this board."""
    import torch
    L = _bench_lib()
    n = mib << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(3):
        L.flb_read(src.data_ptr(), n, sink.data_ptr(), stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        if L.flb_read(src.data_ptr(), n, sink.data_ptr(), stream) != 0:
            raise RuntimeError("flb_read failed")
    e1.record()
    torch.cuda.synchronize()
    return float(n) * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def _read_sysfs_power():
    """(socket power in W, power cap in W) from the amdgpu hwmon files, or (None, None)."""
    import glob
    for d in glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*"):
        try:
            for name in ("power1_average", "power1_input"):
                f = os.path.join(d, name)
                if os.path.exists(f):
                    cap = None
                    if os.path.exists(os.path.join(d, "power1_cap")):
                        cap = int(open(os.path.join(d, "power1_cap")).read()) / 1e6
                    return int(open(f).read()) / 1e6, cap
        except (OSError, ValueError):
            continue
    return None, None


def _read_smi_clock():
    """Mean shader clock in MHz over the gfx_N entries of `amd-smi metric -c --json` (and its socket power), or None."""
    import subprocess
    try:
        out = subprocess.run(["amd-smi", "metric", "-p", "-c", "--json"], capture_output=True, text=True, timeout=10).stdout
        data = json.loads(out[out.index("{"):])
        g = data["gpu_data"][0] if "gpu_data" in data else data[0]
        clks = [v["clk"]["value"] for k, v in g.get("clock", {}).items()
                if k.startswith("gfx_") and isinstance(v, dict) and isinstance(v.get("clk"), dict)
                and isinstance(v["clk"].get("value"), (int, float))]
        pw = g.get("power", {}).get("socket_power", {})
        pw = pw.get("value") if isinstance(pw, dict) else None
        return (float(np.mean(clks)) if clks else None), (float(pw) if isinstance(pw, (int, float)) else None)
    except Exception:
        return None, None


def sustained_power_clock(dw, flops, seconds=1.5, max_seconds=6.0):
    """Runs the workload back to back for `seconds` (until the clock query has returned, at most
    max_seconds) while a thread samples the socket power (hwmon, every 20 ms) and asks amd-smi once for
    the shader clocks.  The clock cannot be pinned from user space: under this kernel the board sits at its
    power limit and lowers the clock, so both numbers go into the record next to the throughput."""
    import threading
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    samples, smi = [], {}
    stop = threading.Event()

    def power_sampler():
        t0 = time.perf_counter()
        while not stop.is_set():
            pw, cap = _read_sysfs_power()
            if pw is not None:
                samples.append((time.perf_counter() - t0, pw, cap))
            time.sleep(0.02)

    def sampler():                                 # the clock query takes a few tenths of a second: three of them
        pt = threading.Thread(target=power_sampler, daemon=True)
        pt.start()
        time.sleep(0.4)
        clks = []
        for _ in range(3):
            if stop.is_set():
                break
            c, pw = _read_smi_clock()
            if c is not None:
                clks.append(c)
            smi["power"] = pw
        smi["clk"] = float(np.mean(clks)) if clks else None
        smi["clk_samples"] = clks
        smi["done"] = True
        pt.join(timeout=5)

    th = threading.Thread(target=sampler, daemon=True)
    th.start()
    t0 = time.perf_counter()
    n = 0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    while True:
        for _ in range(50):
            dw.run_checked(stream)
        n += 50
        torch.cuda.synchronize()
        t = time.perf_counter() - t0
        if (t >= seconds and smi.get("done")) or t >= max_seconds:
            break
    e1.record()
    torch.cuda.synchronize()
    stop.set()
    th.join(timeout=15)
    late = [pw for (t, pw, cap) in samples if t > 0.3]
    cap = next((c for (_, _, c) in samples if c is not None), None)
    return {"socket_power_w": float(np.mean(late)) if late else smi.get("power"),
            "power_cap_w": cap, "sclk_mhz": smi.get("clk"), "sclk_samples_mhz": smi.get("clk_samples"), "sclk_max_mhz": 2400,
            "launches": n, "tflops_sustained": flops * n / (e0.elapsed_time(e1) * 1e-3) / 1e12,
            "source": "hwmon power1_input sampled every 20 ms; mean shader clock of the 8 XCDs from three amd-smi metric -c queries; "
                      "both during a back-to-back run of the same launch"}


def run_grid(steps, warmup):
    """The paper's benchmark grid (Sec. 4.1): every cell timed like the default workload."""
    import torch
    from paper_2511_02043_amd import inputs, runner
    rows = []
    for variant in inputs.GRID_VARIANTS:
        for gqa in (False, True):
            for S in inputs.GRID_SEQ_LENS:
                w = inputs.grid_bf16(variant, S, gqa=gqa)
                flops, byt = flops_and_bytes(w)
                dw = runner.upload(w, out_dtype="same")
                stream = torch.cuda.current_stream().cuda_stream
                for _ in range(warmup):
                    dw.run_checked(stream)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(steps):
                    dw.run_checked(stream)
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1) / steps
                rows.append(dict(variant=variant, heads="gqa" if gqa else "mha", S=S, B=w.dims["B"], ms=ms,
                                 tflops=flops / (ms * 1e-3) / 1e12, gbs=byt / (ms * 1e-3) / 1e9))
                print(f"# {variant:15s} {'gqa' if gqa else 'mha'} S={S:5d} B={w.dims['B']:2d}: {ms:.4f} ms  "
                      f"{rows[-1]['tflops']:.1f} TFLOP/s  {rows[-1]['gbs']:.0f} GB/s", file=sys.stderr, flush=True)
                del dw
    # the variants outside the 7 x 2 grid (Sec. 4.1): DiffAttn on the MHA grid and at head dim 128,
    # Evoformer row-wise gated attention with two biases, plus column-wise gated attention
    extra = [(f"diffattn_d64", "mha", S, lambda S=S: inputs.diffattn_paper_bf16(S=S, D=64)) for S in inputs.GRID_SEQ_LENS]
    extra += [(f"diffattn_d128", "mha", S, lambda S=S: inputs.diffattn_paper_bf16(S=S, D=128)) for S in inputs.GRID_SEQ_LENS]
    extra += [(f"evoformer_d{D}", f"b{B}", 256, lambda B=B, D=D: inputs.evoformer_paper_bf16(B=B, D=D))
              for D in (64, 128) for B in (1, 4, 32)]
    extra += [("columnwise_gated_d32", "b1", 128, lambda: inputs.columnwise_gated_bf16(B=1, Nseq=128, Nres=384, H=8, D=32))]
    for variant, heads, S, make in extra:
        w = make()
        flops, byt = flops_and_bytes(w)
        dw = runner.upload(w, out_dtype="same")
        stream = torch.cuda.current_stream().cuda_stream
        for _ in range(warmup):
            dw.run_checked(stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            dw.run_checked(stream)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        rows.append(dict(variant=variant, heads=heads, S=S, B=w.dims["B"], ms=ms,
                         tflops=flops / (ms * 1e-3) / 1e12, gbs=byt / (ms * 1e-3) / 1e9))
        print(f"# {variant:15s} {heads} S={S:5d} B={w.dims['B']:2d}: {ms:.4f} ms  "
              f"{rows[-1]['tflops']:.1f} TFLOP/s  {rows[-1]['gbs']:.0f} GB/s", file=sys.stderr, flush=True)
        del dw
    os.makedirs(OUT_DIR, exist_ok=True)
    with open(os.path.join(OUT_DIR, "bench_grid.json"), "w") as f:
        json.dump(rows, f, indent=1)
    print(json.dumps({"grid_cells": len(rows), "file": os.path.join(OUT_DIR, "bench_grid.json")}))


def cpu_baseline(w, budget_s=15.0):
    """The oracle as it stands, timed on this host on a bounded sample of heads of the workload."""
    from oracle import attention_oracle as ao
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    d = w.dims
    per_head_flops = flops_and_bytes(w)[0] / (d["B"] * d["G"] * d["H"])
    import dataclasses
    sub = dataclasses.replace(w)
    done, t_used = 0, 0.0
    heads = [(0, h) for h in range(d["H"])]
    for (b, h) in heads:
        for f in ("q", "k", "v", "q2", "k2", "gate"):
            x = getattr(w, f)
            if x is not None:
                hh = h if x.shape[2] == d["H"] else h // (d["H"] // d["Hkv"])
                setattr(sub, f, x[b:b + 1, 0:1, hh:hh + 1])
        sub.biases = tuple(bb[0:1, 0:1, (h if bb.shape[2] > 1 else 0):(h if bb.shape[2] > 1 else 0) + 1] for bb in w.biases)
        if w.alibi is not None:
            sub.alibi = w.alibi[h:h + 1]
        if w.lam is not None:
            sub.lam = w.lam[h:h + 1]
        if w.q_doc is not None:
            sub.q_doc, sub.kv_doc = w.q_doc[b:b + 1], w.kv_doc[b:b + 1]
        t0 = time.perf_counter()
        ao.run_workload(sub)
        t_used += time.perf_counter() - t0
        done += 1
        if t_used > budget_s:
            break
    return dict(value=per_head_flops * done / t_used / 1e12, unit="TFLOP/s", cores=int(threads), kind="oracle",
                sample=f"{done} of {d['B'] * d['G'] * d['H']} (b, g, h) problems of the same workload, "
                       f"{t_used:.1f} s of NumPy fp64")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", default="c2_d128", choices=CONFIGS)
    ap.add_argument("--out-dir", default=None, help="folder for the JSON tables of --all / --grid / --backward (default: bench_out/)")
    ap.add_argument("--all", action="store_true", help="time every configuration (results in bench_all.json under --out-dir)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--grid", action="store_true",
                    help="time the paper's benchmark grid (7 variants x MHA/GQA x S = 512..16k, 16k tokens, D = 64); "
                         "table on stderr, bench_grid.json under --out-dir")
    ap.add_argument("--backward", action="store_true",
                    help="time fl_attn_bwd on the configurations it covers (table on stderr, bench_bwd.json under --out-dir)")
    ap.add_argument("--decode-layout", default="NHD", choices=["NHD", "HND"],
                    help="cache storage order for --decode: [pages, page_size, Hkv, D] or [pages, Hkv, page_size, D]")
    ap.add_argument("--decode-page", type=int, default=16, help="tokens per page for --decode")
    ap.add_argument("--decode-dim", type=int, default=128, choices=[64, 128], help="head dim for --decode")
    ap.add_argument("--decode-batch", type=int, default=64, help="sequences for --decode")
    ap.add_argument("--decode-ctx", type=int, default=8192, help="longest cached sequence for --decode (lengths are uniform on [ctx / 2, ctx])")
    ap.add_argument("--prefill-chunk", type=int, default=0, metavar="ROWS",
                    help="time fl_attn_prefill_paged: the last ROWS query rows of --decode-batch sequences of --decode-ctx cached tokens")
    ap.add_argument("--custom", action="store_true", help="time variants compiled at run time from expressions (ALiBi shapes)")
    ap.add_argument("--decode", action="store_true",
                    help="time fl_attn_decode (64 sequences of 4k-8k cached tokens, 32 / 8 heads, D = 128, 16-token pages)")
    ap.add_argument("--no-gemm-reference", action="store_true",
                    help="skip the bf16 GEMM that shows what the matrix cores sustain on random data")
    ap.add_argument("--window", type=int, default=None,
                    help="override the window of a windowed configuration (c3c): --window 0 leaves one key tile per row "
                         "block, i.e. the launch's memory traffic without its key loop")
    ap.add_argument("--rotate", type=int, default=1,
                    help="cycle the timed launches over this many independent buffer sets (a workload smaller than the "
                         "256 MB Infinity Cache is then timed from HBM)")
    ap.add_argument("--tune", default="", help="comma list key=value passed to fl_set_tuning (sweeps)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="only run a plain device-to-device copy of MIB MiB a few times (scale factor of the "
                         "FETCH_SIZE / WRITE_SIZE counters under rocprofv3 --pmc)")
    args = ap.parse_args()
    global WINDOW_OVERRIDE
    WINDOW_OVERRIDE = args.window
    if args.out_dir:
        global OUT_DIR
        OUT_DIR = os.path.abspath(args.out_dir)
    if args.gpus != 1:
        raise SystemExit("this build runs on one GPU only: no sharding or collectives are part of it (use --gpus 1)")
    import torch
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    if args.calibrate_copy:
        n = args.calibrate_copy * (1 << 20)
        src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": n, "repeats": 5}))
        return
    from paper_2511_02043_amd import binding as fb
    fb.lib()
    for kv in filter(None, args.tune.split(",")):
        k, v = kv.split("=")
        fb.check(fb.fl_set_tuning(k, int(v)))

    if args.custom:
        res = time_custom(args.steps, args.warmup)
        print(json.dumps({"metric": "attention fwd TFLOP/s of run-time compiled variants", "unit": "TFLOP/s", "n_gpus": 1,
                          "steps": args.steps, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic", "results": res}), flush=True)
        return
    if args.prefill_chunk > 0:
        r = time_prefill_paged(args.steps, args.warmup, B=args.decode_batch, ctx=args.decode_ctx, D=args.decode_dim,
                               page_size=args.decode_page, chunk=args.prefill_chunk)
        print(f"# prefill over pages: {r['ms_per_step']:.4f} ms ({r['tflops']:.0f} TFLOP/s); dense keys: {r['ms_dense']:.4f} ms "
              f"({r['tflops_dense']:.0f} TFLOP/s); outputs identical: {r['identical_to_dense']}", file=sys.stderr, flush=True)
        print(json.dumps({"metric": "chunked-prefill attention over a paged KV cache, TFLOP/s of visible scores", "value": r["tflops"],
                          "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": r["ms_per_step"], "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": f"prefill_paged_b{args.decode_batch}_h32_kv8_d{args.decode_dim}_ctx{args.decode_ctx}_chunk{args.prefill_chunk}_page{args.decode_page}",
                                     **r["dims"], "ms_dense_keys": r["ms_dense"], "tflops_dense_keys": r["tflops_dense"],
                                     "identical_to_dense": r["identical_to_dense"]},
                          "roofline": {"bound": "mfma", "achieved": r["tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                       "frac": r["tflops"] / PEAK_BF16_TFLOPS, "traffic": None}}), flush=True)
        return
    if args.decode:
        r = time_decode(args.steps, args.warmup, B=args.decode_batch, ctx=args.decode_ctx, D=args.decode_dim, page_size=args.decode_page,
                        layout=args.decode_layout)
        read_gbs = read_reference()
        print(f"# decode: {r['ms_per_step']:.4f} ms  {r['gbs']:.0f} GB/s  {100 * r['gbs'] / PEAK_HBM_GBS:.1f}% of the HBM peak"
              f"  (a plain read-only kernel on this board: {read_gbs:.0f} GB/s)", file=sys.stderr, flush=True)
        print(json.dumps({"metric": "decode-step attention over a paged KV cache, GB/s of cache read", "value": r["gbs"],
                          "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": r["ms_per_step"], "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": f"decode_b{args.decode_batch}_h32_kv8_d{args.decode_dim}_ctx{args.decode_ctx // 2}-{args.decode_ctx}_page{args.decode_page}",
                                     **r["dims"], "cached_tokens": r["tokens"], "device_read_gb_per_s": read_gbs},
                          "roofline": {"bound": "hbm", "achieved": r["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                       "frac": r["gbs"] / PEAK_HBM_GBS, "traffic": None}}), flush=True)
        return
    if args.grid and args.backward:
        run_grid_backward(args.steps, args.warmup)
        return
    if args.grid:
        run_grid(args.steps, args.warmup)
        return
    if args.backward:
        names = BWD_CONFIGS if args.all else [args.config]
        res = []
        for name in names:
            r = time_backward(name, args.steps, args.warmup)
            res.append(r)
            print(f"# bwd {name}: {r['ms_per_step']:.4f} ms  {r['tflops']:.1f} TFLOP/s  "
                  f"{100 * r['tflops'] / PEAK_BF16_TFLOPS:.1f}% of bf16 peak", file=sys.stderr, flush=True)
        os.makedirs(OUT_DIR, exist_ok=True)
        with open(os.path.join(OUT_DIR, "bench_bwd.json"), "w") as f:
            json.dump(res, f, indent=1)
        print(json.dumps({"metric": "attention bwd TFLOP/s (5 contractions on unmasked pairs)", "unit": "TFLOP/s",
                          "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "dtype": "bf16",
                          "data": "synthetic", "results": res}), flush=True)
        return
    # Reference measurements (what the matrix cores and the HBM of this board sustain, in this run).  They
    # run once the workload is resident, right before its warm-up steps: the board is then in its sustained
    # power state, and the timed steps see the clock a long-running job sees rather than the transient of
    # the first launches after an idle period (the host-side input generation is such a period).
    refs = {}

    def references():
        if args.no_gemm_reference:
            return
        refs["mfma_only_bf16_zeros_tflops"] = mfma_peak_reference(zero_data=True, reps=4)
        refs["device_copy_gb_per_s"] = copy_reference()
        refs["gemm_bf16_random_tflops"] = gemm_reference()
        refs["mfma_only_bf16_random_tflops"] = mfma_peak_reference()
    results = []
    if args.all:
        for name in CONFIGS:
            if name == args.config:
                continue
            r, _ = time_config(name, args.steps, args.warmup)
            r.pop("device_workload")
            results.append(r)
            print(f"# {name}: {r['kernel_ms']:.4f} ms  {r['kernel_tflops']:.1f} TFLOP/s  "
                  f"{100 * r['kernel_tflops'] / PEAK_BF16_TFLOPS:.1f}% of bf16 peak  {r['gbs']:.0f} GB/s",
                  file=sys.stderr, flush=True)
            if r["bytes"] < 256e6 and name in ("c3c_window_doc", "c5_evoformer"):
                # small enough to live in the Infinity Cache between calls: also time it from HBM
                rc, _ = time_config(name, args.steps, args.warmup, rotate=6)
                rc.pop("device_workload")
                rc["config"] = name + "_cold"
                results.append(rc)
                print(f"# {name} over 6 rotating buffer sets: {rc['kernel_ms']:.4f} ms  {rc['gbs']:.0f} GB/s "
                      f"({100 * rc['gbs'] / PEAK_HBM_GBS:.1f}% of the HBM peak)", file=sys.stderr, flush=True)
    r, w = time_config(args.config, args.steps, args.warmup, before=references, rotate=args.rotate)
    dw0 = r.pop("device_workload")
    results.append(r)
    if args.all:
        os.makedirs(OUT_DIR, exist_ok=True)
        with open(os.path.join(OUT_DIR, "bench_all.json"), "w") as f:
            json.dump(results, f, indent=1)

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        entry = json.load(open(tpath)).get(args.config)
        traffic = entry["total"] if entry else None     # HBM bytes per launch, from rocprofv3 --pmc (see profiles/)
    line = {
        "metric": "attention fwd TFLOP/s per variant at 1 GPU; % of bf16 MFMA peak",
        "value": r["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.config, **r["dims"], "variant": w.name, "out_dtype": "bf16", "buffer_sets": args.rotate,
                   "flops_per_step": r["flops"], "pct_of_bf16_mfma_peak": 100 * r["tflops"] / PEAK_BF16_TFLOPS,
                   "hbm_gb_per_s_algorithmic": r["gbs"], "single_launch_us": r["launch_us"]},
        "roofline": {"bound": "mfma", "achieved": r["kernel_tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": r["kernel_tflops"] / PEAK_BF16_TFLOPS, "traffic": traffic},
    }
    if args.config in HBM_BOUND:                   # below the ridge of 315 FLOP per byte once masked tiles are skipped
        line["roofline"] = {"bound": "hbm", "achieved": r["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": r["gbs"] / PEAK_HBM_GBS, "traffic": traffic}
    line["config"].update(refs)
    if not args.no_gemm_reference:
        line["config"]["power_clock"] = sustained_power_clock(dw0, r["flops"])
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
