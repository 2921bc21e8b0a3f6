"""Tensors beyond 4 GiB: the kernels' 64-bit address arithmetic (batch / head / page offsets past
2^32 bytes), on sampled heads and sequences against the oracles.  Inputs are seeded N(0,1) bf16 drawn on
the device (host generation of 4 GiB tensors would dominate the run); only the sampled heads travel
to the host."""
import numpy as np
import pytest

from oracle import attention_backward_oracle as bo
from oracle import attention_oracle as ao
from oracle import decode_oracle as do
from paper_2511_02043_amd import inputs

pytestmark = pytest.mark.gpu


def rel_l2(got, ref):
    d = got - ref
    return float(np.sqrt(np.sum(d * d) / np.sum(ref * ref)))


def test_forward_backward_past_4gib():
    import torch
    from paper_2511_02043_amd.functional import attention
    B, H, S, D = 160, 32, 4096, 128                 # 5 GiB per tensor: head (64, 0) starts at element 2^30, (128, 0) at byte 2^32
    dev = "cuda:0"
    gen = torch.Generator(device=dev).manual_seed(251102043)

    def draw():
        return torch.randn((B, H, S, D), device=dev, dtype=torch.bfloat16, generator=gen)

    q, k, v, dout = draw().requires_grad_(True), draw().requires_grad_(True), draw().requires_grad_(True), draw()
    assert q.numel() * 2 >= 1 << 32
    out = attention(q, k, v, causal=True)
    out.backward(dout)
    torch.cuda.synchronize()
    for b, h in ((0, 0), (64, 0), (128, 0), (159, 31)):
        def head(t):
            return t[b, h].detach().float().cpu().numpy()[None, None, None]      # [1, 1, 1, S, D]
        w = inputs.Workload("causal_bf16_large", "bf16", head(q), head(k), head(v), scale=D ** -0.5, causal=True)
        ref_out, _ = ao.run_workload(w)
        got = head(out)
        err = float(np.max(np.abs(got - ref_out)))
        print(f"head ({b}, {h}): out max_abs={err:.3e}", flush=True)
        assert np.all(np.abs(got - ref_out) <= 1e-2 + 2.0 ** -8 * np.abs(ref_out))
        ref = bo.run_workload_backward(w, head(dout))
        for name, t, r in zip(("dq", "dk", "dv"), (q.grad, k.grad, v.grad), ref):
            e = rel_l2(head(t), r)
            print(f"head ({b}, {h}) {name}: rel_l2={e:.3e}", flush=True)
            assert e <= 5e-3, (b, h, name, e)


def test_decode_cache_past_4gib():
    import torch
    from paper_2511_02043_amd import binding as fb
    dev = "cuda:0"
    P, page, Hkv, H, D = 140000, 16, 8, 32, 128     # 32 KiB per page and cache: pages from 131072 on lie past 4 GiB
    B, max_pages = 32, 96
    gen = torch.Generator(device=dev).manual_seed(251102044)
    kc = torch.randn((P, page, Hkv, D), device=dev, dtype=torch.bfloat16, generator=gen)
    vc = torch.randn((P, page, Hkv, D), device=dev, dtype=torch.bfloat16, generator=gen)
    q = torch.randn((B, H, D), device=dev, dtype=torch.bfloat16, generator=gen)
    rng = np.random.Generator(np.random.PCG64(251102045))
    seq_lens = rng.integers(1, max_pages * page + 1, size=B).astype(np.int32)
    seq_lens[0], seq_lens[1] = max_pages * page, 1
    # every second page of a sequence from the part of the pool past 4 GiB, the others from anywhere
    high = rng.permutation(np.arange(131072, P))[: B * max_pages // 2]
    low = rng.permutation(131072)[: B * max_pages // 2]
    table = np.empty((B, max_pages), dtype=np.int32)
    table[:, 0::2] = high.reshape(B, -1)
    table[:, 1::2] = low.reshape(B, -1)

    q5 = q[:, None, :, None, :]
    k5, v5 = kc.permute(0, 2, 1, 3)[:, None], vc.permute(0, 2, 1, 3)[:, None]
    out = torch.empty((B, 1, H, 1, D), dtype=torch.float32, device=dev)
    lse = torch.empty((B, 1, H, 1, 1), dtype=torch.float32, device=dev)
    d_table, d_lens = torch.from_numpy(table).to(dev), torch.from_numpy(seq_lens).to(dev)
    scale = D ** -0.5
    desc = fb.variant_desc(scale=scale, score_mod=fb.FL_MOD_NONE, mask=fb.FL_MASK_CAUSAL)
    kv = fb.paged_kv(block_table=d_table, page_size=page, seq_lens=d_lens, max_seq_len=int(seq_lens.max()))
    tq, tk, tv, tout, tlse = (fb.tensor_desc(x) for x in (q5, k5, v5, out, lse))
    ws = torch.empty(max(fb.fl_attn_decode_workspace_size(tq, tk, kv), 16), dtype=torch.uint8, device=dev)
    aux = fb.aux_desc(workspace=ws)
    fb.check(fb.fl_attn_decode(tq, tk, tv, kv, desc, aux, tout, tlse, torch.cuda.current_stream().cuda_stream))
    torch.cuda.synchronize()

    # the oracle sees only the pages in use, renumbered in ascending order
    used, inverse = np.unique(table, return_inverse=True)
    small_table = inverse.reshape(table.shape).astype(np.int32)
    idx = torch.from_numpy(used.astype(np.int64)).to(dev)
    k_small = kc.index_select(0, idx).float().cpu().numpy()
    v_small = vc.index_select(0, idx).float().cpu().numpy()
    ref_out, ref_lse = do.decode_attention(q.float().cpu().numpy(), k_small, v_small, small_table, seq_lens, scale=scale)
    got_out, got_lse = out.cpu().numpy()[:, 0, :, 0, :], lse.cpu().numpy()[:, 0, :, 0, 0]
    err, lerr = float(np.max(np.abs(got_out - ref_out))), float(np.max(np.abs(got_lse - ref_lse)))
    print(f"decode past 4 GiB: out max_abs={err:.3e} lse={lerr:.3e}", flush=True)
    assert err <= 1e-2 and lerr <= 1e-3
