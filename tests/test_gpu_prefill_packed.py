"""GPU parity of the in-place paged prefill kernel with the query heads of a kv head packed into one workgroup
(fl_attn_prefill_paged on chunks that leave most of a 128- or 256-row tile empty), through the C-ABI: bit-equal to the
unpacked kernel, and against the fp64 oracle at the forward tolerance (max-abs <= 1e-2, lse <= 1e-3)."""
import pytest

from oracle import decode_oracle as do
from paper_2511_02043_amd import binding as fb
from paper_2511_02043_amd import inputs, runner
from tests.test_gpu_prefill_paged import check

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def restore_tuning():
    yield
    fb.fl_set_tuning("prefill_gather", 0)
    fb.fl_set_tuning("prefill_pack", 0)


PACKED = {
    # chunks that leave a 128- or 256-row tile mostly empty: the in-place kernel packs the query heads of a kv head into
    # one workgroup (rows per head x heads: 64 x 4, 32 x 8, 32 x 4, 64 x 2, 32 x 4 with three tiles per head, 64 x 2 at D = 64)
    "g4_q64": lambda: inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=64, page_size=16, seq_lens=[10, 64, 65, 300, 1500], salt=70),
    "g8_q20": lambda: inputs.prefill_paged_bf16(H=16, Hkv=2, D=128, Sq=20, page_size=16, seq_lens=[5, 20, 21, 900], salt=71),
    "g4_q30": lambda: inputs.prefill_paged_bf16(H=4, Hkv=1, D=128, Sq=30, page_size=8, seq_lens=[29, 30, 31, 700], salt=72),
    "g2_q50": lambda: inputs.prefill_paged_bf16(H=4, Hkv=2, D=128, Sq=50, page_size=32, seq_lens=[49, 64, 1000], salt=73),
    "g4_q96": lambda: inputs.prefill_paged_bf16(H=8, Hkv=2, D=128, Sq=96, page_size=16, seq_lens=[95, 96, 200, 1300], salt=74),
    "g2_q40_d64": lambda: inputs.prefill_paged_bf16(H=4, Hkv=2, D=64, Sq=40, page_size=16, seq_lens=[40, 41, 800], salt=75),
}


@pytest.mark.parametrize("name", list(PACKED))
def test_packed_heads_match_the_unpacked_kernel_and_the_oracle(name):
    """The same rows go through the same arithmetic whether or not the heads of a kv head share a workgroup: bit-equal
    outputs with packing switched off, and parity with the oracle (plain, and one variant instantiated at run time)."""
    import torch
    fb.check(fb.fl_set_tuning("prefill_gather", 2))    # the kernel that reads the pages in place
    for variant in ("plain", "alibi_window"):
        w = PACKED[name]()
        if variant == "alibi_window":
            w.alibi = inputs.alibi_slopes(w.q.shape[1])
            w.window = 200
        outs = []
        for pack_off in (0, 1):
            fb.check(fb.fl_set_tuning("prefill_pack", pack_off))
            try:
                dd = runner.upload_prefill_paged(w)
                dd.out.fill_(float("nan"))
                dd.lse.fill_(float("nan"))
                dd.run_checked()
                torch.cuda.synchronize()
                outs.append((dd.out.clone(), dd.lse.clone()))
            finally:
                fb.fl_set_tuning("prefill_pack", 0)
        assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1]), (name, variant)
        ref, ref_lse = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale, window=w.window,
                                            alibi_slopes=w.alibi)
        check(outs[0][0].cpu().numpy()[:, 0], outs[0][1].cpu().numpy()[:, 0, :, :, 0], ref, ref_lse, f"packed_{name}_{variant}")


def test_packed_and_unpacked_random_shapes():
    """Twenty-four seeded random chunks through the kernel that reads the pages in place: head groups of 1 ... 8, 1 ... 127
    rows, both head dims, page sizes 8 ... 64, lengths from below the chunk to a few thousand tokens -- whatever tile shape
    and head packing the library picks for each, every output against the oracle."""
    import numpy as np
    import torch
    rng = np.random.Generator(np.random.PCG64(2511020431))
    fb.check(fb.fl_set_tuning("prefill_gather", 2))
    for case in range(24):
        group = int(rng.choice([1, 2, 4, 8]))
        Hkv = int(rng.choice([1, 2]))
        D = int(rng.choice([64, 128, 128]))
        Sq = int(rng.integers(1, 128))
        ps = int(rng.choice([8, 16, 32, 64]))
        B = int(rng.integers(1, 4))
        hi = int(rng.choice([150, 1200, 3000]))
        lens = [int(x) for x in rng.integers(1, hi + 1, size=B)]
        w = inputs.prefill_paged_bf16(H=group * Hkv, Hkv=Hkv, D=D, Sq=Sq, page_size=ps, seq_lens=lens, salt=300 + case)
        label = f"case {case}: group={group} Hkv={Hkv} D={D} Sq={Sq} page={ps} lens={lens}"
        print(label, flush=True)
        dd = runner.upload_prefill_paged(w)
        dd.out.fill_(float("nan"))
        dd.lse.fill_(float("nan"))
        dd.run_checked()
        torch.cuda.synchronize()
        ref, ref_lse = do.prefill_attention(w.q, w.k_cache, w.v_cache, w.block_table, w.seq_lens, scale=w.scale)
        check(dd.out.cpu().numpy()[:, 0], dd.lse.cpu().numpy()[:, 0, :, :, 0], ref, ref_lse, label)
