"""CPU tests of the PyTorch wrapper's argument checks: the C ABI reads document ids, sequence
lengths, block tables and ALiBi slopes as raw int32 / float32 arrays, so the wrapper has to refuse
everything that would be reinterpreted silently (torch's default int64, sliced views, wrong shapes)."""
import pytest
import torch

from paper_2511_02043_amd import functional as F

CPU = torch.device("cpu")


def test_accepts_what_the_abi_reads():
    F._check_aux("q_doc_ids", torch.zeros(2, 8, dtype=torch.int32), torch.int32, (2, 8), CPU)
    F._check_aux("alibi_slopes", torch.ones(4), torch.float32, (4,), CPU)
    F._check_aux("nothing", None, torch.int32, (1,), CPU)
    table = torch.zeros(3, 16, dtype=torch.int32)[:, :5]          # row stride 16, unit inner stride
    F._check_aux("block_table", table, torch.int32, (3, 5), CPU, contiguous=False, inner_unit=True)


@pytest.mark.parametrize("name, tensor, dtype, shape, kw", [
    ("int64 ids", torch.zeros(2, 8, dtype=torch.int64), torch.int32, (2, 8), {}),
    ("float64 slopes", torch.ones(4, dtype=torch.float64), torch.float32, (4,), {}),
    ("wrong shape", torch.zeros(2, 7, dtype=torch.int32), torch.int32, (2, 8), {}),
    ("missing batch axis", torch.zeros(8, dtype=torch.int32), torch.int32, (1, 8), {}),
    ("sliced ids", torch.zeros(2, 16, dtype=torch.int32)[:, ::2], torch.int32, (2, 8), {}),
    ("transposed table", torch.zeros(5, 3, dtype=torch.int32).t(), torch.int32, (3, 5),
     dict(contiguous=False, inner_unit=True)),
    ("not a tensor", [1, 2, 3], torch.int32, (3,), {}),
])
def test_rejects(name, tensor, dtype, shape, kw):
    with pytest.raises(ValueError):
        F._check_aux(name, tensor, dtype, shape, CPU, **kw)


def test_rejects_other_device():
    with pytest.raises(ValueError):
        F._check_aux("seq_lens", torch.zeros(3, dtype=torch.int32), torch.int32, (3,), torch.device("cuda:0"))


def test_entry_points_refuse_cpu_tensors():
    q = torch.zeros(1, 2, 8, 64, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        F.attention(q, q, q)
    with pytest.raises(ValueError):
        F.decode_attention(q[0, :, 0], q, q, torch.zeros(2, dtype=torch.int32))
