"""The entry point that allocates nothing (tr_op_topk_static) against tr_op_topk, through the C ABI:
two calls in a row on the library's static device scratch, the second on a smaller input."""
import numpy as np
import pytest
import torch

from paper_2408_08696_amd import synth, tr
from gpu_util import require_gpu, say

pytestmark = pytest.mark.gpu


def test_static_topk_matches_context_topk_twice():
    require_gpu()
    for rows, V, k, dtype, seed in [(80, 32000, 8, torch.bfloat16, 11), (37, 5000, 5, torch.float32, 12)]:
        say("static top-k", rows, V, k, dtype)
        logits = synth.normal_tensor((rows, V), 3.0, seed=seed, dtype=dtype).cuda()
        ctx = tr.Context(V, k, [-1], [-1], 1)
        want = torch.zeros(rows, k, dtype=torch.int32, device="cuda")
        got = torch.full((rows, k), -7, dtype=torch.int32, device="cuda")
        ctx.op_topk(logits, want)
        tr.op_topk_static(logits, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        ctx.close()


def test_static_topk_rejects_sizes_beyond_its_scratch():
    require_gpu()
    x = torch.zeros(4, 64, dtype=torch.float32, device="cuda")
    out = torch.zeros(4, 9, dtype=torch.int32, device="cuda")
    with pytest.raises(tr.TRError) as e:
        tr.op_topk_static(x, out)                              # k = 9 > 8
    assert e.value.status == tr.TR_ECAPACITY
    big = torch.zeros(129, 64, dtype=torch.float32, device="cuda")
    with pytest.raises(tr.TRError) as e:
        tr.op_topk_static(big, torch.zeros(129, 8, dtype=torch.int32, device="cuda"))
    assert e.value.status == tr.TR_ECAPACITY
