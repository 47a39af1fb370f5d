"""wf_op_attention_noalloc (index memory in a device array of the library image, no allocation, asynchronous)
against wf_op_attention on the same inputs: same kernels and same work list, so the results must be
bit-identical.  Two calls in a row on one stream, the second with a smaller batch, so that whatever the first
left in the shared array would show; then the capacity error and a larger batch after it."""
import numpy as np
import pytest

from paper_2412_11272_amd import binding as wf

pytestmark = pytest.mark.gpu


def _case(lens, n_heads, seed, precision):
    import torch
    d = 64 * n_heads
    M = sum(lens)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rng = np.random.default_rng(seed)
    qkv = rng.standard_normal((M, 3 * d)).astype(np.float32)
    qkv[:, :2 * d] *= 2.0
    dt = torch.bfloat16 if precision == wf.WF_PRECISION_BF16 else torch.float32
    return torch.from_numpy(qkv).to(dt).cuda(), cu, torch.full((M, d), float("nan"), dtype=dt, device="cuda"), \
        torch.full((M, d), float("nan"), dtype=dt, device="cuda")


@pytest.mark.parametrize("precision", [wf.WF_PRECISION_BF16, wf.WF_PRECISION_F32], ids=["bf16", "f32"])
def test_noalloc_attention_equals_allocating_entry_point_on_consecutive_calls(precision):
    import torch
    big = [700, 64, 65, 1525, 1, 129, 300, 128]           # 8 streams, 26 query blocks
    small = [75, 2, 130]                                   # fewer streams, fewer blocks: stale entries lie behind it
    q1, cu1, ref1, got1 = _case(big, 3, 1, precision)
    q2, cu2, ref2, got2 = _case(small, 3, 2, precision)
    wf.op_attention(precision, q1, ref1, cu1, 3)
    wf.op_attention(precision, q2, ref2, cu2, 3)
    wf.op_attention_noalloc(precision, q1, got1, cu1, 3)  # back to back on one stream, no sync in between
    wf.op_attention_noalloc(precision, q2, got2, cu2, 3)
    wf.op_attention_noalloc(precision, q1, got1, cu1, 3)  # and the large one again after the small one
    torch.cuda.synchronize()
    assert torch.isfinite(got1).all() and torch.isfinite(got2).all()
    assert torch.equal(got1, ref1)
    assert torch.equal(got2, ref2)


def test_noalloc_attention_rejects_what_the_index_array_cannot_hold():
    import torch
    lens = [1] * 5462                                      # 3 ints per one-token stream: 16387 > 16384
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    qkv = torch.zeros((len(lens), 192), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros((len(lens), 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(wf.WfError) as ei:
        wf.op_attention_noalloc(wf.WF_PRECISION_BF16, qkv, out, cu, 1)
    assert ei.value.code == wf.WF_E_CAPACITY
    # the largest count of one-token streams that fits still runs, and matches
    lens = [1] * 5461
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rng = np.random.default_rng(3)
    qkv = torch.from_numpy(rng.standard_normal((5461, 192)).astype(np.float32)).bfloat16().cuda()
    ref = torch.empty((5461, 64), dtype=torch.bfloat16, device="cuda")
    got = torch.empty_like(ref)
    wf.op_attention(wf.WF_PRECISION_BF16, qkv, ref, cu, 1)
    wf.op_attention_noalloc(wf.WF_PRECISION_BF16, qkv, got, cu, 1)
    torch.cuda.synchronize()
    assert torch.equal(got, ref)
    assert torch.equal(got, qkv[:, 128:192])               # one key per stream: the output is its value row
