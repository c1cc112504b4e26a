"""structkv_select_topk_static (the entry point that allocates nothing: its scratch is an array inside the
library) against structkv_select_topk, through the C ABI, bit for bit, and against the oracle's selection."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(B, oracle, seq_lens, k_per_seq, keep_tail, seed, stream=None):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    total = sum(seq_lens)
    scores = torch.rand(total, generator=g, device="cuda") * 4.0 - 1.0
    m = scores[3::7].numel()
    scores[::7][:m] = scores[3::7]                             # ties, also across the threshold
    cu = [0]
    for n in seq_lens:
        cu.append(cu[-1] + n)
    rows = sum(k + keep_tail for k in k_per_seq)
    ws = torch.empty(B.structkv_workspace_bytes(None, len(seq_lens), total), dtype=torch.uint8, device="cuda")
    ref = torch.full((rows,), -1, dtype=torch.int32, device="cuda")
    got = torch.full((rows,), -2, dtype=torch.int32, device="cuda")
    B.structkv_select_topk(scores, cu, k_per_seq, keep_tail, ref, ws, stream)
    B.structkv_select_topk_static(scores, cu, k_per_seq, keep_tail, got, stream)
    torch.cuda.synchronize()
    assert torch.equal(ref, got), "static-scratch selection differs from the workspace one"
    want = np.concatenate(oracle.select_topk(scores.cpu().numpy(), seq_lens, k_per_seq, keep_tail))
    assert np.array_equal(got.cpu().numpy(), want)


def test_static_scratch_topk_two_calls_in_a_row(oracle):
    from paper_2604_06746_amd import binding as B
    # first a large ragged batch, then a smaller input: the second call finds the first one's leftovers
    _case(B, oracle, [131072, 40000, 77777, 1000], [4096, 2000, 3888, 50], 64, seed=11)
    _case(B, oracle, [5000, 300], [250, 17], 32, seed=12)
    _case(B, oracle, [262144 + 5], [9000], 0, seed=13)
    _case(B, oracle, [97], [96], 1, seed=14)


def test_static_scratch_topk_limit_and_errors():
    from paper_2604_06746_amd import binding as B
    n = 2_200_000                                              # beyond what the 4 MiB scratch covers
    scores = torch.zeros(n, device="cuda")
    idx = torch.empty(10, dtype=torch.int32, device="cuda")
    with pytest.raises(B.StructKVError) as e:
        B.structkv_select_topk_static(scores, [0, n], [10], 0, idx)
    assert e.value.status == B.STRUCTKV_ERR_UNSUPPORTED and "static scratch" in str(e.value)
    with pytest.raises(B.StructKVError) as e:
        B.structkv_select_topk_static(scores, [0, 100], [101], 0, idx)
    assert e.value.status == B.STRUCTKV_ERR_INVALID_ARG
    # the largest documented call is accepted
    m = B.STRUCTKV_STATIC_TOPK_MAX_TOKENS
    lens = [m // 64] * 64
    big = torch.rand(m, device="cuda")
    out = torch.empty(64 * 8, dtype=torch.int32, device="cuda")
    cu = [i * (m // 64) for i in range(65)]
    B.structkv_select_topk_static(big, cu, [8] * 64, 0, out)
    torch.cuda.synchronize()
    top = torch.topk(big.view(64, -1), 8, dim=1).indices.sort(dim=1).values.to(torch.int32).reshape(-1)
    assert torch.equal(out, top)
