"""The entry point that allocates nothing (static device scratch instead of a workspace), through the C ABI,
against the workspace-based rnnlm_sort_segments and the oracle: two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_1502_00512_amd import binding, synth

pytestmark = pytest.mark.gpu


def _static(x, V):
    T, B = x.shape
    M = T * B
    perm = torch.full((M,), -7, dtype=torch.int32, device="cuda")
    seg = torch.full((M + 1,), -7, dtype=torch.int32, device="cuda")
    nseg = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    flag = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    binding.rnnlm_sort_segments_static(x, V, perm, seg, nseg, flag)
    torch.cuda.synchronize()
    n = int(nseg.item())
    return perm, seg[:n + 1], int(flag.item())


def test_static_sort_segments_matches_workspace_call_twice_in_a_row():
    V = 5000
    zeros = np.zeros((V, 8), np.float32)
    for (T, B, seed) in ((32, 256, 5), (7, 37, 6)):      # 8192 positions, then a smaller ragged window
        g = binding.Rnnlm(zeros, np.zeros((8, 8), np.float32), zeros, np.zeros(V, np.float32), B, T, binding.RNNLM_FP32)
        x = synth.zipf_tokens(T * B, V, 1.0, seed).reshape(T, B).astype(np.int32)
        dx = torch.as_tensor(x).cuda()
        perm_w, seg_w = g.rnnlm_sort_segments(dx)
        perm_s, seg_s, flag = _static(dx, V)
        assert flag == 0
        assert torch.equal(perm_s, perm_w) and torch.equal(seg_s, seg_w)
        pr, sr = O.sort_segments(x)
        assert np.array_equal(perm_s.cpu().numpy(), pr) and np.array_equal(seg_s.cpu().numpy(), sr)
        g.rnnlm_check()


def test_static_call_reports_range_and_rejects_oversize():
    x = torch.tensor([[0, 9], [12, 3]], dtype=torch.int32, device="cuda")
    perm, seg, flag = _static(x, 10)          # id 12 is outside [0, 10): clamped to 9 and reported
    assert flag == 1
    assert perm.tolist() == [0, 3, 1, 2] and seg.tolist() == [0, 1, 2, 4]
    perm, seg, flag = _static(x, 13)          # the flag does not stick
    assert flag == 0
    big = torch.zeros(1024, 128, dtype=torch.int32, device="cuda")   # 131072 positions > 65536
    out = torch.empty(1024 * 128 + 1, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.RnnlmError) as e:
        binding.rnnlm_sort_segments_static(big, 10, out, out, out)
    assert e.value.status == -1
