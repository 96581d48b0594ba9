"""The entry point that allocates nothing (anpd_linear_static) against anpd_linear: same kernels, so the
same bits; and against the oracle.  Two calls in a row share the library's built-in scratch, the second
with a smaller input, so the second call must not see what the first left behind."""
import numpy as np
import pytest
import torch

from oracle import decoder as od
from paper_2404_08698_amd import binding as B
from paper_2404_08698_amd import synth

pytestmark = pytest.mark.gpu


def _case(seed, M, N, K):
    X = synth.approx_normal(seed, M * 7 + K, M * K, 1.0).reshape(M, K)
    W = synth.approx_normal(seed + 1, N + K, N * K, 0.02).reshape(N, K).to(torch.bfloat16)
    return X, W


def test_two_calls_in_a_row_match_the_workspace_entry_point_and_the_oracle():
    # the larger input first (17 rows: four operand fragments per k-step, K with a ragged last k-step),
    # then smaller ones (fewer rows, fewer k-steps), then the first again
    cases = [(31, 17, 528, 4104), (33, 3, 64, 1000), (35, 8, 4096 + 16, 4096), (37, 1, 32, 200), (31, 17, 528, 4104)]
    for seed, M, N, K in cases:
        X, W = _case(seed, M, N, K)
        Xc, Wc = X.cuda(), W.cuda()
        packed = B.pack_weights(Wc)
        want = B.linear(Xc, Wc, B.GEMM_MFMA, packed=packed)
        got = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        B.linear_static(Xc, packed, N, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (M, N, K)
        ref = od.linear(X.double().numpy(), od.to_numpy_weight(W))
        assert np.max(np.abs(got.cpu().double().numpy() - ref)) < 1e-4, (M, N, K)


def test_sizes_beyond_the_built_in_scratch_are_rejected():
    K = 16384 + 32
    X = torch.zeros(1, K, dtype=torch.float32, device="cuda")
    Y = torch.zeros(1, 16, dtype=torch.float32, device="cuda")
    packed = torch.zeros(B.lib().anpd_packed_bytes(16, K), dtype=torch.uint8, device="cuda")
    with pytest.raises(B.AnpdError) as e:
        B.linear_static(X, packed, 16, Y)
    assert e.value.code == B.E_CAPACITY
    # the largest size it takes
    K = 16384
    X, W = _case(41, 2, 16, K)
    packed = B.pack_weights(W.cuda())
    want = B.linear(X.cuda(), W.cuda(), B.GEMM_MFMA, packed=packed)
    got = torch.empty(2, 16, dtype=torch.float32, device="cuda")
    B.linear_static(X.cuda(), packed, 16, got)
    torch.cuda.synchronize()
    assert torch.equal(got, want)
