"""GPU check of qvggt_linear_e2m3_own_workspace, the entry point for callers that cannot allocate: its intermediate buffer is a
fixed device array inside the library instead of a workspace argument.  Same kernels as qvggt_linear_e2m3, so Y must be the same
bits; two calls in a row share the array, the second with fewer rows (the array then still holds the first call's tail)."""
import numpy as np
import pytest
import torch

import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu
q = G.q


def _layer(seed, N, K):
    rng = np.random.default_rng(seed)
    W = synth.f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.02).astype(np.float32))
    signs = np.where(rng.random(K) < 0.5, -1, 1).astype(np.int8)
    bias = synth.f32_to_bf16_bits((rng.standard_normal(N) * 0.02).astype(np.float32))
    return W, signs, bias


def _rows(seed, M, K):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(3, (M, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    x[: min(5, M)] *= 20
    return synth.f32_to_bf16_bits(x)


@pytest.mark.parametrize("K,N,M1,M2", [(1024, 3072, 1374, 300), (4096, 1024, 700, 129)])
def test_own_workspace_matches_workspace_argument(K, N, M1, M2):
    W, signs, bias = _layer(K + N, N, K)
    prep = G.gpu_prep(W, _rows(1, 512, K), signs)
    Wf = torch.empty(q.qvggt_e2m3_bytes(N, K), dtype=torch.uint8, device=G.DEV)
    G.codes_to_e2m3(prep["Wq"], N, K, Wf)
    bias_d = G.to_dev(bias)
    q.qvggt_init()
    for call, M in enumerate((M1, M2)):                  # two calls in a row on the same device array, the second smaller
        Xd = G.to_dev(_rows(10 + call, M, K))
        want = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
        ws = torch.empty(q.qvggt_workspace_bytes_e2m3(M, N, K), dtype=torch.uint8, device=G.DEV)
        q.qvggt_linear_e2m3(Xd, prep["signs"], prep["inv"], Wf, prep["sw"], bias_d, want, ws)
        got = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
        torch.cuda.synchronize()
        q.qvggt_linear_e2m3_own_workspace(Xd, prep["signs"], prep["inv"], Wf, prep["sw"], bias_d, got)
        torch.cuda.synchronize()
        assert not torch.isnan(got.float()).any().item(), f"call {call}: rows left unwritten"
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), f"call {call} (M = {M}): Y differs from qvggt_linear_e2m3"


def test_own_workspace_rejects_what_does_not_fit():
    limit = q.qvggt_own_workspace_bytes()
    assert limit == 36 << 20
    K, N = 4096, 1024
    M_fit, M_over = 12160, 12161
    assert q.qvggt_workspace_bytes_e2m3(M_fit, N, K) <= limit < q.qvggt_workspace_bytes_e2m3(M_over, N, K)
    X = torch.zeros(M_over, K, dtype=torch.bfloat16, device=G.DEV)
    Wf = torch.zeros(q.qvggt_e2m3_bytes(N, K), dtype=torch.uint8, device=G.DEV)
    sw = torch.ones(N, dtype=torch.float32, device=G.DEV)
    Y = torch.full((M_over, N), 3.0, dtype=torch.bfloat16, device=G.DEV)
    with pytest.raises(q.QvggtError) as e:
        q.qvggt_linear_e2m3_own_workspace(X, None, None, Wf, sw, None, Y)
    assert e.value.status == 5                                             # QVGGT_ERR_WORKSPACE, nothing launched
    torch.cuda.synchronize()
    assert bool((Y == 3.0).all().item())
    q.qvggt_linear_e2m3_own_workspace(X[:M_fit], None, None, Wf, sw, None, Y[:M_fit])     # the largest shape that fits runs
    torch.cuda.synchronize()
    assert bool((Y[:M_fit] == 0.0).all().item()) and bool((Y[M_fit:] == 3.0).all().item())
