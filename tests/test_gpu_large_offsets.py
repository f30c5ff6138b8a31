"""Tensors of more than 2^31 elements: every index the kernels form must be 64 bits wide.  The benchmark's largest shape
(137400 x 4096) stays below that line, so these cases go past it on purpose: 540000 tokens put kernel 1's input at K = 4096
and the GEMM's output at N = 4096 at 2.2e9 elements each.  The oracle recomputes rows at the start, around the row where the
element offset crosses 2^31 (row 524288) and at the end."""
import numpy as np
import pytest
import torch

import oracle
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

M_BIG = 540000
SEAM = (1 << 31) // 4096


def _rows():
    return np.unique(np.concatenate([np.arange(0, 4), np.arange(SEAM - 130, SEAM + 130, 13), np.arange(M_BIG - 140, M_BIG, 7),
                                     np.array([M_BIG - 1])]))


def test_kernel_1_past_2_31_elements():
    q, K = G.q, 4096
    gen = torch.Generator(device=G.DEV).manual_seed(31)
    X = torch.empty(M_BIG, K, dtype=torch.bfloat16, device=G.DEV)
    for r0 in range(0, M_BIG, 60000):                          # in slabs: the fp32 draw of the whole tensor would be 8.8 GB more
        n = min(60000, M_BIG - r0)
        X[r0:r0 + n] = (torch.randn(n, K, generator=gen, device=G.DEV) * (1.0 + (torch.arange(n, device=G.DEV) % 5)[:, None])).to(torch.bfloat16)
    rng = np.random.default_rng(31)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    c_hat = np.exp(rng.uniform(-1, 1, K))
    inv = (1.0 / (np.sqrt(K) * c_hat)).astype(np.float32)
    rows = _rows()
    idx = torch.from_numpy(rows).to(G.DEV)
    Xs = G.bf16_bits(X[idx])
    dx, qx, _ = oracle.rotate_smooth_quant(Xs, 1.0 / (inv.astype(np.float64) * np.sqrt(K)), pre_signs=signs)
    Xq, sx = G.gpu_rsq(X, G.to_dev(signs), G.to_dev(inv))
    G.check_codes(G.gpu_unpack(Xq[idx].contiguous(), K), qx, "packed codes, 540000 x 4096")
    G.check_scales(sx[idx].cpu().numpy(), dx, "steps, 540000 x 4096")
    # the E2M3 variant of the same launch: the same codes in the other format, every row
    Xf = torch.zeros(q.qvggt_e2m3_bytes(M_BIG, K), dtype=torch.uint8, device=G.DEV)
    sxf = torch.empty(M_BIG, dtype=torch.float32, device=G.DEV)
    q.qvggt_rotate_smooth_quant_e2m3(X, G.to_dev(signs), G.to_dev(inv), Xf, sxf)
    want_f = torch.zeros_like(Xf)
    G.codes_to_e2m3(Xq, M_BIG, K, want_f)
    whole_blocks = (M_BIG // 128) * 128 * K * 3 // 4           # padding rows of the last block are never written
    assert torch.equal(Xf[:whole_blocks], want_f[:whole_blocks])
    assert torch.equal(sxf, sx)
    tail = G.decode_e2m3_rows(Xf[whole_blocks:].cpu().numpy(), M_BIG % 128, K)
    assert np.array_equal(tail, G.decode_e2m3_rows(want_f[whole_blocks:].cpu().numpy(), M_BIG % 128, K))


@pytest.mark.parametrize("path", ["e2m3", "int8"])
def test_gemm_output_past_2_31_elements(path):
    q, N, K = G.q, 4096, 128
    gen = torch.Generator(device="cpu").manual_seed(32)
    qx = torch.randint(-7, 8, (M_BIG, K), generator=gen, dtype=torch.int8).numpy()
    qw = torch.randint(-7, 8, (N, K), generator=gen, dtype=torch.int8).numpy()
    rng = np.random.default_rng(32)
    dx = np.exp(rng.uniform(-3, 1, M_BIG)).astype(np.float32)
    dw = np.exp(rng.uniform(-8, -4, N)).astype(np.float32)
    bias = oracle.bf16_from_f64(rng.normal(0, 0.1, N))
    Xq, Wq = G.gpu_pack(qx), G.gpu_pack(qw)
    Y = torch.full((M_BIG, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
    acc = torch.full((M_BIG, N), 12345, dtype=torch.int32, device=G.DEV)
    sx, sw, b = G.to_dev(dx), G.to_dev(dw), G.to_dev(bias)
    if path == "e2m3":
        Xf = torch.zeros(q.qvggt_e2m3_bytes(M_BIG, K), dtype=torch.uint8, device=G.DEV)
        Wf = torch.zeros(q.qvggt_e2m3_bytes(N, K), dtype=torch.uint8, device=G.DEV)
        G.codes_to_e2m3(Xq, M_BIG, K, Xf)
        G.codes_to_e2m3(Wq, N, K, Wf)
        q.qvggt_e2m3_gemm(Xf, sx, Wf, sw, b, M_BIG, N, K, Y, acc)
    else:
        q.qvggt_w4a4_gemm(Xq, sx, Wq, sw, b, M_BIG, N, K, Y, acc)
    rows = _rows()
    idx = torch.from_numpy(rows).to(G.DEV)
    want = oracle.int_gemm(qx[rows], qw)
    assert np.array_equal(acc[idx].cpu().numpy(), want)
    Yo = oracle.dequant_bias(want, dx[rows], dw, oracle.to_f64(bias))
    ulp_off = np.abs(G.bf16_bits(Y[idx]).astype(np.int32) - Yo.astype(np.int32))
    assert ulp_off.max() <= 1 and (ulp_off != 0).mean() < 5e-3
    # every row written, none twice with something else: the raw sums of all rows against a library product on the device
    ref = (torch.from_numpy(qx).to(G.DEV).float() @ torch.from_numpy(qw).to(G.DEV).float().T)
    assert torch.equal(acc, ref.to(torch.int32))
    assert not torch.isnan(Y[-1].float()).any().item() and not torch.isnan(Y[SEAM].float()).any().item()
