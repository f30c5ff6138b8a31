"""GPU parity of online kernel 2: int32 accumulators bit-exact against the oracle's integer
product given identical codes, and the fused dequant + bias epilogue."""
import numpy as np
import pytest
import torch

import oracle
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _run(qx, qw, dx, dw, bias_bits):
    M, K = qx.shape
    N = qw.shape[0]
    Xq, Wq = G.gpu_pack(qx), G.gpu_pack(qw)
    Y = torch.empty(M, N, dtype=torch.bfloat16, device=G.DEV)
    acc = torch.full((M, N), 12345, dtype=torch.int32, device=G.DEV)
    import paper_2509_21302_amd as q
    q.qvggt_w4a4_gemm(Xq, G.to_dev(dx.astype(np.float32)), Wq, G.to_dev(dw.astype(np.float32)),
                      G.to_dev(bias_bits), M, N, K, Y, acc)
    return acc.cpu().numpy(), G.bf16_bits(Y)


@pytest.mark.parametrize("M,N,K", [(64, 128, 128), (1, 16, 128), (300, 384, 256), (129, 144, 1024),
                                   (1374, 3072, 1024), (257, 1024, 4096), (33, 48, 8192)])
def test_accumulators_bit_exact(M, N, K):
    rng = np.random.default_rng(M * 7 + N)
    qx = rng.integers(-8, 8, (M, K)).astype(np.int8)
    qw = rng.integers(-8, 8, (N, K)).astype(np.int8)
    dx = np.exp(rng.uniform(-3, 1, M))
    dw = np.exp(rng.uniform(-5, -2, N))
    bias = (rng.standard_normal(N) * 0.02).astype(np.float32)
    from synth import f32_to_bf16_bits
    bias_bits = f32_to_bf16_bits(bias)
    acc, Y = _run(qx, qw, dx, dw, bias_bits)
    want = oracle.int_gemm(qx, qw)
    assert np.array_equal(acc, want)
    # epilogue: the oracle applies the same fp32-stored scales in fp64 and rounds once
    Yo = oracle.dequant_bias(want, dx.astype(np.float32), dw.astype(np.float32), oracle.to_f64(bias_bits))
    assert G.rel_fro(Y, Yo) <= 1e-3
    ulp_off = np.abs(Y.astype(np.int32) - Yo.astype(np.int32))
    assert ulp_off.max() <= 1 and (ulp_off != 0).mean() < 5e-3


@pytest.mark.parametrize("M,N,K", [(1, 16, 128), (300, 384, 256), (1374, 3072, 1024), (513, 1040, 1024), (10992, 1024, 4096)])
@pytest.mark.parametrize("with_bias", [True, False])
def test_production_kernel_matches_accumulator_dump_variant(M, N, K, with_bias):
    """The kernel that writes the raw accumulators is a separate instantiation; the one a caller normally gets
    (acc_debug = NULL) must produce the same bf16 output bit for bit, and it is checked against the oracle too."""
    import paper_2509_21302_amd as q
    from synth import f32_to_bf16_bits
    rng = np.random.default_rng(M + 3 * N + K)
    qx = rng.integers(-7, 8, (M, K)).astype(np.int8)
    qw = rng.integers(-7, 8, (N, K)).astype(np.int8)
    dx = np.exp(rng.uniform(-3, 1, M)).astype(np.float32)
    dw = np.exp(rng.uniform(-5, -2, N)).astype(np.float32)
    bias_bits = f32_to_bf16_bits((rng.standard_normal(N) * 0.02).astype(np.float32)) if with_bias else None
    acc_dbg, Y_dbg = _run(qx, qw, dx, dw, bias_bits)
    Xq, Wq = G.gpu_pack(qx), G.gpu_pack(qw)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
    q.qvggt_w4a4_gemm(Xq, G.to_dev(dx), Wq, G.to_dev(dw), G.to_dev(bias_bits), M, N, K, Y, None)
    Y = G.bf16_bits(Y)
    assert np.array_equal(Y, Y_dbg)
    rows = np.unique(np.concatenate([np.arange(min(M, 40)), np.arange(max(M - 40, 0), M), rng.integers(0, M, 64)]))
    want = oracle.int_gemm(qx[rows], qw)
    assert np.array_equal(acc_dbg[rows], want)
    Yo = oracle.dequant_bias(want, dx[rows], dw, None if bias_bits is None else oracle.to_f64(bias_bits))
    ulp_off = np.abs(Y[rows].astype(np.int32) - Yo.astype(np.int32))
    assert ulp_off.max() <= 1 and (ulp_off != 0).mean() < 5e-3


def test_extreme_codes_and_no_bias():
    M, N, K = 40, 32, 4096
    qx = np.full((M, K), -8, np.int8)
    qw = np.full((N, K), -8, np.int8)
    qw[1::2] = 7
    acc, Y = _run(qx, qw, np.ones(M), np.ones(N), None)
    assert np.array_equal(acc, oracle.int_gemm(qx, qw))
    assert acc.max() == 64 * K and acc.min() == -56 * K
    assert np.array_equal(Y, oracle.dequant_bias(acc, np.ones(M), np.ones(N)))


def test_identity_like_weights_reproduce_codes():
    M, K = 70, 128
    rng = np.random.default_rng(1)
    qx = rng.integers(-8, 8, (M, K)).astype(np.int8)
    qw = np.eye(K, dtype=np.int8)
    acc, _ = _run(qx, qw, np.ones(M), np.ones(K), None)
    assert np.array_equal(acc, qx.astype(np.int32))


def test_shape_sweep_both_code_widths():
    """Seeded sweep over ragged shapes (M not a multiple of any tile, N any multiple of 16, every supported K) for the
    4-bit and the 8-bit kernel: accumulators bit-exact, output within one bf16 ulp of the oracle's epilogue."""
    import paper_2509_21302_amd as q
    from synth import f32_to_bf16_bits
    rng = np.random.default_rng(2024)
    Ks = [128, 256, 512, 1024, 2048, 4096, 8192]
    for case in range(36):
        K = Ks[case % len(Ks)]
        M = int(rng.integers(1, 700)) if K <= 2048 else int(rng.integers(1, 300))
        N = 16 * int(rng.integers(1, 66 if K <= 2048 else 20))
        wide = case % 2 == 1
        lim = 128 if wide else 8
        qx = rng.integers(-lim, lim, (M, K)).astype(np.int8)
        qw = rng.integers(-lim, lim, (N, K)).astype(np.int8)
        dx = np.exp(rng.uniform(-3, 1, M)).astype(np.float32)
        dw = np.exp(rng.uniform(-8, -4, N)).astype(np.float32)
        bias_bits = f32_to_bf16_bits((rng.standard_normal(N) * 0.02).astype(np.float32)) if case % 3 else None
        Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
        acc = torch.full((M, N), 12345, dtype=torch.int32, device=G.DEV)
        if wide:
            q.qvggt_i8_gemm(G.gpu_layout_int8(qx, 1), G.to_dev(dx), G.gpu_layout_int8(qw, 1), G.to_dev(dw), G.to_dev(bias_bits), M, N, K, Y, acc)
        else:
            q.qvggt_w4a4_gemm(G.gpu_pack(qx), G.to_dev(dx), G.gpu_pack(qw), G.to_dev(dw), G.to_dev(bias_bits), M, N, K, Y, acc)
        want = oracle.int_gemm(qx, qw)
        what = f"case {case}: M={M} N={N} K={K} wide={wide}"
        assert np.array_equal(acc.cpu().numpy(), want), what
        Yo = oracle.dequant_bias(want, dx, dw, None if bias_bits is None else oracle.to_f64(bias_bits))
        ulp_off = np.abs(G.bf16_bits(Y).astype(np.int32) - Yo.astype(np.int32))
        assert ulp_off.max() <= 1 and (ulp_off != 0).mean() < 5e-3, what


@pytest.mark.parametrize("M,N,K,wide", [(66000, 512, 256, False), (33000, 1024, 512, True), (65700, 768, 128, False)])
def test_rows_split_between_the_two_tile_shapes(M, N, K, wide):
    """Shapes whose 256 x 256 tiles fill whole rounds of 256 plus a small remainder: the remainder rows go to the 128 x 128
    configuration in a second launch.  Accumulators of rows on both sides of the seam, and the last rows, are bit-exact."""
    import paper_2509_21302_amd as q
    tiles_n = (N + 255) // 256
    seam = ((M + 255) // 256 * tiles_n // 256 * 256 // tiles_n) * 256
    assert 0 < seam < M
    gen = torch.Generator(device="cpu").manual_seed(M)
    lim = 128 if wide else 8
    qx = torch.randint(-lim, lim, (M, K), generator=gen, dtype=torch.int8).numpy()
    qw = torch.randint(-lim, lim, (N, K), generator=gen, dtype=torch.int8).numpy()
    rng = np.random.default_rng(M)
    dx = np.exp(rng.uniform(-3, 1, M)).astype(np.float32)
    dw = np.exp(rng.uniform(-8, -4, N)).astype(np.float32)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=G.DEV)
    acc = torch.full((M, N), 12345, dtype=torch.int32, device=G.DEV)
    if wide:
        q.qvggt_i8_gemm(G.gpu_layout_int8(qx, 1), G.to_dev(dx), G.gpu_layout_int8(qw, 1), G.to_dev(dw), None, M, N, K, Y, acc)
    else:
        q.qvggt_w4a4_gemm(G.gpu_pack(qx), G.to_dev(dx), G.gpu_pack(qw), G.to_dev(dw), None, M, N, K, Y, acc)
    rows = np.unique(np.concatenate([np.arange(0, 8), np.arange(seam - 300, min(seam + 300, M)), np.arange(M - 200, M),
                                     rng.choice(M, 200, replace=False)]))
    idx = torch.from_numpy(rows).to(G.DEV)
    want = oracle.int_gemm(qx[rows], qw)
    assert np.array_equal(acc[idx].cpu().numpy(), want)
    Yo = oracle.dequant_bias(want, dx[rows], dw, None)
    ulp_off = np.abs(G.bf16_bits(Y[idx]).astype(np.int32) - Yo.astype(np.int32))
    assert ulp_off.max() <= 1 and (ulp_off != 0).mean() < 5e-3
    assert not torch.isnan(Y.float()).any().item()                      # every row of Y was written by one of the launches


@pytest.mark.parametrize("kind", [0, 1])
def test_matrix_ceiling_helper_runs_and_repeats(kind):
    """The benchmark's register-only matrix loop: finishes, writes every slot of its sink, and gives the same sums twice
    (integer sums for kind 0; the fp32 sums of kind 1 are order-independent only by being the same instruction stream)."""
    import paper_2509_21302_amd as q
    sink = torch.full((65536,), float("nan"), dtype=torch.float32, device=G.DEV)
    q.qvggt_mfma_ceiling(kind, 50, sink)
    torch.cuda.synchronize()
    first = sink.clone()
    assert torch.isfinite(first).all().item()
    sink.fill_(float("nan"))
    q.qvggt_mfma_ceiling(kind, 50, sink)
    torch.cuda.synchronize()
    assert torch.equal(first, sink)
