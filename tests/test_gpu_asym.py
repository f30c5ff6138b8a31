"""GPU parity of the asymmetric setting (affine activation codes with a zero point per token, symmetric weights) against
the CPU oracle, through the C ABI: kernel 1's codes / steps / zero points, the weight code sums, the GEMM's corrected sum."""
import numpy as np
import pytest
import torch

import oracle
import synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def _rows(rows, K, seed, dtype, one_sided):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(3, (rows, K)).astype(np.float32)
    x[:, rng.choice(K, max(1, K // 100), replace=False)] *= 50
    x[: min(5, rows)] *= 20
    if one_sided:
        x = np.abs(x)                      # what a GELU hands on: the rotated row has a large first column
    else:
        x += rng.uniform(-2, 4, (rows, 1)).astype(np.float32)
    return synth.f32_to_bf16_bits(x) if dtype == "bf16" else x


def _check_asym_codes(Xq, sx, zx, K, dx, zp, u, what):
    """Zero points may differ by one on a knife edge of rne(-lo / step); what is unique is the effective code u - zp."""
    got_u = G.gpu_unpack(Xq, K).astype(np.int16) + 8
    got_zp = zx.cpu().numpy()
    assert np.array_equal(got_zp, np.rint(got_zp)) and got_zp.min() >= 0 and got_zp.max() <= 15
    assert got_u.min() >= 0 and got_u.max() <= 15
    dz = np.abs(got_zp - zp)
    assert dz.max(initial=0) <= 1 and (dz != 0).mean() <= 1e-3, f"{what}: zero points differ on {(dz != 0).mean():.2e} of the rows"
    G.check_codes(got_u - got_zp[:, None].astype(np.int16), u.astype(np.int16) - zp[:, None].astype(np.int16), what)
    G.check_scales(sx.cpu().numpy(), dx, what)


@pytest.mark.parametrize("K", [128, 512, 1024, 2048, 4096, 8192])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("one_sided", [False, True])
def test_asym_rotate_quant(K, dtype, one_sided):
    rows = 1031 if K == 1024 else (37 if K >= 2048 else 203)
    X = _rows(rows, K, 700 + K, dtype, one_sided)
    rng = np.random.default_rng(K + 9)
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    c_hat = np.exp(rng.uniform(-1, 1, K))
    inv = (1.0 / (np.sqrt(K) * c_hat)).astype(np.float32)
    dx, zp, u, _ = oracle.rotate_smooth_quant_asym(X, 1.0 / (inv.astype(np.float64) * np.sqrt(K)), pre_signs=signs)
    Xq, sx, zx = G.gpu_rsq_asym(G.to_dev(X), G.to_dev(signs), G.to_dev(inv))
    _check_asym_codes(Xq, sx, zx, K, dx, zp, u, f"K={K} {dtype} one_sided={one_sided}")


def test_asym_rotate_quant_degenerate_rows():
    """Zeros: step 0, zero point 0, u = 0 (stored -8).  No rotation signs or smoothing.  One row."""
    K = 1024
    X = _rows(9, K, 5, "bf16", False)
    X[2] = 0
    dx, zp, u, _ = oracle.rotate_smooth_quant_asym(X)
    Xq, sx, zx = G.gpu_rsq_asym(G.to_dev(X), None, None)
    _check_asym_codes(Xq, sx, zx, K, dx, zp, u, "plain")
    assert sx[2].item() == 0.0 and zx[2].item() == 0.0 and (G.gpu_unpack(Xq, K)[2] == -8).all()
    Xq1, sx1, zx1 = G.gpu_rsq_asym(G.to_dev(X[:1]), None, None)
    assert torch.equal(Xq1, Xq[:1]) and torch.equal(sx1, sx[:1]) and torch.equal(zx1, zx[:1])


@pytest.mark.parametrize("N,K", [(16, 128), (3072, 1024), (1024, 4096), (48, 768)])
def test_weight_code_sums(N, K):
    rng = np.random.default_rng(N + K)
    qw = rng.integers(-8, 8, (N, K)).astype(np.int8)
    qw[0] = -8
    qw[N - 1] = 7
    got = G.gpu_code_sums(G.gpu_pack(qw), N, K).cpu().numpy()
    assert np.array_equal(got, oracle.weight_code_sums(qw).astype(np.float32))


def _run_gemm_asym(u, zp, qw, dx, dw, bias_bits):
    M, K = u.shape
    N = qw.shape[0]
    Xq = G.gpu_pack((u.astype(np.int16) - 8).astype(np.int8))
    Wq = G.gpu_pack(qw)
    Y = torch.empty(M, N, dtype=torch.bfloat16, device=G.DEV)
    G.q.qvggt_w4a4_gemm_asym(Xq, G.to_dev(dx.astype(np.float32)), G.to_dev(zp.astype(np.float32)), Wq,
                             G.to_dev(dw.astype(np.float32)), G.gpu_code_sums(Wq, N, K), G.to_dev(bias_bits), M, N, K, Y)
    return G.bf16_bits(Y)


@pytest.mark.parametrize("M,N,K", [(70, 48, 128), (300, 272, 1024), (5000, 4096, 128)])
def test_gemm_asym_small_integers_are_exact(M, N, K):
    """Unit scales, no bias and effective codes u - zp in {-1, 0, 1}, mostly 0: the corrected sum stays below 256 in magnitude
    and is a bf16 value, while the stored codes u - 8, the accumulator and the correction term are large and cancel."""
    rng = np.random.default_rng(M + N + K)
    zp = rng.integers(0, 16, M)
    d = rng.choice([-1, 0, 1], size=(M, K), p=[0.01, 0.98, 0.01])
    u = np.clip(zp[:, None] + d, 0, 15).astype(np.uint8)
    qw = rng.integers(-8, 8, (N, K)).astype(np.int8)
    want = oracle.int_gemm_asym(u, zp, qw)
    assert np.abs(want).max() <= 256
    Y = _run_gemm_asym(u, zp, qw, np.ones(M), np.ones(N), None)
    assert np.array_equal(Y, oracle.bf16_from_f64(want.astype(np.float64)))


@pytest.mark.parametrize("M,N,K", [(64, 128, 128), (1374, 3072, 1024), (257, 1024, 4096), (4200, 4096, 1024)])
def test_gemm_asym_against_the_oracle_on_identical_codes(M, N, K):
    """Random codes and zero points, the oracle's integer sum with the same fp32-stored scales applied in double; the largest
    shape runs the 256 x 256 kernel and the tail kernel and is compared on sampled token rows (rows are independent)."""
    rng = np.random.default_rng(M * 3 + N)
    u = rng.integers(0, 16, (M, K)).astype(np.uint8)
    zp = rng.integers(0, 16, M)
    qw = rng.integers(-8, 8, (N, K)).astype(np.int8)
    dx = np.exp(rng.uniform(-3, 1, M)).astype(np.float32)
    dw = np.exp(rng.uniform(-5, -2, N)).astype(np.float32)
    bias_bits = synth.f32_to_bf16_bits((rng.standard_normal(N) * 0.02).astype(np.float32))
    Y = _run_gemm_asym(u, zp, qw, dx, dw, bias_bits)
    rows = np.arange(M) if M <= 1400 else np.unique(np.concatenate([np.arange(0, 260), np.arange(M - 140, M), rng.integers(0, M, 200)]))
    acc = oracle.int_gemm_asym(u[rows], zp[rows], qw)
    y = acc.astype(np.float64) * dx[rows].astype(np.float64)[:, None] * dw.astype(np.float64)[None, :] + oracle.to_f64(bias_bits)[None, :]
    Yo = oracle.bf16_from_f64(y)
    ulp_off = np.abs(Y[rows].astype(np.int32) - Yo.astype(np.int32))
    assert G.rel_fro(Y[rows], Yo) <= 1e-3
    assert ulp_off.max() <= 1 and (ulp_off != 0).mean() < 5e-3


def test_asym_layer_end_to_end():
    """Kernel 1 (asymmetric) -> code sums -> GEMM against the oracle's asymmetric layer on post-GELU-like rows."""
    K, N, rows = 4096, 1024, 600
    rng = np.random.default_rng(31)
    X = _rows(rows, K, 32, "bf16", True)
    W = rng.standard_normal((N, K)).astype(np.float32) * 0.03
    bias = synth.f32_to_bf16_bits(rng.normal(0, 0.1, N).astype(np.float32))
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    act = oracle.rotated_col_absmax(X, pre_signs=signs)
    prep_o = oracle.prepare_weights(W, act, pre_signs=signs)
    want = oracle.linear_asym(X, prep_o, bias, pre_signs=signs)[0]
    prep = G.gpu_prep(W, X, signs)
    Xq, sx, zx = G.gpu_rsq_asym(G.to_dev(X), prep["signs"], prep["inv"])
    Y = torch.empty(rows, N, dtype=torch.bfloat16, device=G.DEV)
    G.q.qvggt_w4a4_gemm_asym(Xq, sx, zx, prep["Wq"], prep["sw"], G.gpu_code_sums(prep["Wq"], N, K), G.to_dev(bias), rows, N, K, Y)
    assert G.rel_fro(G.bf16_bits(Y), want) <= G.Y_REL_FRO
