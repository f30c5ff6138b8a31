"""GPU parity of the calibration-set arithmetic (Sec. 3.3) against the float64 oracle, through the C ABI.
Tolerances: the kernels sum in double and return floats, so results agree with the oracle to float rounding
(relative 1e-6 here); labels, masks and counts are integers and must be identical."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2509_21302_amd as q
from oracle import nfds
from tests import gpu_util as G

pytestmark = pytest.mark.gpu
RTOL = 1e-6


def _ws(rows, count, t):
    code = q.QVGGT_BF16 if t.dtype == torch.bfloat16 else q.QVGGT_F32
    return torch.empty(q.qvggt_nfds_workspace_bytes(rows, count, code), dtype=torch.uint8, device=G.DEV)


@pytest.mark.parametrize("rows,count,dtype", [(1, 8, "bf16"), (3, 4096, "bf16"), (5, 100000, "f32"), (2, 1374 * 1024, "bf16"),
                                              (37, 24, "f32"), (1, 1374 * 1024 * 20, "bf16")])
def test_moments(rows, count, dtype):
    rng = np.random.default_rng(rows * 31 + count % 1000)
    x = (rng.standard_t(3, (rows, count)) * rng.uniform(0.1, 3, (rows, 1)) + rng.uniform(-20, 20, (rows, 1))).astype(np.float32)
    x[0, : min(5, count)] *= 40                                  # a few salient values, as the special tokens produce
    X = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    Xd = G.to_dev(X)
    mean = torch.empty(rows, dtype=torch.float32, device=G.DEV)
    var = torch.empty(rows, dtype=torch.float32, device=G.DEV)
    q.qvggt_nfds_moments(Xd, mean, var, _ws(rows, count, Xd))
    Xo = oracle.to_f64(X)
    for r in range(rows):
        m, s = nfds.layer_moments(Xo[r])
        assert mean[r].item() == pytest.approx(m, rel=RTOL, abs=1e-7 * np.sqrt(s)), (r, "mean")
        assert var[r].item() == pytest.approx(s, rel=RTOL), (r, "var")


def test_moments_large_mean_small_spread():
    """E[x^2] - E[x]^2 in double: a mean 1e3 times the standard deviation must not hurt the variance."""
    rng = np.random.default_rng(5)
    x = (1000.0 + rng.standard_normal((2, 1 << 18))).astype(np.float32)
    Xd = G.to_dev(x)
    mean = torch.empty(2, dtype=torch.float32, device=G.DEV)
    var = torch.empty(2, dtype=torch.float32, device=G.DEV)
    q.qvggt_nfds_moments(Xd, mean, var, _ws(2, 1 << 18, Xd))
    for r in range(2):
        m, s = nfds.layer_moments(x[r])
        assert var[r].item() == pytest.approx(s, rel=1e-5) and mean[r].item() == pytest.approx(m, rel=RTOL)


@pytest.mark.parametrize("samples,frames,tokens,d,dtype", [(1, 2, 1, 8, "bf16"), (3, 5, 37, 64, "f32"), (2, 20, 1374, 1024, "bf16"),
                                                           (4, 3, 200, 256, "bf16")])
def test_frame_correlation(samples, frames, tokens, d, dtype):
    rng = np.random.default_rng(samples + frames)
    base = rng.standard_normal((samples, 1, tokens * d))
    mix = rng.uniform(-1, 1, (samples, frames, 1))
    x = (mix * base + np.sqrt(1 - mix ** 2) * rng.standard_normal((samples, frames, tokens * d))).astype(np.float32)
    X = synth.f32_to_bf16_bits(x) if dtype == "bf16" else x
    Xd = G.to_dev(X)
    c = torch.empty(samples, frames - 1, dtype=torch.float32, device=G.DEV)
    q.qvggt_nfds_frame_correlation(Xd, c, _ws(samples * frames, tokens * d, Xd))
    got = c.cpu().numpy()
    Xo = oracle.to_f64(X)
    for i in range(samples):
        want = nfds.frame_correlation(Xo[i].reshape(frames * tokens, d), frames)
        assert np.allclose(got[i], want, rtol=RTOL, atol=2e-7), i


def test_frame_correlation_on_synthetic_vggt_frames():
    """The recipe's fc1 input (100 frames of 1374 x 1024, special tokens salient) as one sample's feature map."""
    s = synth.layer_spec(3, "fc1")
    X = synth.make_activation_frames(s)
    frames = s.frames
    Xd = G.to_dev(X).view(1, frames, -1)
    c = torch.empty(1, frames - 1, dtype=torch.float32, device=G.DEV)
    q.qvggt_nfds_frame_correlation(Xd, c, _ws(frames, Xd.shape[2], Xd))
    want = nfds.frame_correlation(oracle.to_f64(X), frames)
    assert np.allclose(c.cpu().numpy()[0], want, rtol=RTOL, atol=2e-7)


@pytest.mark.parametrize("D,L", [(2, 1), (40, 7), (400, 48), (1000, 300)])
def test_scores_and_filter(D, L):
    rng = np.random.default_rng(D + L)
    m = rng.standard_normal((D, L)).astype(np.float32)
    s = rng.uniform(0.5, 2, (D, L)).astype(np.float32)
    m[rng.integers(0, D, max(1, D // 20))] += 9.0
    md, sd = G.to_dev(m), G.to_dev(s)
    score = torch.empty(D, dtype=torch.float32, device=G.DEV)
    q.qvggt_nfds_scores(md, sd, 1e-6, score)
    want = nfds.noise_scores(m, s, 1e-6)
    assert np.allclose(score.cpu().numpy(), want, rtol=RTOL)
    # the filter is an integer decision on the scores: both sides rank the SAME float scores
    sc32 = score.cpu().numpy()
    for p in (0.0, 0.2, 0.5, 0.7, 1.0):
        keep = torch.empty(D, dtype=torch.uint8, device=G.DEV)
        q.qvggt_nfds_keep_lowest(score, p, keep)
        assert np.array_equal(keep.cpu().numpy().astype(bool), nfds.keep_lowest(sc32, p)), p


def test_filter_ties_by_index():
    sc = np.array([5.0, 1.0, 3.0, 1.0, 9.0, 2.0, 7.0, 4.0, 6.0, 8.0], dtype=np.float32)
    for p in (0.19, 0.2, 0.3):
        keep = torch.empty(10, dtype=torch.uint8, device=G.DEV)
        q.qvggt_nfds_keep_lowest(G.to_dev(sc), p, keep)
        assert np.array_equal(keep.cpu().numpy().astype(bool), nfds.keep_lowest(sc, p))


@pytest.mark.parametrize("n,dim,K", [(5, 1, 2), (80, 19, 8), (400, 99, 8), (3000, 7, 64)])
def test_kmeans_iterations(n, dim, K):
    rng = np.random.default_rng(n)
    if n == 5:
        c = np.array([[0.0], [1.0], [10.0], [11.0], [5.0]], dtype=np.float32)      # 5 is a tie between the two centres
        cen = np.array([[0.0], [10.0]], dtype=np.float32)
    else:
        blobs = rng.uniform(-1, 1, (K, dim))
        c = (blobs[rng.integers(0, K, n)] + 0.15 * rng.standard_normal((n, dim))).astype(np.float32)
        cen = c[:K].copy()
    cd = G.to_dev(c)
    a, b = G.to_dev(cen), torch.empty(K, dim, dtype=torch.float32, device=G.DEV)
    labels = torch.empty(n, dtype=torch.int32, device=G.DEV)
    cen_o = cen.astype(np.float64)
    for it in range(6):
        q.qvggt_nfds_kmeans_step(cd, a, b, labels)
        # the oracle starts every iteration from the centres the GPU iteration started from (floats), so a last-bit
        # difference in a centre cannot grow into a different label later
        lab_o, new_o = nfds.kmeans_step(c, a.cpu().numpy())
        assert np.array_equal(labels.cpu().numpy(), lab_o), it
        assert np.allclose(b.cpu().numpy(), new_o, rtol=RTOL, atol=1e-7), it
        a, b = b, a
