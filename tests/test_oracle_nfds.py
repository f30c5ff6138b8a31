"""Pins of the oracle's sampling arithmetic (Sec. 3.3) against closed forms, invariances and hand-worked cases."""
import numpy as np
import pytest

from oracle import nfds


def test_moments_closed_forms():
    assert nfds.layer_moments(np.full((7, 9), 3.25)) == (3.25, 0.0)
    n, step, start = 1001, 0.5, -3.0
    m, s = nfds.layer_moments(start + step * np.arange(n))
    assert m == pytest.approx(start + step * (n - 1) / 2, rel=1e-14)
    assert s == pytest.approx(step ** 2 * (n * n - 1) / 12, rel=1e-13)          # population variance of an arithmetic progression
    # population, not sample, variance: two points at +-1
    assert nfds.layer_moments([1.0, -1.0]) == (0.0, 1.0)
    # shift and scale laws
    rng = np.random.default_rng(0)
    x = rng.standard_normal(5000)
    m0, s0 = nfds.layer_moments(x)
    m1, s1 = nfds.layer_moments(3.0 * x + 7.0)
    assert m1 == pytest.approx(3 * m0 + 7, rel=1e-12) and s1 == pytest.approx(9 * s0, rel=1e-12)


def test_scores_two_samples_and_invariance():
    L = 5
    rng = np.random.default_rng(1)
    # two samples: every z-score is +-1 (eps -> 0), so both scores are sqrt(2 L)
    m, s = rng.standard_normal((2, L)), rng.uniform(1, 2, (2, L))
    sc = nfds.noise_scores(m, s, 0.0)
    assert np.allclose(sc, np.sqrt(2 * L), rtol=1e-12)
    # z-scores do not change under a per-layer affine map of the moments (eps = 0)
    m, s = rng.standard_normal((40, L)), rng.uniform(1, 2, (40, L))
    a, b = rng.uniform(0.5, 2, L), rng.standard_normal(L)
    assert np.allclose(nfds.noise_scores(m, s, 0.0), nfds.noise_scores(m * a + b, s * a, 0.0), rtol=1e-10)
    # sum of squared z-scores over the pool is D per statistic: sum_i score_i^2 = 2 L D
    assert np.sum(nfds.noise_scores(m, s, 0.0) ** 2) == pytest.approx(2 * L * 40, rel=1e-12)
    # a planted outlier has the highest score; eps only shrinks the scores
    m[17] += 25.0
    sc = nfds.noise_scores(m, s, 1e-6)
    assert sc.argmax() == 17 and np.all(sc <= nfds.noise_scores(m, s, 0.0) + 1e-12)


def test_score_hand_worked():
    # one layer, three samples: m = 0, 3, 6 -> mu 3, sigma sqrt(6); s = 1, 1, 4 -> nu 2, tau sqrt(2)
    sc = nfds.noise_scores([[0.0], [3.0], [6.0]], [[1.0], [1.0], [4.0]], 0.0)
    want = [np.sqrt(9 / 6 + 1 / 2), np.sqrt(0 + 1 / 2), np.sqrt(9 / 6 + 4 / 2)]
    assert np.allclose(sc, want, rtol=1e-14)


def test_keep_lowest():
    sc = np.array([5.0, 1.0, 3.0, 1.0, 9.0, 2.0, 7.0, 4.0, 6.0, 8.0])
    assert nfds.keep_lowest(sc, 0.2).tolist() == [False, True, False, True] + [False] * 6
    assert nfds.keep_lowest(sc, 0.3).sum() == 3 and nfds.keep_lowest(sc, 0.3)[5]
    assert nfds.keep_lowest(sc, 0.19).sum() == 1 and nfds.keep_lowest(sc, 0.19)[1]      # tie: the lower index wins
    assert nfds.keep_lowest(sc, 1.0).all() and not nfds.keep_lowest(sc, 0.0).any()


def test_frame_correlation_closed_forms():
    d = 64
    e1, e2 = np.eye(d)[0], np.eye(d)[1]
    thetas = [0.0, 0.3, np.pi / 2, 2.0, np.pi]
    frames = [e1] + [3.7 * (np.cos(t) * e1 + np.sin(t) * e2) for t in thetas]
    c = nfds.frame_correlation(np.stack(frames), len(frames))
    assert np.allclose(c, np.cos(thetas), atol=1e-15)
    # scale of any frame does not matter; frame vectors are whole frames (tokens x channels flattened)
    rng = np.random.default_rng(2)
    A = rng.standard_normal((4 * 6, 8))                     # f = 4 frames of s = 6 tokens, d = 8
    c0 = nfds.frame_correlation(A, 4)
    B = A.copy()
    B[6:12] *= 5.0
    B[:6] *= 0.1
    assert np.allclose(nfds.frame_correlation(B, 4), c0, rtol=1e-12)
    flat = A.reshape(4, 48)
    assert c0[1] == pytest.approx(sum(flat[0][k] * flat[2][k] for k in range(48))
                                  / np.sqrt(sum(v * v for v in flat[0]) * sum(v * v for v in flat[2])), rel=1e-12)


def test_kmeans_step_hand_worked():
    pts = np.array([[0.0], [1.0], [10.0], [11.0], [5.0]])
    labels, new = nfds.kmeans_step(pts, np.array([[0.0], [10.0]]))
    assert labels.tolist() == [0, 0, 1, 1, 0]               # 5 is at distance 5 from both: the lower index wins
    assert new.ravel().tolist() == [2.0, 10.5]
    labels, new = nfds.kmeans_step(pts, np.array([[0.0], [10.0], [100.0]]))
    assert new[2, 0] == 100.0 and 2 not in labels           # an empty cluster keeps its centre
    # a fixed point of the iteration stays fixed, and the within-cluster sum of squares never increases
    rng = np.random.default_rng(3)
    c = rng.standard_normal((60, 5))
    cen = c[:4].copy()
    prev = None
    for _ in range(12):
        lab, cen2 = nfds.kmeans_step(c, cen)
        cost = sum(((c[i] - cen2[lab[i]]) ** 2).sum() for i in range(60))
        assert prev is None or cost <= prev * (1 + 1e-12)
        prev, cen = cost, cen2
    lab2, cen3 = nfds.kmeans_step(c, cen)
    if np.array_equal(lab, lab2):
        assert np.allclose(cen3, cen, rtol=1e-12)
