"""CPU oracle of the arithmetic of Noise-Filtered Diverse Sampling (paper Sec. 3.3, the calibration-set
construction).  Test infrastructure only: plain numpy in float64, one function per equation, no blocking.

Readings where the paper leaves a choice (also listed in the design notes):
  * var(.) is the population variance (divide by the number of elements);
  * "keep the lowest p% scores" keeps the floor(p * |D|) samples of lowest score, ties broken by index;
  * K-Means is Lloyd's iteration from centres the caller supplies; a point on equal distance from two
    centres goes to the one with the lower index; a centre that loses all its points stays where it is.
"""
from __future__ import annotations

import numpy as np


def layer_moments(A) -> tuple:
    """m = mean(layer_j(x_i)), s = var(layer_j(x_i)) over every element of one activation tensor
    (Sec. 3.3, first equation of the noise filter)."""
    a = np.asarray(A, dtype=np.float64).ravel()
    m = a.sum() / a.size
    s = ((a - m) ** 2).sum() / a.size
    return float(m), float(s)


def noise_scores(m, s, eps: float) -> np.ndarray:
    """score(x_i) from the per-sample, per-layer moments m[i, j], s[i, j] (Sec. 3.3, second equation):
    z-scores of m and s against their means and standard deviations over the candidate pool, root of the
    sum of squares over the layers."""
    m = np.asarray(m, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    D = m.shape[0]
    mu = m.sum(axis=0) / D
    sigma = np.sqrt(((m - mu) ** 2).sum(axis=0) / D + eps)
    nu = s.sum(axis=0) / D
    tau = np.sqrt(((s - nu) ** 2).sum(axis=0) / D + eps)
    return np.sqrt((((m - mu) / sigma) ** 2).sum(axis=1) + (((s - nu) / tau) ** 2).sum(axis=1))


def keep_lowest(score, p: float) -> np.ndarray:
    """D_filtered (Sec. 3.3, Eq. "filter"): boolean mask of the floor(p * |D|) samples with the lowest
    score (threshold T at that percentile); equal scores are ordered by index."""
    score = np.asarray(score, dtype=np.float64)
    n_keep = int(np.floor(p * score.size))
    order = sorted(range(score.size), key=lambda i: (score[i], i))
    keep = np.zeros(score.size, dtype=bool)
    keep[order[:n_keep]] = True
    return keep


def frame_correlation(A, f: int) -> np.ndarray:
    """Frame-aware correlation vector c in R^(f-1) (Sec. 3.3, third equation): the feature [n, d] of one
    sample, n = s * f tokens frame after frame, is cut into f frame vectors of s * d values; c_t is the cosine
    between frame 0 and frame t."""
    a = np.asarray(A, dtype=np.float64).reshape(f, -1)
    out = np.empty(f - 1, dtype=np.float64)
    n0 = np.sqrt((a[0] * a[0]).sum())
    for t in range(1, f):
        out[t - 1] = (a[0] * a[t]).sum() / (n0 * np.sqrt((a[t] * a[t]).sum()))
    return out


def kmeans_step(c, centres):
    """One Lloyd iteration on the correlation vectors c[i, :] (Sec. 3.3, Eq. "cluster"): label = nearest
    centre in squared Euclidean distance, new centre = mean of its points.  Returns (labels, new centres)."""
    c = np.asarray(c, dtype=np.float64)
    centres = np.asarray(centres, dtype=np.float64)
    n, K = c.shape[0], centres.shape[0]
    labels = np.empty(n, dtype=np.int32)
    for i in range(n):
        best, best_d = 0, None
        for k in range(K):
            d = float(((c[i] - centres[k]) ** 2).sum())
            if best_d is None or d < best_d:
                best, best_d = k, d
        labels[i] = best
    new = centres.copy()
    for k in range(K):
        pts = c[labels == k]
        if len(pts):
            new[k] = pts.sum(axis=0) / len(pts)
    return labels, new
