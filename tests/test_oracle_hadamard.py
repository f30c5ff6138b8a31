"""Pins of the oracle's Hadamard matrix and rotation (paper Sec. 3.2, Pre-Global-Rotation)."""
import os

import numpy as np
import pytest
import scipy.linalg

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_h2_is_the_printed_matrix():
    rows = [l.split() for l in open(os.path.join(GOLD, "hadamard_h2.txt")) if l.strip() and l[0] != "#"]
    printed = np.array(rows, dtype=np.int64)
    assert np.array_equal(oracle.hadamard(2).astype(np.int64), printed)


@pytest.mark.parametrize("K", [1, 2, 4, 8, 64, 128, 512, 1024])
def test_hht_is_k_identity_in_integers(K):
    H = oracle.hadamard(K).astype(np.int32)
    assert set(np.unique(H)) <= {-1, 1}
    assert np.array_equal(H @ H.T, K * np.eye(K, dtype=np.int32))


def test_hht_is_k_identity_4096():
    H = oracle.hadamard(4096).astype(np.float32)        # exact: all partial sums are integers < 2^24
    G = H @ H.T
    assert np.array_equal(G, 4096 * np.eye(4096, dtype=np.float32))


@pytest.mark.parametrize("K", [2, 16, 128, 1024, 4096])
def test_recursion_equals_closed_form_and_library(K):
    Hr = oracle.hadamard(K, "recursive")
    Hp = oracle.hadamard(K, "popcount")
    assert np.array_equal(Hr, Hp)
    assert np.array_equal(Hr, Hr.T)
    assert np.all(Hr[0] == 1) and np.all(Hr[:, 0] == 1)
    if K <= 1024:
        assert np.array_equal(Hr.astype(np.int64), scipy.linalg.hadamard(K).astype(np.int64))


def test_kronecker_structure():
    # H_2n = H_2 (x) H_n, as the recursion in the paper states it
    for n in (1, 4, 32):
        assert np.array_equal(np.kron(oracle.hadamard(2), oracle.hadamard(n)), oracle.hadamard(2 * n))


@pytest.mark.parametrize("K", [64, 128, 1024])
def test_rotation_matches_dense_library_product(K):
    rng = np.random.default_rng(K)
    X = rng.standard_normal((7, K))
    ref = X @ scipy.linalg.hadamard(K).astype(np.float64) / np.sqrt(K)
    got = oracle.rotate(X)
    assert np.allclose(got, ref, rtol=0, atol=1e-12 * np.abs(ref).max())


def test_rotation_sign_conventions():
    K = 128
    rng = np.random.default_rng(1)
    X = rng.standard_normal((5, K))
    u = rng.integers(0, 2, K).astype(np.int8) * 2 - 1
    v = rng.integers(0, 2, K).astype(np.int8) * 2 - 1
    Hn = scipy.linalg.hadamard(K) / np.sqrt(K)
    # pre-rotation signs act on input channels, post-rotation signs on output channels
    assert np.allclose(oracle.rotate(X, pre_signs=u), (X * u) @ Hn, atol=1e-12)
    assert np.allclose(oracle.rotate(X, post_signs=v), (X @ Hn) * v, atol=1e-12)
    assert np.allclose(oracle.rotate(X, u, v), ((X * u) @ Hn) * v, atol=1e-12)
    # a random-sign Hadamard is still orthogonal: H^T H = I
    Hfull = oracle.rotate(np.eye(K), u, v)
    assert np.allclose(Hfull.T @ Hfull, np.eye(K), atol=1e-12)
    # and not symmetric any more, so a transposed use would show
    assert not np.allclose(Hfull, Hfull.T)


@pytest.mark.parametrize("K", [128, 1024])
def test_rotation_invariance_of_the_product(K):
    # X W^T = (X H)(W H)^T
    rng = np.random.default_rng(2)
    X = rng.standard_normal((9, K)) * rng.choice([1.0, 50.0], size=K)
    W = rng.standard_normal((11, K)) * 0.02
    u = rng.integers(0, 2, K).astype(np.int8) * 2 - 1
    ref = X @ W.T
    for pre, post in ((None, None), (u, None), (None, u), (u, u[::-1].copy())):
        got = oracle.rotate(X, pre, post) @ oracle.rotate(W, pre, post).T
        assert np.abs(got - ref).max() <= 1e-10 * np.abs(ref).max()


def test_norm_preserved_and_one_hot_dispersed():
    K = 1024
    rng = np.random.default_rng(3)
    X = rng.standard_normal((4, K))
    Xr = oracle.rotate(X)
    assert np.allclose(np.linalg.norm(Xr, axis=1), np.linalg.norm(X, axis=1), rtol=1e-12)
    e = np.zeros((1, K))
    e[0, 37] = 3.0
    y = oracle.rotate(e)
    assert np.allclose(np.abs(y), 3.0 / np.sqrt(K), rtol=1e-14)       # an outlier spreads evenly
    assert np.array_equal(np.sign(y[0]).astype(np.int8), oracle.hadamard(K)[37])


# ----------------------------------------------------------------- sizes 2^n m (Sec. 3.2: H_d = H_{2^n} (x) H_m)
@pytest.mark.parametrize("m", [12, 20, 28])
def test_paley_matrices_are_hadamard(m):
    H = oracle.hadamard_paley(m).astype(np.int64)
    assert set(np.unique(H)) == {-1, 1}
    assert np.array_equal(H @ H.T, m * np.eye(m, dtype=np.int64))
    assert np.array_equal(H.T @ H, m * np.eye(m, dtype=np.int64))
    # any two distinct rows agree in exactly m / 2 places
    for i in range(m):
        for j in range(i + 1, m):
            assert int((H[i] == H[j]).sum()) == m // 2


def test_paley_type_one_structure_from_brute_force_squares():
    """q = 11, 19: H - I is skew with the quadratic character of GF(q) in its core, the squares found by enumeration."""
    for m in (12, 20):
        q = m - 1
        squares = {(k * k) % q for k in range(1, q)}
        H = oracle.hadamard_paley(m).astype(int)
        S = H - np.eye(m, dtype=int)
        assert np.array_equal(S, -S.T)
        assert S[0, 1:].tolist() == [1] * q and S[1:, 0].tolist() == [-1] * q
        for i in range(q):
            for j in range(q):
                want = 0 if i == j else (1 if (i - j) % q in squares else -1)
                assert S[1 + i, 1 + j] == want


def test_paley_type_two_structure_from_brute_force_squares():
    q = 13
    squares = {(k * k) % q for k in range(1, q)}
    H = oracle.hadamard_paley(28).astype(int)
    assert np.array_equal(H, H.T)                               # q = 1 mod 4: symmetric
    for i in range(14):
        for j in range(14):
            blk = H[2 * i:2 * i + 2, 2 * j:2 * j + 2]
            if i == j:
                assert blk.tolist() == [[1, -1], [-1, -1]]
            else:
                c = 1 if (i == 0 or j == 0 or ((i - 1) - (j - 1)) % q in squares) else -1
                assert blk.tolist() == [[c, c], [c, -c]]


@pytest.mark.parametrize("K", [768, 1280, 1792, 1536])
def test_general_size_is_the_kronecker_product(K):
    m = {3: 12, 5: 20, 7: 28}[K // (K & -K)]
    n2 = K // m
    H = oracle.hadamard_general(K)
    assert np.array_equal(H, np.kron(oracle.hadamard(n2), oracle.hadamard_paley(m)))
    Hl = H.astype(np.int64)
    assert np.array_equal(Hl @ Hl.T, K * np.eye(K, dtype=np.int64))


@pytest.mark.parametrize("K", [768, 2560])
def test_rotation_general_size_is_orthonormal_and_dense(K):
    rng = np.random.default_rng(K)
    X = rng.standard_normal((6, K))
    W = rng.standard_normal((5, K))
    signs = (rng.integers(0, 2, K) * 2 - 1).astype(np.int8)
    Xr, Wr = oracle.rotate(X, pre_signs=signs), oracle.rotate(W, pre_signs=signs)
    assert np.allclose(Xr @ Wr.T, X @ W.T, rtol=0, atol=1e-10 * np.abs(X @ W.T).max())
    assert np.allclose((Xr ** 2).sum(axis=1), (X ** 2).sum(axis=1), rtol=1e-12)
    dense = (X * signs) @ oracle.hadamard_general(K).astype(np.float64) / np.sqrt(K)
    assert np.allclose(Xr, dense, rtol=0, atol=1e-12 * np.abs(dense).max())
    # one-hot input: the row of the matrix, all entries +-1 / sqrt(K)
    e = np.zeros((1, K)); e[0, 5] = 1.0
    assert np.allclose(np.abs(oracle.rotate(e)), 1.0 / np.sqrt(K), rtol=1e-14)


def test_sizes_without_a_construction_are_refused():
    for K in (1000, 1408, 2304, 96 * 11):
        with pytest.raises(oracle.OracleError):
            oracle.rotate(np.zeros((1, K)))
