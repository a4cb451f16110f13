"""Pins for the oracle at widths d = 12 * 2^m  (CPU only).

The paper trains widths 768 and 1536 (Table 2) and does not say which matrix replaces the Sylvester
matrix there.  This library's reading: H_raw = P12 (x) S_{2^m}, P12 the symmetric order-12 Hadamard
matrix of Paley's second construction over GF(5), normalised to a constant first row and column.
What is pinned here is what Sec. 4.1 requires of H -- entries +-1/sqrt(d), orthogonal, symmetric --
plus the Kronecker structure, each checked by brute force or against a library routine, and the
backward formulas by finite differences.
"""
import numpy as np
import pytest
import scipy.linalg

import oracle

RNG = np.random.default_rng(2468)
WIDTHS = [12, 24, 48, 96, 192, 768]


def _paley2_order12_independent():
    """Order-12 Hadamard matrix built a second way, with numpy only: squares mod 5 -> Jacobsthal
    matrix -> bordered conference matrix C -> C (x) [[1,1],[1,-1]] + I (x) [[1,-1],[-1,-1]]."""
    squares = {(a * a) % 5 for a in range(1, 5)}
    Q = np.zeros((5, 5), dtype=np.int64)
    for i in range(5):
        for j in range(5):
            if i != j:
                Q[i, j] = 1 if (i - j) % 5 in squares else -1
    C = np.zeros((6, 6), dtype=np.int64)
    C[0, 1:] = 1
    C[1:, 0] = 1
    C[1:, 1:] = Q
    H = np.kron(C, np.array([[1, 1], [1, -1]])) + np.kron(np.eye(6, dtype=np.int64),
                                                           np.array([[1, -1], [-1, -1]]))
    s = H[0].copy()                       # negate rows/columns where row 0 is -1
    return s[:, None] * H * s[None, :]


def test_h12_is_a_normalised_symmetric_hadamard_matrix():
    P = oracle.h12()
    assert P.shape == (12, 12) and set(np.unique(P)) == {-1, 1}
    assert np.array_equal(P @ P.T, 12 * np.eye(12, dtype=np.int64))      # rows orthogonal, exactly
    assert np.array_equal(P, P.T)
    assert np.all(P[0] == 1) and np.all(P[:, 0] == 1)
    # every other row is balanced (orthogonal to the all-ones row)
    assert np.all(P[1:].sum(axis=1) == 0)


def test_h12_equals_independent_paley_construction():
    assert np.array_equal(oracle.h12(), _paley2_order12_independent())


@pytest.mark.parametrize("d", [12, 24, 96, 192])
def test_sign_matrix_is_kron_of_h12_and_scipy_sylvester(d):
    m = d // 12
    expect = np.kron(oracle.h12(), scipy.linalg.hadamard(m).astype(np.int64) if m > 1
                     else np.ones((1, 1), dtype=np.int64))
    H = oracle.hadamard_matrix(d)
    assert np.array_equal(H, expect)
    assert np.array_equal(H @ H.T, d * np.eye(d, dtype=np.int64))
    assert np.array_equal(H, H.T)
    assert np.all(H[0] == 1)


@pytest.mark.parametrize("d", [12, 48, 192])
@pytest.mark.parametrize("method", ["matrix", "fast"])
def test_transform_equals_numpy_matmul_with_kron_matrix(d, method):
    m = d // 12
    S = scipy.linalg.hadamard(m).astype(np.float64) if m > 1 else np.ones((1, 1))
    H = np.kron(_paley2_order12_independent().astype(np.float64), S) / np.sqrt(d)
    x = RNG.standard_normal((5, d))
    assert np.allclose(oracle.transform(x, method), x @ H.T, rtol=0, atol=1e-12 * np.sqrt(d))


@pytest.mark.parametrize("d", WIDTHS + [1536])
def test_fast_equals_matrix(d):
    x = RNG.standard_normal((3, d))
    a, b = oracle.transform(x, "matrix"), oracle.transform(x, "fast")
    assert np.max(np.abs(a - b)) <= 1e-12 * np.max(np.abs(a))


@pytest.mark.parametrize("d", WIDTHS + [1536, 3072, 12288])
def test_involution_and_norm_preservation(d):
    x = RNG.standard_normal((4, d))
    z = oracle.transform(x, "fast")
    assert np.allclose(oracle.transform(z, "fast"), x, rtol=0, atol=1e-12 * np.sqrt(d))
    assert np.allclose(np.linalg.norm(z, axis=1), np.linalg.norm(x, axis=1), rtol=1e-12)


@pytest.mark.parametrize("d", [12, 96, 768])
def test_unit_vectors_constants_blocks(d):
    m = d // 12
    # H 1 = sqrt(d) e_0 (first row and column of H_raw are all +1, every other row is balanced)
    z = oracle.transform(np.ones((1, d)), "fast")[0]
    expect = np.zeros(d)
    expect[0] = np.sqrt(d)
    assert np.allclose(z, expect, atol=1e-12 * np.sqrt(d))
    # H e_k is column k: entries +-1/sqrt(d) with the Kronecker sign
    for k in (0, 1, m - 1, m, 5 * m + 3 % m, d - 1):
        e = np.zeros((1, d))
        e[0, k] = 1.0
        col = oracle.transform(e, "fast")[0]
        assert np.allclose(np.abs(col), 1 / np.sqrt(d), rtol=1e-14)
        j = np.arange(d)
        sylv = (-1.0) ** np.array([bin((jj % m) & (k % m)).count("1") for jj in j])
        assert np.array_equal(np.sign(col), oracle.h12()[j // m, k // m] * sylv)
    # an input confined to one block of 2^m features: each output block is +- the block's own
    # Sylvester transform, scaled by 1/sqrt(12)
    if m > 1:
        x = np.zeros((1, d))
        blk = RNG.standard_normal(m)
        x[0, 3 * m:4 * m] = blk
        z = oracle.transform(x, "fast")[0].reshape(12, m)
        inner = oracle.transform(blk[None, :], "fast")[0] / np.sqrt(12)
        for a in range(12):
            assert np.allclose(z[a], oracle.h12()[a, 3] * inner, atol=1e-13 * np.sqrt(d))


def test_affine_and_residual_special_cases():
    d = 96
    x = RNG.standard_normal((3, d))
    alpha, beta = RNG.uniform(0.5, 1.5, d), RNG.standard_normal(d)
    z = oracle.transform(x, "fast")
    assert np.array_equal(oracle.forward(x, np.ones(d), np.zeros(d)), z)
    assert np.array_equal(oracle.forward(np.zeros((2, d)), alpha, beta), np.tile(beta, (2, 1)))
    assert np.allclose(oracle.forward(x, alpha, beta), alpha * z + beta, rtol=0, atol=1e-15)
    resid = RNG.standard_normal((3, d))
    assert np.allclose(oracle.forward_residual(x, alpha, beta, resid), resid + alpha * z + beta,
                       rtol=0, atol=1e-14)


def _loss(x, alpha, beta, dy, method):
    return float(np.sum(dy * oracle.forward(x, alpha, beta, method)))


@pytest.mark.parametrize("method", ["matrix", "fast"])
@pytest.mark.parametrize("N,d", [(2, 12), (3, 24)])
def test_backward_matches_finite_differences(method, N, d):
    x, dy = RNG.standard_normal((N, d)), RNG.standard_normal((N, d))
    alpha, beta = RNG.uniform(0.5, 1.5, d), 0.02 * RNG.standard_normal(d)
    dx, dalpha, dbeta = oracle.backward(dy, x, alpha, method)
    h = 1e-5

    def fd(arr, idx):
        save = arr[idx]
        arr[idx] = save + h
        up = _loss(x, alpha, beta, dy, method)
        arr[idx] = save - h
        dn = _loss(x, alpha, beta, dy, method)
        arr[idx] = save
        return (up - dn) / (2 * h)

    fd_dx = np.array([[fd(x, (n, k)) for k in range(d)] for n in range(N)])
    fd_da = np.array([fd(alpha, j) for j in range(d)])
    fd_db = np.array([fd(beta, j) for j in range(d)])
    scale = lambda a: max(1.0, np.max(np.abs(a)))
    assert np.max(np.abs(dx - fd_dx)) <= 1e-7 * scale(fd_dx)
    assert np.max(np.abs(dalpha - fd_da)) <= 1e-7 * scale(fd_da)
    assert np.max(np.abs(dbeta - fd_db)) <= 1e-7 * scale(fd_db)


@pytest.mark.parametrize("N,d", [(5, 48), (33, 768)])
def test_backward_identities(N, d):
    x, dy = RNG.standard_normal((N, d)), RNG.standard_normal((N, d))
    alpha = RNG.uniform(0.5, 1.5, d)
    dx, dalpha, dbeta = oracle.backward(dy, x, alpha, "fast")
    assert np.allclose(dbeta, dy.sum(axis=0), rtol=0, atol=1e-12 * np.sqrt(N))
    lhs = np.sum(dy * oracle.forward(x, alpha, np.zeros(d), "fast"))
    assert abs(lhs - np.sum(dx * x)) <= 1e-10 * max(1.0, abs(lhs))         # adjoint identity
    assert abs(np.dot(dalpha, alpha) - lhs) <= 1e-10 * max(1.0, abs(lhs))
    assert np.allclose(oracle.transform(dx, "fast"), alpha * dy, atol=1e-12 * np.sqrt(d))
    a = oracle.backward(dy, x, alpha, "matrix")
    for u, v in zip(a, (dx, dalpha, dbeta)):
        assert np.max(np.abs(u - v)) <= 1e-12 * max(1.0, np.max(np.abs(v)))


def test_pins_reject_planted_mistakes():
    """The checks above must fail for plausible wrong order-12 factors (planted here, on the CPU)."""
    P = oracle.h12()

    def is_good(M):
        return (np.array_equal(M @ M.T, 12 * np.eye(12, dtype=np.int64)) and np.array_equal(M, M.T)
                and np.all(M[0] == 1) and np.array_equal(M, _paley2_order12_independent()))

    assert is_good(P)
    flipped = P.copy()
    flipped[5, 7] *= -1                                   # one wrong sign
    assert not is_good(flipped)
    rolled = np.roll(P, 1, axis=1)                        # columns off by one
    assert not is_good(rolled)
    swapped = P.copy()
    swapped[[3, 4]] = swapped[[4, 3]]                     # two rows exchanged: still Hadamard, not symmetric
    assert not is_good(swapped)
    perm = P[np.ix_([0, 2, 1] + list(range(3, 12)), [0, 2, 1] + list(range(3, 12)))]
    assert not is_good(perm)                              # a different (equivalent) order-12 matrix
