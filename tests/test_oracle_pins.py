"""Pins for the CPU oracle: everything here checks oracle/ against facts fixed by the paper or by
mathematics, never against the oracle's own formula retyped and never against the GPU path.

  ordering / sign pattern ... the 4x4 block printed in Fig. 1; scipy's Sylvester construction
  butterfly network ......... the pairs and the rule printed in Fig. 2
  normalisation ............. H^T H = I (Sec. 4.1): H_raw H_raw = d I, involution, norm preservation
  Eq. 1 ..................... hand-worked d = 2, 4, 8 examples, special cases
  backward .................. central finite differences in fp64, the adjoint identity, column sums
  mutants ................... plausible mistakes (sequency order, missing 1/sqrt d, transposed use,
                              swapped sign in the butterfly) must fail at least one pin
"""
import os

import numpy as np
import pytest
import scipy.linalg

import oracle

RNG = np.random.default_rng(12345)


# ---------------------------------------------------------------- ordering: Fig. 1 and Sylvester

def _read_signs(path):
    rows = []
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        rows.append([+1 if s == "+" else -1 for s in line.split()])
    return np.array(rows, dtype=np.int64)


def test_sign_matrix_d4_equals_fig1(golden_dir):
    printed = _read_signs(os.path.join(golden_dir, "fig1_hadamard4_signs.txt"))
    assert printed.shape == (4, 4)
    assert np.array_equal(oracle.hadamard_matrix(4), printed)
    # the transform itself, not only the sign helper: column k of H_raw is sqrt(d) * H e_k
    for method in ("matrix", "fast"):
        cols = np.stack([oracle.transform(np.eye(4)[k], method) for k in range(4)], axis=1)
        assert np.array_equal(np.rint(cols * 2.0).astype(np.int64), printed)


@pytest.mark.parametrize("d", [1, 2, 4, 8, 16, 64, 256])
def test_sign_matrix_equals_scipy_sylvester(d):
    assert np.array_equal(oracle.hadamard_matrix(d), scipy.linalg.hadamard(d).astype(np.int64))


@pytest.mark.parametrize("d", [2, 8, 32, 128])
@pytest.mark.parametrize("method", ["matrix", "fast"])
def test_transform_equals_scipy_matmul(d, method):
    x = RNG.standard_normal((5, d))
    want = x @ scipy.linalg.hadamard(d).astype(np.float64) / np.sqrt(d)      # Y H, as in Eq. 1
    assert np.allclose(oracle.transform(x, method), want, rtol=0, atol=1e-12 * np.sqrt(d))


# ---------------------------------------------------------------- butterfly network: Fig. 2

def _read_butterfly(path):
    stages = []
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        stages.append((int(tok[1]), [tuple(int(v) for v in p.split("-")) for p in tok[2:]]))
    return stages


def test_butterfly_pairs_and_rule_equal_fig2(golden_dir):
    stages = _read_butterfly(os.path.join(golden_dir, "fig2_butterfly8.txt"))
    assert [s for s, _ in stages] == [1, 2, 4]
    for stride, pairs in stages:
        # which inputs reach which outputs: feed unit vectors through one stage
        touched = set()
        for i in range(8):
            out = oracle.butterfly_stage(np.eye(8)[i], stride)
            nz = tuple(int(v) + 1 for v in np.flatnonzero(out))
            touched.add(nz)
        assert touched == set(pairs)
        # the rule: upper gets the sum, lower gets upper minus lower
        a = np.arange(1.0, 9.0) ** 2
        out = oracle.butterfly_stage(a, stride)
        for (i, j) in pairs:
            assert out[i - 1] == a[i - 1] + a[j - 1]
            assert out[j - 1] == a[i - 1] - a[j - 1]


# ---------------------------------------------------------------- hand-worked examples

def test_hand_worked_d2():
    s = np.sqrt(2.0)
    for method in ("matrix", "fast"):
        assert np.allclose(oracle.transform(np.array([1.0, 2.0]), method), [3 / s, -1 / s], atol=1e-15)
        assert np.allclose(oracle.transform(np.array([1.0, 0.0]), method), [1 / s, 1 / s], atol=1e-15)


def test_hand_worked_d4():
    x = np.array([[1.0, 2.0, 3.0, 4.0]])
    for method in ("matrix", "fast"):
        z = oracle.transform(x, method)
        assert np.array_equal(z, [[5.0, -1.0, -2.0, 0.0]])          # (10,-2,-4,0)/2
        y = oracle.forward(x, np.array([1.0, 2.0, 3.0, 4.0]), np.full(4, 0.5), method)
        assert np.array_equal(y, [[5.5, -1.5, -5.5, 0.5]])


def test_hand_worked_d8():
    x = np.arange(1.0, 9.0)
    want_raw = np.array([36.0, -4.0, -8.0, 0.0, -16.0, 0.0, 0.0, 0.0])
    for method in ("matrix", "fast"):
        z = oracle.transform(x, method)
        assert np.allclose(z * np.sqrt(8.0), want_raw, atol=1e-13)
    assert np.sum(want_raw ** 2) == 8 * np.sum(x ** 2)


# ---------------------------------------------------------------- normalisation and structure

@pytest.mark.parametrize("d", [1, 2, 4, 16, 64, 256])
def test_Hraw_squared_is_d_times_identity(d):
    H = oracle.hadamard_matrix(d)
    assert np.array_equal(H @ H, d * np.eye(d, dtype=np.int64))
    assert np.array_equal(H, H.T)


@pytest.mark.parametrize("d", [2 ** k for k in range(0, 11)])
def test_fast_equals_matrix(d):
    x = RNG.standard_normal((3, d))
    a, b = oracle.transform(x, "fast"), oracle.transform(x, "matrix")
    assert np.max(np.abs(a - b)) <= 1e-12 * max(1.0, np.max(np.abs(b)))


@pytest.mark.parametrize("d", [2, 64, 1024, 4096, 8192])
def test_involution_and_norm_preservation(d):
    x = RNG.standard_normal((4, d))
    z = oracle.transform(x, "fast")
    assert np.allclose(np.linalg.norm(z, axis=1), np.linalg.norm(x, axis=1), rtol=1e-12)
    assert np.max(np.abs(oracle.transform(z, "fast") - x)) <= 1e-12 * np.max(np.abs(x))


@pytest.mark.parametrize("d", [8, 128, 2048])
def test_unit_vectors_constants_linearity(d):
    for k in (0, 1, d // 2 + 1, d - 1):
        e = np.zeros(d)
        e[k] = 1.0
        col = oracle.transform(e, "fast")
        signs = np.array([(-1) ** bin(j & k).count("1") for j in range(d)], dtype=np.float64)
        assert np.allclose(col, signs / np.sqrt(d), atol=1e-15)
    ones = oracle.transform(np.ones(d), "fast")
    want = np.zeros(d)
    want[0] = np.sqrt(d)
    assert np.allclose(ones, want, atol=1e-12)
    x, w = RNG.standard_normal(d), RNG.standard_normal(d)
    lhs = oracle.transform(2.5 * x - 0.75 * w, "fast")
    rhs = 2.5 * oracle.transform(x, "fast") - 0.75 * oracle.transform(w, "fast")
    assert np.allclose(lhs, rhs, atol=1e-12 * np.sqrt(d))


def test_rejects_widths_without_a_definition():
    # 2^n and 12 * 2^m have one; nothing else does (no Hadamard matrix of order 3, 6, 10 ...)
    for d in (3, 6, 10, 20, 36, 100, 1000):
        with pytest.raises(ValueError):
            oracle.transform(np.zeros((2, d)))
        with pytest.raises(ValueError):
            oracle.forward(np.zeros((2, d)), np.ones(d), np.zeros(d))


# ---------------------------------------------------------------- Eq. 1 special cases

@pytest.mark.parametrize("method", ["matrix", "fast"])
def test_affine_special_cases(method):
    d = 64
    x = RNG.standard_normal((6, d))
    alpha, beta = RNG.uniform(0.5, 1.5, d), 0.02 * RNG.standard_normal(d)
    assert np.array_equal(oracle.forward(x, np.ones(d), np.zeros(d), method), oracle.transform(x, method))
    assert np.array_equal(oracle.forward(np.zeros((6, d)), alpha, beta, method), np.tile(beta, (6, 1)))
    z = oracle.transform(x, method)
    assert np.allclose(oracle.forward(x, alpha, beta, method), alpha * z + beta, rtol=0, atol=1e-15)
    k = 37
    e = np.zeros(d)
    e[k] = 1.0
    col = scipy.linalg.hadamard(d)[:, k] / np.sqrt(d)
    assert np.allclose(oracle.forward(e, alpha, beta, method), alpha * col + beta, atol=1e-15)


def test_forward_residual_special_cases():
    d = 32
    x, resid = RNG.standard_normal((5, d)), RNG.standard_normal((5, d))
    alpha, beta = RNG.uniform(0.5, 1.5, d), 0.02 * RNG.standard_normal(d)
    for method in ("matrix", "fast"):
        # zero residual: the plain layer; zero input: residual + beta; hand-worked d = 4
        assert np.array_equal(oracle.forward_residual(x, alpha, beta, np.zeros((5, d)), method),
                              oracle.forward(x, alpha, beta, method))
        assert np.allclose(oracle.forward_residual(np.zeros((5, d)), alpha, beta, resid, method), resid + beta,
                           rtol=0, atol=1e-15)
        y = oracle.forward_residual(np.array([[1.0, 2.0, 3.0, 4.0]]), np.array([1.0, 2.0, 3.0, 4.0]),
                                    np.full(4, 0.5), np.array([[10.0, 20.0, 30.0, 40.0]]), method)
        assert np.array_equal(y, [[15.5, 18.5, 24.5, 40.5]])
        # the gradient with respect to the residual is the identity: finite difference of sum(w*y)
        w = RNG.standard_normal((5, d))
        base = np.sum(w * oracle.forward_residual(x, alpha, beta, resid, method))
        bumped = resid.copy()
        bumped[2, 7] += 1e-3
        assert abs((np.sum(w * oracle.forward_residual(x, alpha, beta, bumped, method)) - base) / 1e-3 - w[2, 7]) < 1e-9


# ---------------------------------------------------------------- stored dtypes are widened exactly

def test_forward_residual_stats_special_cases():
    """sumsq[n] = sum_j y[n,j]^2: with alpha = 1, beta = 0 and no residual it is ||x_n||^2 (H preserves
    the norm, Sec. 4.1); with x = 0 and no residual it is ||beta||^2; in general numpy's row sums."""
    N, d = 5, 256
    x, resid = RNG.standard_normal((N, d)), RNG.standard_normal((N, d))
    alpha, beta = RNG.uniform(0.5, 1.5, d), RNG.standard_normal(d)
    zero = np.zeros((N, d))
    y, s = oracle.forward_residual_stats(x, np.ones(d), np.zeros(d), zero)
    assert np.allclose(s, np.sum(x * x, axis=1), rtol=1e-12)
    y, s = oracle.forward_residual_stats(zero, alpha, beta, zero)
    assert np.allclose(s, np.full(N, np.dot(beta, beta)), rtol=1e-14)
    y, s = oracle.forward_residual_stats(x, alpha, beta, resid)
    assert np.array_equal(y, oracle.forward_residual(x, alpha, beta, resid))
    assert np.allclose(s, np.einsum("nj,nj->n", y, y), rtol=1e-14)
    # twelve-block width and a hand-worked row: y = (3, -4) -> 25
    y, s = oracle.forward_residual_stats(np.zeros((1, 2)), np.ones(2), np.array([3.0, -4.0]), np.zeros((1, 2)))
    assert s.tolist() == [25.0]
    y, s = oracle.forward_residual_stats(RNG.standard_normal((2, 96)), np.ones(96), np.zeros(96), np.zeros((2, 96)))
    assert s.shape == (2,) and np.all(s > 0)


def test_bf16_and_f32_inputs_widen_exactly():
    import torch
    bits = RNG.integers(0, 1 << 16, size=4096, dtype=np.uint16)
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.bf16_bits_to_float64(bits)
    finite = np.isfinite(t)
    assert np.array_equal(got[finite], t[finite])
    assert np.array_equal(np.isnan(got), np.isnan(t))
    # through the transform: bf16 / f32 storage gives the same result as pre-widened float64
    d = 32
    xb = RNG.integers(0x3C00, 0x4100, size=(3, d), dtype=np.uint16)          # moderate positive values
    xb[:, ::2] |= 0x8000                                                       # some negative
    wide = torch.from_numpy(xb.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oracle.transform(xb, "fast"), oracle.transform(wide, "fast"))
    xf = RNG.standard_normal((3, d)).astype(np.float32)
    assert np.array_equal(oracle.transform(xf, "fast"), oracle.transform(xf.astype(np.float64), "fast"))


# ---------------------------------------------------------------- backward

def _loss(x, alpha, beta, dy, method):
    return float(np.sum(dy * oracle.forward(x, alpha, beta, method)))


@pytest.mark.parametrize("method", ["matrix", "fast"])
@pytest.mark.parametrize("N,d", [(1, 2), (3, 8), (4, 16)])
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


@pytest.mark.parametrize("N,d", [(1, 4), (7, 64), (129, 256), (33, 2048)])
def test_backward_identities(N, d):
    x, dy = RNG.standard_normal((N, d)), RNG.standard_normal((N, d))
    alpha = RNG.uniform(0.5, 1.5, d)
    dx, dalpha, dbeta = oracle.backward(dy, x, alpha, "fast")
    # dbeta is a plain column sum
    assert np.allclose(dbeta, dy.sum(axis=0), rtol=0, atol=1e-12 * np.sqrt(N))
    # adjoint identity  <dy, alpha (.) H x> = <H(alpha (.) dy), x>
    lhs = np.sum(dy * oracle.forward(x, alpha, np.zeros(d), "fast"))
    assert abs(lhs - np.sum(dx * x)) <= 1e-10 * max(1.0, abs(lhs))
    # <dalpha, alpha> = same scalar  (sum_j alpha_j sum_n dy z)
    assert abs(np.dot(dalpha, alpha) - lhs) <= 1e-10 * max(1.0, abs(lhs))
    # dy = 1: dalpha is the column sum of z
    _, da1, db1 = oracle.backward(np.ones((N, d)), x, alpha, "fast")
    assert np.allclose(da1, oracle.transform(x, "fast").sum(axis=0), atol=1e-11 * np.sqrt(N * d))
    assert np.array_equal(db1, np.full(d, float(N)))
    # dx is H applied to alpha*dy: undo it with the involution
    assert np.allclose(oracle.transform(dx, "fast"), alpha * dy, atol=1e-12 * np.sqrt(d))
    # skipping outputs changes nothing else
    dx2, none_a, none_b = oracle.backward(dy, x, alpha, "fast", want_param_grads=False)
    assert none_a is None and none_b is None and np.array_equal(dx2, dx)
    none_x, da3, db3 = oracle.backward(dy, x, alpha, "fast", want_dx=False)
    assert none_x is None and np.array_equal(da3, dalpha) and np.array_equal(db3, dbeta)


def test_backward_matrix_equals_fast():
    N, d = 5, 128
    x, dy = RNG.standard_normal((N, d)), RNG.standard_normal((N, d))
    alpha = RNG.uniform(0.5, 1.5, d)
    a = oracle.backward(dy, x, alpha, "matrix")
    b = oracle.backward(dy, x, alpha, "fast")
    for u, v in zip(a, b):
        assert np.max(np.abs(u - v)) <= 1e-12 * max(1.0, np.max(np.abs(v)))


def test_thread_count_does_not_change_results():
    N, d = 37, 256
    x, dy = RNG.standard_normal((N, d)), RNG.standard_normal((N, d))
    alpha = RNG.uniform(0.5, 1.5, d)
    before = oracle.num_threads()
    try:
        oracle.set_num_threads(1)
        one = oracle.backward(dy, x, alpha, "fast")
        oracle.set_num_threads(3)
        three = oracle.backward(dy, x, alpha, "fast")
    finally:
        oracle.set_num_threads(before)
    assert np.array_equal(one[0], three[0])
    for u, v in zip(one[1:], three[1:]):
        assert np.allclose(u, v, rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- planted mistakes must be caught

def _mutants(d):
    """Plausible wrong versions of H (as explicit matrices), each paired with a name."""
    H = scipy.linalg.hadamard(d).astype(np.float64)
    n = int(np.log2(d))
    bitrev = [int(format(i, f"0{n}b")[::-1], 2) for i in range(d)]
    gray = [i ^ (i >> 1) for i in range(d)]
    seq = H[[bitrev[g] for g in gray], :]                          # sequency (Walsh) order
    swapped = np.array([[(-1) ** (bin(j & k).count("1") + (j != 0)) for k in range(d)]
                        for j in range(d)], dtype=np.float64)       # lower-minus-upper butterflies
    return {
        "sequency_order": seq / np.sqrt(d),
        "no_normalisation": H,
        "normalised_by_d": H / d,
        "bit_reversed_rows": H[bitrev, :] / np.sqrt(d),
        "difference_sign_flipped": swapped / np.sqrt(d),
    }


def test_pins_reject_planted_mistakes(golden_dir):
    printed = _read_signs(os.path.join(golden_dir, "fig1_hadamard4_signs.txt"))
    x8 = np.arange(1.0, 9.0)
    want8 = np.array([36.0, -4.0, -8.0, 0.0, -16.0, 0.0, 0.0, 0.0]) / np.sqrt(8.0)
    for name, M4 in _mutants(4).items():
        M8 = _mutants(8)[name]
        fails_fig1 = not np.array_equal(np.rint(M4 * 2.0), printed)
        fails_d8 = not np.allclose(M8 @ x8, want8, atol=1e-12)
        fails_orth = not np.allclose(M8 @ M8.T, np.eye(8), atol=1e-12)
        assert fails_fig1 or fails_d8 or fails_orth, name
