"""Pins for the oracle's butterfly variance equaliser: the output condition of Section 5.1
(diag(R Sigma R^T) = c 1, the equality case of Theorem 4.1), closed forms (2 x 2, diagonal and scalar
covariances), the structure (R is the product of the log2 B rounds rebuilt from the returned
tangents), and the effect on the sample it was computed from.
"""
import math

import numpy as np
import pytest

import oracle


def _sample_cov(B, seed, n=300):
    rng = np.random.default_rng(seed)
    A = rng.standard_t(3, size=(n, B)) * np.exp(rng.normal(size=B) * 1.5)
    A[:, 1:] += 0.5 * A[:, :-1]                  # correlation between neighbouring blocks
    return A, A.T @ A / n


@pytest.mark.parametrize("B", [2, 4, 16, 64, 128, 256])
def test_butterfly_meets_the_output_condition(B):
    _, S = _sample_cov(B, B)
    R, S2, tan = oracle.equalize_butterfly(S)
    c = np.trace(S) / B
    assert np.abs(R @ R.T - np.eye(B)).max() <= 1e-12
    assert np.abs(S2 - R @ S @ R.T).max() <= 1e-9 * np.abs(S).max()         # the returned matrix is R Sigma R^T
    assert np.abs(np.diag(R @ S @ R.T) - c).max() <= 1e-10 * c              # constant diagonal
    assert abs(np.trace(S2) - np.trace(S)) <= 1e-10 * np.trace(S)
    assert tan.shape == (int(math.log2(B)), B // 2) and np.abs(tan).max() <= 1.0 + 1e-15
    assert np.diag(S).max() / np.diag(S).min() > (5.0 if B >= 16 else 1.5)  # the input was far from equal


@pytest.mark.parametrize("B", [4, 32, 128])
def test_butterfly_is_the_product_of_its_rounds(B):
    _, S = _sample_cov(B, 100 + B)
    R, _, tan = oracle.equalize_butterfly(S)
    want = np.eye(B)
    h, t = B // 2, 0
    while h >= 1:
        J = np.eye(B)
        pairs = [p for p in range(B) if not p & h]
        for i, p in enumerate(pairs):
            th = math.atan(tan[t, i])
            J[p, p] = J[p + h, p + h] = math.cos(th)
            J[p, p + h] = math.sin(th)
            J[p + h, p] = -math.sin(th)
        want = J @ want
        h //= 2
        t += 1
    assert np.abs(R - want).max() <= 1e-13


def test_butterfly_two_by_two_closed_form():
    a, b, g = 5.0, 1.0, 1.5
    R, S2, tan = oracle.equalize_butterfly(np.array([[a, g], [g, b]]))
    th = 0.5 * math.atan((b - a) / (2 * g))
    assert tan[0, 0] == pytest.approx(math.tan(th), abs=1e-15)
    assert np.allclose(R, [[math.cos(th), math.sin(th)], [-math.sin(th), math.cos(th)]], atol=1e-15)
    assert S2[0, 0] == pytest.approx(3.0, abs=1e-12) and S2[1, 1] == pytest.approx(3.0, abs=1e-12)


def test_butterfly_on_diagonal_and_scalar_covariances():
    B = 16
    R, S2, tan = oracle.equalize_butterfly(np.diag(np.arange(1.0, B + 1)))
    # no correlation anywhere: every pair is turned by 45 degrees, R has Hadamard magnitudes
    assert np.allclose(tan, 1.0, atol=1e-15)
    assert np.allclose(np.abs(R), 1 / math.sqrt(B), atol=1e-15)
    assert np.allclose(np.diag(S2), (B + 1) / 2, atol=1e-12)
    R, S2, tan = oracle.equalize_butterfly(3.0 * np.eye(B))
    assert np.array_equal(R, np.eye(B)) and np.all(tan == 0.0)


def test_butterfly_rotation_equalizes_the_samples_block_energies():
    # blocks of a sample -> Gram matrix -> butterfly R -> rotate that sample: equal block energies
    G, M = 32, 64
    rng = np.random.default_rng(9)
    X = (rng.standard_t(3, size=(M, G, 32)) * np.exp(rng.normal(size=(1, G, 1)) * 1.2))
    xb = oracle.f32_to_bf16(X.reshape(M, G * 32).astype(np.float32))
    Xq = oracle.bf16_to_f32(xb).astype(np.float64).reshape(M, G, 32)
    Sigma = np.einsum("mbk,mck->bc", Xq, Xq) / M
    R, _, _ = oracle.equalize_butterfly(Sigma)
    Y = oracle.rotate_inter(Xq.reshape(M, G * 32), G, R.astype(np.float32).astype(np.float64))
    energies = (Y.reshape(M, G, 32) ** 2).sum(axis=2).mean(axis=0)
    c = np.trace(Sigma) / G
    assert np.abs(energies - c).max() <= 1e-5 * c        # R went through fp32 on the way in
    assert np.diag(Sigma).max() / np.diag(Sigma).min() > 5.0
