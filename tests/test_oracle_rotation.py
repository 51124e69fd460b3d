"""Pins for the oracle's two-level rotation (Appendix A.3, Algorithm 3, steps 1-3)
and for the variance equaliser (Section 5.1, Algorithm 1 / Theorem 4.1).

The oracle is compared with: the explicit Kronecker matrix built by numpy on a
tiny case, closed forms for Hadamard rotations, invariants of orthogonal maps
(norm, inner product, trace), and the equal-diagonal condition of Theorem 4.1.
"""
import numpy as np
import scipy.linalg
import torch

from paper_2605_19561_amd import synth


def _bits(a32):
    """float32 array -> bf16 patterns (torch's conversion) and the values they hold"""
    t = torch.from_numpy(np.ascontiguousarray(a32, np.float32)).to(torch.bfloat16)
    return synth.bf16_bits(t), t.to(torch.float64).numpy()


def test_generated_rotations_are_orthogonal():
    for n, seed in ((128, 1), (32, 2), (80, 3), (256, 4)):
        R = synth.random_orthogonal(n, seed).astype(np.float64)
        assert np.abs(R @ R.T - np.eye(n)).max() < 1e-6      # Appendix A.2 constraint 1
        assert np.abs(R.T @ R - np.eye(n)).max() < 1e-6
        assert not np.allclose(R, R.T, atol=1e-2)            # not symmetric: transposes matter


def test_identity_rotation_is_identity(oracle):
    rng = np.random.default_rng(0)
    bits, vals = _bits(rng.standard_normal((3, 512)))
    z32, z64 = oracle.rotate(bits, 16, np.eye(16, dtype=np.float32), np.eye(32, dtype=np.float32), want_f64=True)
    assert np.array_equal(z64, vals)
    assert np.array_equal(z32.astype(np.float64), vals)


def test_matches_explicit_kronecker_matrix(oracle):
    # Section 5: R = R_inter (x) R_intra acting on the row-major vec of the B x 32 view.
    # Algorithm 3: Z = R_inter X R_intra  <=>  vec_r(Z) = (R_inter (x) R_intra^T) vec_r(X).
    rng = np.random.default_rng(1)
    B = 4
    d = 32 * B
    Ri = synth.random_orthogonal(B, 10)
    Ra = synth.random_orthogonal(32, 11)
    bits, vals = _bits(rng.standard_normal((5, d)) * 3)
    z64 = oracle.rotate(bits, B, Ri, Ra, want_f64=True)[1]
    K = np.kron(Ri.astype(np.float64), Ra.astype(np.float64).T)
    ref = vals @ K.T
    assert np.abs(z64 - ref).max() < 1e-12
    # a transposed operand anywhere would give one of these instead
    for wrong in (np.kron(Ri.T, Ra.T), np.kron(Ri, Ra), np.kron(Ri.T, Ra), np.kron(Ra.T, Ri)):
        assert np.abs(z64 - vals @ wrong.astype(np.float64).T).max() > 1e-2


def test_group_structure_when_G_smaller_than_B(oracle):
    # G x G matrix acting on each run of G consecutive blocks == block-diagonal B x B matrix
    rng = np.random.default_rng(2)
    G, B = 4, 12
    d = 32 * B
    Ri = synth.random_orthogonal(G, 20)
    Ra = synth.random_orthogonal(32, 21)
    bits, vals = _bits(rng.standard_normal((4, d)))
    z64 = oracle.rotate(bits, G, Ri, Ra, want_f64=True)[1]
    big = scipy.linalg.block_diag(*[Ri.astype(np.float64)] * (B // G))
    zfull = oracle.rotate(bits, B, big.astype(np.float32), Ra, want_f64=True)[1]
    assert np.abs(z64 - zfull).max() < 1e-12
    X = vals.reshape(4, B, 32)
    ref = np.einsum("ij,mjk,kl->mil", big, X, Ra.astype(np.float64)).reshape(4, d)
    assert np.abs(z64 - ref).max() < 1e-12


def test_hadamard_rotations_closed_forms(oracle):
    # R_inter = H_G / sqrt(G), R_intra = H_32 / sqrt(32): the two-level map is a
    # Walsh-Hadamard transform of length 32 G (Sylvester ordering), for which
    #   one-hot at position p -> +-1/sqrt(32 G) everywhere, sign = H[p, :]
    #   constant c            -> c sqrt(32 G) at index 0, zero elsewhere
    G = 16
    d = 32 * G
    Hi = (scipy.linalg.hadamard(G) / np.sqrt(G)).astype(np.float32)     # exact in fp32
    Ha = (scipy.linalg.hadamard(32) / np.sqrt(32)).astype(np.float32)
    x = np.zeros((3, d), np.float32)
    p = 5 * 32 + 9
    x[0, p] = 1.0
    x[1, :] = 0.5
    rng = np.random.default_rng(3)
    x[2] = rng.standard_normal(d)
    bits, vals = _bits(x)
    z64 = oracle.rotate(bits, G, Hi, Ha, want_f64=True)[1]
    Hd = scipy.linalg.hadamard(d).astype(np.float64)
    scale = float(Hi[0, 0]) * float(Ha[0, 0])
    assert np.abs(z64[0] - Hd[p] * scale).max() < 1e-15
    want1 = np.zeros(d)
    want1[0] = 0.5 * d * scale
    assert np.abs(z64[1] - want1).max() < 1e-12
    assert np.abs(z64[2] - (Hd @ vals[2]) * scale).max() < 1e-12       # H_d = H_G (x) H_32, symmetric


def test_norm_and_inner_product_preserved(oracle):
    # orthogonal map: ||z|| = ||x|| and <rot(x), rot(w)> = <x, w>  (Section 5.2: the
    # rotate / inverse-rotate link is an identity under full precision)
    G = 16
    d = 32 * G * 2
    Ri, Ra = synth.rotations(G, seed=33)
    x = synth.activations(6, d, nu=3.0, outliers=4, outlier_scale=50.0, seed=5)
    w = synth.weights(6, d, std=0.02, seed=6)
    zx = oracle.rotate(synth.bf16_bits(x), G, Ri, Ra, want_f64=True)[1]
    zw = oracle.rotate(synth.bf16_bits(w), G, Ri, Ra, want_f64=True)[1]
    xv, wv = x.to(torch.float64).numpy(), w.to(torch.float64).numpy()
    nx = np.linalg.norm(xv, axis=1)
    assert np.abs(np.linalg.norm(zx, axis=1) - nx).max() / nx.max() < 1e-6
    assert np.abs(zx @ zw.T - xv @ wv.T).max() < 1e-5 * np.abs(xv @ wv.T).max() + 1e-6
    # explicit inverse (Algorithm 3 step 5 option A) recovers x
    back = oracle.rotate_inverse(zx, G, Ri, Ra)
    assert np.abs(back - xv).max() < 1e-5 * np.abs(xv).max()


def test_inter_and_intra_commute(oracle):
    # the two factors of a Kronecker product act on different indices
    G = 16
    d = 32 * G
    Ri, Ra = synth.rotations(G, seed=44)
    rng = np.random.default_rng(4)
    x = rng.standard_normal((3, d))
    a = oracle.rotate_intra(oracle.rotate_inter(x, G, Ri), Ra)
    b = oracle.rotate_inter(oracle.rotate_intra(x, Ra), G, Ri)
    assert np.abs(a - b).max() < 1e-12
    # each alone against numpy
    X = x.reshape(3, G, 32)
    assert np.abs(oracle.rotate_inter(x, G, Ri).reshape(3, G, 32)
                  - np.einsum("ij,mjk->mik", Ri.astype(np.float64), X)).max() < 1e-12
    assert np.abs(oracle.rotate_intra(x, Ra).reshape(3, G, 32)
                  - np.einsum("mbk,kl->mbl", X, Ra.astype(np.float64))).max() < 1e-12


def test_fp32_output_is_rounded_double(oracle):
    G = 16
    Ri, Ra = synth.rotations(G, seed=55)
    x = synth.activations(4, 32 * G, seed=8)
    z32, z64 = oracle.rotate(synth.bf16_bits(x), G, Ri, Ra, want_f64=True)
    assert np.array_equal(z32, z64.astype(np.float32))


# ------------------------------------------------------- Algorithm 1 --------

def _sample_gram(M, B, seed):
    x = synth.activations(M, 32 * B, nu=3.0, outliers=max(1, B // 8), outlier_scale=50.0, seed=seed)
    X = x.to(torch.float64).numpy().reshape(M, B, 32)
    # block Gram matrix: Sigma[b, b'] = mean over tokens of <x_b, x_b'>
    return X, np.einsum("mbk,mck->bc", X, X) / M


def test_equalizer_meets_theorem_4_1_condition(oracle):
    for B, seed in ((16, 1), (64, 2), (128, 3)):
        X, Sigma = _sample_gram(256, B, seed)
        c = np.trace(Sigma) / B
        R, S_after, steps = oracle.equalize(Sigma, eps=1e-12 * c)
        assert 0 < steps <= B - 1
        assert np.abs(R @ R.T - np.eye(B)).max() < 1e-12
        # the oracle's updated Sigma is R Sigma R^T (numpy recomputes it)
        RSR = R @ Sigma @ R.T
        assert np.abs(RSR - S_after).max() < 1e-9 * c
        assert np.abs(np.diag(RSR) - c).max() < 1e-10 * c              # diag = c 1
        assert abs(np.trace(RSR) - np.trace(Sigma)) < 1e-10 * np.trace(Sigma)   # Appendix A.1 step 1
        # Schur-Horn: rotating the sample itself equalises its block energies
        Y = oracle.rotate_inter(X.reshape(256, -1), B, R.astype(np.float32)).reshape(256, B, 32)
        energy = (Y ** 2).sum(axis=(0, 2)) / 256
        assert np.abs(energy - c).max() < 1e-5 * c                     # R was rounded to fp32
        before = (X ** 2).sum(axis=(0, 2)) / 256
        assert before.max() / before.min() > 20.0                      # the input was unbalanced


def test_equalizer_on_fresh_samples_reduces_imbalance(oracle):
    B = 64
    # one draw of 1024 tokens (one outlier-channel set): calibrate on the first half,
    # look at the second half
    x_all = synth.activations(1024, 32 * B, nu=3.0, outliers=B // 8, outlier_scale=50.0, seed=7)
    Xa = x_all.to(torch.float64).numpy()
    Sigma_a = np.einsum("mbk,mck->bc", Xa[:512].reshape(512, B, 32), Xa[:512].reshape(512, B, 32)) / 512
    R, _, _ = oracle.equalize(Sigma_a, eps=0.0)
    fresh = Xa[512:]
    e0 = (fresh.reshape(512, B, 32) ** 2).sum(axis=(0, 2))
    Y = oracle.rotate_inter(fresh, B, R.astype(np.float32)).reshape(512, B, 32)
    e1 = (Y ** 2).sum(axis=(0, 2))
    assert abs(e0.sum() - e1.sum()) < 1e-5 * e0.sum()
    assert (e1.max() / e1.min()) < 0.2 * (e0.max() / e0.min())         # direction only


def test_equalizer_trivial_cases(oracle):
    R, S, steps = oracle.equalize(np.eye(8) * 3.0)
    assert steps == 0 and np.array_equal(R, np.eye(8))
    # 2 x 2 diagonal: the equalising angle is 45 degrees
    R, S, steps = oracle.equalize(np.diag([4.0, 2.0]), eps=1e-15)
    assert steps == 1
    assert np.allclose(np.abs(R), np.sqrt(0.5))
    assert np.allclose(np.diag(S), 3.0)


# ------------------------------------------------- block Gram (Section 5.1) -

def test_block_gram_against_its_definition_and_invariants(oracle):
    # several runs of G blocks per row, outlier channels: compared with the same contraction written
    # with numpy's einsum on the widened values (a library routine, not the oracle's loops)
    M, d, G = 24, 3072, 32
    x = synth.activations(M, d, nu=3.0, outliers=12, outlier_scale=50.0, seed=41)
    S = oracle.block_gram(synth.bf16_bits(x), G)
    X = x.to(torch.float64).numpy().reshape(M * (d // 32 // G), G, 32)
    want = np.einsum("tbk,tck->bc", X, X) / X.shape[0]
    assert np.abs(S - want).max() <= 1e-12 * np.abs(want).max()
    assert np.array_equal(S, S.T)                                       # same products, same order
    assert np.linalg.eigvalsh(S).min() > -1e-9 * np.trace(S)            # a Gram matrix
    # the diagonal is the mean block energy; the trace the mean energy of a run
    assert np.allclose(np.diag(S), (X ** 2).sum(axis=2).mean(axis=0), rtol=1e-12)
    assert abs(np.trace(S) - (X ** 2).sum() / X.shape[0]) <= 1e-12 * np.trace(S)


def test_block_gram_closed_forms(oracle):
    G = 16
    # every block equal to one vector v: Sigma = |v|^2 * ones (rank one)
    v = np.arange(1, 33, dtype=np.float32) / 8.0                          # exact in bf16
    x = torch.from_numpy(np.tile(v, (5, G))).to(torch.bfloat16)
    S = oracle.block_gram(synth.bf16_bits(x), G)
    assert np.array_equal(S, np.full((G, G), float((v.astype(np.float64) ** 2).sum())))
    # one-hot rows: row m has a 1 at element 32 * (m % G): Sigma = I / G (mean over G rows)
    x = torch.zeros((G, 32 * G), dtype=torch.bfloat16)
    for m in range(G):
        x[m, 32 * m] = 1.0
    assert np.array_equal(oracle.block_gram(synth.bf16_bits(x), G), np.eye(G) / G)
    # blocks b and b+1 carry the same vector with opposite sign in one run: off-diagonal -|v|^2
    x = torch.zeros((1, 32 * G), dtype=torch.bfloat16)
    x[0, 32 * 3:32 * 4] = torch.from_numpy(v).to(torch.bfloat16)
    x[0, 32 * 4:32 * 5] = -torch.from_numpy(v).to(torch.bfloat16)
    S = oracle.block_gram(synth.bf16_bits(x), G)
    e = float((v.astype(np.float64) ** 2).sum())
    assert S[3, 3] == e and S[4, 4] == e and S[3, 4] == -e and S[4, 3] == -e and np.count_nonzero(S) == 4


def test_block_gram_positions_against_its_definition_and_closed_forms(oracle):
    # Sigma_k of Theorem 4.1, one matrix per position inside a block: numpy's einsum on the widened values,
    # the sum over k (the block Gram, pinned above), and inputs whose answer can be written down
    M, d, G = 24, 3072, 32
    x = synth.activations(M, d, nu=3.0, outliers=12, outlier_scale=50.0, seed=43)
    xb = synth.bf16_bits(x)
    P = oracle.block_gram_positions(xb, G)
    X = x.to(torch.float64).numpy().reshape(M * (d // 32 // G), G, 32)
    want = np.einsum("tbk,tck->kbc", X, X) / X.shape[0]
    assert P.shape == (32, G, G) and np.abs(P - want).max() <= 1e-12 * np.abs(want).max()
    assert np.abs(P.sum(axis=0) - oracle.block_gram(xb, G)).max() <= 1e-12 * np.abs(want).max()
    assert all(np.array_equal(P[k], P[k].T) for k in range(32))
    # position k of block b varies over the rows as a known sequence: x[m][32 b + k] = (b + 1) * s_k(m)
    # with s_k(m) = 1 if m % 32 == k else 0: Sigma_k[b][b'] = (b + 1)(b' + 1) / 32 for every k
    G2 = 16
    x2 = torch.zeros((32, 32 * G2), dtype=torch.float32)
    for m in range(32):
        for b in range(G2):
            x2[m, 32 * b + m] = b + 1.0
    P2 = oracle.block_gram_positions(synth.bf16_bits(x2.to(torch.bfloat16)), G2)
    outer = np.outer(np.arange(1, G2 + 1), np.arange(1, G2 + 1)) / 32.0
    assert all(np.array_equal(P2[k], outer) for k in range(32))
    # only position 5 is ever non-zero: every other matrix is zero, and an antisymmetric pair of blocks
    # gives a negative off-diagonal entry (the order of the two factors and their signs)
    x3 = torch.zeros((2, 32 * G2), dtype=torch.float32)
    x3[0, 32 * 3 + 5], x3[0, 32 * 9 + 5] = 2.0, -3.0
    x3[1, 32 * 3 + 5] = 1.0
    P3 = oracle.block_gram_positions(synth.bf16_bits(x3.to(torch.bfloat16)), G2)
    assert np.count_nonzero(P3[np.arange(32) != 5]) == 0
    assert P3[5, 3, 3] == 2.5 and P3[5, 9, 9] == 4.5 and P3[5, 3, 9] == -3.0 and P3[5, 9, 3] == -3.0
    assert np.count_nonzero(P3[5]) == 4


def test_rotating_with_the_equalizer_of_the_sample_gram_equalizes_block_energies(oracle):
    # Sections 4.2 / 5.1 end to end on the oracle: Gram of a sample -> Algorithm 1 -> rotate that
    # sample -> Gram of the result has a constant diagonal (and is R Sigma R^T)
    M, d, G = 96, 2048, 32
    x = synth.activations(M, d, nu=3.0, outliers=10, outlier_scale=50.0, seed=43)
    xb = synth.bf16_bits(x)
    Sigma = oracle.block_gram(xb, G)
    c = np.trace(Sigma) / G
    R, _, steps = oracle.equalize(Sigma, eps=1e-12 * c)
    assert 0 < steps <= G - 1
    X = x.to(torch.float64).numpy()
    Y = oracle.rotate_inter(X, G, R.astype(np.float32))
    Yg = Y.reshape(M * (d // 32 // G), G, 32)
    energies = (Yg ** 2).sum(axis=2).mean(axis=0)
    assert np.abs(energies - c).max() < 1e-5 * c
    before = np.diag(Sigma)
    assert before.max() / before.min() > 20.0
