"""Pins for the oracle's intra-block calibration pieces (Section 5.2, Algorithm 2, Appendix A.4 and
A.5): closed forms worked by hand, brute force over a dense grid of angles on tiny inputs, the
symmetries of the problem, and the link back to the pinned quantiser (the occupancy that Algorithm 2
reports must be the occupancy of the codes that the quantiser emits for the rotated sample).
"""
import math

import numpy as np
import pytest

import oracle

THRESH = [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]


# ------------------------------------------------------------------ magnitude codeword --

def test_mag_code_agrees_with_the_pinned_element_quantiser():
    vals = list(np.linspace(-7.0, 7.0, 2801))
    for t in THRESH:
        f = np.float32(t)
        vals += [t, -t, float(np.nextafter(f, np.float32(10))), float(np.nextafter(f, np.float32(0)))]
    vals += [0.0, -0.0, 1e-30, 6.0, 6.5, 1e9, -1e9]
    for a in vals:
        a = float(np.float32(a))
        assert oracle.mag_code(a) == (oracle.e2m1_from_f32(a) & 7), a


def test_mag_code_is_decided_in_double():
    # a double that rounds to the boundary as a float still lies on its own side of it
    assert oracle.mag_code(0.25 + 1e-12) == 1
    assert oracle.mag_code(0.75 - 1e-12) == 1
    assert oracle.mag_code(5.0 + 1e-12) == 7


# ------------------------------------------------------------------ histogram --

def _pack(codes):
    codes = np.asarray(codes, np.uint8)
    return (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)


def test_histogram_of_constructed_codes():
    M, d = 5, 96
    codes = np.zeros((M, d), np.uint8)
    for j in range(d):
        codes[:, j] = (j % 32) % 8            # position k always carries codeword k % 8
    h = oracle.code_histogram(_pack(codes), d)
    want = np.zeros((32, 8), np.uint64)
    for k in range(32):
        want[k, k % 8] = M * (d // 32)
    assert np.array_equal(h, want)


def test_histogram_ignores_sign_and_matches_bincount():
    rng = np.random.default_rng(5)
    M, d = 37, 160
    codes = rng.integers(0, 16, size=(M, d), dtype=np.uint8)
    h = oracle.code_histogram(_pack(codes), d)
    assert np.array_equal(h, oracle.code_histogram(_pack(codes ^ 8), d))
    assert h.sum() == M * d and np.all(h.sum(axis=1) == M * d // 32)
    for k in range(32):
        col = codes[:, k::32].reshape(-1) & 7
        assert np.array_equal(h[k], np.bincount(col, minlength=8).astype(np.uint64))


def test_histogram_separates_the_two_nibbles():
    d = 32
    codes = np.zeros((1, d), np.uint8)
    codes[0, 0] = 3                            # even element: low nibble of byte 0
    codes[0, 1] = 5                            # odd element: high nibble of byte 0
    h = oracle.code_histogram(_pack(codes), d)
    assert h[0, 3] == 1 and h[1, 5] == 1 and h[0, 5] == 0 and h[1, 3] == 0


# ------------------------------------------------------------------ loss and scores --

def test_code_loss_closed_forms():
    assert oracle.code_loss(np.full(8, 7)) == 0.0
    one_hot = np.zeros(8, np.uint64)
    one_hot[3] = 11
    assert oracle.code_loss(one_hot) == pytest.approx((7 / 8) ** 2 + 7 / 64, abs=1e-15)
    two = np.zeros(8, np.uint64)
    two[0] = two[7] = 5
    assert oracle.code_loss(two) == pytest.approx(2 * (3 / 8) ** 2 + 6 / 64, abs=1e-15)
    # identity with the sum of squares: sum (p - 1/8)^2 = sum p^2 - 1/8
    n = np.array([5, 0, 9, 1, 1, 30, 2, 4], np.uint64)
    p = n / n.sum()
    assert oracle.code_loss(n) == pytest.approx(float((p * p).sum() - 1 / 8), abs=1e-15)


def test_pair_scores_closed_forms():
    counts = np.full((32, 8), 10, np.uint64)
    counts[0] = 0
    counts[0, 0] = 80                          # column 0: everything on codeword 0
    counts[1] = 0
    counts[1, 1] = 80                          # column 1: everything on codeword 1
    counts[2] = counts[0]                      # column 2: a copy of column 0
    lam = 0.5
    h, H = oracle.pair_scores(counts, lam)
    assert h[0] == pytest.approx(0.875) and h[1] == pytest.approx(0.875) and np.all(h[3:] == 0.0)
    # c_01 = -[2 (7/8)(-1/8) + 6/64] = 1/8 ; c_02 = -h_0 ; a uniform partner contributes nothing
    assert H[0, 1] == pytest.approx(1.75 + lam * 0.125)
    assert H[0, 2] == pytest.approx(1.75 - lam * 0.875)
    assert H[0, 5] == pytest.approx(0.875)
    assert H[4, 5] == 0.0
    assert np.allclose(H, H.T, atol=0)
    assert H[0, 1] > H[0, 2]                   # the complementary partner is preferred to the similar one


def test_pair_scores_do_not_depend_on_the_sample_count():
    rng = np.random.default_rng(1)
    counts = rng.integers(1, 50, size=(32, 8)).astype(np.uint64)
    h1, H1 = oracle.pair_scores(counts, 2.0)
    h2, H2 = oracle.pair_scores(counts * 3, 2.0)
    assert np.allclose(h1, h2, atol=1e-15) and np.allclose(H1, H2, atol=1e-15)


# ------------------------------------------------------------------ exact angle solver --

def _loss_numpy(u, v, rest, theta):
    """Occupancy loss of one angle, written with library calls only (digitize on the interval
    midpoints is safe here because grid angles never put a sample exactly on a boundary)."""
    c, s = math.cos(theta), math.sin(theta)
    a = np.abs(np.concatenate([u * c + v * s, -u * s + v * c]))
    n = np.bincount(np.digitize(a, THRESH), minlength=8) + np.asarray(rest, np.int64)
    p = n / n.sum()
    return float(((p - 0.125) ** 2).sum())


def test_best_angle_single_sample_by_hand():
    # one sample (3, 0): near theta = 0 the pair reads (3, 0) -> codewords 5 and 0, two different
    # bins, the best possible for two counts: loss 2 (1/2 - 1/8)^2 + 6/64 = 3/8.  The interval that
    # holds theta = 0 wraps around 2 pi and its midpoint is the smallest candidate.
    th, lo, k = oracle.best_angle([3.0], [0.0], np.zeros(8, np.uint64))
    assert lo == pytest.approx(0.375, abs=1e-15)
    assert min(th, 2 * math.pi - th) < 1e-12
    # critical angles: boundaries 0.25 .. 2.5 are below r = 3 -> 5 boundaries x 2 axes x 4 angles
    assert k == 40


def test_best_angle_without_critical_angles():
    th, lo, k = oracle.best_angle([0.1, -0.05], [0.02, 0.1], np.array([0, 3, 0, 0, 0, 0, 0, 0], np.uint64))
    assert k == 0 and th == 0.0
    n = np.array([4, 3, 0, 0, 0, 0, 0, 0])
    p = n / 7
    assert lo == pytest.approx(float(((p - 0.125) ** 2).sum()), abs=1e-15)


@pytest.mark.parametrize("seed,n,scale", [(0, 6, 2.0), (1, 12, 1.0), (2, 25, 3.0), (3, 40, 0.7)])
def test_best_angle_beats_a_dense_grid(seed, n, scale):
    rng = np.random.default_rng(seed)
    u = rng.standard_normal(n) * scale
    v = rng.standard_normal(n) * scale * 0.3
    rest = rng.integers(0, 3 * n, size=8).astype(np.uint64)
    th, lo, k = oracle.best_angle(u, v, rest)
    assert 0.0 <= th < 2 * math.pi and k > 0
    assert lo == pytest.approx(_loss_numpy(u, v, rest, th), abs=1e-14)       # the reported loss is the loss there
    grid = [_loss_numpy(u, v, rest, t) for t in np.linspace(0, 2 * math.pi, 40001)[:-1] + 1e-7]
    assert lo <= min(grid) + 1e-14
    # with this few samples the grid is finer than almost every interval: it reaches the optimum too
    assert min(grid) <= lo + 1e-14 or n >= 25
    # the loss is constant on the interval around the midpoint
    assert _loss_numpy(u, v, rest, th + 1e-9) == pytest.approx(lo, abs=1e-14)
    assert _loss_numpy(u, v, rest, th - 1e-9) == pytest.approx(lo, abs=1e-14)


def test_best_angle_symmetries():
    rng = np.random.default_rng(9)
    u = rng.standard_normal(15) * 2
    v = rng.standard_normal(15)
    rest = rng.integers(0, 20, size=8).astype(np.uint64)
    _, lo, k = oracle.best_angle(u, v, rest)
    for uu, vv in ((v, u), (-u, v), (u, -v), (-u, -v)):
        _, l2, k2 = oracle.best_angle(uu, vv, rest)
        assert l2 == pytest.approx(lo, abs=1e-15) and k2 == k


def test_best_angle_never_worse_than_no_rotation():
    rng = np.random.default_rng(4)
    for _ in range(5):
        u = rng.standard_t(3, size=30)
        v = rng.standard_t(3, size=30) * 0.2
        rest = rng.integers(0, 60, size=8).astype(np.uint64)
        _, lo, _ = oracle.best_angle(u, v, rest)
        assert lo <= _loss_numpy(u, v, rest, 0.0) + 1e-15


def test_best_angle_depends_on_rest():
    # two samples (1, 0) and (1, 0).  Unrotated the pair fills codewords 2 and 0.  If the other
    # columns already crowd codewords 0 and 2, some other angle is strictly better.
    u, v = [1.0, 1.0], [0.0, 0.0]
    crowded = np.array([50, 0, 50, 0, 0, 0, 0, 0], np.uint64)
    th, lo, _ = oracle.best_angle(u, v, crowded)
    assert lo < _loss_numpy(np.array(u), np.array(v), crowded, 0.0) - 1e-6
    # at 45 degrees both coordinates are 0.707 -> codeword 1, which is empty: that is the optimum
    want = _loss_numpy(np.array(u), np.array(v), crowded, math.pi / 4)
    assert lo == pytest.approx(want, abs=1e-15)


# ------------------------------------------------------------------ Algorithm 2 --

def _loss_through_quantiser(X, R):
    """Occupancy loss of the sample under R, from the codes the pinned quantiser emits."""
    Z = (X @ R).astype(np.float32)
    codes, _ = oracle.quantize(Z)
    return oracle.code_loss(oracle.code_histogram(codes, 32).sum(axis=0))


def _sample(seed, n):
    rng = np.random.default_rng(seed)
    X = rng.standard_t(3, size=(n, 32))
    X[:, 5] *= 6.0                             # one heavy column, as activation channels have
    return X


def test_algorithm2_zero_iterations_is_identity():
    X = _sample(0, 50)
    R, losses = oracle.intra_rotation(X, 0, 16, 8, 1.0, 0.0)
    assert np.array_equal(R, np.eye(32)) and len(losses) == 1
    assert losses[0] == pytest.approx(_loss_through_quantiser(X, np.eye(32)), abs=1e-12)


def test_algorithm2_reports_the_quantisers_occupancy_and_descends():
    X = _sample(1, 240)
    R, losses = oracle.intra_rotation(X, 4, 16, 8, 1.0, 0.0)
    assert np.abs(R.T @ R - np.eye(32)).max() < 1e-13
    assert len(losses) == 5 and np.all(np.diff(losses) < 0)
    assert losses[0] == pytest.approx(_loss_through_quantiser(X, np.eye(32)), abs=1e-12)
    # the sample values are doubles but the quantiser reads floats: away from ties (measure zero
    # for this sample) both see the same codes
    assert min(losses) == pytest.approx(_loss_through_quantiser(X, R), abs=1e-12)
    assert min(losses) < 0.6 * losses[0]


def test_algorithm2_stops_when_the_loss_stalls():
    X = _sample(2, 120)
    _, losses = oracle.intra_rotation(X, 6, 16, 8, 1.0, 1e9)     # no drop can exceed eps
    assert len(losses) == 2                     # the first pass always takes its R-step, the second stops


def test_algorithm2_pool_and_pair_limits():
    X = _sample(3, 120)
    # one pair from a pool of two: exactly the two most imbalanced columns are turned
    R, losses = oracle.intra_rotation(X, 1, 2, 1, 1.0, 0.0)
    moved = [k for k in range(32) if not np.array_equal(R[:, k], np.eye(32)[:, k])]
    Z = X / np.exp2(np.floor(np.log2(np.abs(X).max(axis=1, keepdims=True))) - 2)
    counts = np.stack([np.bincount(np.digitize(np.abs(Z[:, k]), THRESH), minlength=8) for k in range(32)])
    h, _ = oracle.pair_scores(counts.astype(np.uint64), 1.0)
    top2 = sorted(np.argsort(-h, kind="stable")[:2].tolist())
    assert moved == top2
    # the 2x2 block that moved is a rotation by one angle
    p, q = moved
    blk = R[np.ix_([p, q], [p, q])]
    assert blk[0, 0] == pytest.approx(blk[1, 1]) and blk[0, 1] == pytest.approx(-blk[1, 0])
    assert np.linalg.det(blk) == pytest.approx(1.0)
    # that one turn is the exact solver's answer for those two columns of the normalised sample
    rest = (counts.sum(axis=0) - counts[p] - counts[q]).astype(np.uint64)
    th, lo, _ = oracle.best_angle(Z[:, p], Z[:, q], rest)
    assert blk[0, 0] == pytest.approx(math.cos(th), abs=1e-12) and blk[1, 0] == pytest.approx(math.sin(th), abs=1e-12)
    assert losses[1] <= losses[0]


@pytest.mark.parametrize("seed,n,k_top,P", [(4, 150, 6, 3), (100, 10, 8, 4), (101, 10, 8, 4), (101, 24, 8, 4), (102, 10, 8, 4)])
def test_algorithm2_later_pairs_see_the_earlier_turns(seed, n, k_top, P):
    """Replay one R-step of several pairs outside the oracle: every pair's turn must be the exact
    solver's answer for the columns and the occupancy as the earlier turns of the same step left them.  The small samples are the sensitive ones:
    with few counts per bin a stale occupancy changes the best interval."""
    X = _sample(seed, n)
    lam = 1.5
    R, _ = oracle.intra_rotation(X, 1, k_top, P, lam, 0.0)
    Z = X / np.exp2(np.floor(np.log2(np.abs(X).max(axis=1, keepdims=True))) - 2)

    def hist(Z):
        return np.stack([np.bincount(np.digitize(np.abs(Z[:, k]), THRESH), minlength=8) for k in range(32)]).astype(np.uint64)

    counts = hist(Z)
    h, H = oracle.pair_scores(counts, lam)
    pool = sorted(np.argsort(-h, kind="stable")[:k_top].tolist())
    used, want = set(), np.eye(32)
    for _ in range(P):
        cand = [(H[p, q], -p, -q) for p in pool for q in pool if p < q and p not in used and q not in used]
        _, p, q = max(cand)
        p, q = -p, -q
        used |= {p, q}
        counts = hist(Z)
        rest = (counts.sum(axis=0) - counts[p] - counts[q]).astype(np.uint64)
        th, _, _ = oracle.best_angle(Z[:, p], Z[:, q], rest)
        G = np.eye(32)
        G[p, p] = G[q, q] = math.cos(th)
        G[q, p] = math.sin(th)
        G[p, q] = -math.sin(th)
        Z = Z @ G
        want = want @ G
    assert len(used) == 2 * P
    assert np.abs(R - want).max() < 1e-12
