"""Pins for oracle/boundary.py: hand-worked cases, exhaustive scan, invariants of Sec. 4.2."""
import numpy as np
import pytest

from oracle.boundary import block_boundary, dependency_score, normalise, smooth

RNG = np.random.default_rng(2)


def test_hand_worked_raw_scores():
    I, H = [4.0, 2.0, 1.0, 1.0], [1.0, 1.0, 2.0, 4.0]
    L, S, m = block_boundary(I, H, lam=1.0, l_min=1, r=0, norm_mode=3)
    assert S.tolist() == [3.0, 1.0, -1.0, -3.0] and L == 2 and m == 1.0
    assert block_boundary(I, H, 1.0, 3, 0, 3)[0] == 3  # clipped up to L_min
    assert block_boundary(I, H, 1.0, 9, 0, 3)[0] == 4  # the window wins over L_min
    assert block_boundary(I, H, 0.1, 1, 0, 3)[0] == 4  # no crossing: whole window
    assert block_boundary(I, H, 5.0, 1, 0, 3)[0] == 1  # crossing at k = 0 then L_min
    # cumulative rule: partial sums 3, 4, 3, 0 -> never negative; with lam = 2: 2, 2, -1 -> L_raw = 2
    assert block_boundary(I, H, 1.0, 1, 0, 3, rule=1)[0] == 4
    L, _, m = block_boundary(I, H, 2.0, 1, 0, 3, rule=1)
    assert L == 2 and m == 1.0
    assert block_boundary(I, H, 1.0, 2, cold_start=True)[0] == 2
    assert block_boundary(I, H, 1.0, 8, cold_start=True)[0] == 4


def test_hand_worked_smoothing_and_normalisation():
    np.testing.assert_allclose(smooth([4.0, 2.0, 1.0, 1.0], 1), [3.0, 7 / 3, 4 / 3, 1.0], rtol=1e-15)
    np.testing.assert_allclose(smooth([4.0, 2.0, 1.0, 1.0], 2), [7 / 3, 2.0, 2.0, 4 / 3], rtol=1e-15)
    x = np.array([1.0, 3.0, 4.0])
    np.testing.assert_allclose(normalise(x, 0), x / (8 / 3), rtol=1e-11)
    np.testing.assert_allclose(normalise(x, 1), x / 4, rtol=1e-11)
    np.testing.assert_allclose(normalise(x, 2), [0, 2 / 3, 1.0], atol=1e-11)
    # mean-normalised, r = 0, lam = 1: S_k = I_k/mean(I) - H_k/mean(H)
    S = dependency_score([2.0, 1.0, 0.0], [1.0, 1.0, 4.0], 1.0, 0, 0)
    np.testing.assert_allclose(S, [2 - 0.5, 1 - 0.5, 0 - 2.0], atol=1e-10)


def _exhaustive(I, H, lam, l_min, r, mode, rule):
    W = len(I)
    sm = lambda x: np.array([np.mean(x[max(0, k - r): k + r + 1]) for k in range(W)])
    Is, Hs = sm(np.asarray(I)), sm(np.asarray(H))
    def nrm(x):
        if mode == 0: return x / (x.sum() / W + 1e-12)
        if mode == 1: return x / (x.max() + 1e-12)
        if mode == 2: return (x - x.min()) / (x.max() - x.min() + 1e-12)
        return x
    S = nrm(Is) - lam * nrm(Hs)
    best = W
    for k in range(W - 1, -1, -1):  # scan every k, keep the smallest negative one
        q = S[k] if rule == 0 else S[: k + 1].sum()
        if q < 0:
            best = k
    return min(max(best, l_min), W)


@pytest.mark.parametrize("rule", [0, 1])
@pytest.mark.parametrize("mode", [0, 1, 2, 3])
def test_exhaustive_scan(mode, rule):
    for trial in range(200):
        W = int(RNG.integers(1, 40))
        I = RNG.exponential(0.3, W) * np.exp(-np.arange(W) / RNG.uniform(2, 30))
        H = RNG.uniform(0.1, 5.0, W)
        lam = float(RNG.choice([0.6, 0.8, 1.0, 1.2, 1.4, 1.6]))
        r, l_min = int(RNG.integers(0, 4)), int(RNG.integers(1, 12))
        L, S, m = block_boundary(I, H, lam, l_min, r, mode, rule)
        assert L == _exhaustive(I, H, lam, l_min, r, mode, rule)
        assert min(l_min, W) <= L <= W and m >= 0


def test_invariants():
    for trial in range(100):
        W = int(RNG.integers(2, 64))
        I = RNG.exponential(0.3, W) * np.exp(-np.arange(W) / 10.0) + 1e-3
        H = RNG.uniform(0.5, 5.0, W)
        for lam in (0.6, 1.2):
            S = dependency_score(I, H, lam, 1, 0)
            np.testing.assert_allclose(S.sum(), W * (1 - lam), rtol=1e-9, atol=1e-9)
        # positive rescaling of either signal changes nothing under mean normalisation
        a = block_boundary(I, H, 0.9, 4)
        b = block_boundary(I * 7.5, H * 0.01, 0.9, 4)
        assert a[0] == b[0]
        np.testing.assert_allclose(a[1], b[1], rtol=1e-9, atol=1e-9)
        # more uncertainty penalty never lengthens the block
        Ls = [block_boundary(I, H, lam, 1)[0] for lam in (0.2, 0.6, 0.8, 1.0, 1.2, 1.6)]
        assert all(x >= y for x, y in zip(Ls, Ls[1:]))
        assert block_boundary(I, H, 1e-9, 1)[0] == W
        np.testing.assert_array_equal(smooth(I, 0), I)
    W = 16
    H = RNG.uniform(0.5, 5.0, W)
    assert block_boundary(np.zeros(W), H, 1.2, 8)[0] == 8  # identical steps: no support, L = L_min
    assert block_boundary(np.zeros(W), np.zeros(W), 1.2, 8)[0] == W  # S == 0 is not negative
