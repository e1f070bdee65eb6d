"""Pins for oracle/select.py: a hand-worked case, an independent set-recursive Alg. 1, invariants."""
import itertools
import math

import numpy as np
import pytest

from oracle.select import conflict_score, select_parallel
from oracle.stats import vocab_stats
from paper_2604_15750_amd.inputs import peaked_logits

RNG = np.random.default_rng(3)


def _stats(z, mask):
    st = vocab_stats(z, mask)
    return st["lse"], st["conf"], st["argmax"]


def _logits_from_probs(P):
    """Rows of probabilities over V-1 real tokens -> logits with a trailing mask column."""
    P = np.asarray(P, dtype=np.float64)
    return np.concatenate([np.log(P), np.zeros((P.shape[0], 1))], axis=1)


def test_hand_worked_case():
    # 4 tokens + mask.  rows 0,1: confident (0.96 on token 0 / token 1); row 2: 0.85 on token 2;
    # row 3: 0.84 on token 0; row 4: 0.5 (below tau_low).
    P = [[0.96, 0.02, 0.01, 0.01],
         [0.01, 0.96, 0.02, 0.01],
         [0.05, 0.05, 0.85, 0.05],
         [0.84, 0.01, 0.05, 0.10],
         [0.5, 0.3, 0.1, 0.1]]
    z = _logits_from_probs(P)
    lse, conf, yh = _stats(z, 4)
    assert yh.tolist() == [0, 1, 2, 0, 0]
    # D_03 = log p0(y3=0) + log p3(y0=0) = log .96 + log .84;  D_23 = log p2(0) + log p3(2) = log .05 + log .05
    np.testing.assert_allclose(conflict_score(z, lse, yh, 0, 3), math.log(0.96) + math.log(0.84), rtol=1e-13)
    np.testing.assert_allclose(conflict_score(z, lse, yh, 2, 3), 2 * math.log(0.05), rtol=1e-13)
    elig = np.ones(5, dtype=bool)
    # gamma = -1: only (0,3) conflicts [-0.215]; D_01 = log .02 + log .01 = -8.5; D_02 = log .01 + log .05 = -7.6 ...
    sel, _ = select_parallel(z, lse, conf, yh, elig, 0.8, 0.95, -1.0)
    assert sel.tolist() == [True, True, True, False, False]  # 3 dropped by phase 1, 2 taken in phase 2
    # gamma = -7: (0,3), (2,3) [-6.0], and (1,2) [log .02 + log .05 = -6.9] conflict; (0,2) [-7.6] does not
    sel, _ = select_parallel(z, lse, conf, yh, elig, 0.8, 0.95, -7.0)
    assert sel.tolist() == [True, True, False, False, False]
    # phase 1 keeps both 0 and 1 even if they conflict with each other (gamma below D_01)
    sel, _ = select_parallel(z, lse, conf, yh, elig, 0.8, 0.95, -9.0)
    assert sel.tolist() == [True, True, False, False, False]
    # no phase-1 member: greedy by confidence 0 (.96), 1 (.96, later index), 2, 3
    sel, _ = select_parallel(z, lse, conf, yh, elig, 0.8, 0.99, -1.0)
    assert sel.tolist() == [True, True, True, False, False]
    sel, _ = select_parallel(z, lse, conf, yh, elig, 0.8, 0.99, -8.0)  # 0 first; drops 3 (-0.2) and 2 (-7.6); 1 stays (-8.5)
    assert sel.tolist() == [True, True, False, False, False]
    # row 0 already decoded: pool {1,2,3}
    elig[0] = False
    sel, _ = select_parallel(z, lse, conf, yh, elig, 0.8, 0.99, -7.0)  # 1 first, drops 2 (-6.9); 3 vs 1: log .01+log .01
    assert sel.tolist() == [False, True, False, True, False]
    # fallback: thresholds out of reach -> the single most confident eligible position
    sel, _ = select_parallel(z, lse, conf, yh, elig, 0.97, 0.99, -7.0)
    assert sel.tolist() == [False, True, False, False, False]
    assert not select_parallel(z, lse, conf, yh, np.zeros(5, bool), 0.8, 0.95, -7.0)[0].any()
    # comparison rules
    elig[:] = True
    assert select_parallel(z, lse, conf, yh, elig, 0.8, 0.9, 0.0, mode=1)[0].tolist() == [True, True, False, False, False]
    assert select_parallel(z, lse, conf, yh, elig, 0.8, 0.999, 0.0, mode=1)[0].tolist() == [True, False, False, False, False]
    assert select_parallel(z, lse, conf, yh, elig, 0.8, 0.9, 0.0, mode=2)[0].tolist() == [True, False, False, False, False]


def _alg1_sets(z, mask, elig, tau_low, tau_high, gamma):
    """Alg. 1 written over Python sets with p computed directly (independent of the oracle's path)."""
    zz = np.array(z, dtype=np.float64)
    zz[:, mask] = -np.inf
    p = np.exp(zz - zz.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    c, yh = p.max(-1), p.argmax(-1)
    MB = {i for i in range(len(c)) if elig[i]}
    C = {i for i in MB if c[i] >= tau_low}
    D = {(i, j): math.log(p[i, yh[j]]) + math.log(p[j, yh[i]]) for i in C for j in C if i != j}
    S = {i for i in C if c[i] >= tau_high}
    C = {j for j in C - S if all(D[(i, j)] <= gamma for i in S)}

    def greedy(C, S):
        if not C:
            return S
        i = min(C, key=lambda i: (-c[i], i))
        return greedy({j for j in C if j != i and D[(i, j)] <= gamma}, S | {i})

    S = greedy(C, S)
    if not S and MB:
        S = {min(MB, key=lambda i: (-c[i], i))}
    return S, D, c


def _random_case(seed):
    rng = np.random.default_rng(seed)
    L, V = int(rng.integers(1, 11)), 40
    peaks = []
    for r in range(L):
        if rng.random() < 0.7:
            peaks.append((r, int(rng.integers(0, 6)), float(rng.uniform(4, 16))))
        if rng.random() < 0.5:  # a strong runner-up makes pairs entangled
            peaks.append((r, int(rng.integers(0, 6)), float(rng.uniform(6, 12))))
    z = peaked_logits(L, V, seed, peaks, sigma=2.0, dtype=np.float64)
    elig = rng.random(L) < 0.8
    return z, elig, V - 1


@pytest.mark.parametrize("gamma", [-4.0, -8.0, -16.0])
def test_against_set_recursive_alg1(gamma):
    fired = dict(phase1=0, phase2=0, fallback=0, dropped=0)
    for seed in range(400):
        z, elig, mask = _random_case(seed)
        lse, conf, yh = _stats(z, mask)
        tau_low, tau_high = 0.6, 0.93
        sel, margin = select_parallel(z, lse, conf, yh, elig, tau_low, tau_high, gamma)
        S, D, c = _alg1_sets(z, mask, elig, tau_low, tau_high, gamma)
        assert set(np.nonzero(sel)[0]) == S
        # invariants
        E = set(np.nonzero(elig)[0])
        assert S <= E and (len(S) >= 1) == (len(E) >= 1)
        if E:
            assert min(E, key=lambda i: (-c[i], i)) in S
        pool = {i for i in E if c[i] >= tau_low}
        S1 = {i for i in pool if c[i] >= tau_high}
        for i, j in itertools.combinations(sorted(S), 2):
            if not (i in S1 and j in S1):
                assert D[(i, j)] <= gamma  # conflict-free outside phase 1
        for j in pool - S:
            assert any(D[(i, j)] > gamma for i in S)  # maximal
        for (i, j), v in D.items():
            assert v == D[(j, i)]
        fired["phase1"] += bool(S1)
        fired["phase2"] += bool(S - S1 and pool)
        fired["fallback"] += bool(E and not pool)
        fired["dropped"] += bool(pool - S)
    assert all(v > 10 for v in fired.values()), fired


def test_limits_reduce_to_simpler_rules():
    for seed in range(100):
        z, elig, mask = _random_case(seed)
        lse, conf, yh = _stats(z, mask)
        E = np.nonzero(elig)[0]
        if E.size == 0:
            continue
        top = min(E, key=lambda i: (-conf[i], i))
        pool = {i for i in E if conf[i] >= 0.6}
        # gamma = +inf: nothing conflicts -> the whole pool (confidence-threshold decoding at tau_low)
        sel, _ = select_parallel(z, lse, conf, yh, elig, 0.6, 0.93, np.inf)
        assert set(np.nonzero(sel)[0]) == (pool or {top})
        assert sel.tolist() == select_parallel(z, lse, conf, yh, elig, 0.0, 0.6, 0.0, mode=1)[0].tolist()
        # gamma = -inf: everything conflicts -> phase 1 set, or one position
        sel, _ = select_parallel(z, lse, conf, yh, elig, 0.6, 0.93, -np.inf)
        S1 = {i for i in pool if conf[i] >= 0.93}
        assert set(np.nonzero(sel)[0]) == (S1 or {top})
        # tau_low > 1: top-1 per step
        sel, _ = select_parallel(z, lse, conf, yh, elig, 1.5, 2.0, -16.0)
        assert set(np.nonzero(sel)[0]) == {top}
        assert sel.tolist() == select_parallel(z, lse, conf, yh, elig, 0, 0, 0, mode=2)[0].tolist()
