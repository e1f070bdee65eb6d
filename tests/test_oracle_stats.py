"""Pins for oracle/stats.py: closed forms, library routines, the MI identity of Sec. 4.4."""
import math

import numpy as np
import scipy.special
import scipy.stats

from oracle.stats import vocab_stats

RNG = np.random.default_rng(1)


def test_uniform_and_peak():
    V, mask = 50, 49
    st = vocab_stats(np.zeros((2, V)), mask)
    np.testing.assert_allclose(st["entropy"], math.log(V - 1), rtol=1e-14)
    np.testing.assert_allclose(st["conf"], 1.0 / (V - 1), rtol=1e-14)
    assert st["argmax"].tolist() == [0, 0]  # ties: lowest id
    st = vocab_stats(np.zeros((1, V)), 0)
    assert st["argmax"].tolist() == [1]  # never the mask id
    z = RNG.standard_normal((1, V))
    z[0, 7] += 100
    st = vocab_stats(z, mask)
    assert st["argmax"][0] == 7 and st["entropy"][0] < 1e-30 and abs(st["conf"][0] - 1) < 1e-15
    # a huge logit on the mask id must not matter
    z2 = z.copy()
    z2[0, mask] = 1e4
    st2 = vocab_stats(z2, mask)
    assert st2["argmax"][0] == 7 and st2["lse"][0] == st["lse"][0]


def test_two_point_closed_forms():
    # V = 3 with mask id 2: a Bernoulli with p = sigmoid(a - b)
    a, b, a2, b2 = 0.3, -1.1, 2.0, 0.5
    z, zp = np.array([[a, b, 5.0]]), np.array([[a2, b2, -3.0]])
    p = 1 / (1 + math.exp(-(a - b)))
    q = 1 / (1 + math.exp(-(a2 - b2)))
    st = vocab_stats(z, 2, zp)
    np.testing.assert_allclose(st["entropy"], -p * math.log(p) - (1 - p) * math.log(1 - p), rtol=1e-14)
    np.testing.assert_allclose(st["kl"], p * math.log(p / q) + (1 - p) * math.log((1 - p) / (1 - q)), rtol=1e-13)
    np.testing.assert_allclose(st["conf"], p, rtol=1e-14)
    np.testing.assert_allclose(st["lse"], math.log(math.exp(a) + math.exp(b)), rtol=1e-14)
    # direction of the divergence: KL(curr || prev), not the reverse (hand values)
    z = np.log(np.array([[0.5, 0.5, 1.0]]))
    zp = np.log(np.array([[0.9, 0.1, 1.0]]))
    np.testing.assert_allclose(vocab_stats(z, 2, zp)["kl"], 0.5108256237659907, rtol=1e-13)
    np.testing.assert_allclose(vocab_stats(zp, 2, z)["kl"], 0.3680642071684971, rtol=1e-13)


def test_library_routines_and_invariances():
    V, mask = 300, 299
    z, zp = RNG.standard_normal((6, V)) * 4, RNG.standard_normal((6, V)) * 4
    st = vocab_stats(z, mask, zp)
    p = scipy.special.softmax(z[:, :mask], axis=-1)
    q = scipy.special.softmax(zp[:, :mask], axis=-1)
    np.testing.assert_allclose(st["lse"], scipy.special.logsumexp(z[:, :mask], axis=-1), rtol=1e-14)
    np.testing.assert_allclose(st["entropy"], scipy.stats.entropy(p, axis=-1), rtol=1e-13)
    np.testing.assert_allclose(st["kl"], scipy.special.rel_entr(p, q).sum(-1), rtol=1e-12)
    np.testing.assert_allclose(st["conf"], p.max(-1), rtol=1e-14)
    assert (st["argmax"] == p.argmax(-1)).all() and (st["max_logit"] == z[:, :mask].max(-1)).all()
    assert (st["kl"] > 0).all()
    assert (vocab_stats(z, mask, z)["kl"] == 0).all()
    sh = vocab_stats(z + 3.25, mask, zp - 7.5)
    for key in ("entropy", "kl", "conf"):
        np.testing.assert_allclose(sh[key], st[key], rtol=1e-11)
    np.testing.assert_allclose(sh["lse"], st["lse"] + 3.25, rtol=1e-13)
    # KL to the uniform distribution ties the KL and entropy paths together
    ku = vocab_stats(z, mask, np.zeros_like(z))["kl"]
    np.testing.assert_allclose(ku, math.log(V - 1) - st["entropy"], rtol=1e-12)


def test_expected_influence_is_conditional_mutual_information():
    """E_B[KL(p(Z|c,B) || p(Z|c))] = I(Z;B|c) (Sec. 4.4), on a toy joint."""
    nz, nb = 6, 4
    joint = RNG.random((nb, nz))
    joint /= joint.sum()
    pb, pz = joint.sum(1), joint.sum(0)
    cond = joint / pb[:, None]
    zl = np.concatenate([np.log(cond), np.zeros((nb, 1))], axis=1)  # extra column = mask id
    zprev = np.concatenate([np.log(pz)[None].repeat(nb, 0), np.zeros((nb, 1))], axis=1)
    st = vocab_stats(zl, nz, zprev)
    mi = scipy.stats.entropy(pz) + scipy.stats.entropy(pb) - scipy.stats.entropy(joint.ravel())
    np.testing.assert_allclose(np.sum(pb * st["kl"]), mi, rtol=1e-12)
    # and H(Z|B) from the per-row entropies
    np.testing.assert_allclose(np.sum(pb * st["entropy"]), scipy.stats.entropy(joint.ravel()) - scipy.stats.entropy(pb), rtol=1e-12)
