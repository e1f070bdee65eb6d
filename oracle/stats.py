"""Oracle: per-position predictive statistics over the vocabulary.

TEST INFRASTRUCTURE (see oracle/__init__.py).  fp64, natural logarithm.

Definitions (paper Sec. 4.2 and 4.3): confidence c = max_v p(v), prediction
y = argmax_v p(v), predictive uncertainty H = Shannon entropy of p^curr,
last-block influence I = KL(p^curr || p^prev) (Eq. 3).  p = softmax(z) with the
mask token excluded (the final sequence must be mask-free, Sec. 3), i.e.
z[mask_id] = -inf before anything else.  argmax ties go to the lowest token id.
"""
import numpy as np

from .forward import widen


def log_softmax_masked(z, mask_id):
    """log p over the vocabulary with the mask token's probability forced to 0."""
    z = widen(z).copy()
    z[..., mask_id] = -np.inf
    m = z.max(axis=-1, keepdims=True)
    lse = m + np.log(np.sum(np.exp(z - m), axis=-1, keepdims=True))
    return z - lse, lse[..., 0], m[..., 0]


def vocab_stats(z, mask_id, z_prev=None):
    """Statistics of each row of logits z [rows, V].

    Returns dict: max_logit, lse, argmax, conf, entropy, and kl (Eq. 3, only if
    z_prev [rows, V] is given; the same mask suppression applies to z_prev).
    """
    logp, lse, m = log_softmax_masked(z, mask_id)
    p = np.exp(logp)
    yhat = np.argmax(logp, axis=-1)  # first occurrence = lowest token id
    rows = np.arange(logp.shape[0])
    conf = p[rows, yhat]
    keep = np.ones(logp.shape[-1], dtype=bool)
    keep[mask_id] = False  # p = 0 there; 0 * log 0 := 0
    entropy = -np.sum(p[:, keep] * logp[:, keep], axis=-1)
    out = dict(max_logit=m, lse=lse, argmax=yhat, conf=conf, entropy=entropy)
    if z_prev is not None:
        logq, _, _ = log_softmax_masked(z_prev, mask_id)
        out["kl"] = np.sum(p[:, keep] * (logp[:, keep] - logq[:, keep]), axis=-1)
    return out
