"""Oracle: DepGA-Block boundary decision (paper Sec. 4.2, Eq. 4; Sec. 4.4 for rule 1).

TEST INFRASTRUCTURE (see oracle/__init__.py).  fp64.

Given last-block influence I_k and entropy H_k for the W = L_window candidate
positions after the frontier (k = 0 is the frontier itself), both signals are
smoothed and normalised inside the window, the dependency score
S_k = I~_k - lambda * H~_k is formed, and the next block ends immediately
before the first position whose score is negative; the length is clipped to
[L_min, W] (upper bound wins when W < L_min).

The paper does not define the smoothing or the normalisation.  This build's
reading (parity with the authors' behaviour is unpinned):
  smoothing     centred moving average of radius r, truncated at the window
                edges (divide by the number of taps present); r = 0 disables
  norm_mode 0   divide by the window mean of the smoothed signal (+ eps)
  norm_mode 1   divide by the window maximum (+ eps)
  norm_mode 2   min-max: (x - min) / (max - min + eps)
  norm_mode 3   none (raw nats, the appendix form S_k = I_k - lambda H_k)
  rule 0        first k with S_k < 0; L_raw = k (number of leading k with S_k >= 0)
  rule 1        first L >= 1 with sum_{k<L} S_k < 0; L_raw = L - 1 (cumulative form, Sec. 4.4)
"""
import numpy as np

EPS = 1e-12


def smooth(x, r):
    x = np.asarray(x, dtype=np.float64)
    W = x.shape[0]
    out = np.empty(W)
    for k in range(W):
        lo, hi = max(0, k - r), min(W - 1, k + r)
        out[k] = np.sum(x[lo : hi + 1]) / (hi - lo + 1)
    return out


def normalise(x, mode):
    if mode == 0:
        return x / (np.mean(x) + EPS)
    if mode == 1:
        return x / (np.max(x) + EPS)
    if mode == 2:
        return (x - np.min(x)) / (np.max(x) - np.min(x) + EPS)
    if mode == 3:
        return x.copy()
    raise ValueError("norm_mode")


def dependency_score(I, H, lam, r=1, norm_mode=0):
    """S_k of Eq. 4 for the whole window."""
    It = normalise(smooth(I, r), norm_mode)
    Ht = normalise(smooth(H, r), norm_mode)
    return It - lam * Ht


def block_boundary(I, H, lam, l_min, r=1, norm_mode=0, rule=0, cold_start=False):
    """Returns (L, S, margin).

    len(I) = len(H) = W = min(L_max, L_remain) >= 1 (the caller sizes the
    window).  cold_start: the first block uses L = L_min (clipped to W) and the
    signals are ignored.  margin = smallest |decision quantity| among those
    examined up to and including the crossing: the perturbation below which L
    cannot change.
    """
    W = len(I)
    assert W >= 1 and len(H) == W
    if cold_start:
        return min(l_min, W), np.zeros(W), np.inf
    S = dependency_score(I, H, lam, r, norm_mode)
    q = S if rule == 0 else np.cumsum(S)  # q[k] decides position k (rule 0) / length k+1 (rule 1)
    neg = np.nonzero(q < 0)[0]
    if neg.size:
        kstar = int(neg[0])
        L_raw = kstar
        margin = float(np.min(np.abs(q[: kstar + 1])))
    else:
        L_raw = W
        margin = float(np.min(np.abs(q)))
    L = min(max(L_raw, l_min), W)
    return L, S, margin
