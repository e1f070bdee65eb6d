"""Oracle: CAP-Decoding, the conflict-aware choice of positions to decode (paper Sec. 4.3, Alg. 1).

TEST INFRASTRUCTURE (see oracle/__init__.py).  fp64.

For the masked positions of the current block: pool the positions whose
confidence reaches tau_low (Eq. 5); two pooled positions i, j conflict when
D_ij = log p_i(y_j) + log p_j(y_i) > gamma (Eq. 6, strict); phase 1 takes every
pooled position with confidence >= tau_high and drops from the pool whatever
conflicts with one of them; phase 2 walks the rest in descending confidence
(ties: lower position first), taking a position and dropping its conflicts;
if nothing was taken the most confident masked position is decoded alone.

mode 0 is the algorithm above.  mode 1 (confidence threshold: every masked
position with c >= tau_high, else the single most confident one) and mode 2
(the single most confident one) are the comparison rules of Sec. 5.1.
"""
import numpy as np


def conflict_score(z, lse, yhat, i, j):
    """D_ij of Eq. 6 with log p_i(v) = z[i, v] - lse[i]."""
    return (float(z[i, yhat[j]]) - float(lse[i])) + (float(z[j, yhat[i]]) - float(lse[j]))


def select_parallel(z, lse, conf, yhat, eligible, tau_low, tau_high, gamma, mode=0):
    """Returns (selected bool [L], margin).

    z [L, V] logits of the block rows, lse/conf/yhat [L] their statistics,
    eligible [L] bool = position still holds the mask token.
    margin = smallest distance of any examined quantity from the threshold or
    neighbour that decides it.
    """
    L = len(conf)
    conf = np.asarray(conf, dtype=np.float64)
    lse = np.asarray(lse, dtype=np.float64)
    E = [i for i in range(L) if eligible[i]]
    sel = np.zeros(L, dtype=bool)
    margin = np.inf
    if not E:
        return sel, margin
    order_E = sorted(E, key=lambda i: (-conf[i], i))
    top = order_E[0]
    top_gap = np.inf  # exact ties are decided by position on both sides, so they limit nothing
    if len(E) > 1 and conf[order_E[0]] != conf[order_E[1]]:
        top_gap = conf[order_E[0]] - conf[order_E[1]]

    if mode == 2:
        sel[top] = True
        return sel, float(top_gap)
    if mode == 1:
        for i in E:
            margin = min(margin, abs(conf[i] - tau_high))
            sel[i] = conf[i] >= tau_high
        if not sel.any():
            sel[top] = True
            margin = min(margin, top_gap)
        return sel, float(margin)

    for i in E:
        margin = min(margin, abs(conf[i] - tau_low), abs(conf[i] - tau_high))
    pool = [i for i in E if conf[i] >= tau_low]
    D = {}
    for a in pool:
        for b in pool:
            if a != b:
                D[(a, b)] = conflict_score(z, lse, yhat, a, b)
                margin = min(margin, abs(D[(a, b)] - gamma))

    def conflicts(a, b):
        return D[(a, b)] > gamma

    S1 = [i for i in pool if conf[i] >= tau_high]
    for i in S1:
        sel[i] = True
    rest = [j for j in pool if j not in S1 and not any(conflicts(i, j) for i in S1)]
    rest.sort(key=lambda i: (-conf[i], i))
    for a, b in zip(rest, rest[1:]):
        if conf[a] != conf[b]:
            margin = min(margin, conf[a] - conf[b])
    while rest:
        i = rest.pop(0)
        sel[i] = True
        rest = [j for j in rest if not conflicts(i, j)]
    if not sel.any():
        sel[top] = True
        margin = min(margin, top_gap)
    return sel, float(margin)
