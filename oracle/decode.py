"""Oracle: block-wise decode of one sequence with DepGA-Block + CAP-Decoding.

TEST INFRASTRUCTURE (see oracle/__init__.py).

Update rules: Eq. 1 / Eq. 2 (only masked positions of the current block may be
written, each with its predicted token).  Blocks are decoded one after another
(Sec. 3, "Block-wise decoding").  The paper leaves the pass schedule to the
host block-wise process; this build's reading, computable with a prefix KV
cache (parity with the authors' behaviour is unpinned):

  pass 0 (prefill)   span = prompt + look-ahead masks [0, P+Lk), Lk = min(2*L_max, N);
                     the prompt rows are committed to the cache; the look-ahead logits
                     are kept as p^prev; the first block has L = min(L_min, N) (cold
                     start, Sec. 4.2) and the first L look-ahead rows double as the
                     block's first denoising step.
  in-block pass      span = the block [F, F+L) in its current state, against the cache;
                     nothing committed; then CAP-Decoding on the still-masked rows.
  boundary pass      once the block is mask-free and R > 0 masks remain:
                     span = block + look-ahead [F, F+L+Lk'), Lk' = min(2*L_max, R);
                     the L block rows are committed; the first W = min(L_max, R)
                     look-ahead rows are the candidates: p^curr from this pass, p^prev
                     from the previous boundary pass (when the block just decoded was
                     still all masks), giving I_k (Eq. 3) and H_k; block_boundary gives
                     the next L; the look-ahead logits become the new p^prev and the
                     first L rows double as the new block's first denoising step.

NFE counts forward passes (Sec. 5.1, metrics).

prm["dual_cache"] = 1: in-block passes also attend to the look-ahead positions after the block with the
keys and values the last prefill / boundary pass computed for them (the suffix half of a dual cache,
Sec. 5.2, Q2: DepCap is compatible with such caches), instead of seeing nothing after the block.

prm["fixed_block"] = B > 0 replaces DepGA-Block by the fixed block size of the comparison methods of
Sec. 5.1 (vanilla and confidence-threshold decoding with block size 16 / 32 / 64; CAP-Decoding alone
with block size 32): every block has min(B, remaining) positions and the boundary pass only commits
the finished block and gives the next block's first denoising step.
"""
import numpy as np

from .boundary import block_boundary
from .forward import KVCache, forward_span
from .select import select_parallel
from .stats import vocab_stats


def decode_full(cfg, W, prompt, n_gen, prm, trace=None, max_passes=None, stop_after=None):
    """prm: dict(l_min, l_max, lam, smooth_radius, norm_mode, rule, tau_low, tau_high, gamma, mode).

    Returns dict(tokens [P+N], nfe, blocks [list of L], steps [tokens written per
    denoising step]).  If trace is a list, one record per forward pass and per
    decision is appended (inputs and outputs, for replay against another
    implementation).  max_passes stops the decode early after that many forward
    passes (for sampling the first passes of a large model); the result is then partial.
    stop_after = "boundary" (or another pass kind) stops it, likewise, once a pass of that kind and
    the decisions that follow it have been taken.
    """
    mask = cfg["mask_id"]
    P, N = len(prompt), n_gen
    END = P + N
    y = np.concatenate([np.asarray(prompt, dtype=np.int64), np.full(N, mask, dtype=np.int64)])
    cache = KVCache(cfg)
    nfe, blocks, steps = 0, [], []
    l_min, l_max = prm["l_min"], prm["l_max"]
    fixed = int(prm.get("fixed_block", 0))
    dual = bool(prm.get("dual_cache", 0))
    look_end = 0  # end of the positions the last prefill / boundary pass covered
    seen_stop_kind = False

    class _Stop(Exception):
        pass

    def run_pass(kind, start, rows, commit):
        nonlocal nfe, look_end, seen_stop_kind
        if (max_passes is not None and nfe >= max_passes) or seen_stop_kind:
            raise _Stop
        seen_stop_kind = stop_after is not None and kind == stop_after
        toks = y[start : start + rows].copy()
        suffix = look_end - (start + rows) if (dual and kind == "inblock") else 0
        z = forward_span(cfg, W, cache, toks, start, commit, suffix)
        if kind != "inblock":
            look_end = start + rows
        nfe += 1
        if trace is not None:
            trace.append(dict(op="pass", kind=kind, span_start=start, tokens=toks, commit_len=commit, suffix_len=suffix, logits=z))
        return z

    try:
        Lk = min(2 * l_max, N)
        z = run_pass("prefill", 0, P + Lk, P)
        prev_base, prev_z = P, z[P:]
        F = P
        if fixed:
            L = min(fixed, N)
        else:
            L, _, _ = block_boundary(np.zeros(min(l_max, N)), np.zeros(min(l_max, N)), prm["lam"], l_min, cold_start=True)
        zb = prev_z[:L]
        while True:
            blocks.append(L)
            while True:  # denoising steps of block [F, F+L)
                st = vocab_stats(zb, mask)
                elig = y[F : F + L] == mask
                sel, mrg = select_parallel(
                    zb, st["lse"], st["conf"], st["argmax"], elig,
                    prm["tau_low"], prm["tau_high"], prm["gamma"], prm.get("mode", 0),
                )
                if trace is not None:
                    trace.append(dict(op="select", F=F, L=L, stats=st, eligible=elig.copy(), selected=sel.copy(), margin=mrg))
                idx = np.nonzero(sel)[0]
                assert idx.size >= 1 and elig[idx].all()
                y[F + idx] = st["argmax"][idx]  # Eq. 2
                steps.append(int(idx.size))
                if not (y[F : F + L] == mask).any():
                    break
                zb = run_pass("inblock", F, L, 0)
            R = END - (F + L)
            if R == 0:
                break
            Lk = min(2 * l_max, R)
            Wn = min(l_max, R)
            z = run_pass("boundary", F, L + Lk, L)
            look = z[L:]
            if fixed:
                Lnext = min(fixed, R)
            else:
                off = F + L - prev_base
                st = vocab_stats(look[:Wn], mask, z_prev=prev_z[off : off + Wn])
                Lnext, S, mrg = block_boundary(
                    st["kl"], st["entropy"], prm["lam"], l_min, prm["smooth_radius"], prm["norm_mode"], prm["rule"]
                )
                if trace is not None:
                    trace.append(dict(op="boundary", F=F + L, W=Wn, kl=st["kl"], entropy=st["entropy"], L=Lnext, S=S, margin=mrg))
            prev_base, prev_z = F + L, look
            F, L = F + L, Lnext
            zb = look[:L]
    except _Stop:
        pass
    return dict(tokens=y, nfe=nfe, blocks=blocks, steps=steps)
