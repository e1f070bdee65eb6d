"""Pins for oracle/decode.py: the structural facts Sec. 3 and Sec. 4.2 fix (Eq. 1, Eq. 2, block rules)."""
import numpy as np
import pytest

from oracle.decode import decode_full
from paper_2604_15750_amd import inputs


@pytest.fixture(scope="module")
def tiny():
    cfg = inputs.TINY
    return cfg, inputs.weights_to_numpy(inputs.make_weights(cfg)), inputs.make_prompts(cfg, 1, 64)[0]


PARAM_SETS = {
    "paper": dict(inputs.PAPER_PARAMS, l_max=32),
    "scaled": dict(inputs.PAPER_PARAMS, l_max=32, lam=0.9, tau_low=0.05, tau_high=0.3, gamma=-14.0),
    "cumulative": dict(inputs.PAPER_PARAMS, l_max=16, lam=0.98, rule=1, tau_low=0.1, tau_high=0.5, gamma=-12.0),
    "threshold": dict(inputs.PAPER_PARAMS, l_max=32, lam=0.8, tau_high=0.2, mode=1),
    "dual_cache": dict(inputs.PAPER_PARAMS, l_max=24, lam=0.9, tau_low=0.05, tau_high=0.3, gamma=-14.0, dual_cache=1),
}


@pytest.mark.parametrize("name", list(PARAM_SETS))
def test_decode_invariants(tiny, name):
    cfg, W, prompt = tiny
    prm = PARAM_SETS[name]
    N, P, mask = 64, 64, cfg["mask_id"]
    trace = []
    r = decode_full(cfg, W, prompt, N, prm, trace)
    y = r["tokens"]
    assert (y[:P] == prompt).all() and not (y == mask).any()  # final sequence is mask-free
    assert sum(r["blocks"]) == N and r["blocks"][0] == prm["l_min"]  # partition + cold start
    assert all(prm["l_min"] <= L <= prm["l_max"] for L in r["blocks"][:-1]) and r["blocks"][-1] <= prm["l_max"]
    assert sum(r["steps"]) == N and min(r["steps"]) >= 1  # every step decodes at least one token
    assert len(r["blocks"]) <= r["nfe"] <= N and r["nfe"] == sum(t["op"] == "pass" for t in trace)
    # Eq. 2: a step writes only masked positions of the current block, each with its own prediction
    for t in trace:
        if t["op"] == "select":
            assert not (t["selected"] & ~t["eligible"]).any()
            assert t["eligible"].any() and t["selected"][np.argmax(np.where(t["eligible"], t["stats"]["conf"], -1))]
        if t["op"] == "pass":
            assert t["span_start"] + t["commit_len"] <= P + N
            if t["kind"] == "inblock":
                assert (t["tokens"] == mask).any() and t["commit_len"] == 0
            else:
                assert not (t["tokens"][: t["commit_len"]] == mask).any()  # only clean tokens reach the cache
        if t["op"] == "boundary":
            assert (t["kl"] >= 0).all() and min(t["W"], prm["l_min"]) <= t["L"] <= t["W"] <= prm["l_max"]
    again = decode_full(cfg, W, prompt, N, prm)
    assert (again["tokens"] == y).all() and again["nfe"] == r["nfe"]
    if name != "paper":
        assert max(r["steps"]) > 1 and len(set(r["blocks"][:-1])) > 1, (r["blocks"], r["steps"])  # both decisions are exercised


@pytest.mark.parametrize("block,mode", [(16, 2), (32, 1), (24, 0)])
def test_fixed_block_comparison_rules(tiny, block, mode):
    """The comparison methods of Sec. 5.1: fixed block size with vanilla (top-1), confidence-threshold or CAP selection.
    Vanilla decoding takes exactly one token per pass: NFE = N (the paper's NFE 256 at generation length 256)."""
    cfg, W, prompt = tiny
    prm = dict(inputs.PAPER_PARAMS, l_max=32, fixed_block=block, mode=mode, tau_low=0.05, tau_high=0.2, gamma=-14.0)
    N, mask = 64, cfg["mask_id"]
    trace = []
    r = decode_full(cfg, W, prompt, N, prm, trace)
    assert not (r["tokens"] == mask).any() and sum(r["steps"]) == N
    assert r["blocks"] == [block] * (N // block) + ([N % block] if N % block else [])
    assert not any(t["op"] == "boundary" for t in trace)  # no DepGA-Block decision is taken
    if mode == 2:
        assert r["nfe"] == N and set(r["steps"]) == {1}
    else:
        assert r["nfe"] < N and max(r["steps"]) > 1
        vanilla = decode_full(cfg, W, prompt, N, dict(prm, mode=2))
        assert r["nfe"] < vanilla["nfe"]


def test_stored_decodes_are_what_the_oracle_writes():
    """tests/golden/tiny_decode.json is the committed script's output and nothing else: re-deriving two of its cases gives
    the stored values, and every stored case satisfies the decode's invariants (Sec. 3, Sec. 4.2)."""
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_decode_golden", os.path.join(here, "make_decode_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(here, "tiny_decode.json")) as f:
        gold = json.load(f)
    assert set(gold["cases"]) == set(mod.CASES)
    for name in ("scaled", "threshold_block16"):
        assert mod.decode(name) == gold["cases"][name]
    N, mask = gold["gen_len"], inputs.TINY["mask_id"]
    for name, r in gold["cases"].items():
        prm = mod.CASES[name]
        assert sum(r["blocks"]) == N and sum(r["steps"]) == N and min(r["steps"]) >= 1 and mask not in r["tokens"]
        first = prm.get("fixed_block") or prm["l_min"]
        assert r["blocks"][0] == first and max(r["blocks"]) <= prm["l_max"]
        # one pass per selection step, the prefill's and each boundary pass's selection included (Sec. 4.2)
        assert r["nfe"] == len(r["steps"])


# ---- which passes give p^prev and p^curr (Sec. 4.2; App. A.3) ---------------------------------------
def _kl_entropy(z_curr, z_prev, mask):
    """KL(p^curr || p^prev) (Eq. 3) and H(p^curr) of one position, from scipy's routines (not the oracle's formulae)."""
    from scipy.special import rel_entr, softmax
    from scipy.stats import entropy
    keep = np.arange(z_curr.shape[0]) != mask
    p, q = softmax(z_curr[keep]), softmax(z_prev[keep])
    return float(rel_entr(p, q).sum()), float(entropy(p))


def _check_alignment(trace, cfg, P, N, prm):
    """Rebuilds every boundary record of a decode trace from its pass records alone, with bookkeeping by ABSOLUTE position
    written here: `retained[pos]` = (logits row, index of the pass that produced it) for every uncommitted row of the last
    prefill / boundary pass.  Raises AssertionError when the trace's KL / entropy rows, window or pass pairing differ."""
    mask, lmax = cfg["mask_id"], prm["l_max"]
    retained = {}
    passes = []
    frontier = P  # first position not in a finished block
    checked = 0
    pending = None  # the boundary pass whose decision record comes next
    for t in trace:
        if t["op"] == "pass":
            passes.append(t)
            if t["kind"] == "inblock":
                continue
            start, commit, rows = t["span_start"], t["commit_len"], len(t["tokens"])
            new = {start + r: (t["logits"][r], len(passes) - 1) for r in range(commit, rows)}
            if t["kind"] == "boundary":
                pending = (t, dict(retained), start + commit)
            retained = new  # the look-ahead rows of this pass replace what was retained before
            frontier = start + commit
        elif t["op"] == "boundary":
            assert pending is not None, "a boundary decision without its boundary pass"
            bp, old, f_new = pending
            pending = None
            remaining = P + N - f_new
            assert t["F"] == f_new and t["W"] == min(lmax, remaining)
            assert len(t["kl"]) == t["W"] == len(t["entropy"])
            block = range(bp["span_start"], bp["span_start"] + bp["commit_len"])  # the block this pass has just committed
            for k in range(t["W"]):
                pos = f_new + k
                z_curr = bp["logits"][pos - bp["span_start"]]
                assert pos in old, f"candidate {pos} has no retained distribution"
                z_prev, src = old[pos]
                kl, H = _kl_entropy(z_curr, z_prev, mask)
                assert abs(kl - t["kl"][k]) <= 1e-9 * max(1.0, abs(kl)), (pos, kl, t["kl"][k])
                assert abs(H - t["entropy"][k]) <= 1e-9 * max(1.0, H), (pos, H, t["entropy"][k])
                # p^prev: from the pass taken while the block just decoded was still all masks; p^curr: from the pass right
                # after it was fully decoded, the rest of the state unchanged (positions after the block still masked)
                sp = passes[src]
                seen_then = [sp["tokens"][b - sp["span_start"]] for b in block]
                assert all(v == mask for v in seen_then), "p^prev was taken after part of the block had been decoded"
                assert not any(bp["tokens"][b - bp["span_start"]] == mask for b in block), "p^curr was taken before the block was finished"
                assert sp["tokens"][pos - sp["span_start"]] == mask and bp["tokens"][pos - bp["span_start"]] == mask
                checked += 1
    return checked


@pytest.mark.parametrize("name", ["scaled", "cumulative", "dual_cache"])
def test_boundary_signal_pairs_the_right_passes_and_positions(tiny, name):
    cfg, W, prompt = tiny
    prm = PARAM_SETS[name]
    trace = []
    r = decode_full(cfg, W, prompt, 64, prm, trace)
    n = _check_alignment(trace, cfg, 64, 64, prm)
    assert n >= 3 * (len(r["blocks"]) - 1) and len(r["blocks"]) >= 3  # every boundary decision after the cold start, several candidates each


def _mutant(replacements):
    """oracle/decode.py with a planted mistake (CPU only): returns the mutated module's decode_full."""
    import importlib.util
    import os
    import types
    import oracle.decode as real
    src = open(real.__file__).read()
    for old, new in replacements:
        assert src.count(old) == 1, old
        src = src.replace(old, new)
    mod = types.ModuleType("oracle._decode_mutant")
    mod.__package__ = "oracle"
    mod.__file__ = os.path.join(os.path.dirname(real.__file__), "_decode_mutant.py")
    exec(compile(src, mod.__file__, "exec"), mod.__dict__)
    return mod.decode_full


@pytest.mark.parametrize("planted", [
    [("off = F + L - prev_base", "off = min(F + L - prev_base + 1, len(prev_z) - Wn)")],  # p^prev of the neighbouring position
    [("off = F + L - prev_base", "off = F + L - prev_base - 1")],
    [("Wn = min(l_max, R)", "Wn = min(l_max - 1, R)")],                                  # a shorter candidate window
    [("st = vocab_stats(look[:Wn], mask, z_prev=prev_z[off : off + Wn])", "st = vocab_stats(look[min(1, len(look) - Wn) :][:Wn], mask, z_prev=prev_z[off : off + Wn])")],  # p^curr shifted
    [("            prev_base, prev_z = F + L, look\n", "            prev_base, prev_z = (F + L, look) if len(blocks) % 2 == 0 else (prev_base, prev_z)\n"),
     ("off = F + L - prev_base", "off = min(F + L - prev_base, len(prev_z) - Wn)")],     # p^prev not refreshed after every other block
])
def test_alignment_check_catches_planted_mistakes(tiny, planted):
    """The check above is only a pin if a plausible mistake in the schedule arithmetic fails it: plant one in a copy of the
    oracle's source and see it fail, while the decode's structural invariants (partition, NFE, Eq. 2) still hold."""
    cfg, W, prompt = tiny
    prm = PARAM_SETS["scaled"]
    trace = []
    r = _mutant(planted)(cfg, W, prompt, 64, prm, trace)
    assert sum(r["blocks"]) == 64 and not (r["tokens"] == cfg["mask_id"]).any()  # the invariants do not notice
    with pytest.raises(AssertionError):
        _check_alignment(trace, cfg, 64, 64, prm)
