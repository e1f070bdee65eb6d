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
