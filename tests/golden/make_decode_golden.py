#!/usr/bin/env python3
"""Writes tests/golden/tiny_decode.json: whole decodes of the tiny fp32 model by the CPU oracle.

The paper prints no worked example (no numeric trace of a decode, a boundary search or a selection),
so there are no paper values to store; what is stored here is the oracle's own output, written by
this script, which calls only oracle/ and the seeded input generators.  The file pins the oracle
against silent change (a CPU test re-derives it) and gives the GPU path a stored target (a GPU test
decodes the same inputs and must reproduce it exactly: the tiny model is fp32 on both sides and
every decision margin is far above the rounding differences).

  python tests/golden/make_decode_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import decode as o_decode  # noqa: E402
from paper_2604_15750_amd import inputs  # noqa: E402  (seeded synthetic weights and prompts only)

CASES = {
    # the defaults of Sec. 5.1 (a random-init model then decodes one token per pass)
    "paper": dict(inputs.PAPER_PARAMS, l_max=32),
    # thresholds inside a random-init model's confidence range: every branch of Alg. 1 is taken
    "scaled": dict(inputs.PAPER_PARAMS, l_max=32, lam=0.9, tau_low=0.05, tau_high=0.3, gamma=-14.0),
    # in-block passes that also see the look-ahead suffix (Sec. 5.2, Q2)
    "dual_cache": dict(inputs.PAPER_PARAMS, l_max=24, lam=0.9, tau_low=0.05, tau_high=0.3, gamma=-14.0, dual_cache=1),
    # the comparison rules of Sec. 5.1 at a fixed block size
    "threshold_block16": dict(inputs.PAPER_PARAMS, l_max=32, fixed_block=16, mode=1, tau_low=0.05, tau_high=0.2, gamma=-14.0),
    "vanilla_block32": dict(inputs.PAPER_PARAMS, l_max=32, fixed_block=32, mode=2),
}
PROMPT_LEN = GEN_LEN = 64


def f32(prm):
    """The thresholds as the fp32 values both sides compare against."""
    return {k: (float(np.float32(v)) if k in ("lam", "tau_low", "tau_high", "gamma") else v) for k, v in prm.items()}


def decode(name):
    cfg = inputs.TINY
    W = inputs.weights_to_numpy(inputs.make_weights(cfg, seed=0, device="cpu"))
    prompt = inputs.make_prompts(cfg, 1, PROMPT_LEN)[0]
    r = o_decode.decode_full(cfg, W, prompt, GEN_LEN, f32(CASES[name]))
    return dict(blocks=[int(b) for b in r["blocks"]], steps=[int(s) for s in r["steps"]], nfe=int(r["nfe"]),
                tokens=[int(t) for t in r["tokens"]])


if __name__ == "__main__":
    out = {name: decode(name) for name in CASES}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_decode.json")
    with open(path, "w") as f:
        json.dump(dict(model="inputs.TINY, weights seed 0", prompt_len=PROMPT_LEN, gen_len=GEN_LEN, cases=out), f, indent=1)
    for name, r in out.items():
        print(name, "NFE", r["nfe"], "blocks", r["blocks"])
