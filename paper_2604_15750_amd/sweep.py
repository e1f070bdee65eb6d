#!/usr/bin/env python3
"""Decoding-strategy comparison and hyper-parameter sweeps on a synthetic (random-init) model.

Mirrors the rows of the paper's Table 1 (Sec. 5.2: vanilla and confidence-threshold decoding at
fixed block sizes, CAP-Decoding alone, DepGA-Block alone, full DepCap) and the sweeps of App. B
(generation length, lambda, L_max, tau_low, gamma), reporting what the hot path can report without
trained weights or datasets: forward passes per sequence (NFE), tokens per pass and decoded
tokens/s.  Accuracy is out of reach here (no trained weights), so this says nothing about quality.

A random-init model never reaches the paper's confidence thresholds; by default the thresholds are
the scaled set of inputs.SCALED_THRESHOLDS (--thresholds paper uses Sec. 5.1's values: everything
then decodes one token per pass).

  python -m paper_2604_15750_amd.sweep [--workload NAME] [--layers N] [--what methods,l_gen,lam,l_max,tau_low,gamma]
"""
import argparse
import json
import time

import numpy as np
import torch

from . import api, inputs
from .decode import Decoder


def run(model, cfg, B, P, N, prm, dev, prompts):
    prm = dict(prm)
    for k in ("lam", "tau_low", "tau_high", "gamma"):
        prm[k] = float(np.float32(prm[k]))
    dec = Decoder(model, B, P, N, prm, dev)
    dec.run(prompts)  # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    res = dec.run(prompts)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    dec.close()
    nfe = float(np.mean(res["nfe"]))
    return dict(nfe=nfe, tokens_per_pass=N / nfe, tokens_per_s=B * N / dt, blocks=float(np.mean([len(b) for b in res["blocks"]])))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="llada8b_p256_g256")
    ap.add_argument("--layers", type=int, default=0, help="override the depth (0: the workload's)")
    ap.add_argument("--thresholds", default="scaled", choices=["scaled", "paper"])
    ap.add_argument("--what", default="methods,l_gen,lam,l_max,tau_low,gamma")
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    cfg, B, P, N, lmax = inputs.WORKLOADS[args.workload]
    if args.layers:
        cfg = inputs.with_depth(cfg, args.layers)
    base = dict(inputs.PAPER_PARAMS, l_max=lmax)
    if args.thresholds == "scaled":
        base.update(inputs.SCALED_THRESHOLDS)
    W = inputs.make_weights(cfg, seed=0, device=dev)
    model = api.Model(cfg, W)
    del W
    torch.cuda.empty_cache()
    prompts = inputs.make_prompts(cfg, B, P)
    what = set(args.what.split(","))
    rows = []

    def emit(group, name, prm, n=N):
        r = run(model, cfg, B, P, n, prm, dev, prompts)
        rows.append(dict(group=group, setting=name, **r))
        print(f"{group:10s} {name:34s} NFE {r['nfe']:7.1f}  tokens/pass {r['tokens_per_pass']:6.2f}  blocks {r['blocks']:5.1f}  "
              f"{r['tokens_per_s']:8.1f} tokens/s", flush=True)

    if "methods" in what:  # Table 1: the decoding strategies
        emit("methods", "vanilla, block 32", dict(base, fixed_block=32, mode=2))
        for b in (16, 32, 64):
            emit("methods", f"confidence threshold, block {b}", dict(base, fixed_block=b, mode=1))
        emit("methods", "CAP-Decoding, block 32", dict(base, fixed_block=32, mode=0))
        emit("methods", "DepGA-Block + confidence threshold", dict(base, mode=1))
        emit("methods", "DepCap (DepGA-Block + CAP-Decoding)", dict(base, mode=0))
        emit("methods", "DepCap, suffix visible in the block", dict(base, mode=0, dual_cache=1))  # the dual cache of Sec. 5.2
    if "l_gen" in what:  # App. B.1
        for n in (128, 256, 512, 1024):
            if P + n <= 4096:
                emit("l_gen", f"L_gen {n}", base, n)
    if "lam" in what:  # App. B.2
        for lam in (0.6, 0.8, 1.0, 1.2, 1.4, 1.6):
            emit("lambda", f"lambda {lam}", dict(base, lam=lam))
    if "l_max" in what:  # App. B.3
        for lm in (16, 32, 64, 128, 256):
            if lm <= 128:  # the boundary window is at most 256 positions and the look-ahead is 2 L_max
                emit("l_max", f"L_max {lm}", dict(base, l_max=lm))
    if "tau_low" in what:  # App. B.4: the paper moves tau_low over 0.65 .. 0.85 around its default 0.8; same ratios here
        for f in (0.8125, 0.875, 0.9375, 1.0, 1.0625):
            emit("tau_low", f"tau_low {base['tau_low'] * f:.4f}", dict(base, tau_low=base["tau_low"] * f))
    if "gamma" in what:  # App. B.5: the paper moves gamma over -8 .. -24 around its default -16; same ratios here
        for f in (0.5, 0.75, 1.0, 1.25, 1.5):
            emit("gamma", f"gamma {base['gamma'] * f:.1f}", dict(base, gamma=base["gamma"] * f))
    print(json.dumps({"workload": args.workload, "n_layers": cfg["n_layers"], "thresholds": args.thresholds, "rows": rows}))
    model.close()


if __name__ == "__main__":
    main()
