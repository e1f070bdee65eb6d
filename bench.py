#!/usr/bin/env python3
"""Benchmark of the DepCap denoising-step hot path on one MI355X.

One "step" is one complete block-wise decode of the workload (every row of the hot path: prefill,
in-block denoising passes, boundary passes, vocabulary statistics, block_boundary, select_parallel
and the token write), inputs resident in HBM.  value = decoded tokens per second over the timed
steps.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--layers N] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def gemm_shapes(cfg):
    """(N, K) of every GEMM of one pass, in launch order per layer, then the LM head."""
    d, hd, ffn = cfg["d_model"], cfg["head_dim"], cfg["d_ffn"]
    qd, kvd = cfg["n_q_heads"] * hd, cfg["n_kv_heads"] * hd
    per_layer = [(qd + 2 * kvd, d), (d, qd), (2 * ffn, d), (d, ffn)]
    return per_layer * cfg["n_layers"] + [(cfg["vocab"], d)]


def gemm_algorithmic(cfg, rows):
    """Algorithmic HBM bytes and flops of all GEMM launches of one pass over `rows` rows:
    weights once (2 B), activations in once (2 B), outputs out once (fp32 partial sums are not
    algorithmic: an ideal kernel writes the bf16 / fp32 result once; counted as 2 B)."""
    by = fl = 0
    for n, k in gemm_shapes(cfg):
        by += 2 * n * k + 2 * rows * k + 2 * rows * n
        fl += 2 * rows * n * k
    return by, fl


def cpu_baseline(cfg, W_host, prompt, prm, sample_layers):
    """The oracle, as it stands, on a bounded sample: prefill + the first in-block pass of the same
    workload through the first `sample_layers` layers and the LM head; the in-block pass time is
    extrapolated linearly in depth to the full model.  Returns tokens/s of in-block decoding."""
    from oracle import forward as ofw, select as osel, stats as ost
    from paper_2604_15750_amd import inputs
    import threadpoolctl

    twin = inputs.with_depth(cfg, sample_layers)
    mask, P = cfg["mask_id"], len(prompt)
    look = min(2 * prm["l_max"], 256)
    cache = ofw.KVCache(twin)
    y = np.concatenate([prompt, np.full(look, mask, dtype=np.int64)])
    t0 = time.perf_counter()
    z = ofw.forward_span(twin, W_host, cache, y, 0, P)
    t_prefill = time.perf_counter() - t0
    L = prm["l_min"]
    blk = y[P: P + L].copy()
    st = ost.vocab_stats(z[P: P + L], mask)
    sel, _ = osel.select_parallel(z[P: P + L], st["lse"], st["conf"], st["argmax"], blk == mask, prm["tau_low"], prm["tau_high"],
                                  prm["gamma"], prm["mode"])
    blk[sel] = st["argmax"][sel]
    # in-block pass, timed in two parts so that depth can be extrapolated
    t0 = time.perf_counter()
    zb = ofw.forward_span(twin, W_host, cache, blk, P, 0)
    st = ost.vocab_stats(zb, mask)
    sel2, _ = osel.select_parallel(zb, st["lse"], st["conf"], st["argmax"], blk == mask, prm["tau_low"], prm["tau_high"], prm["gamma"],
                                   prm["mode"])
    t_pass = time.perf_counter() - t0
    t0 = time.perf_counter()
    head_only = inputs.with_depth(cfg, 0)
    ofw.forward_span(head_only, W_host, ofw.KVCache(head_only), blk, 0, 0)
    t_head = time.perf_counter() - t0
    t_full = (t_pass - t_head) * cfg["n_layers"] / sample_layers + t_head
    threads = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
    return dict(value=float(sel2.sum()) / t_full, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=f"prefill ({P}+{look} rows, {t_prefill:.1f} s) then one in-block denoising pass ({L} rows, kv {P}) with statistics "
                       f"and selection, through {sample_layers} of {cfg['n_layers']} layers + LM head ({t_pass:.2f} s, head {t_head:.2f} s); "
                       f"layer time scaled to {cfg['n_layers']} layers: {t_full:.2f} s per pass, {int(sel2.sum())} token(s) per pass")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llada8b_p256_g256")
    ap.add_argument("--layers", type=int, default=0, help="override depth (debug only; makes the result non-comparable)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--cpu-layers", type=int, default=2)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2604_15750_amd import api, inputs
    from paper_2604_15750_amd.decode import Decoder

    dev = torch.device("cuda:0")
    cfg, B, P, N, lmax = inputs.WORKLOADS[args.workload]
    if args.layers:
        cfg = inputs.with_depth(cfg, args.layers)
    prm = dict(inputs.PAPER_PARAMS, l_max=lmax)
    for k in ("lam", "tau_low", "tau_high", "gamma"):
        prm[k] = float(np.float32(prm[k]))
    prompts = inputs.make_prompts(cfg, B, P)

    t0 = time.perf_counter()
    W = inputs.make_weights(cfg, seed=0, device=dev)
    W_host = None
    if not args.no_cpu:
        nl = min(args.cpu_layers, cfg["n_layers"])
        W_host = {k: ([inputs.tensor_to_numpy(t) for t in v[:nl]] if isinstance(v, list) else inputs.tensor_to_numpy(v))
                  for k, v in W.items()}
    model = api.Model(cfg, W)
    del W
    torch.cuda.empty_cache()
    t_setup = time.perf_counter() - t0

    dec = Decoder(model, B, P, N, prm, dev)
    for _ in range(args.warmup):
        res = dec.run(prompts)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = dec.run(prompts)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    tokens = B * N * args.steps
    passes = sum(res["nfe"])

    # per-kernel-class durations: one more decode with every class bracketed by HIP events on the
    # launch stream (events cost queue time, so they stay out of the timed steps)
    dec.state.profile_enable(True)
    dec.state.profile_read(reset=True)
    res_p = dec.run(prompts)
    prof = dec.state.profile_read(reset=True)
    dec.state.profile_enable(False)
    # algorithmic bytes of the GEMM launches of that decode
    rows_hist = dec.rows_log
    gbytes = gflops = 0
    for rows in rows_hist:
        b_, f_ = gemm_algorithmic(cfg, rows)
        gbytes += b_
        gflops += f_
    gemm_ms, gemm_launches = prof["gemm"]
    achieved = gbytes / (gemm_ms * 1e-3) / 1e9
    out = {
        "metric": "decoded tokens/s + denoise-step latency, 8B-shaped DLM, gen 256, 1 GPU",
        "value": tokens / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, "batch": B, "prompt_len": P, "gen_len": N, "l_max": lmax, "n_layers": cfg["n_layers"],
                   "thresholds": "paper defaults (lambda 1.2, L_min 8, tau 0.8/0.95, gamma -16)"},
        "nfe": passes / B, "tokens_per_pass": B * N / passes, "launches_per_decode": res["launches"],
        "denoise_step_ms": elapsed / args.steps * 1e3 / res["launches"],
        "roofline": {"bound": "hbm", "kernel": "gemm_bf16_kernel (all GEMM launches of a decode)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "avg_launch_us": gemm_ms * 1e3 / max(gemm_launches, 1), "launches": gemm_launches,
                     "mfma_tflops": gflops / (gemm_ms * 1e-3) / 1e12},
        "kernel_ms_per_decode": {k: v[0] for k, v in prof.items()},
        "setup_s": t_setup,
    }
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, W_host, prompts[0], prm, min(args.cpu_layers, cfg["n_layers"]))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
