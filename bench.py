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
DOMINANT = "gemm_gate_up"  # the kernel class with the largest share of a decode (rocprofv3 summary under profiles/)


GEMM_CLASSES = ("gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down", "gemm_lm_head")


def gemm_shapes(cfg):
    """class -> (N, K, launches per pass) of the GEMMs of one pass."""
    d, hd, ffn, L = cfg["d_model"], cfg["head_dim"], cfg["d_ffn"], cfg["n_layers"]
    qd, kvd = cfg["n_q_heads"] * hd, cfg["n_kv_heads"] * hd
    return {"gemm_qkv": (qd + 2 * kvd, d, L), "gemm_o": (d, qd, L), "gemm_gate_up": (2 * ffn, d, L), "gemm_down": (d, ffn, L),
            "gemm_lm_head": (cfg["vocab"], d, 1)}


def gemm_algorithmic(cfg, cls, rows):
    """Algorithmic HBM bytes and flops of ONE launch of GEMM class `cls` over `rows` rows: weights once (2 B), activations in
    once (2 B), results out once (2 B; the gate/up launch writes only the d_ffn gated columns).  fp32 partial sums, the fp32
    residual stream and the norm statistics are not algorithmic."""
    n, k, _ = gemm_shapes(cfg)[cls]
    n_out = n // 2 if cls == "gemm_gate_up" else n
    return 2 * n * k + 2 * rows * k + 2 * rows * n_out, 2 * rows * n * k


def pass_floor_us(cfg, rows_per_seq, kv_per_seq):
    """Roofline floor of one pass: every GEMM at max(HBM time of its algorithmic bytes, MFMA time of its flops), attention at
    the HBM time of its K/V reads, the vocabulary statistics at the HBM time of one read of the logits."""
    rows = sum(rows_per_seq)
    t = 0.0
    for cls, (n, k, launches) in gemm_shapes(cfg).items():
        by, fl = gemm_algorithmic(cfg, cls, rows)
        t += launches * max(by / (HBM_PEAK_GBS * 1e9), fl / (MFMA_BF16_PEAK_TFLOPS * 1e12))
    kvw = cfg["n_kv_heads"] * cfg["head_dim"]
    t += cfg["n_layers"] * sum(2 * (kv + r) * kvw * 2 for r, kv in zip(rows_per_seq, kv_per_seq)) / (HBM_PEAK_GBS * 1e9)
    t += rows * cfg["vocab"] * 2 / (HBM_PEAK_GBS * 1e9)
    return t * 1e6


def traffic_from_profile(workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, if there is one for this
    workload (two --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by a copy kernel of known size)."""
    path = os.path.join(ROOT, "profiles", f"gemm_gate_up_{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    vals = {}
    for line in open(path):
        if "=" in line and not line.startswith("#"):
            k, v = line.split("=", 1)
            vals[k.strip()] = v.strip()
    try:
        return float(vals["fetch_bytes_per_launch"]) + float(vals["write_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def micro_vocab_stats(args):
    """The vocabulary-statistics kernel alone at a batched-pass shape (HBM-bound: the logits are read once, plus the retained
    p^prev logits on KL rows).  Buffers rotate over more than the 256 MB memory-side cache.  Prints one JSON line."""
    import torch
    from paper_2604_15750_amd import api, inputs

    dev = torch.device("cuda:0")
    V = inputs.WORKLOADS[args.workload][0]["vocab"]
    rows, with_prev = args.rows, bool(args.prev)
    nb = max(2, min(8, int(1.2e9 // (rows * V * 2))))
    mk = lambda: torch.randn(rows, V, device=dev, dtype=torch.float32).mul_(4).to(torch.bfloat16)
    zs = [mk() for _ in range(nb)]
    ps = [mk() for _ in range(nb)] if with_prev else None
    ws = torch.empty(api.lib().dlm_vocab_stats_workspace(rows), dtype=torch.uint8, device=dev)
    run = lambda i: api.dlm_vocab_stats(zs[i % nb], V - 1, prev=ps[i % nb] if ps else None, workspace=ws)
    for i in range(args.warmup + 2):
        run(i)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    iters = max(args.steps, 1) * 10
    a.record()
    for i in range(iters):
        run(i)
    b.record()
    torch.cuda.synchronize()
    us = a.elapsed_time(b) * 1e3 / iters
    by = rows * V * 2 * (2 if with_prev else 1)
    gbs = by / (us * 1e-6) / 1e9
    print(json.dumps({"micro": "vocab_stats", "rows": rows, "vocab": V, "kl_rows": with_prev, "launches": iters, "avg_launch_us": us,
                      "bytes_per_launch": by,
                      "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}}))


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
    ap.add_argument("--cpu-layers", type=int, default=12, help="layers of the model the oracle leg runs (about 11 s of host time at 12 on 16 cores)")
    ap.add_argument("--thresholds", default="paper", choices=["paper", "scaled"],
                    help="paper: the defaults of Sec. 5.1; scaled: thresholds placed inside the confidence range of a random-init model, "
                         "so that CAP-Decoding commits several tokens per pass")
    ap.add_argument("--stats", default="epilogue", choices=["epilogue", "streamed"],
                    help="where passes that compare and retain no row (at most 64 rows) take their vocabulary statistics: the LM head's "
                         "epilogue (the default) or the streamed reduction every other pass uses")
    ap.add_argument("--weight-copies", type=int, default=1, choices=[0, 1],
                    help="0: no step-major second copies of the layer matrices (DLM_W_STEPS=0 for dlm_model_create)")
    ap.add_argument("--micro", default="", choices=["", "vocab_stats", "peaks"],
                    help="time one kernel alone instead of the decode (peaks: a plain HBM read and a matrix-core loop, what the GPU achieves)")
    ap.add_argument("--rows", type=int, default=3072, help="--micro: rows of the pass (3072 = 16 sequences x 192 rows, the widest batched pass)")
    ap.add_argument("--prev", type=int, default=1, help="--micro vocab_stats: 1 = every row is a KL row (reads the retained logits too)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run out = in + 1 over 1 GiB three times (a kernel of known HBM traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if args.micro == "vocab_stats":
        micro_vocab_stats(args)
        return
    if args.micro == "peaks":
        import torch
        from paper_2604_15750_amd import api
        buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda:0")
        print(json.dumps({"micro": "peaks", "hbm_read_GBs": api.probe_hbm_read(buf, reps=20), "hbm_published_GBs": HBM_PEAK_GBS,
                          "mfma_bf16_TFLOPs": api.probe_mfma_bf16(reps=10), "mfma_bf16_published_TFLOPs": 2500.0}))
        return

    import torch
    from paper_2604_15750_amd import api, inputs
    from paper_2604_15750_amd.decode import Decoder

    dev = torch.device("cuda:0")
    cfg, B, P, N, lmax = inputs.WORKLOADS[args.workload]
    if args.layers:
        cfg = inputs.with_depth(cfg, args.layers)
    prm = dict(inputs.PAPER_PARAMS, l_max=lmax)
    if args.thresholds == "scaled":
        prm.update(inputs.SCALED_THRESHOLDS)
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
    model = api.Model(cfg, W, weight_copies=bool(args.weight_copies))
    del W
    torch.cuda.empty_cache()
    t_setup = time.perf_counter() - t0

    dec = Decoder(model, B, P, N, prm, dev)
    dec.state.fuse_stats(args.stats == "epilogue")
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

    # Per-kernel-class durations: one more decode with every class bracketed by HIP events on the launch stream, and one with
    # only the dominant class (the gate/up GEMM) bracketed: events cost queue time, so they stay out of the timed steps, and
    # the dominant kernel's own figure comes from the run in which nothing else is bracketed.
    st = dec.state
    st.profile_enable(True)
    st.profile_read(reset=True)
    dec.run(prompts)
    prof = st.profile_read(reset=True)
    st.profile_enable([DOMINANT])
    dec.run(prompts)
    dom_ms, dom_launches = st.profile_read(reset=True)[DOMINANT]
    st.profile_enable(False)
    rows_hist = dec.rows_log
    shapes = gemm_shapes(cfg)

    def class_roofline(cls, ms, launches):
        by = fl = 0
        for rows in rows_hist:
            b_, f_ = gemm_algorithmic(cfg, cls, rows)
            by += b_ * shapes[cls][2]
            fl += f_ * shapes[cls][2]
        gbs = by / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                "avg_launch_us": ms * 1e3 / max(launches, 1), "launches": launches, "bytes_per_launch": by / max(launches, 1),
                "mfma_tflops": fl / (ms * 1e-3) / 1e12}

    roof = class_roofline(DOMINANT, dom_ms, dom_launches)
    roof["kernel"] = "gemm_mid_kernel / gemm_macro_kernel with the SwiGLU epilogue (gate/up GEMM, every launch of one decode)"
    roof["traffic"] = traffic_from_profile(args.workload)
    # what this GPU achieves on the same resources with kernels that do nothing else (a plain streaming read of 2 GiB; matrix-core
    # products out of registers): the published peaks are not reachable by any kernel
    probe_buf = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    achievable = {"hbm_read_GBs": api.probe_hbm_read(probe_buf, reps=10), "mfma_bf16_TFLOPs": api.probe_mfma_bf16(reps=5)}
    del probe_buf
    roof["achievable_peak"] = achievable["hbm_read_GBs"]
    roof["frac_of_achievable"] = roof["achieved"] / achievable["hbm_read_GBs"]
    others = {cls: class_roofline(cls, *prof[cls]) for cls in GEMM_CLASSES}
    # attention against the HBM time of its K/V reads (cached prefix + the span's own rows, every layer); vocabulary statistics
    # against one read of the logits (plus the retained logits on KL rows)
    kvw = cfg["n_kv_heads"] * cfg["head_dim"]
    att_bytes = cfg["n_layers"] * sum(2 * (kv + r) * kvw * 2 for rows_l, kv_l in dec.pass_log for r, kv in zip(rows_l, kv_l))
    att_flops = cfg["n_layers"] * sum(4 * r * (kv + r) * cfg["n_q_heads"] * cfg["head_dim"] for rows_l, kv_l in dec.pass_log for r, kv in zip(rows_l, kv_l))
    att_ms, att_n = prof["attention"]
    others["attention"] = {"bound": "hbm", "achieved": att_bytes / (att_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": att_bytes / (att_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "avg_launch_us": att_ms * 1e3 / max(att_n, 1), "launches": att_n,
                           "bytes_per_launch": att_bytes / max(att_n, 1), "mfma_tflops": att_flops / (att_ms * 1e-3) / 1e12}
    vs_ms, vs_n = prof["vocab_stats"]
    # passes whose statistics come from the LM head's epilogue read no logits here: their launch is the merge of the per-group states
    streamed = [r for r, special in dec.stat_log if args.stats == "streamed" or special or r > 64]
    vs_bytes = sum(streamed) * cfg["vocab"] * 2 + dec.kl_rows * cfg["vocab"] * 2
    others["vocab_stats"] = {"bound": "hbm", "achieved": vs_bytes / (vs_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": vs_bytes / (vs_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "avg_launch_us": vs_ms * 1e3 / max(vs_n, 1), "launches": vs_n,
                             "bytes_per_launch": vs_bytes / max(vs_n, 1), "source": args.stats, "streamed_launches": len(streamed),
                             "note": "narrow passes: launch-bound, and the logits were just written (cache hits); see --micro vocab_stats for the batched shape"}
    # the whole decode against the sum of its passes' roofline floors
    floor_ms = sum(pass_floor_us(cfg, rows_l, kv_l) for rows_l, kv_l in dec.pass_log) * 1e-3
    out = {
        "metric": "decoded tokens/s + denoise-step latency, 8B-shaped DLM, gen 256, 1 GPU",
        "value": tokens / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, "batch": B, "prompt_len": P, "gen_len": N, "l_max": lmax, "n_layers": cfg["n_layers"], "weight_copies": args.weight_copies, "stats": args.stats,
                   "thresholds": "paper defaults (lambda 1.2, L_min 8, tau 0.8/0.95, gamma -16)" if args.thresholds == "paper" else
                                 "scaled to a random-init model (lambda 0.9, L_min 8, tau 0.04/0.25, gamma -36)"},
        "nfe": passes / B, "tokens_per_pass": B * N / passes, "launches_per_decode": res["launches"],
        "denoise_step_ms": elapsed / args.steps * 1e3 / res["launches"],
        "roofline": roof,
        "achievable": achievable,
        "roofline_other_kernels": others,
        "decode_floor_ms": floor_ms, "decode_floor_frac": floor_ms / (elapsed / args.steps * 1e3),
        "kernel_ms_per_decode": {k: v[0] for k, v in prof.items()},
        "setup_s": t_setup,
    }
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.int32, device=dev)  # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)  # an elementwise kernel (CUDAFunctor_add) that reads 1 GiB and writes 1 GiB
        torch.cuda.synchronize()
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, W_host, prompts[0], prm, min(args.cpu_layers, cfg["n_layers"]))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
