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
    # KL rows: the retained logits come with their log-sum-exp, as in dlm_step (an earlier pass computed it as that row's lse);
    # --prev 2 leaves it out and has the kernel recompute it from the retained logits in the same pass
    # (set-up, not the timed path: computed here with torch so that every launch of the kernel in a profile of this run is a KL launch)
    def lse_of(p):
        z = p.float()
        z[:, V - 1] = float("-inf")
        return torch.logsumexp(z, dim=-1)
    pl = [lse_of(p) for p in ps] if (ps and args.prev == 1) else None
    run = lambda i: api.dlm_vocab_stats(zs[i % nb], V - 1, prev=ps[i % nb] if ps else None, workspace=ws, prev_lse=pl[i % nb] if pl else None)
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
    print(json.dumps({"micro": "vocab_stats", "rows": rows, "vocab": V, "kl_rows": with_prev, "prev_lse": "given" if pl else ("recomputed" if with_prev else None), "launches": iters, "avg_launch_us": us,
                      "bytes_per_launch": by,
                      "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}}))


def micro_wide_pass(args):
    """The matrix-core-bound regime on its own: one pass of dlm_step over 16 packed sequences of rows / 16 rows each (no cached
    prefix: the shape of the batched workload's widest launches) through the full model, repeated; every GEMM class timed by
    the start / end stamps of its own launches (dlm_profile_*).  Reports each class against max(bytes / HBM peak, flops / bf16
    matrix-core peak).  Prints one JSON line."""
    import torch
    from paper_2604_15750_amd import api, inputs

    dev = torch.device("cuda:0")
    cfg = inputs.WORKLOADS[args.workload][0]
    rows, nseq = args.rows, 16
    per = rows // nseq
    assert per * nseq == rows and per >= 1, "--rows must be a multiple of 16"
    W = inputs.make_weights(cfg, seed=0, device=dev)
    model = api.Model(cfg, W)
    del W
    torch.cuda.empty_cache()
    state = api.State(model, nseq, per, rows, 0)
    out = api.StepOutputs(rows, cfg["vocab"], model.torch_dtype, dev)
    tokens = torch.from_numpy(inputs.make_prompts(cfg, nseq, per).astype(np.int32)).to(dev)
    off = [b * per for b in range(nseq + 1)]
    reps = max(args.steps, 1) * 2

    def one():
        for b in range(nseq):
            state.reset(b)
        api.dlm_step(state, tokens, out, off, [0] * nseq, [0] * nseq, [b * per for b in range(nseq)], slot=list(range(nseq)))

    for _ in range(max(args.warmup, 1)):
        one()
    torch.cuda.synchronize()
    state.profile_enable(list(GEMM_CLASSES))
    state.profile_read(reset=True)
    for _ in range(reps):
        one()
    torch.cuda.synchronize()
    prof = state.profile_read(reset=True)
    res = {}
    for cls in GEMM_CLASSES:
        ms, n = prof[cls]
        by, fl = gemm_algorithmic(cfg, cls, rows)
        us = ms * 1e3 / max(n, 1)
        tfl, gbs = fl / (us * 1e-6) / 1e12, by / (us * 1e-6) / 1e9
        bound = "mfma" if fl / (MFMA_BF16_PEAK_TFLOPS * 1e12) >= by / (HBM_PEAK_GBS * 1e9) else "hbm"
        res[cls] = {"launches": n, "avg_launch_us": us, "bound": bound, "achieved": tfl if bound == "mfma" else gbs,
                    "peak": MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else HBM_PEAK_GBS, "unit": "TFLOP/s" if bound == "mfma" else "GB/s",
                    "frac": tfl / MFMA_BF16_PEAK_TFLOPS if bound == "mfma" else gbs / HBM_PEAK_GBS}
    print(json.dumps({"micro": "wide_pass", "workload": args.workload, "rows": rows, "sequences": nseq, "passes": reps, "gemm": res}))
    state.close()
    model.close()


def cpu_baseline(cfg, W_host, prompt, prm, sample_layers, n_gen, gpu_pass_counts):
    """The oracle, as it stands, on a bounded sample of the same workload: the prefill pass, two in-block denoising passes
    of the first block and the first boundary pass (with their statistics, selection and boundary decision), through the
    first `sample_layers` layers and the LM head.  Each pass time is scaled linearly in depth to the full model (the LM head,
    timed alone, is not scaled), and the time of a whole decode is extrapolated as sum over pass kinds of (passes of that
    kind in the GPU's decode) x (sampled time of that kind).  Returns decoded tokens/s of that extrapolated decode."""
    from oracle import boundary as obd, forward as ofw, select as osel, stats as ost
    from paper_2604_15750_amd import inputs
    import threadpoolctl

    twin = inputs.with_depth(cfg, sample_layers)
    mask, P = cfg["mask_id"], len(prompt)
    lmax = prm["l_max"]
    look = min(2 * lmax, n_gen)
    cache = ofw.KVCache(twin)
    y = np.concatenate([prompt, np.full(n_gen, mask, dtype=np.int64)])
    times = {}

    def select(z, blk_tokens):
        st = ost.vocab_stats(z, mask)
        sel, _ = osel.select_parallel(z, st["lse"], st["conf"], st["argmax"], blk_tokens == mask, prm["tau_low"], prm["tau_high"],
                                      prm["gamma"], prm["mode"])
        return sel, st["argmax"]

    t0 = time.perf_counter()
    z = ofw.forward_span(twin, W_host, cache, y[: P + look], 0, P)
    prev_z = z[P:]
    L = min(prm["l_min"], n_gen)
    sel, am = select(z[P: P + L], y[P: P + L])
    y[P: P + L][sel] = am[sel]
    times["prefill"] = time.perf_counter() - t0
    t_in = []
    for _ in range(2):  # two in-block passes (the second one's tokens follow from the first one's selection)
        t0 = time.perf_counter()
        zb = ofw.forward_span(twin, W_host, cache, y[P: P + L], P, 0)
        sel, am = select(zb, y[P: P + L])
        y[P: P + L][sel] = am[sel]
        t_in.append(time.perf_counter() - t0)
    times["inblock"] = sum(t_in) / len(t_in)
    y[P: P + L] = np.where(y[P: P + L] == mask, 0, y[P: P + L])  # finish the block (any tokens: only the time is sampled)
    R = n_gen - L
    Lk, Wn = min(2 * lmax, R), min(lmax, R)
    t0 = time.perf_counter()
    zbd = ofw.forward_span(twin, W_host, cache, y[P: P + L + Lk], P, L)
    st = ost.vocab_stats(zbd[L: L + Wn], mask, z_prev=prev_z[L: L + Wn])
    Lnext, _, _ = obd.block_boundary(st["kl"], st["entropy"], prm["lam"], prm["l_min"], prm["smooth_radius"], prm["norm_mode"], prm["rule"])
    select(zbd[L: L + Lnext], y[P + L: P + L + Lnext])
    times["boundary"] = time.perf_counter() - t0
    head_only = inputs.with_depth(cfg, 0)
    t_head = {}
    for kind, rows in (("prefill", P + look), ("inblock", L), ("boundary", L + Lk)):
        t0 = time.perf_counter()
        ofw.forward_span(head_only, W_host, ofw.KVCache(head_only), y[:rows], 0, 0)
        t_head[kind] = time.perf_counter() - t0
    full = {k: (times[k] - t_head[k]) * cfg["n_layers"] / sample_layers + t_head[k] for k in times}
    decode_s = sum(gpu_pass_counts[k] * full[k] for k in full)
    threads = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
    sampled_s = sum(times.values()) + times["inblock"] + sum(t_head.values())
    return dict(value=n_gen / decode_s, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=f"prefill ({P}+{look} rows, {times['prefill']:.1f} s), two in-block passes ({L} rows, {times['inblock']:.1f} s each) and the first "
                       f"boundary pass ({L}+{Lk} rows, {times['boundary']:.1f} s) with statistics and decisions, through {sample_layers} of "
                       f"{cfg['n_layers']} layers + LM head ({sampled_s:.0f} s of host time in all); layer time scaled to {cfg['n_layers']} layers "
                       f"({full['prefill']:.1f} / {full['inblock']:.1f} / {full['boundary']:.1f} s per pass) and a decode extrapolated as "
                       f"{gpu_pass_counts['prefill']} prefill + {gpu_pass_counts['inblock']} in-block + {gpu_pass_counts['boundary']} boundary passes "
                       f"(the GPU decode's pass counts): {decode_s:.0f} s per {n_gen} tokens")


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
    ap.add_argument("--micro", default="", choices=["", "vocab_stats", "peaks", "wide_pass"],
                    help="time one kernel alone instead of the decode (peaks: a plain HBM read and a matrix-core loop, what the GPU achieves; "
                         "wide_pass: one pass of --rows rows over 16 packed sequences, the matrix-core-bound regime, per GEMM class)")
    ap.add_argument("--rows", type=int, default=3072, help="--micro: rows of the pass (3072 = 16 sequences x 192 rows, the widest batched pass)")
    ap.add_argument("--prev", type=int, default=1, help="--micro vocab_stats: 1 = every row is a KL row (reads the retained logits too; their log-sum-exp is given, as in dlm_step), 2 = the same with that log-sum-exp recomputed in the pass, 0 = no KL rows")
    ap.add_argument("--extras", type=int, default=1, choices=[0, 1],
                    help="1 (default workload only): also time the scaled-threshold decode and the batched workload on the same model")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run out = in + 1 over 1 GiB three times (a kernel of known HBM traffic, to scale rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (every box has one); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if args.micro == "vocab_stats":
        micro_vocab_stats(args)
        return
    if args.micro == "wide_pass":
        micro_wide_pass(args)
        return
    if args.micro == "peaks":
        import torch
        from paper_2604_15750_amd import api
        buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda:0")
        print(json.dumps({"micro": "peaks", "hbm_read_GBs": api.probe_hbm_read(buf, reps=20), "hbm_published_GBs": HBM_PEAK_GBS,
                          "mfma_f16_random_operands_TFLOPs": api.probe_mfma(reps=10), "mfma_f16_published_TFLOPs": 2500.0}))
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
        """Achieved rate of a GEMM class over all its launches of one decode, against the roof that bounds it: each launch
        is charged max(algorithmic bytes / HBM peak, flops / bf16 matrix-core peak); the class is "hbm" bound when the byte
        term is the larger share of that floor, else "mfma", and achieved / peak are quoted in that roof's unit."""
        by = fl = 0
        t_hbm = t_mfma = floor = 0.0
        for rows in rows_hist:
            b_, f_ = gemm_algorithmic(cfg, cls, rows)
            n = shapes[cls][2]
            by += b_ * n
            fl += f_ * n
            tb, tf = b_ / (HBM_PEAK_GBS * 1e9), f_ / (MFMA_BF16_PEAK_TFLOPS * 1e12)
            t_hbm += n * tb
            t_mfma += n * tf
            floor += n * max(tb, tf)
        gbs, tfl = by / (ms * 1e-3) / 1e9, fl / (ms * 1e-3) / 1e12
        common = {"avg_launch_us": ms * 1e3 / max(launches, 1), "launches": launches, "bytes_per_launch": by / max(launches, 1),
                  "flops_per_launch": fl / max(launches, 1), "hbm_GBs": gbs, "mfma_tflops": tfl,
                  "floor_frac": floor / (ms * 1e-3)}  # sum of the launches' roofline times / measured time
        if t_hbm >= t_mfma:
            return dict({"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}, **common)
        return dict({"bound": "mfma", "achieved": tfl, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tfl / MFMA_BF16_PEAK_TFLOPS}, **common)

    roof = class_roofline(DOMINANT, dom_ms, dom_launches)
    roof["kernel"] = "gemm_mid_kernel / gemm_macro_kernel with the SwiGLU epilogue (gate/up GEMM, every launch of one decode)"
    roof["traffic"] = traffic_from_profile(args.workload)
    # what this GPU achieves on the same resources with kernels that do nothing else (a plain streaming read of 2 GiB; matrix-core
    # products out of registers): the published peaks are not reachable by any kernel
    probe_buf = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
    achievable = {"hbm_read_GBs": api.probe_hbm_read(probe_buf, reps=10), "mfma_f16_random_operands_TFLOPs": api.probe_mfma(reps=5)}
    del probe_buf
    roof["achievable_peak"] = achievable["hbm_read_GBs"] if roof["bound"] == "hbm" else achievable["mfma_f16_random_operands_TFLOPs"]
    roof["frac_of_achievable"] = roof["achieved"] / roof["achievable_peak"]
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
        # what the matrix cores multiply: a bf16 model's operands are IEEE half (bf16 weights converted once, activations rounded
        # to half), accumulated in fp32; weights, embeddings and logits are bf16 in the caller's memory
        "dtype": "f16" if cfg["dtype"] == "bf16" else cfg["dtype"], "storage_dtype": cfg["dtype"], "data": "synthetic",
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
    pass_counts = dict(dec.kind_counts)  # of the last decode (every decode of a workload takes the same passes)
    out["pass_counts"] = pass_counts
    dec.close()
    if args.extras and args.workload == "llada8b_p256_g256" and not args.layers:
        # Beside the headline (paper thresholds: a random-init model commits one token per pass), on the same model: the same
        # workload with the thresholds scaled into such a model's confidence range (CAP-Decoding then commits several tokens
        # per pass), and the batched workload (16 sequences, ragged blocks packed per launch: the matrix-core-bound regime).
        def one(name, B2, P2, N2, lmax2, prm2, steps):
            d2 = Decoder(model, B2, P2, N2, prm2, dev)
            pr2 = inputs.make_prompts(cfg, B2, P2)
            d2.run(pr2)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(steps):
                r2 = d2.run(pr2)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t1) / steps
            fl_ms = sum(pass_floor_us(cfg, rows_l, kv_l) for rows_l, kv_l in d2.pass_log) * 1e-3
            res2 = {"workload": name, "tokens_per_s": B2 * N2 / dt, "ms_per_decode": dt * 1e3, "nfe": sum(r2["nfe"]) / B2,
                    "tokens_per_pass": B2 * N2 / sum(r2["nfe"]), "launches_per_decode": r2["launches"], "denoise_step_ms": dt * 1e3 / r2["launches"],
                    "mean_rows_per_launch": float(np.mean(d2.rows_log)), "decode_floor_frac": fl_ms / (dt * 1e3)}
            d2.close()
            return res2
        scaled = dict(prm, **inputs.SCALED_THRESHOLDS)
        for k in ("lam", "tau_low", "tau_high", "gamma"):
            scaled[k] = float(np.float32(scaled[k]))
        out["scaled_thresholds"] = one("llada8b_p256_g256, thresholds scaled to a random-init model (lambda 0.9, tau 0.04/0.25, gamma -36)",
                                       B, P, N, lmax, scaled, max(1, min(args.steps, 3)))
        _, B4, P4, N4, lmax4 = inputs.WORKLOADS["llada8b_b16_p256_g512"]
        out["batched"] = one("llada8b_b16_p256_g512 (paper thresholds)", B4, P4, N4, lmax4, dict(prm, l_max=lmax4), 1)
    model.close()
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, W_host, prompts[0], prm, min(args.cpu_layers, cfg["n_layers"]), N, pass_counts)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
