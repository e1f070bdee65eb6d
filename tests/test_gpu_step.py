"""dlm_step / block_boundary / select_parallel against the oracle's block-wise decode.

Teacher-forced replay: the oracle decodes on the CPU and records every pass and decision; the HIP
path is fed the same tokens pass by pass through the C ABI and every output is compared:
  logits            against the oracle's, per row: |dz| <= tol * max(|z_ref|_inf, sigma_logit)
                    (tol = 2e-2 for bf16 models, the benchmark spec's bound; 2e-4 for the fp32 model)
  statistics        stage-isolated: the oracle's statistics of the GPU's own logits, 1e-5
  KL                stage-isolated against the GPU's own retained logits
  decisions         the oracle's rule applied to the GPU's statistics: exact where the margin allows
Then the free-running HIP decode (paper_2604_15750_amd.decode) is compared with the oracle's result.
"""
import numpy as np
import pytest
import torch

from oracle import boundary as o_boundary
from oracle import decode as o_decode
from oracle import forward as o_fwd
from oracle import select as o_select
from oracle import stats as o_stats
from paper_2604_15750_amd import api, inputs
from paper_2604_15750_amd.decode import Decoder

pytestmark = pytest.mark.gpu

SIGMA_LOGIT = 4.0


def _weights(cfg, seed, device):
    """Small models: drawn on the CPU (same bytes wherever the test runs), then moved."""
    W = inputs.make_weights(cfg, seed=seed, device="cpu")
    return {k: [t.to(device) for t in v] if isinstance(v, list) else v.to(device) for k, v in W.items()}


def _f32(prm):
    """Thresholds as the fp32 values the kernels receive."""
    out = dict(prm)
    for k in ("lam", "tau_low", "tau_high", "gamma"):
        out[k] = float(np.float32(prm[k]))
    return out


def replay(cfg, W_dev, prompt, N, prm, device, logit_tol, max_passes=None, stats_out=None, stop_after=None):
    prm = _f32(prm)
    P, END, lmax, mask = len(prompt), len(prompt) + N, prm["l_max"], cfg["mask_id"]
    Wn = inputs.weights_to_numpy(W_dev)
    trace = []
    o_decode.decode_full(cfg, Wn, prompt, N, prm, trace, max_passes=max_passes, stop_after=stop_after)
    model = api.Model(cfg, W_dev)
    look = min(2 * lmax, N)
    max_rows = max(P + look, lmax + look)
    state = api.State(model, 1, END, max_rows, look)
    out = api.StepOutputs(max_rows, cfg["vocab"], model.torch_dtype, device)
    tokens = torch.full((END,), mask, dtype=torch.int32, device=device)
    sel = torch.zeros(max_rows, dtype=torch.uint8, device=device)
    nsel = torch.zeros(1, dtype=torch.int32, device=device)
    mg = torch.zeros(1, dtype=torch.float32, device=device)
    L_dev = torch.zeros(1, dtype=torch.int32, device=device)
    prev = None  # (base position, GPU logits fp64) retained by the previous prefill / boundary pass
    worst = rms = 0.0
    n_pass = n_bnd = n_sel = 0
    last = None
    for rec in trace:
        if rec["op"] == "pass":
            s0, toks, commit = rec["span_start"], rec["tokens"], rec["commit_len"]
            rows = len(toks)
            tokens[s0: s0 + rows] = torch.from_numpy(toks.astype(np.int32)).to(device)
            klf = klc = svf = svc = 0
            if rec["kind"] == "prefill":
                svf, svc = P, rows - P
            elif rec["kind"] == "boundary":
                klf, klc = commit, min(lmax, END - (s0 + commit))
                svf, svc = commit, rows - commit
            assert state.kv_len(0) == s0
            api.dlm_step(state, tokens, out, [0, rows], [s0], [commit], [s0], kl_first=[klf], kl_count=[klc], save_first=[svf],
                         save_count=[svc], suffix_len=[rec.get("suffix_len", 0)])
            torch.cuda.synchronize()
            assert state.kv_len(0) == s0 + commit
            z = o_fwd.widen(inputs.tensor_to_numpy(out.logits[:rows]))
            ref = rec["logits"]
            scale = np.maximum(np.abs(ref).max(-1, keepdims=True), SIGMA_LOGIT)
            err = (np.abs(z - ref) / scale).max()
            worst = max(worst, err)
            rms = max(rms, float((np.sqrt(np.mean((z - ref) ** 2, -1)) / np.sqrt(np.mean(ref ** 2, -1))).max()))
            if stats_out is not None:
                stats_out.append(dict(kind=rec["kind"], rows=rows, worst=float(err), rms=rms,
                                      p999=float(np.quantile(np.abs(z - ref) / scale, 0.999)), frac_over=float((np.abs(z - ref) / scale > logit_tol).mean())))
            assert err <= logit_tol, (rec["kind"], s0, rows, err)
            st = o_stats.vocab_stats(z, mask)
            got = {k: getattr(out, k)[:rows].cpu().numpy() for k in ("max_logit", "lse", "entropy", "conf", "argmax", "kl")}
            for key in ("max_logit", "lse", "entropy", "conf"):
                assert (np.abs(got[key] - st[key]) <= 1e-5 * np.maximum(1.0, np.abs(st[key]))).all(), key
            assert (got["argmax"] == st["argmax"]).all()
            kl_ref = np.zeros(rows)
            if klc:
                zp = prev[1][s0 + klf - prev[0]: s0 + klf - prev[0] + klc]
                kst = o_stats.vocab_stats(z[klf: klf + klc], mask, zp)
                kl_ref[klf: klf + klc] = kst["kl"]
                logp, _, _ = o_stats.log_softmax_masked(z[klf: klf + klc], mask)
                logq, _, _ = o_stats.log_softmax_masked(zp, mask)
                spread = np.zeros(rows)
                spread[klf: klf + klc] = np.sum(np.exp(logp) * np.abs(np.where(np.isfinite(logp), logp, 0.0) - np.where(np.isfinite(logq), logq, 0.0)), -1)
                assert (np.abs(got["kl"] - kl_ref) <= 1e-5 * np.maximum(1.0, np.abs(kl_ref)) + 1e-5 * spread).all()
            else:
                assert (got["kl"] == 0).all()
            if svc:
                prev = (s0 + svf, z[svf: svf + svc])
            last = dict(rec=rec, got=got, z=z, rows=rows)
            n_pass += 1
        elif rec["op"] == "boundary":
            g, W = last["got"], rec["W"]
            c = last["rec"]["commit_len"]
            api.block_boundary(out.kl, out.entropy, [c], [W], L_dev, prm["lam"], prm["l_min"], prm["smooth_radius"], prm["norm_mode"],
                               prm["rule"], margin_out=mg)
            torch.cuda.synchronize()
            Lr, _, mr = o_boundary.block_boundary(g["kl"][c: c + W], g["entropy"][c: c + W], prm["lam"], prm["l_min"],
                                                  prm["smooth_radius"], prm["norm_mode"], prm["rule"])
            if mr > 1e-4:
                assert int(L_dev[0]) == Lr
            if rec["margin"] > 20 * logit_tol:  # end to end: the GPU's own signals lead to the oracle's decision
                assert int(L_dev[0]) == rec["L"], (int(L_dev[0]), rec["L"], rec["margin"])
            n_bnd += 1
        elif rec["op"] == "select":
            g, F, L = last["got"], rec["F"], rec["L"]
            r0 = F - last["rec"]["span_start"]
            tok_before = tokens.clone()
            api.select_parallel(out.logits, out.lse, out.conf, out.argmax, tokens, [r0], [F], [L], mask, prm["tau_low"], prm["tau_high"],
                                prm["gamma"], prm.get("mode", 0), sel, nsel, apply_tokens=True, margin_out=mg)
            torch.cuda.synchronize()
            got_sel = sel[r0: r0 + L].cpu().numpy().astype(bool)
            elig = tok_before[F: F + L].cpu().numpy() == mask
            assert (elig == rec["eligible"]).all()
            ref_sel, mr = o_select.select_parallel(last["z"][r0: r0 + L], g["lse"][r0: r0 + L], g["conf"][r0: r0 + L],
                                                   g["argmax"][r0: r0 + L], elig, prm["tau_low"], prm["tau_high"], prm["gamma"],
                                                   prm.get("mode", 0))
            if mr > 1e-5:
                assert (got_sel == ref_sel).all() and int(nsel[0]) == ref_sel.sum()
                after = tokens[F: F + L].cpu().numpy()
                assert (after == np.where(ref_sel, g["argmax"][r0: r0 + L], tok_before[F: F + L].cpu().numpy())).all()  # Eq. 2
            n_sel += 1
    state.close()
    model.close()
    return dict(worst=worst, rms=rms, passes=n_pass, boundaries=n_bnd, selects=n_sel, trace=trace)


TINY_SETS = {
    "paper": dict(inputs.PAPER_PARAMS, l_max=32),
    "dual_cache": dict(inputs.PAPER_PARAMS, l_max=24, lam=0.9, tau_low=0.05, tau_high=0.3, gamma=-14.0, dual_cache=1),
    "scaled": dict(inputs.PAPER_PARAMS, l_max=32, lam=0.9, tau_low=0.05, tau_high=0.3, gamma=-14.0),
    "cumulative": dict(inputs.PAPER_PARAMS, l_max=16, lam=0.98, rule=1, tau_low=0.1, tau_high=0.5, gamma=-12.0),
}


@pytest.mark.parametrize("name", list(TINY_SETS))
def test_tiny_f32_replay(device, name):
    cfg = inputs.TINY
    W = _weights(cfg, 0, device)
    prompt = inputs.make_prompts(cfg, 1, 64)[0]
    r = replay(cfg, W, prompt, 64, TINY_SETS[name], device, logit_tol=2e-4)
    assert r["passes"] >= 8 and r["boundaries"] == len([t for t in r["trace"] if t["op"] == "boundary"]) >= 1
    print(name, "worst relative logit error", r["worst"], "passes", r["passes"])


MID = inputs.model_config(2, 512, 4, 2, 128, 1536, 4096, "bf16")


@pytest.mark.parametrize("name", ["paper", "scaled", "dual_cache"])
def test_mid_bf16_gqa_replay(device, name):
    W = _weights(MID, 5, device)
    prompt = inputs.make_prompts(MID, 1, 100, seed=5)[0]
    prm = dict(TINY_SETS[name], l_max=24)
    r = replay(MID, W, prompt, 90, prm, device, logit_tol=2e-2)
    print(name, "worst relative logit error", r["worst"], "passes", r["passes"])


# many heads (48 query heads over 12 kv heads of 128 dims: 9216 QKV columns, so the QKV weights take the interleaved-pair
# packing of the wide matrices) on a narrow model
WIDE_HEADS = inputs.model_config(2, 256, 48, 12, 128, 512, 2048, "bf16")


@pytest.mark.parametrize("l_max", [12, 24])
def test_wide_heads_bf16_gqa_replay(device, l_max):
    """Grouped-query attention with groups of four, blocks of one and of two query tiles, QKV weights in the wide packing;
    every pass against the oracle."""
    W = _weights(WIDE_HEADS, 7, device)
    prompt = inputs.make_prompts(WIDE_HEADS, 1, 70, seed=7)[0]
    prm = dict(TINY_SETS["scaled"], l_max=l_max, l_min=4)
    r = replay(WIDE_HEADS, W, prompt, 60, prm, device, logit_tol=2e-2)
    kinds = [t["kind"] for t in r["trace"] if t["op"] == "pass"]
    assert kinds.count("inblock") >= 5 and kinds.count("boundary") >= 2
    print("worst relative logit error", r["worst"], "passes", r["passes"])


def _free_run_matches(cfg, W_dev, prompts, N, prm, device, exact):
    prm = _f32(prm)
    Wn = inputs.weights_to_numpy(W_dev)
    model = api.Model(cfg, W_dev)
    dec = Decoder(model, len(prompts), prompts.shape[1], N, prm, device)
    got = dec.run(prompts)
    again = dec.run(prompts)
    assert (again["tokens"] == got["tokens"]).all() and again["nfe"] == got["nfe"]  # rerun is bit-identical
    mask = cfg["mask_id"]
    for b in range(len(prompts)):
        y = got["tokens"][b]
        assert (y[: prompts.shape[1]] == prompts[b]).all() and not (y == mask).any()
        assert sum(got["blocks"][b]) == N and got["blocks"][b][0] == min(prm.get("fixed_block") or prm["l_min"], N)
        assert sum(got["steps"][b]) == N and min(got["steps"][b]) >= 1
        if exact:
            ref = o_decode.decode_full(cfg, Wn, prompts[b], N, prm)
            assert got["blocks"][b] == ref["blocks"] and got["steps"][b] == ref["steps"] and got["nfe"][b] == ref["nfe"]
            assert (y == ref["tokens"]).all()
    dec.close()
    model.close()
    return got


@pytest.mark.parametrize("name", list(TINY_SETS))
def test_tiny_f32_free_run_equals_oracle(device, name):
    cfg = inputs.TINY
    W = _weights(cfg, 0, device)
    _free_run_matches(cfg, W, inputs.make_prompts(cfg, 1, 64), 64, TINY_SETS[name], device, exact=True)


@pytest.mark.parametrize("block,mode", [(16, 2), (32, 1), (24, 0)])
def test_tiny_f32_fixed_block_rules_equal_oracle(device, block, mode):
    """The comparison methods of Sec. 5.1 (fixed block size; vanilla, confidence-threshold or CAP selection) decode exactly
    as the oracle does."""
    cfg = inputs.TINY
    W = _weights(cfg, 0, device)
    prm = dict(inputs.PAPER_PARAMS, l_max=32, fixed_block=block, mode=mode, tau_low=0.05, tau_high=0.2, gamma=-14.0)
    _free_run_matches(cfg, W, inputs.make_prompts(cfg, 1, 64), 64, prm, device, exact=True)


def test_tiny_f32_ragged_batch(device):
    """Independent sequences packed into shared launches decode exactly as they do alone."""
    cfg = inputs.TINY
    W = _weights(cfg, 0, device)
    prompts = inputs.make_prompts(cfg, 5, 40, seed=9)
    prm = dict(TINY_SETS["scaled"], lam=1.0, l_max=16)
    got = _free_run_matches(cfg, W, prompts, 56, prm, device, exact=True)
    assert len({tuple(b) for b in got["blocks"]}) > 1 and len(set(got["nfe"])) > 1  # the sequences really are in different phases
    assert got["launches"] < sum(got["nfe"])  # and really share launches


def test_mid_bf16_batch_invariants(device):
    W = _weights(MID, 5, device)
    prompts = inputs.make_prompts(MID, 3, 64, seed=6)
    _free_run_matches(MID, W, prompts, 48, dict(TINY_SETS["scaled"], l_max=16), device, exact=False)


def test_step_errors_leave_state_untouched(device):
    cfg = inputs.TINY
    model = api.Model(cfg, _weights(cfg, 0, device))
    state = api.State(model, 2, 64, 48, 16)
    out = api.StepOutputs(48, cfg["vocab"], torch.float32, device)
    tokens = torch.zeros(64, dtype=torch.int32, device=device)
    ok = dict(row_offsets=[0, 8], span_start=[0], commit_len=[4], tok_start=[0])
    bad = [
        (dict(ok, row_offsets=[0, 49]), -3), (dict(ok, span_start=[3]), -1), (dict(ok, commit_len=[9]), -1),
        (dict(ok, row_offsets=[0, 0]), -1), (dict(ok, slot=[2]), -1), (dict(ok, kl_first=[0], kl_count=[2]), -1),
        (dict(ok, save_first=[0], save_count=[17], row_offsets=[0, 40]), -3), (dict(ok, save_first=[4], save_count=[8]), -1),
        (dict(row_offsets=[0, 8, 16], span_start=[0, 0], commit_len=[0, 0], tok_start=[0, 0], slot=[1, 1]), -1),
    ]
    for kw, code in bad:
        with pytest.raises(api.DlmError) as e:
            api.dlm_step(state, tokens, out, **kw)
        assert e.value.code == code, (kw, e.value)
        assert state.kv_len(0) == 0
    api.dlm_step(state, tokens, out, **ok)
    torch.cuda.synchronize()
    assert state.kv_len(0) == 4
    api.dlm_step(state, tokens, out, row_offsets=[0, 48], span_start=[4], commit_len=[44], tok_start=[0])
    assert state.kv_len(0) == 48
    with pytest.raises(api.DlmError) as e:  # span beyond max_seq_len
        api.dlm_step(state, tokens, out, row_offsets=[0, 48], span_start=[48], commit_len=[0], tok_start=[0])
    assert e.value.code == -3
    with pytest.raises(api.DlmError) as e:  # a suffix no pass has covered (positions [0, 52) have been)
        api.dlm_step(state, tokens, out, row_offsets=[0, 4], span_start=[48], commit_len=[0], tok_start=[0], suffix_len=[1])
    assert e.value.code == -1
    state.reset(0)
    assert state.kv_len(0) == 0
    torch.cuda.synchronize()
    state.close()
    model.close()


@pytest.mark.parametrize("which", ["f32", "bf16"])
def test_profile_classes_time_their_launches(device, which):
    """dlm_profile_enable / dlm_profile_read: every class counts its launches, the times are positive and together no more
    than the wall time of the passes, a masked class stays at zero, and profiling changes no output bit."""
    import time
    cfg = inputs.WORKLOADS["tiny_f32_p64_g64"][0] if which == "f32" else MID
    W = inputs.make_weights(cfg, seed=0, device=device)
    model = api.Model(cfg, W)
    rows, passes = 40, 5
    state = api.State(model, 1, 64, rows, 0)
    out = api.StepOutputs(rows, cfg["vocab"], model.torch_dtype, device)
    tokens = torch.from_numpy(inputs.make_prompts(cfg, 1, 64)[0].astype(np.int32)).to(device)

    def run():
        for _ in range(passes):
            api.dlm_step(state, tokens, out, [0, rows], [0], [0], [0])
        torch.cuda.synchronize()
        return out.logits[:rows].clone(), out.entropy[:rows].clone()

    plain = run()
    state.profile_enable(True)
    state.profile_read(reset=True)
    t0 = time.perf_counter()
    timed = run()
    wall_ms = (time.perf_counter() - t0) * 1e3
    prof = state.profile_read(reset=True)
    L = cfg["n_layers"]
    for name, per_pass in (("gemm_qkv", L), ("gemm_o", L), ("gemm_gate_up", L), ("gemm_down", L), ("gemm_lm_head", 1), ("attention", L),
                           ("vocab_stats", 1)):
        ms, n = prof[name]
        assert n == per_pass * passes and ms > 0, (name, prof[name])
    assert sum(ms for ms, _ in prof.values()) <= wall_ms, (prof, wall_ms)
    state.profile_enable(["gemm_gate_up"])
    only = run()
    prof = state.profile_read(reset=True)
    assert prof["gemm_gate_up"][1] == L * passes and prof["gemm_gate_up"][0] > 0
    assert all(v == (0.0, 0) for k, v in prof.items() if k != "gemm_gate_up"), prof
    state.profile_enable(False)
    for a, b in ((plain, timed), (plain, only)):
        assert torch.equal(a[0].view(torch.int16 if which == "bf16" else torch.int32), b[0].view(torch.int16 if which == "bf16" else torch.int32))
        assert torch.equal(a[1], b[1])
    state.close()
    model.close()


def test_tiny_f32_full_batch_of_32(device):
    """The largest batch a state holds (32 sequences) packed into shared launches, each decoding exactly as it does alone."""
    cfg = inputs.TINY
    W = _weights(cfg, 0, device)
    prompts = inputs.make_prompts(cfg, 32, 24, seed=3)
    got = _free_run_matches(cfg, W, prompts, 24, dict(TINY_SETS["scaled"], lam=1.0, l_max=8), device, exact=True)
    assert got["launches"] < sum(got["nfe"]) / 8


def test_tiny_f32_ragged_batch_with_visible_suffix(device):
    """Packed sequences with the look-ahead suffix visible to in-block passes: every sequence attends to its own suffix only."""
    cfg = inputs.TINY
    W = _weights(cfg, 0, device)
    prompts = inputs.make_prompts(cfg, 4, 40, seed=11)
    _free_run_matches(cfg, W, prompts, 56, dict(TINY_SETS["dual_cache"], l_max=16), device, exact=True)


@pytest.mark.parametrize("P,N", [(1, 1), (3, 5), (64, 8), (5, 9)])
def test_tiny_f32_degenerate_lengths(device, P, N):
    """Prompts of one token, generations shorter than L_min or than the look-ahead window: the window and the last block
    are cut at the end of the sequence."""
    cfg = inputs.TINY
    W = _weights(cfg, 0, device)
    _free_run_matches(cfg, W, inputs.make_prompts(cfg, 1, P, seed=P + N), N, TINY_SETS["scaled"], device, exact=True)


def _golden():
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_decode_golden", os.path.join(here, "make_decode_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    with open(os.path.join(here, "tiny_decode.json")) as f:
        return mod, json.load(f)


@pytest.mark.parametrize("name", ["paper", "scaled", "dual_cache", "threshold_block16", "vanilla_block32"])
def test_tiny_f32_free_run_equals_stored_decode(device, name):
    """The stored decodes (written from the oracle alone by tests/golden/make_decode_golden.py): block lengths, tokens
    written per pass, NFE and every token, exactly."""
    mod, gold = _golden()
    cfg = inputs.TINY
    W = _weights(cfg, 0, device)
    model = api.Model(cfg, W)
    P, N = gold["prompt_len"], gold["gen_len"]
    dec = Decoder(model, 1, P, N, _f32(mod.CASES[name]), device)
    got = dec.run(inputs.make_prompts(cfg, 1, P))
    ref = gold["cases"][name]
    assert got["blocks"][0] == ref["blocks"] and got["steps"][0] == ref["steps"] and got["nfe"][0] == ref["nfe"]
    assert got["tokens"][0].tolist() == ref["tokens"]
    dec.close()
    model.close()


# a vocabulary of 129 column groups of the LM head, the last one a quarter full; the mask token sits inside a group
WIDE_VOCAB = inputs.model_config(1, 256, 2, 2, 128, 512, 16416, "bf16")


@pytest.mark.parametrize("L", [1, 8, 24, 64])
def test_statistics_from_the_lm_head_epilogue(device, L):
    """An in-block pass (no row compared, none retained) takes its statistics from the LM head's epilogue: the same pass with that
    switched off gives the same logits bit for bit and the same statistics to rounding, and both agree with the oracle's statistics
    of those logits (Sec. 4.2 entropy; Sec. 4.3 confidence and prediction)."""
    cfg = WIDE_VOCAB
    W = _weights(cfg, 11, device)
    model = api.Model(cfg, W)
    P, look, mask = 40, 64, cfg["mask_id"]
    prompt = inputs.make_prompts(cfg, 1, P, seed=11)[0]
    tokens = torch.full((P + look,), mask, dtype=torch.int32, device=device)
    tokens[:P] = torch.from_numpy(prompt.astype(np.int32)).to(device)
    results = []
    for fused in (True, False):
        state = api.State(model, 1, P + look, P + look, look)
        state.fuse_stats(fused)
        out = api.StepOutputs(P + look, cfg["vocab"], model.torch_dtype, device)
        api.dlm_step(state, tokens, out, [0, P + look], [0], [P], [0], kl_first=[0], kl_count=[0], save_first=[P], save_count=[look])
        api.dlm_step(state, tokens, out, [0, L], [P], [0], [P], kl_first=[0], kl_count=[0], save_first=[0], save_count=[0])
        torch.cuda.synchronize()
        results.append({k: getattr(out, k)[:L].cpu().numpy() for k in ("max_logit", "lse", "entropy", "conf", "argmax", "kl")})
        results[-1]["z"] = o_fwd.widen(inputs.tensor_to_numpy(out.logits[:L]))
        state.close()
    a, b = results
    assert (a["z"] == b["z"]).all()
    st = o_stats.vocab_stats(a["z"], mask)
    for got in (a, b):
        for key in ("max_logit", "lse", "entropy", "conf"):
            assert (np.abs(got[key] - st[key]) <= 1e-5 * np.maximum(1.0, np.abs(st[key]))).all(), key
        assert (got["argmax"] == st["argmax"]).all() and (got["kl"] == 0).all()
    assert (a["max_logit"] == b["max_logit"]).all()
    model.close()


def test_sweep_harness_reports_the_oracles_counts(device):
    """The hyper-parameter / strategy sweep harness (App. B; the comparison methods of Sec. 5.1) on the tiny fp32 model: the NFE,
    tokens per pass and number of blocks it reports for each setting are the oracle's whole decode of the same setting."""
    from paper_2604_15750_amd import sweep
    cfg = inputs.TINY
    W = _weights(cfg, 0, device)
    Wn = inputs.weights_to_numpy(W)
    model = api.Model(cfg, W)
    P = 64
    prompts = inputs.make_prompts(cfg, 1, P)
    base = dict(inputs.PAPER_PARAMS, l_max=32, lam=0.9, tau_low=0.05, tau_high=0.3, gamma=-14.0)
    settings = [("DepCap", base, 64), ("DepCap, lambda 1.2", dict(base, lam=1.2), 64), ("confidence threshold, block 16", dict(base, fixed_block=16, mode=1, tau_high=0.2), 64),
                ("vanilla, block 32", dict(base, fixed_block=32, mode=2), 64), ("DepCap, L_gen 40", base, 40), ("DepCap, gamma -10", dict(base, gamma=-10.0), 64)]
    seen = set()
    for name, prm, n_gen in settings:
        got = sweep.run(model, cfg, 1, P, n_gen, prm, device, prompts)
        ref = o_decode.decode_full(cfg, Wn, prompts[0], n_gen, _f32(prm))
        assert got["nfe"] == ref["nfe"] and got["blocks"] == len(ref["blocks"]), (name, got, ref["nfe"], ref["blocks"])
        assert abs(got["tokens_per_pass"] - n_gen / ref["nfe"]) < 1e-12 and got["tokens_per_s"] > 0
        seen.add((got["nfe"], got["blocks"]))
    assert len(seen) >= 4  # the settings really decode differently
    model.close()
