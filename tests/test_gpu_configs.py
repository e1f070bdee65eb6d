"""The benchmark configurations at their full widths, vocabularies, prompt / generation lengths and
launch shapes, against the oracle.

The oracle needs about a minute for two passes through 32 layers of an 8B-shaped model, so only
configurations 1 and 2 are also run at full depth (the first passes, up to the first boundary pass for
configuration 1); each configuration is run as a
depth-reduced twin (same widths, heads, vocabulary, prompt and block sizes; 2 layers) and the oracle
decodes the first passes of it: the prefill pass (prompt + look-ahead rows, the widest launch), the
in-block denoising passes of the first block and the first boundary pass.  Every pass is fed to the
HIP path with the oracle's tokens and every output is compared (see test_gpu_step.replay: logits
2e-2 of the row maximum, statistics 1e-5 stage-isolated, KL against the retained logits, decisions
exact where the margin allows).
"""
import numpy as np
import pytest
import torch

from oracle import decode as o_decode
from oracle import forward as o_fwd
from paper_2604_15750_amd import api, inputs
from paper_2604_15750_amd.decode import Decoder
from test_gpu_step import SIGMA_LOGIT, _f32, replay

pytestmark = pytest.mark.gpu

# thresholds that let CAP-Decoding take several tokens per pass on random-init weights (their confidences are a few
# per cent to a few tens of per cent); lambda below 1 so that blocks grow beyond L_min
SCALED = dict(inputs.PAPER_PARAMS, **inputs.SCALED_THRESHOLDS)


def _twin(name, layers=2):
    cfg, B, P, N, lmax = inputs.WORKLOADS[name]
    return inputs.with_depth(cfg, layers), B, P, N, lmax


@pytest.mark.parametrize("name,passes", [("llada8b_p256_g256", 10), ("dream7b_p512_g256", 10), ("llada8b_p1024_g1024", 4)])
def test_twin_replay(device, name, passes):
    cfg, _, P, N, lmax = _twin(name)
    W = inputs.make_weights(cfg, seed=0, device=device)
    prompt = inputs.make_prompts(cfg, 1, P)[0]
    r = replay(cfg, W, prompt, N, dict(SCALED, l_max=lmax), device, logit_tol=2e-2, max_passes=passes)
    kinds = [t["kind"] for t in r["trace"] if t["op"] == "pass"]
    assert r["passes"] == passes and kinds[0] == "prefill" and "inblock" in kinds and "boundary" in kinds
    print(name, "passes", kinds, "worst relative logit error", r["worst"])


@pytest.mark.parametrize("name,rows", [("llada8b_p256_g256", 24), ("llada8b_p256_g256", 40), ("llada8b_p256_g256", 64), ("llada8b_p256_g256", 100),
                                       ("llada8b_p256_g256", 136), ("llada8b_p256_g256", 160), ("llada8b_p256_g256", 200), ("llada8b_p256_g256", 256),
                                       ("dream7b_p512_g256", 40), ("dream7b_p512_g256", 150),
                                       ("llada8b_p256_g256", 368), ("llada8b_p256_g256", 768)])  # 192 x 256 macro tiles, every epilogue
def test_twin_row_counts(device, name, rows):
    """One prefill pass of exactly `rows` rows at full widths (prompt of rows - 16 tokens, look-ahead 16), then the first
    in-block pass: the row counts at which the GEMM dispatcher changes kernel or tile shape, every fused epilogue included."""
    cfg, _, _, _, _ = _twin(name)
    W = inputs.make_weights(cfg, seed=0, device=device)
    prompt = inputs.make_prompts(cfg, 1, rows - 16)[0]
    r = replay(cfg, W, prompt, 32, dict(SCALED, l_max=8), device, logit_tol=2e-2, max_passes=2)
    first = [t for t in r["trace"] if t["op"] == "pass"][0]
    assert first["kind"] == "prefill" and len(first["tokens"]) == rows
    print(name, rows, "worst relative logit error", r["worst"])


def _bf16_dataflow(cfg, W, tokens, device):
    """The pass over `tokens` (no cached prefix) in exact fp32 torch operations with the activations rounded to bf16 at the
    points where a bf16 matrix-core path has to round them (every GEMM input, Q / K / V, the unnormalised attention
    probabilities, the logits); the residual stream, the norms, the rotary embedding and the softmax stay fp32.  An
    independent statement of what bf16 costs, with none of the kernels' code."""
    import math
    torch.backends.cuda.matmul.allow_tf32 = False
    r = lambda t: t.to(torch.bfloat16).float()
    hd, nq, nkv, ffn, eps = cfg["head_dim"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["d_ffn"], cfg["rms_eps"]
    rows = len(tokens)
    h = W["embed"][torch.from_numpy(np.asarray(tokens)).to(device)].float()
    inv = cfg["rope_theta"] ** (-2.0 * torch.arange(hd // 2, device=device, dtype=torch.float64) / hd)
    ang = torch.arange(rows, device=device, dtype=torch.float64)[:, None] * inv[None, :]
    cos, sin = torch.cos(ang).float()[:, None, :], torch.sin(ang).float()[:, None, :]
    rope = lambda x: torch.cat([x[..., : hd // 2] * cos - x[..., hd // 2:] * sin, x[..., hd // 2:] * cos + x[..., : hd // 2] * sin], -1)
    rinv_of = lambda t: torch.rsqrt((t * t).mean(-1, keepdim=True) + eps)
    for l in range(cfg["n_layers"]):
        qkv = (r(h * W["norm1"][l].float()) @ W["wqkv"][l].float().T) * rinv_of(h)
        q = r(rope(qkv[:, : nq * hd].view(rows, nq, hd)))
        k = r(rope(qkv[:, nq * hd: (nq + nkv) * hd].view(rows, nkv, hd))).repeat_interleave(nq // nkv, 1)
        v = r(qkv[:, (nq + nkv) * hd:].view(rows, nkv, hd)).repeat_interleave(nq // nkv, 1)
        s = torch.einsum("ahd,thd->hat", q, k) / math.sqrt(hd)
        e = torch.exp(s - s.max(-1, keepdim=True).values)
        o = torch.einsum("hat,thd->ahd", r(e), v) / e.sum(-1).permute(1, 0)[:, :, None]
        h = h + r(o.reshape(rows, nq * hd)) @ W["wo"][l].float().T
        gu = (r(h * W["norm2"][l].float()) @ W["w_gate_up"][l].float().T) * rinv_of(h)
        g, u = gu[:, :ffn], gu[:, ffn:]
        h = h + r(g / (1 + torch.exp(-g)) * u) @ W["w_down"][l].float().T
    return r((r(h * W["final_norm"].float()) @ W["lm_head"].float().T) * rinv_of(h)).double().cpu().numpy()


def test_full_depth_first_passes(device):
    """Configuration 1 at its full size (32 layers, 15 GB of bf16 weights): the prefill pass (384 rows, the launch
    configuration of the benchmark's first pass), the in-block denoising passes of the first block (8 rows: the kernels the
    benchmark spends its time in) and the first boundary pass (136 rows, KL rows against the retained prefill logits), every
    logit and statistic against the oracle run at full depth on the host, at the benchmark spec's tolerance: 2e-2 of
    max(row maximum, sigma_logit) for the worst logit of every row.

    What keeps the path well inside that bound at this depth is what the kernels feed the matrix cores: IEEE half (11
    significant bits) for every GEMM input, the packed weights and the attention operands, instead of bf16's 8 bits; the
    measured worst logit error is 0.5e-2, and the test also holds the path to 1e-2 so that a lost bit somewhere shows.  The
    same pass in exact fp32 torch operations with every activation rounded to bf16 between the GEMMs is printed beside it, as
    information: that dataflow is about 2.3e-2 (relative L2 per row) from the oracle, whoever does the arithmetic."""
    cfg, _, P, N, lmax = inputs.WORKLOADS["llada8b_p256_g256"]
    W = inputs.make_weights(cfg, seed=0, device=device)
    prompt = inputs.make_prompts(cfg, 1, P)[0]
    st = []
    r = replay(cfg, W, prompt, N, dict(SCALED, l_max=lmax), device, logit_tol=2e-2, max_passes=12, stats_out=st, stop_after="boundary")
    kinds = [t["kind"] for t in r["trace"] if t["op"] == "pass"]
    assert kinds[0] == "prefill" and kinds[-1] == "boundary" and "inblock" in kinds, kinds
    assert r["boundaries"] == 1 and r["worst"] <= 2e-2
    assert r["worst"] <= 1e-2 and r["rms"] <= 6e-3, st  # (measured 0.5e-2 and 0.37e-2)
    pre = [t for t in r["trace"] if t["op"] == "pass"][0]
    ref = pre["logits"]
    emu = _bf16_dataflow(cfg, W, pre["tokens"], device)
    emu_rms = float((np.sqrt(np.mean((emu - ref) ** 2, -1)) / np.sqrt(np.mean(ref ** 2, -1))).max())
    print("full depth:", kinds, st, "all-bf16 dataflow in fp32 torch operations (information):", emu_rms)


def test_full_depth_grouped_query_first_passes(device):
    """Configuration 2 at its full size (Dream-7B shape: 28 layers, 28 query / 4 kv heads, FFN 18944, vocabulary 152064):
    the prefill pass (512 + 128 = 640 rows) and the first in-block pass (8 rows against 512 cached keys), every logit and
    statistic against the oracle at full depth, at the benchmark spec's tolerance."""
    cfg, _, P, N, lmax = inputs.WORKLOADS["dream7b_p512_g256"]
    W = inputs.make_weights(cfg, seed=0, device=device)
    prompt = inputs.make_prompts(cfg, 1, P)[0]
    st = []
    r = replay(cfg, W, prompt, N, dict(SCALED, l_max=lmax), device, logit_tol=2e-2, max_passes=2, stats_out=st)
    kinds = [t["kind"] for t in r["trace"] if t["op"] == "pass"]
    assert kinds == ["prefill", "inblock"] and r["worst"] <= 2e-2
    assert r["worst"] <= 1e-2, st  # (measured 0.54e-2)
    print("full depth, grouped-query shape:", st)


def _widened(Wn):
    """The bf16 weights widened to fp64 once (exactly, by the oracle's own routine) instead of on every use: the oracle then
    spends its time on the arithmetic, and many passes of a depth-reduced twin fit a test."""
    return {k: [o_fwd.widen(t) for t in v] if isinstance(v, list) else o_fwd.widen(v) for k, v in Wn.items()}


def _compare_pass(out, r0, rows, ref_logits, mask, prev_gpu, klf, klc, tol):
    """One sequence's rows [r0, r0 + rows) of a launch against the oracle: every logit within tol of max(row maximum,
    sigma_logit); statistics stage-isolated (the oracle's statistics of the GPU's own logits) at 1e-5; KL rows against the
    oracle's KL of the GPU's own current and retained logits.  Returns (worst relative logit error, the GPU's logits fp64)."""
    from oracle import stats as o_stats
    z = o_fwd.widen(inputs.tensor_to_numpy(out.logits[r0: r0 + rows]))
    scale = np.maximum(np.abs(ref_logits).max(-1, keepdims=True), SIGMA_LOGIT)
    err = float((np.abs(z - ref_logits) / scale).max())
    assert err <= tol, err
    st = o_stats.vocab_stats(z, mask)
    got = {k: getattr(out, k)[r0: r0 + rows].cpu().numpy() for k in ("max_logit", "lse", "entropy", "conf", "argmax", "kl")}
    for key in ("max_logit", "lse", "entropy", "conf"):
        assert (np.abs(got[key] - st[key]) <= 1e-5 * np.maximum(1.0, np.abs(st[key]))).all(), key
    assert (got["argmax"] == st["argmax"]).all()
    kl_ref, spread = np.zeros(rows), np.zeros(rows)
    if klc:
        kst = o_stats.vocab_stats(z[klf: klf + klc], mask, prev_gpu)
        kl_ref[klf: klf + klc] = kst["kl"]
        logp, _, _ = o_stats.log_softmax_masked(z[klf: klf + klc], mask)
        logq, _, _ = o_stats.log_softmax_masked(prev_gpu, mask)
        fin = lambda a: np.where(np.isfinite(a), a, 0.0)
        spread[klf: klf + klc] = np.sum(np.exp(logp) * np.abs(fin(logp) - fin(logq)), -1)
    assert (np.abs(got["kl"] - kl_ref) <= 1e-5 * np.maximum(1.0, np.abs(kl_ref)) + 1e-5 * spread).all()
    return err, z


def test_long_context_late_passes(device):
    """Configuration 3 (prompt 1024 + generation 1024, L_max 128) late in its decode, on the depth-reduced twin: passes whose
    key counts run from 1784 to the full 2048 positions - a 1912-row prefill, in-block passes of 128 and 8 rows, a 384-row
    boundary pass over 2040 keys with 128 KL rows, and the last boundary pass of the sequence - teacher-forced with the same
    tokens on both sides and compared row by row with the oracle's forward pass, statistics and KL."""
    cfg, _, P, N, lmax = _twin("llada8b_p1024_g1024")
    T, mask, V = P + N, cfg["mask_id"], cfg["vocab"]
    W = inputs.make_weights(cfg, seed=0, device=device)
    Wn = _widened(inputs.weights_to_numpy(W))
    model = api.Model(cfg, W)
    del W
    rng = np.random.default_rng(3)
    y = np.full(T, mask, dtype=np.int64)
    F0 = 1656
    y[:F0] = rng.integers(0, V - 1, F0)
    look = 2 * lmax
    state = api.State(model, 1, T, F0 + look, look)
    out = api.StepOutputs(F0 + look, V, model.torch_dtype, device)
    tokens = torch.empty(T, dtype=torch.int32, device=device)
    cache = o_fwd.KVCache(cfg)
    prev = None  # (first position, GPU logits) retained by the last prefill / boundary pass
    worst, keys_seen = 0.0, []

    def run(kind, s0, rows, commit):
        nonlocal prev, worst
        klf = klc = svf = svc = 0
        if kind == "prefill":
            svf, svc = commit, rows - commit
        elif kind == "boundary":
            klf, klc = commit, min(lmax, T - (s0 + commit))
            svf, svc = commit, rows - commit
        tokens.copy_(torch.from_numpy(y.astype(np.int32)))
        api.dlm_step(state, tokens, out, [0, rows], [s0], [commit], [s0], kl_first=[klf], kl_count=[klc], save_first=[svf], save_count=[svc])
        torch.cuda.synchronize()
        ref = o_fwd.forward_span(cfg, Wn, cache, y[s0: s0 + rows], s0, commit)
        zp = prev[1][s0 + klf - prev[0]: s0 + klf - prev[0] + klc] if klc else None
        err, z = _compare_pass(out, 0, rows, ref, mask, zp, klf, klc, 2e-2)
        worst = max(worst, err)
        keys_seen.append(s0 + rows)
        if svc:
            prev = (s0 + svf, z[svf: svf + svc])
        assert state.kv_len(0) == s0 + commit

    run("prefill", 0, F0 + look, F0)                      # 1912 rows; look-ahead [1656, 1912) retained
    y[F0: F0 + 40] = rng.integers(0, V - 1, 40)           # the block [1656, 1784) partly decoded
    run("inblock", F0, lmax, 0)                           # 128 rows against 1656 cached keys
    y[F0: F0 + lmax] = rng.integers(0, V - 1, lmax)       # block finished
    run("boundary", F0, lmax + look, lmax)                # 384 rows, 2040 keys; KL rows [1784, 1912)
    F1 = F0 + lmax
    y[F1 + 3] = int(rng.integers(0, V - 1))
    run("inblock", F1, 8, 0)                              # 8 rows against 1784 cached keys
    y[F1: F1 + 50] = rng.integers(0, V - 1, 50)
    run("inblock", F1, lmax, 0)                           # 128 rows, 1912 keys
    y[F1: F1 + lmax] = rng.integers(0, V - 1, lmax)
    run("boundary", F1, lmax + (T - F1 - lmax), lmax)     # the last boundary pass: 264 rows up to position 2048
    assert max(keys_seen) == T and min(keys_seen[1:]) >= 1784
    print("keys per pass", keys_seen, "worst relative logit error", worst)
    state.close()
    model.close()


def test_batch16_packed_replay(device):
    """Config 4: 16 independent sequences (prompt 256, generation 512, L_max 64) of the depth-reduced twin.  The oracle decodes
    the first passes of every sequence alone; the HIP path is fed the oracle's tokens (teacher-forced: a low-margin selection
    cannot make the two sides diverge) with the k-th pass of EVERY sequence packed into shared launches - two launches of
    eight 384-row prefill spans, then launches that mix sequences on boundary passes (KL rows, retained rows, commits) with
    sequences on in-block passes of ragged lengths.  Every pass of every sequence is compared (logits, statistics, KL), and
    block_boundary / select_parallel run packed on the GPU's own statistics must take the oracle rule's decisions."""
    from oracle import boundary as o_boundary, select as o_select
    cfg, B, P, N, lmax = _twin("llada8b_b16_p256_g512")
    prm = _f32(dict(SCALED, l_max=lmax))
    T, mask, look, iters = P + N, cfg["mask_id"], 2 * lmax, 4
    W = inputs.make_weights(cfg, seed=0, device=device)
    Wn = _widened(inputs.weights_to_numpy(W))
    prompts = inputs.make_prompts(cfg, B, P)
    model = api.Model(cfg, W)
    del W
    traces = []
    for b in range(B):
        tr = []
        o_decode.decode_full(cfg, Wn, prompts[b], N, prm, tr, max_passes=iters)
        traces.append(tr)
    max_rows = 8 * (P + look)
    state = api.State(model, B, T, max_rows, look)
    out = api.StepOutputs(max_rows, cfg["vocab"], model.torch_dtype, device)
    tokens = torch.full((B, T), mask, dtype=torch.int32, device=device)
    sel = torch.zeros(max_rows, dtype=torch.uint8, device=device)
    nsel = torch.zeros(B, dtype=torch.int32, device=device)
    L_dev = torch.zeros(B, dtype=torch.int32, device=device)
    mg = torch.zeros(B, dtype=torch.float32, device=device)
    prev = [None] * B
    compared, mixed_launches, worst = 0, 0, 0.0
    # per sequence: its records grouped by pass (a pass record followed by the decisions taken on it)
    per_pass = []
    for tr in traces:
        groups = []
        pending = []  # decisions recorded before the pass they belong to come after it in the trace: select follows its pass,
        for rec in tr:  # but the prefill's / boundary's records are [pass, (boundary), select]
            if rec["op"] == "pass":
                groups.append(dict(p=rec, boundary=None, select=None))
            elif rec["op"] == "boundary":
                groups[-1]["boundary"] = rec
            elif groups:
                if groups[-1]["select"] is None:
                    groups[-1]["select"] = rec
        per_pass.append(groups[:iters])
    assert all(len(g) == iters for g in per_pass)
    for k in range(iters):
        todo = list(range(B))
        while todo:
            group, rows_total = [], 0
            while todo and rows_total + len(per_pass[todo[0]][k]["p"]["tokens"]) <= max_rows:
                b = todo.pop(0)
                group.append(b)
                rows_total += len(per_pass[b][k]["p"]["tokens"])
            row_off, desc = [0], dict(span=[], commit=[], klf=[], klc=[], svf=[], svc=[])
            for b in group:
                rec = per_pass[b][k]["p"]
                s0, rows, commit = rec["span_start"], len(rec["tokens"]), rec["commit_len"]
                tokens[b, s0: s0 + rows] = torch.from_numpy(rec["tokens"].astype(np.int32)).to(device)
                klf = klc = svf = svc = 0
                if rec["kind"] == "prefill":
                    svf, svc = P, rows - P
                elif rec["kind"] == "boundary":
                    klf, klc = commit, min(lmax, T - (s0 + commit))
                    svf, svc = commit, rows - commit
                row_off.append(row_off[-1] + rows)
                for key, v in zip(("span", "commit", "klf", "klc", "svf", "svc"), (s0, commit, klf, klc, svf, svc)):
                    desc[key].append(v)
            kinds = {per_pass[b][k]["p"]["kind"] for b in group}
            mixed_launches += len(kinds) > 1
            api.dlm_step(state, tokens, out, row_off, desc["span"], desc["commit"], [b * T + s for b, s in zip(group, desc["span"])], slot=group,
                         kl_first=desc["klf"], kl_count=desc["klc"], save_first=desc["svf"], save_count=desc["svc"])
            torch.cuda.synchronize()
            zs = {}
            for i, b in enumerate(group):
                rec = per_pass[b][k]["p"]
                s0, rows = desc["span"][i], row_off[i + 1] - row_off[i]
                klf, klc = desc["klf"][i], desc["klc"][i]
                zp = prev[b][1][s0 + klf - prev[b][0]: s0 + klf - prev[b][0] + klc] if klc else None
                err, z = _compare_pass(out, row_off[i], rows, rec["logits"], mask, zp, klf, klc, 2e-2)
                worst = max(worst, err)
                zs[b] = z
                if desc["svc"][i]:
                    prev[b] = (s0 + desc["svf"][i], z[desc["svf"][i]: desc["svf"][i] + desc["svc"][i]])
                compared += 1
            # DepGA-Block, packed over the sequences of this launch that have just finished a block (or the prompt)
            bnd = [i for i, b in enumerate(group) if per_pass[b][k]["p"]["kind"] != "inblock"]
            if bnd:
                starts, lens, cold = [], [], []
                for i in bnd:
                    b = group[i]
                    if per_pass[b][k]["p"]["kind"] == "prefill":
                        starts.append(row_off[i] + P); lens.append(min(lmax, N)); cold.append(1)
                    else:
                        starts.append(row_off[i] + desc["klf"][i]); lens.append(desc["klc"][i]); cold.append(0)
                api.block_boundary(out.kl, out.entropy, starts, lens, L_dev, prm["lam"], prm["l_min"], prm["smooth_radius"], prm["norm_mode"],
                                   prm["rule"], cold=cold, margin_out=mg)
                torch.cuda.synchronize()
                Ls = L_dev[: len(bnd)].cpu().numpy()
                for j, i in enumerate(bnd):
                    b = group[i]
                    kl = out.kl[starts[j]: starts[j] + lens[j]].cpu().numpy().astype(np.float64)
                    H = out.entropy[starts[j]: starts[j] + lens[j]].cpu().numpy().astype(np.float64)
                    Lr, _, mr = o_boundary.block_boundary(kl, H, prm["lam"], prm["l_min"], prm["smooth_radius"], prm["norm_mode"], prm["rule"],
                                                          cold_start=bool(cold[j]))
                    if cold[j] or mr > 1e-4:
                        assert int(Ls[j]) == Lr, (b, k, int(Ls[j]), Lr, mr)
            # CAP-Decoding, packed over every sequence of the launch, on the block the oracle's trace names
            row_start, tok_start, blen = [], [], []
            for i, b in enumerate(group):
                srec = per_pass[b][k]["select"]
                row_start.append(row_off[i] + srec["F"] - desc["span"][i]); tok_start.append(b * T + srec["F"]); blen.append(srec["L"])
            before = tokens.clone()
            api.select_parallel(out.logits, out.lse, out.conf, out.argmax, tokens, row_start, tok_start, blen, mask, prm["tau_low"],
                                prm["tau_high"], prm["gamma"], prm.get("mode", 0), sel, nsel, apply_tokens=True, margin_out=mg)
            torch.cuda.synchronize()
            for i, b in enumerate(group):
                srec = per_pass[b][k]["select"]
                F, L, r0 = srec["F"], srec["L"], row_start[i]
                elig = before[b, F: F + L].cpu().numpy() == mask
                assert (elig == srec["eligible"]).all()
                zb = zs[b][r0 - row_off[i]: r0 - row_off[i] + L]
                g = {kk: getattr(out, kk)[r0: r0 + L].cpu().numpy() for kk in ("lse", "conf", "argmax")}
                ref_sel, mr = o_select.select_parallel(zb, g["lse"], g["conf"], g["argmax"], elig, prm["tau_low"], prm["tau_high"], prm["gamma"],
                                                       prm.get("mode", 0))
                got_sel = sel[r0: r0 + L].cpu().numpy().astype(bool)
                assert got_sel.sum() >= 1 and not (got_sel & ~elig).any()
                if mr > 1e-5:
                    assert (got_sel == ref_sel).all() and int(nsel[i]) == ref_sel.sum(), (b, k, mr)
                    after = tokens[b, F: F + L].cpu().numpy()
                    assert (after == np.where(ref_sel, g["argmax"], before[b, F: F + L].cpu().numpy())).all()  # Eq. 2
    assert compared == B * iters and mixed_launches >= 1, (compared, mixed_launches)
    print("passes compared", compared, "launches mixing pass kinds", mixed_launches, "worst relative logit error", worst)
    state.close()
    model.close()


def test_step_rerun_is_bit_identical(device):
    """The same pass launched repeatedly gives the same bits: reductions have a fixed order, and the partial tiles
    and tickets that cross workgroups inside a launch are coherent (a stale read would show up as a difference)."""
    cfg, _, P, N, lmax = _twin("llada8b_p256_g256")
    W = inputs.make_weights(cfg, seed=0, device=device)
    model = api.Model(cfg, W)
    del W
    mask = cfg["mask_id"]
    look = 2 * lmax
    for rows_block in (8, 40, 64):  # skinny kernels; then with the look-ahead rows the tiled ones
        state = api.State(model, 1, P + N, P + look, look)
        out = api.StepOutputs(P + look, cfg["vocab"], model.torch_dtype, device)
        tokens = torch.full((P + N,), mask, dtype=torch.int32, device=device)
        tokens[:P] = torch.from_numpy(inputs.make_prompts(cfg, 1, P)[0].astype(np.int32)).to(device)
        api.dlm_step(state, tokens, out, [0, P + look], [0], [P], [0], save_first=[P], save_count=[look])
        first = {}
        for rep in range(12):
            for rows in (rows_block, rows_block + look):
                api.dlm_step(state, tokens, out, [0, rows], [P], [0], [P])
                torch.cuda.synchronize()
                got = (out.logits[:rows].view(torch.int16).clone(), out.lse[:rows].clone(), out.argmax[:rows].clone())
                if rows not in first:
                    first[rows] = got
                else:
                    for x, y in zip(got, first[rows]):
                        assert torch.equal(x, y), (rows, rep)
        state.close()
    # 257 .. 512 rows: the macro-tile kernel splits K for the narrow matrices (O, down)
    state = api.State(model, 1, P + N, 400, 0)
    out = api.StepOutputs(400, cfg["vocab"], model.torch_dtype, device)
    tokens = torch.from_numpy(inputs.make_prompts(cfg, 1, P + N)[0].astype(np.int32)).to(device)
    first = {}
    for rep in range(8):
        for rows in (300, 400):
            api.dlm_step(state, tokens, out, [0, rows], [0], [0], [0])
            torch.cuda.synchronize()
            got = (out.logits[:rows].view(torch.int16).clone(), out.lse[:rows].clone(), out.argmax[:rows].clone())
            if rows not in first:
                first[rows] = got
            else:
                for x, y in zip(got, first[rows]):
                    assert torch.equal(x, y), (rows, rep)
    state.close()
    model.close()


@pytest.mark.parametrize("thresholds", ["scaled", "paper"])
def test_full_depth_decode_invariants_and_decisions(device, thresholds):
    """A whole decode of configuration 1 at full depth on the GPU (the run the benchmark times), checked without an oracle
    forward pass: the invariants of the decode schedule, and every decision re-taken by the oracle from the GPU's own
    outputs of that pass - the statistics of the block's logits recomputed in fp64, DepGA-Block on the GPU's KL / entropy
    profile, CAP-Decoding on the GPU's logits - exact wherever the oracle's decision margin exceeds the fp32 tolerance."""
    from oracle import boundary as o_boundary, select as o_select, stats as o_stats
    cfg, B, P, N, lmax = inputs.WORKLOADS["llada8b_p256_g256"]
    prm = _f32(dict(SCALED if thresholds == "scaled" else inputs.PAPER_PARAMS, l_max=lmax))
    W = inputs.make_weights(cfg, seed=0, device=device)
    model = api.Model(cfg, W)
    del W
    prompts = inputs.make_prompts(cfg, 1, P)
    dec = Decoder(model, 1, P, N, prm, device)
    trace = []
    got = dec.run(prompts, trace)
    mask = cfg["mask_id"]
    y, blocks, steps, nfe = got["tokens"][0], got["blocks"][0], got["steps"][0], got["nfe"][0]
    # schedule invariants (Sec. 3, 4.2): the prompt is kept, nothing stays masked, the blocks partition the generation, every
    # block but the last lies in [L_min, L_max], the first is L_min, every pass decodes at least one token
    assert (y[:P] == prompts[0]).all() and not (y == mask).any()
    assert sum(blocks) == N and blocks[0] == prm["l_min"] and all(prm["l_min"] <= b <= lmax for b in blocks[:-1]) and 1 <= blocks[-1] <= lmax
    assert sum(steps) == N and min(steps) >= 1 and len(blocks) <= nfe <= N and nfe == len(steps)
    n_sel = n_bnd = exact_sel = exact_bnd = 0
    last = None
    for rec in trace:
        if rec["op"] == "pass":
            last = rec
        elif rec["op"] == "boundary":
            Lr, _, mr = o_boundary.block_boundary(rec["kl"].astype(np.float64), rec["entropy"].astype(np.float64), prm["lam"], prm["l_min"],
                                                  prm["smooth_radius"], prm["norm_mode"], prm["rule"], cold_start=rec["cold"])
            n_bnd += 1
            if mr > 1e-4:
                exact_bnd += 1
                assert rec["L"] == Lr, (rec["F"], rec["L"], Lr, mr)
        elif rec["op"] == "select":
            F, L = rec["F"], rec["L"]
            r0 = F - last["span_start"]
            z = o_fwd.widen(inputs.tensor_to_numpy(last["logits"][r0: r0 + L]))
            st = o_stats.vocab_stats(z, mask)
            elig = last["tokens"][r0: r0 + L] == mask
            ref_sel, mr = o_select.select_parallel(z, st["lse"], st["conf"], st["argmax"], elig, prm["tau_low"], prm["tau_high"], prm["gamma"],
                                                   prm.get("mode", 0))
            n_sel += 1
            assert rec["selected"].sum() >= 1 and not (rec["selected"] & ~elig).any()
            if mr > 1e-5:
                exact_sel += 1
                assert (rec["selected"] == ref_sel).all(), (F, L, mr)
    assert n_sel == nfe and n_bnd == len(blocks)  # the first block's (cold-start) decision included
    assert exact_sel >= 0.9 * n_sel and exact_bnd >= 0.8 * n_bnd, (exact_sel, n_sel, exact_bnd, n_bnd)
    print(thresholds, "NFE", nfe, "blocks", blocks, "selections checked exactly", exact_sel, "of", n_sel, "boundaries", exact_bnd, "of", n_bnd)
    dec.close()
    model.close()


@pytest.mark.parametrize("name", ["llada8b_p256_g256", "dream7b_p512_g256"])
def test_step_major_weight_copies_change_no_bit(device, name):
    """The second, step-major copies of the layer matrices that narrow passes read (all four matrices at these widths) hold the
    same fragments in another order, and the kernels add the same products in the same order: a prefill pass (standard layout
    either way) and in-block passes of 8 to 64 rows give bit-identical logits and statistics with and without the copies."""
    cfg, _, _, _, _ = _twin(name)
    W = inputs.make_weights(cfg, seed=0, device=device)
    P, look = 48, 64
    tokens = torch.full((P + look,), cfg["mask_id"], dtype=torch.int32, device=device)
    tokens[:P] = torch.from_numpy(inputs.make_prompts(cfg, 1, P)[0].astype(np.int32)).to(device)
    results = []
    for copies in (True, False):
        model = api.Model(cfg, W, weight_copies=copies)
        got = []
        for L in (8, 16, 32, 48, 64):
            state = api.State(model, 1, P + look, P + look, look)
            out = api.StepOutputs(P + look, cfg["vocab"], model.torch_dtype, device)
            api.dlm_step(state, tokens, out, [0, P + look], [0], [P], [0], kl_first=[0], kl_count=[0], save_first=[P], save_count=[look])
            api.dlm_step(state, tokens, out, [0, L], [P], [0], [P], kl_first=[0], kl_count=[0], save_first=[0], save_count=[0])
            torch.cuda.synchronize()
            got.append([out.logits[:L].clone()] + [getattr(out, k)[:L].clone() for k in ("max_logit", "lse", "entropy", "conf", "argmax")])
            state.close()
        results.append(got)
        model.close()
    for a, b in zip(*results):
        for x, y in zip(a, b):
            assert torch.equal(x, y)
    assert float(results[0][0][0].float().abs().max()) > 0
