"""Seeded synthetic inputs: model shapes, random-init weights, prompts.

Holds none of the method's arithmetic.  Both the HIP path and the CPU checker
are fed from here, so that they read the same bytes.  The shapes are those of
the five benchmark configurations; weights are N(0, 0.02^2) with the LM head at
N(0, (4/sqrt(d))^2) so that logits have standard deviation about 4 (the final
RMSNorm output has unit RMS); norm gains are 1; prompts are uniform token ids
on [0, V-1); generation slots hold the mask id V-1.
"""
import math

import numpy as np
import torch


def model_config(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, dtype):
    return dict(
        n_layers=n_layers, d_model=d_model, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
        head_dim=head_dim, d_ffn=d_ffn, vocab=vocab, mask_id=vocab - 1, dtype=dtype,
        rms_eps=1e-5, rope_theta=10000.0,
    )


TINY = model_config(2, 128, 4, 4, 32, 384, 1024, "f32")
LLADA_8B = model_config(32, 4096, 32, 32, 128, 12288, 126464, "bf16")
DREAM_7B = model_config(28, 3584, 28, 4, 128, 18944, 152064, "bf16")

# name -> (model, batch, prompt_len, gen_len, l_max)
WORKLOADS = {
    "tiny_f32_p64_g64": (TINY, 1, 64, 64, 32),
    "llada8b_p256_g256": (LLADA_8B, 1, 256, 256, 64),
    "dream7b_p512_g256": (DREAM_7B, 1, 512, 256, 64),
    "llada8b_p1024_g1024": (LLADA_8B, 1, 1024, 1024, 128),
    "llada8b_b16_p256_g512": (LLADA_8B, 16, 256, 512, 64),
}

# hyper-parameters of Sec. 5.1 of the paper (L_max comes with the workload)
PAPER_PARAMS = dict(l_min=8, lam=1.2, smooth_radius=1, norm_mode=0, rule=0,
                    tau_low=0.8, tau_high=0.95, gamma=-16.0, mode=0)
# A random-init model never reaches those confidences (it commits one token per pass).  This second set puts the thresholds
# inside the confidence range such a model does reach at the benchmark vocabularies, so that every branch of the selection
# rule runs and passes commit several tokens.
SCALED_THRESHOLDS = dict(lam=0.9, tau_low=0.04, tau_high=0.25, gamma=-36.0)


def with_depth(cfg, n_layers):
    """Same widths and vocabulary, fewer layers (a twin the CPU checker can run whole)."""
    c = dict(cfg)
    c["n_layers"] = n_layers
    return c


def _gen(device, *key):
    g = torch.Generator(device=device)
    seed = 0
    for k in key:  # mix the key into one 63-bit seed
        seed = (seed * 1000003 + int(k) + 12345) % (2**63 - 1)
    g.manual_seed(seed)
    return g


def _normal(shape, std, dt, device, *key):
    n = 1
    for s in shape:
        n *= s
    out = torch.empty(shape, dtype=dt, device=device)
    flat = out.view(-1)
    g = _gen(device, *key)
    chunk = 1 << 26  # bound the fp32 temporary
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        flat[lo:hi] = (torch.randn(hi - lo, generator=g, dtype=torch.float32, device=device) * std).to(dt)
    return out


def make_weights(cfg, seed=0, device="cpu"):
    """Dict of torch tensors in the model dtype, row-major [out, in]; per-layer entries are lists."""
    dt = torch.float32 if cfg["dtype"] == "f32" else torch.bfloat16
    d, hd, ffn, V = cfg["d_model"], cfg["head_dim"], cfg["d_ffn"], cfg["vocab"]
    nq, nkv = cfg["n_q_heads"], cfg["n_kv_heads"]
    W = dict(
        embed=_normal((V, d), 0.02, dt, device, seed, 0, 0),
        final_norm=torch.ones(d, dtype=dt, device=device),
        lm_head=_normal((V, d), 4.0 / math.sqrt(d), dt, device, seed, 0, 1),
        wqkv=[], wo=[], w_gate_up=[], w_down=[], norm1=[], norm2=[],
    )
    for l in range(cfg["n_layers"]):
        W["wqkv"].append(_normal(((nq + 2 * nkv) * hd, d), 0.02, dt, device, seed, 1 + l, 0))
        W["wo"].append(_normal((d, nq * hd), 0.02, dt, device, seed, 1 + l, 1))
        W["w_gate_up"].append(_normal((2 * ffn, d), 0.02, dt, device, seed, 1 + l, 2))
        W["w_down"].append(_normal((d, ffn), 0.02, dt, device, seed, 1 + l, 3))
        W["norm1"].append(torch.ones(d, dtype=dt, device=device))
        W["norm2"].append(torch.ones(d, dtype=dt, device=device))
    return W


def make_prompts(cfg, batch, prompt_len, seed=0):
    """int64 numpy [batch, prompt_len], uniform on [0, V-1) (never the mask id)."""
    out = np.empty((batch, prompt_len), dtype=np.int64)
    for b in range(batch):
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 1000 + b])))
        out[b] = rng.integers(0, cfg["vocab"] - 1, size=prompt_len)
    return out


def tensor_to_numpy(t):
    """Host numpy view for the CPU checker: fp32 as is, bf16 as its uint16 bit pattern."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def weights_to_numpy(W):
    return {k: [tensor_to_numpy(x) for x in v] if isinstance(v, list) else tensor_to_numpy(v) for k, v in W.items()}


def peaked_logits(rows, vocab, seed, peak=None, sigma=4.0, dtype=np.float32):
    """Logits ~ N(0, sigma^2) with an optional planted peak per row.

    peak: list of (row, token, height) triples added on top; gives confident
    rows so that every branch of the selection rule is reachable.
    """
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 77])))
    z = (rng.standard_normal((rows, vocab)) * sigma).astype(dtype)
    for r, tok, hgt in peak or []:
        z[r, tok] += hgt
    return z
