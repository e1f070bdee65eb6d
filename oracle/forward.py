"""Oracle: forward pass of the masked-diffusion transformer over one span.

TEST INFRASTRUCTURE (see oracle/__init__.py).  fp64 throughout.

The paper (Sec. 3, "Diffusion language model inference") treats the model as a
black box that maps prompt + current target sequence to per-position predictive
distributions using bidirectional context.  The architecture is the one the
benchmark configurations name: pre-norm transformer, RMSNorm, rotary position
embedding (half-split pairs), multi-/grouped-query attention without a causal
mask, SwiGLU feed-forward, untied LM head, no biases.

Weights are a dict of numpy arrays, row-major [out, in]:
  embed [V,d]; per layer (lists): wqkv [(Hq+2Hkv)*hd, d] (Q rows, then K rows,
  then V rows), wo [d, Hq*hd], w_gate_up [2*ffn, d] (gate rows, then up rows),
  w_down [d, ffn], norm1 [d], norm2 [d]; final_norm [d]; lm_head [V,d].
A uint16 array holds bfloat16 bit patterns and is widened exactly.
"""
import numpy as np


def widen(a):
    """Exact widening to fp64.  uint16 = bfloat16 bits (upper half of an fp32)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def matmul_nt(x, w):
    """y[r, o] = sum_i x[r, i] * w[o, i]."""
    return widen(x) @ widen(w).T


def rmsnorm(x, g, eps):
    """x / sqrt(mean(x^2) + eps) * g, per row."""
    x = widen(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * widen(g)


def rope(x, pos, theta):
    """Rotary embedding, half-split pairing.

    x [rows, heads, hd]; pos [rows] absolute positions.  Pair (i, i+hd/2),
    i < hd/2, is rotated by the angle pos * theta**(-2i/hd).
    """
    x = widen(x)
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]
    cos = np.cos(ang)[:, None, :]
    sin = np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * cos - x2 * sin, x2 * cos + x1 * sin], axis=-1)


def attention(q, k, v):
    """Bidirectional softmax attention (no causal mask).

    q [A, Hq, hd]; k, v [T, Hkv, hd]; query head h reads kv head h // (Hq//Hkv).
    Every query row sees all T keys.  Scale 1/sqrt(hd).
    """
    q, k, v = widen(q), widen(k), widen(v)
    A, Hq, hd = q.shape
    Hkv = k.shape[1]
    group = Hq // Hkv
    out = np.empty_like(q)
    for h in range(Hq):
        g = h // group
        s = q[:, h, :] @ k[:, g, :].T / np.sqrt(hd)
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True)
        out[:, h, :] = p @ v[:, g, :]
    return out


def swiglu(gate, up):
    """silu(gate) * up, silu(a) = a / (1 + exp(-a))."""
    gate, up = widen(gate), widen(up)
    return gate / (1.0 + np.exp(-gate)) * up


class KVCache:
    """Post-RoPE keys and values of committed positions, per layer: [kv_len, Hkv, hd].

    tail_k / tail_v keep what the last pass computed for the rows it did NOT commit (positions from
    tail_start on): the "suffix" entries of a dual cache (Sec. 5.2, Q2: cache compatibility), visible to a
    later pass only when it asks for them."""

    def __init__(self, cfg):
        shape = (0, cfg["n_kv_heads"], cfg["head_dim"])
        self.k = [np.zeros(shape) for _ in range(cfg["n_layers"])]
        self.v = [np.zeros(shape) for _ in range(cfg["n_layers"])]
        self.tail_start = 0
        self.tail_k = [np.zeros(shape) for _ in range(cfg["n_layers"])]
        self.tail_v = [np.zeros(shape) for _ in range(cfg["n_layers"])]

    @property
    def kv_len(self):
        return self.k[0].shape[0] if self.k else 0


def forward_span(cfg, W, cache, tokens, span_start, commit_len, suffix_len=0):
    """One forward pass over span rows [span_start, span_start+len(tokens)).

    The span attends to the cached prefix [0, kv_len) (kv_len must equal
    span_start), to all of its own rows and, if suffix_len > 0, to the suffix_len
    positions right after the span with the keys and values an EARLIER pass computed
    for them (they are not recomputed: the dual-cache approximation).  Afterwards K
    (post-RoPE) and V of the first commit_len rows are appended to the cache and
    those of the other rows replace the tail entries from their positions on
    (tail entries beyond the span's end are kept).  Returns logits [rows, V].
    """
    tokens = np.asarray(tokens, dtype=np.int64)
    A = tokens.shape[0]
    assert cache.kv_len == span_start
    assert 0 <= commit_len <= A
    end = span_start + A
    s0 = end - cache.tail_start  # index of the first suffix position in the tail
    assert suffix_len == 0 or (s0 >= 0 and s0 + suffix_len <= cache.tail_k[0].shape[0]), "suffix positions have no cached keys"
    Hq, Hkv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    eps, theta = cfg["rms_eps"], cfg["rope_theta"]
    pos = span_start + np.arange(A)

    h = widen(W["embed"][tokens])
    for l in range(cfg["n_layers"]):
        x = rmsnorm(h, W["norm1"][l], eps)
        qkv = matmul_nt(x, W["wqkv"][l])
        q = qkv[:, : Hq * hd].reshape(A, Hq, hd)
        k = qkv[:, Hq * hd : (Hq + Hkv) * hd].reshape(A, Hkv, hd)
        v = qkv[:, (Hq + Hkv) * hd :].reshape(A, Hkv, hd)
        q = rope(q, pos, theta)
        k = rope(k, pos, theta)
        keys = np.concatenate([cache.k[l], k, cache.tail_k[l][s0 : s0 + suffix_len] if suffix_len else k[:0]], axis=0)
        vals = np.concatenate([cache.v[l], v, cache.tail_v[l][s0 : s0 + suffix_len] if suffix_len else v[:0]], axis=0)
        o = attention(q, keys, vals).reshape(A, Hq * hd)
        h = h + matmul_nt(o, W["wo"][l])
        x = rmsnorm(h, W["norm2"][l], eps)
        gu = matmul_nt(x, W["w_gate_up"][l])
        ffn = cfg["d_ffn"]
        h = h + matmul_nt(swiglu(gu[:, :ffn], gu[:, ffn:]), W["w_down"][l])
        cache.k[l] = np.concatenate([cache.k[l], k[:commit_len]], axis=0)
        cache.v[l] = np.concatenate([cache.v[l], v[:commit_len]], axis=0)
        # the tail now starts at the first uncommitted row: this pass's values up to the span's end, older ones beyond it
        keep = max(s0, 0)
        old_k, old_v = cache.tail_k[l][keep:], cache.tail_v[l][keep:]
        if s0 < 0:  # (a gap between the span's end and the old tail: nothing beyond the span survives)
            old_k, old_v = k[:0], v[:0]
        cache.tail_k[l] = np.concatenate([k[commit_len:], old_k], axis=0)
        cache.tail_v[l] = np.concatenate([v[commit_len:], old_v], axis=0)
    cache.tail_start = span_start + commit_len
    x = rmsnorm(h, W["final_norm"], eps)
    return matmul_nt(x, W["lm_head"])
