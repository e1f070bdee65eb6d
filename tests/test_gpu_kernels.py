"""Parity of each HIP kernel (through the C ABI) against the CPU oracle, element by element.

Tolerances (derivations in the design doc):
  bf16 GEMM / attention   2e-2 * max(|ref| over the row, sigma)  (spec bound for bf16 logits)
  fp32 GEMM / attention   1e-4 * max(|ref| over the row)          (fp32 accumulation over K <= 4096)
  fp32 statistics         1e-5 * max(1, |ref|), KL additionally 1e-5 * sum p |log p - log p'|
  decisions               exact where the oracle's margin exceeds 1e-4 (boundary) / 1e-5 (selection)
"""
import numpy as np
import pytest
import torch

from oracle import boundary as o_boundary
from oracle import forward as o_fwd
from oracle import select as o_select
from oracle import stats as o_stats
from paper_2604_15750_amd import api, inputs

pytestmark = pytest.mark.gpu


def _np(t):
    return inputs.tensor_to_numpy(t)


def _rowtol(ref, rel, floor=0.0):
    return rel * np.maximum(np.abs(ref).max(axis=-1, keepdims=True), floor)


# ---- GEMM ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("M,N,K", [(1, 32, 32), (7, 64, 96), (16, 128, 128), (64, 4096, 4096), (100, 160, 4096 + 64),
                                   (192, 1024, 1536), (300, 96, 512), (33, 12288, 256),
                                   # 65 .. 160 rows: the mid kernel (every row-tile count; wide matrices with 128- and 96-column groups and a ragged
                                   # last group; narrow ones with and without a K split; k ranges that leave wavefronts idle)
                                   (65, 4096, 4096), (81, 24576, 512), (97, 4096, 1024), (112, 12288, 2048), (113, 4096, 12288),
                                   (136, 12288, 4096), (150, 8224, 1024), (160, 4096, 4096), (80, 126464, 64), (144, 64, 96),
                                   (161, 4096, 4096), (200, 1024, 2048), (225, 4096, 12288), (256, 4096, 512),
                                   (17, 16384, 256), (40, 24576, 1024), (33, 4096, 8192), (64, 256, 12288), (8, 4608, 3584), (16, 6144, 512),
                                   # more than 256 rows: the macro-tile kernel (ragged rows, column tails, both weight packings, short K)
                                   (257, 4096, 4096), (513, 8224, 1024), (700, 160, 4096 + 64), (1100, 640, 64), (384, 12288, 32),
                                   # ... with 192 x 256 tiles (two or four row blocks of 192 instead of three or six of 128)
                                   (368, 24576, 256), (700, 12288, 128)])
def test_gemm_bf16(device, M, N, K):
    g = torch.Generator(device="cpu").manual_seed(M * 7 + N + K)
    x = torch.randn(M, K, generator=g).to(torch.bfloat16).to(device)
    w = (torch.randn(N, K, generator=g) * 0.05).to(torch.bfloat16).to(device)
    y = api.dlm_gemm_nt(x, w)
    torch.cuda.synchronize()
    ref = o_fwd.matmul_nt(_np(x), _np(w))
    got = o_fwd.widen(_np(y))
    assert (np.abs(got - ref) <= _rowtol(ref, 2e-2, 0.05 * np.sqrt(K))).all(), np.abs(got - ref).max()
    # the output is the bf16 rounding of an fp32 accumulation: far tighter on average
    assert np.abs(got - ref).mean() <= 4e-3 * np.abs(ref).mean() + 1e-6


@pytest.mark.parametrize("M", [8, 100, 300])
def test_gemm_operand_conversion_at_the_ends_of_halfs_range(device, M):
    """A bf16 model's matrix-core operands are IEEE half.  Weights far below half's smallest normal number (2^-14) land on its
    subnormal grid: each keeps an absolute error of at most 2^-25.  Activations beyond half's largest number saturate at
    +-65504 instead of becoming infinite.  Everything in between converts exactly (covered by test_gemm_bf16)."""
    N, K = 256, 512
    g = torch.Generator(device="cpu").manual_seed(M)
    x = torch.randn(M, K, generator=g).to(torch.bfloat16)
    w = (torch.randn(N, K, generator=g) * 2.0 ** -17).to(torch.bfloat16)  # most of them subnormal in half, many below its resolution
    y = api.dlm_gemm_nt(x.to(device), w.to(device))
    torch.cuda.synchronize()
    ref = o_fwd.matmul_nt(_np(x), _np(w))
    got = o_fwd.widen(_np(y))
    bound = 2.0 ** -25 * np.abs(o_fwd.widen(_np(x))).sum(-1, keepdims=True) + 2.0 ** -8 * np.abs(ref) + 1e-12
    assert (np.abs(got - ref) <= bound).all(), (np.abs(got - ref) / bound).max()
    assert np.abs(ref).max() > 0 and np.abs(got).max() > 0.25 * np.abs(ref).max()  # (not flushed to zero)
    # saturation: one activation per row far beyond 65504
    x2 = x.clone()
    x2[:, 3] = 3.0e5
    w2 = (torch.randn(N, K, generator=g) * 0.05).to(torch.bfloat16)
    y2 = api.dlm_gemm_nt(x2.to(device), w2.to(device))
    torch.cuda.synchronize()
    got2 = o_fwd.widen(_np(y2))
    assert np.isfinite(got2).all()
    xc = o_fwd.widen(_np(x2)).clip(-65504.0, 65504.0)
    ref2 = xc @ o_fwd.widen(_np(w2)).T
    assert (np.abs(got2 - ref2) <= _rowtol(ref2, 2e-2)).all()


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (5, 7, 3), (64, 128, 128), (130, 1024, 384), (67, 384, 129)])
def test_gemm_f32(device, M, N, K):
    g = torch.Generator(device="cpu").manual_seed(M + N + K)
    x = torch.randn(M, K, generator=g).to(device)
    w = torch.randn(N, K, generator=g).to(device)
    y = api.dlm_gemm_nt(x, w)
    torch.cuda.synchronize()
    ref = o_fwd.matmul_nt(_np(x), _np(w))
    assert (np.abs(_np(y) - ref) <= _rowtol(ref, 1e-5, 1.0)).all()


# ---- attention -----------------------------------------------------------------------------------
@pytest.mark.parametrize("dt,A,T,nq,nkv,hd", [
    ("f32", 1, 1, 1, 1, 32), ("f32", 8, 72, 4, 4, 32), ("f32", 37, 101, 4, 2, 64), ("f32", 64, 320, 8, 2, 128),
    ("bf16", 8, 264, 4, 4, 128), ("bf16", 64, 320, 8, 8, 128), ("bf16", 50, 700, 28, 4, 128), ("bf16", 192, 448, 4, 1, 128),
    # head dims of 64 and 32 (a head's output dims split over two workgroups / not split), and enough (tile, head) pairs that
    # nothing is split (4 x 32, 40 x 16)
    ("bf16", 24, 300, 4, 2, 64), ("bf16", 9, 77, 8, 8, 32), ("bf16", 64, 200, 32, 8, 128), ("bf16", 640, 640, 16, 4, 128),
])
def test_attention(device, dt, A, T, nq, nkv, hd):
    tdt = torch.float32 if dt == "f32" else torch.bfloat16
    g = torch.Generator(device="cpu").manual_seed(A * 3 + T)
    q = (torch.randn(A, nq, hd, generator=g) * 1.5).to(tdt).to(device)
    k = (torch.randn(T, nkv, hd, generator=g) * 1.5).to(tdt).to(device)
    v = torch.randn(T, nkv, hd, generator=g).to(tdt).to(device)
    out = api.dlm_attention(q, k, v)
    torch.cuda.synchronize()
    ref = o_fwd.attention(_np(q), _np(k), _np(v))
    got = o_fwd.widen(_np(out))
    tol = 1e-5 if dt == "f32" else 2e-2
    assert (np.abs(got - ref) <= tol * np.maximum(np.abs(ref).max(-1, keepdims=True), 0.1)).all(), np.abs(got - ref).max()


# ---- vocabulary statistics -------------------------------------------------------------------------
def _check_stats(got, ref, z64, zp64, mask_id):
    for key in ("max_logit", "lse", "entropy", "conf"):
        r = ref[key]
        assert (np.abs(got[key].cpu().numpy() - r) <= 1e-5 * np.maximum(1.0, np.abs(r))).all(), key
    assert (got["argmax"].cpu().numpy() == ref["argmax"]).all()
    if zp64 is not None:
        logp, _, _ = o_stats.log_softmax_masked(z64, mask_id)
        logq, _, _ = o_stats.log_softmax_masked(zp64, mask_id)
        keep = np.arange(z64.shape[1]) != mask_id
        spread = np.sum(np.exp(logp[:, keep]) * np.abs(logp[:, keep] - logq[:, keep]), axis=-1)
        r = ref["kl"]
        assert (np.abs(got["kl"].cpu().numpy() - r) <= 1e-5 * np.maximum(1.0, np.abs(r)) + 1e-5 * spread).all()
    else:
        assert (got["kl"].cpu().numpy() == 0).all()


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("rows,V,mask_id", [(1, 8, 7), (3, 1024, 1023), (5, 1001, 17), (64, 126464, 126463), (300, 4096, 0), (9, 152064, 152063)])
@pytest.mark.parametrize("with_prev", [False, True])
def test_vocab_stats(device, dt, rows, V, mask_id, with_prev):
    tdt = torch.float32 if dt == "f32" else torch.bfloat16
    z = torch.from_numpy(inputs.peaked_logits(rows, V, rows + V, [(0, min(5, V - 2), 30.0)])).to(tdt)
    z[:, mask_id] = 50.0  # a huge logit on the mask token must not matter
    if rows > 2:
        z[2, :] = 1.25  # a flat row: argmax ties go to the lowest id
    zp = None
    if with_prev:
        zp = (z.float() + 0.5 * torch.from_numpy(inputs.peaked_logits(rows, V, 99 + rows))).to(tdt)
        if rows > 1:
            zp[1] = z[1]  # identical rows: KL = 0
    got = api.dlm_vocab_stats(z.to(device), mask_id, None if zp is None else zp.to(device))
    torch.cuda.synchronize()
    z64 = o_fwd.widen(_np(z))
    zp64 = None if zp is None else o_fwd.widen(_np(zp))
    ref = o_stats.vocab_stats(z64, mask_id, zp64)
    _check_stats(got, ref, z64, zp64, mask_id)
    if with_prev and rows > 1:
        assert abs(got["kl"][1].item()) <= 1e-6
    if with_prev:  # the previous rows' log-sum-exp handed in (what dlm_step keeps with the retained logits) instead of recomputed
        lse_prev = api.dlm_vocab_stats(zp.to(device), mask_id)["lse"]
        got2 = api.dlm_vocab_stats(z.to(device), mask_id, zp.to(device), prev_lse=lse_prev)
        torch.cuda.synchronize()
        _check_stats(got2, ref, z64, zp64, mask_id)


# ---- block_boundary ----------------------------------------------------------------------------------
@pytest.mark.parametrize("norm_mode", [0, 1, 2, 3])
@pytest.mark.parametrize("rule", [0, 1])
def test_block_boundary(device, norm_mode, rule):
    rng = np.random.default_rng(norm_mode * 2 + rule)
    for trial in range(6):
        n = int(rng.integers(1, 17))
        Ws = [int(rng.choice([1, 2, 5, 31, 64, 65, 128, 200, 256])) for _ in range(n)]
        off = np.concatenate([[0], np.cumsum(Ws)])
        I = (rng.exponential(0.3, off[-1]) * np.exp(-rng.uniform(0, 3, off[-1]))).astype(np.float32)
        H = rng.uniform(0.1, 6.0, off[-1]).astype(np.float32)
        if trial == 0:
            I[off[0]:off[1]] = 0.0  # identical steps in the first window
        cold = [int(rng.random() < 0.2) for _ in range(n)]
        lam = float(np.float32(rng.choice([0.6, 0.9, 1.0, 1.2, 1.6])))
        l_min, r = int(rng.integers(1, 12)), int(rng.integers(0, 4))
        L = torch.empty(n, dtype=torch.int32, device=device)
        S = torch.empty(int(off[-1]), dtype=torch.float32, device=device)
        mg = torch.empty(n, dtype=torch.float32, device=device)
        api.block_boundary(torch.from_numpy(I).to(device), torch.from_numpy(H).to(device), off[:-1].tolist(), Ws, L, lam, l_min, r, norm_mode,
                           rule, cold=cold, S_out=S, margin_out=mg)
        torch.cuda.synchronize()
        L, S, mg = L.cpu().numpy(), S.cpu().numpy(), mg.cpu().numpy()
        for b in range(n):
            sl = slice(off[b], off[b + 1])
            Lr, Sr, mr = o_boundary.block_boundary(I[sl], H[sl], lam, l_min, r, norm_mode, rule, cold_start=bool(cold[b]))
            assert (np.abs(S[sl] - Sr) <= 1e-5 * np.maximum(1.0, np.abs(Sr))).all()
            if mr > 1e-4:
                assert L[b] == Lr, (b, Ws[b], L[b], Lr, mr)
            assert min(l_min, Ws[b]) <= L[b] <= Ws[b]
            if np.isfinite(mr):
                assert abs(mg[b] - mr) <= 1e-5 * max(1.0, mr)


# ---- select_parallel -----------------------------------------------------------------------------------
def _select_case(rng, L, V, dt):
    peaks = []
    for r in range(L):
        if rng.random() < 0.7:
            peaks.append((r, int(rng.integers(0, 6)), float(rng.uniform(4, 16))))
        if rng.random() < 0.5:
            peaks.append((r, int(rng.integers(0, 6)), float(rng.uniform(6, 12))))
    z = torch.from_numpy(inputs.peaked_logits(L, V, int(rng.integers(1 << 30)), peaks, sigma=2.0))
    return z.to(torch.float32 if dt == "f32" else torch.bfloat16)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_select_parallel(device, dt, mode):
    rng = np.random.default_rng(17 + mode)
    V, mask_id = 512, 511
    fired = dict(multi=0, fallback=0, dropped=0)
    for trial in range(12):
        n = int(rng.integers(1, 9))
        lens = [int(rng.choice([0, 1, 3, 8, 32, 64, 100, 256])) for _ in range(n)]
        pad = [int(rng.integers(0, 5)) for _ in range(n)]  # unrelated rows between blocks
        row_start, rows = [], 0
        for b in range(n):
            rows += pad[b]
            row_start.append(rows)
            rows += lens[b]
        rows = max(rows, 1)
        z = _select_case(rng, rows, V, dt)
        tokens = np.where(rng.random(rows) < 0.75, mask_id, 5).astype(np.int32)
        z64 = o_fwd.widen(_np(z))
        st = api.dlm_vocab_stats(z.to(device), mask_id)
        tok_d = torch.from_numpy(tokens).to(device)
        sel = torch.zeros(rows, dtype=torch.uint8, device=device)
        nsel = torch.empty(n, dtype=torch.int32, device=device)
        mg = torch.empty(n, dtype=torch.float32, device=device)
        tl, th, gm = float(np.float32(0.6)), float(np.float32(0.93)), float(np.float32(rng.choice([-4.0, -8.0, -16.0])))
        api.select_parallel(z.to(device), st["lse"], st["conf"], st["argmax"], tok_d, row_start, row_start, lens, mask_id, tl, th, gm,
                            mode, sel, nsel, apply_tokens=True, margin_out=mg)
        torch.cuda.synchronize()
        lse, conf, yh = st["lse"].cpu().numpy(), st["conf"].cpu().numpy(), st["argmax"].cpu().numpy()
        sel, nsel, mg, tok_after = sel.cpu().numpy(), nsel.cpu().numpy(), mg.cpu().numpy(), tok_d.cpu().numpy()
        expect_tok = tokens.copy()
        for b in range(n):
            sl = slice(row_start[b], row_start[b] + lens[b])
            ref, mr = o_select.select_parallel(z64[sl], lse[sl], conf[sl], yh[sl], tokens[sl] == mask_id, tl, th, gm, mode)
            if mr > 1e-5:
                assert (sel[sl].astype(bool) == ref).all(), (trial, b, lens[b], mr)
                assert nsel[b] == ref.sum()
                expect_tok[sl] = np.where(ref, yh[sl], tokens[sl])
                assert (tok_after[sl] == expect_tok[sl]).all()  # Eq. 2
                if np.isfinite(mr):
                    assert abs(mg[b] - mr) <= 1e-5 * max(1.0, mr) + 2e-6 * 20
            E = tokens[sl] == mask_id
            pool = E & (conf[sl] >= tl)
            fired["multi"] += int(ref.sum() > 1)
            fired["fallback"] += int(E.any() and not pool.any())
            fired["dropped"] += int((pool & ~ref).any())
        # rows outside every block are untouched
        outside = np.ones(rows, dtype=bool)
        for b in range(n):
            outside[row_start[b]: row_start[b] + lens[b]] = False
        assert (tok_after[outside] == tokens[outside]).all() and (sel[outside] == 0).all()
    assert fired["multi"] > 3 or mode == 2
    if mode == 0:
        assert fired["fallback"] > 0 and fired["dropped"] > 3, fired


# ---- measurement helpers --------------------------------------------------------------------------
def test_probes_report_plausible_rates(device):
    """The two probes bench.py quotes rooflines against: a plain streaming read reaches most of, and no more than, the
    published 8 TB/s; the matrix-core loop (operands of pseudo-random values: power-limited) a good part of, and no more
    than, the published 2.5 PFLOP/s."""
    buf = torch.empty(1 << 30, dtype=torch.uint8, device=device)
    gbs = api.probe_hbm_read(buf, reps=5)
    tf = api.probe_mfma(reps=2)
    assert 3000 < gbs < 8000, gbs
    assert 1000 < tf < 2600, tf
    with pytest.raises(api.DlmError):
        api.probe_hbm_read(torch.empty(1 << 20, dtype=torch.uint8, device=device))
