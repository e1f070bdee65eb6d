"""dlm_vocab_stats_static, the entry point that allocates nothing (its partial states live in a file-scope device array of the
library), against dlm_vocab_stats with a caller workspace: same kernels, so every output must be bit-identical.  Two calls
in a row on the shared scratch, the second with a smaller input (what the first call left behind must not leak into it)."""
import numpy as np
import pytest
import torch

from oracle import forward as o_fwd, stats as o_stats
from paper_2604_15750_amd import api, inputs
from test_gpu_kernels import _check_stats

pytestmark = pytest.mark.gpu

KEYS = ("max_logit", "lse", "entropy", "kl", "conf", "argmax")


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_scratch_matches_workspace_entry_point(device, dtype):
    V, mask = 12640, 12639
    g = torch.Generator(device="cpu").manual_seed(5)
    for rows in (40, 7):  # both are cut into several chunks per row: the partial states go through the scratch
        z = (torch.randn(rows, V, generator=g) * 4).to(dtype).to(device)
        p = (z.float() + 0.3 * torch.randn(rows, V, generator=g).to(device)).to(dtype)
        outs = {k: torch.full((rows,), -7, dtype=torch.int32 if k == "argmax" else torch.float32, device=device) for k in KEYS}
        lse_p = api.dlm_vocab_stats(p, mask)["lse"] if rows == 7 else None  # the second call also takes the previous rows' lse
        got = api.dlm_vocab_stats_static(z, mask, prev=p, out=outs, prev_lse=lse_p)
        ref = api.dlm_vocab_stats(z, mask, prev=p, prev_lse=lse_p)
        torch.cuda.synchronize()
        for k in KEYS:
            assert torch.equal(got[k], ref[k]), (rows, k)
        # and against the oracle at the fp32 statistics tolerance
        z64, p64 = o_fwd.widen(inputs.tensor_to_numpy(z)), o_fwd.widen(inputs.tensor_to_numpy(p))
        _check_stats(got, o_stats.vocab_stats(z64, mask, p64), z64, p64, mask)
    # without previous-step logits: kl = 0
    z = (torch.randn(9, V, generator=g) * 4).to(dtype).to(device)
    got, ref = api.dlm_vocab_stats_static(z, mask), api.dlm_vocab_stats(z, mask)
    torch.cuda.synchronize()
    for k in KEYS:
        assert torch.equal(got[k], ref[k]), k
    assert float(got["kl"].abs().max()) == 0.0
