"""The allocation-free softmax backward (its scratch is a fixed array inside the library's
device image) against the workspace-taking entry point it is a variant of, through the C ABI:
two calls in a row, the second with a smaller input, so that stale scratch contents of the
first call would show."""
import numpy as np
import pytest
import torch

import paper_2409_04431_amd as sa
from oracle import sattn_oracle as orc
from paper_2409_04431_amd import workloads as W

pytestmark = pytest.mark.gpu


def _both(B, H, N, d, causal, alibi, seed):
    g = torch.Generator().manual_seed(seed)
    q, k, v, do = (torch.randn(B, H, N, d, generator=g).bfloat16().cuda() for _ in range(4))
    sl = W.alibi_slopes(H).cuda() if alibi else None
    o = torch.empty_like(q)
    lse = torch.empty(B, H, N, dtype=torch.float32, device="cuda")
    sa.softmax_attn_fwd(q, k, v, o, lse, causal, sl)
    ref = [torch.full_like(q, float("nan")) for _ in range(3)]
    got = [torch.full_like(q, float("nan")) for _ in range(3)]
    sa.softmax_attn_bwd(q, k, v, o, lse, do, *ref, causal, sl)
    sa.softmax_attn_bwd_noalloc(q, k, v, o, lse, do, *got, causal, sl)
    torch.cuda.synchronize()
    return (q, k, v, do, sl), ref, got


def test_noalloc_softmax_backward_equals_the_workspace_entry_point_twice():
    # first call: many rows (fills a large part of the scratch); second call: fewer, shorter rows
    for (B, H, N, d, causal, alibi, seed) in ((2, 4, 1000, 128, True, True, 1), (1, 2, 333, 64, False, False, 2)):
        inp, ref, got = _both(B, H, N, d, causal, alibi, seed)
        for name, r, x in zip(("dq", "dk", "dv"), ref, got):
            assert not torch.isnan(x).any(), name
            assert torch.equal(r, x), f"{name} differs from softmax_attn_bwd at N={N}"   # same kernels, same inputs
        # and the oracle's bar for the new entry point itself
        q, k, v, do, sl = inp
        rq, rk, rv = orc.softmax_attn_bwd(q.cpu(), k.cpu(), v.cpu(), do.cpu(), causal,
                                          sl.cpu().numpy() if sl is not None else None)
        for name, r, x in zip(("dq", "dk", "dv"), (rq, rk, rv), got):
            e = float(np.abs(x.float().cpu().numpy() - r).max() / np.abs(r).max())
            assert e <= 2e-2, f"{name}: {e:.3e}"


def test_noalloc_rejects_problems_beyond_its_scratch():
    lim = sa.softmax_attn_bwd_noalloc_max_rows()
    assert lim == 1 << 20
    B, H, N, d = 1, 1, 64, 64
    t = torch.zeros(B, H, N, d, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(B, H, N, device="cuda")
    lib = sa.load_library()
    # B*H*roundup(N,64) = 2^20 + 64 rows: refused before anything is launched (fake sizes, real pointers)
    rc = lib.softmax_attn_bwd_noalloc(t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), lse.data_ptr(),
                                      t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), 1, 1, lim + 64, d, 0, 0,
                                      None, *([None] * 8), None)
    assert rc == -7 and "scratch" in sa.sattn_strerror(rc)
