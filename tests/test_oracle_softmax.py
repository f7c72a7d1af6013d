"""Pins for the fp64 CPU oracle of softmax attention (the comparison system)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import sattn_oracle as orc

RNG = np.random.default_rng(715)


def _rand(B, H, N, d):
    return RNG.standard_normal((B, H, N, d))


def test_zero_logits_give_mean_of_visible_values_and_log_count():
    B, H, N, d = 1, 2, 9, 4
    v = _rand(B, H, N, d)
    z = np.zeros_like(v)
    o, lse = orc.softmax_attn_fwd(z, z, v)
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(2, keepdims=True), v.shape), rtol=1e-13)
    np.testing.assert_allclose(lse, math.log(N), rtol=1e-14)
    oc, lsec = orc.softmax_attn_fwd(z, z, v, causal=True)
    cnt = np.arange(1, N + 1)[None, None, :, None]
    np.testing.assert_allclose(oc, np.cumsum(v, 2) / cnt, rtol=1e-13)
    np.testing.assert_allclose(lsec, np.broadcast_to(np.log(cnt[..., 0]), lsec.shape), rtol=1e-14)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(2, 2, 31, 8), (1, 3, 128, 64)])
def test_against_torch_sdpa_fp64_with_autograd(causal, shape):
    # torch's scaled_dot_product_attention on CPU is the library routine this reduces to
    B, H, N, d = shape
    q, k, v, dout = (_rand(B, H, N, d) for _ in range(4))
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    to = F.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)
    (to * torch.tensor(dout)).sum().backward()
    o, lse = orc.softmax_attn_fwd(q, k, v, causal)
    np.testing.assert_allclose(o, to.detach().numpy(), rtol=1e-11, atol=1e-13)
    dq, dk, dv = orc.softmax_attn_bwd(q, k, v, dout, causal)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-13)
    # LSE against torch.logsumexp of the masked logits
    s = (tq @ tk.transpose(-1, -2) / math.sqrt(d)).detach()
    if causal:
        idx = torch.arange(N)
        s = s.masked_fill(idx[None, :] > idx[:, None], float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), rtol=1e-12)


def test_alibi_matches_additive_mask_in_sdpa():
    B, H, N, d = 1, 2, 20, 8
    q, k, v = _rand(B, H, N, d), _rand(B, H, N, d), _rand(B, H, N, d)
    slopes = np.array([0.5, 0.0625])
    idx = torch.arange(N)
    mask = -torch.tensor(slopes)[None, :, None, None] * (idx[:, None] - idx[None, :]).abs().double()
    to = F.scaled_dot_product_attention(torch.tensor(q), torch.tensor(k), torch.tensor(v), attn_mask=mask)
    o, _ = orc.softmax_attn_fwd(q, k, v, False, slopes)
    np.testing.assert_allclose(o, to.numpy(), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_backward_with_alibi_against_sdpa_autograd(causal):
    # the gradients with ALiBi slopes: autograd through SDPA with the additive mask
    # -m_h |i - j| (plus -inf above the diagonal when causal)
    B, H, N, d = 2, 3, 37, 8
    q, k, v, dout = (_rand(B, H, N, d) for _ in range(4))
    slopes = np.array([2.0 ** (-8.0 * (h + 1) / H) for h in range(H)])
    idx = torch.arange(N)
    mask = -torch.tensor(slopes)[None, :, None, None] * (idx[:, None] - idx[None, :]).abs().double()
    if causal:
        mask = mask.masked_fill(idx[None, :] > idx[:, None], float("-inf"))
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    to = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask.expand(B, H, N, N))
    (to * torch.tensor(dout)).sum().backward()
    o, _ = orc.softmax_attn_fwd(q, k, v, causal, slopes)
    np.testing.assert_allclose(o, to.detach().numpy(), rtol=1e-11, atol=1e-13)
    dq, dk, dv = orc.softmax_attn_bwd(q, k, v, dout, causal, slopes)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-13)
    # and the slopes matter: without them the gradients differ
    dq0, _, _ = orc.softmax_attn_bwd(q, k, v, dout, causal)
    assert np.abs(dq0 - dq).max() > 1e-3


def test_shift_invariance_and_rows_entry_point():
    B, H, N, d = 1, 1, 40, 8
    q, k, v = _rand(B, H, N, d), _rand(B, H, N, d), _rand(B, H, N, d)
    o, lse = orc.softmax_attn_fwd(q, k, v, True)
    rows = [0, 3, 39]
    ro, rl = orc.softmax_attn_fwd_rows(q[0, 0], k[0, 0], v[0, 0], True, 0.0, rows)
    np.testing.assert_allclose(ro, o[0, 0, rows], rtol=1e-13)
    np.testing.assert_allclose(rl, lse[0, 0, rows], rtol=1e-13)
    # huge logits must not overflow (row max is subtracted)
    o2, lse2 = orc.softmax_attn_fwd(1e3 * q, k, v)
    assert np.isfinite(o2).all() and np.isfinite(lse2).all()
