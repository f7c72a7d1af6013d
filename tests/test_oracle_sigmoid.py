"""Pins for the fp64 CPU oracle of sigmoid attention.

None of these re-types the oracle's loop: each pins it to a closed form, an identity, a
limit, a library routine (PyTorch fp64 CPU ops + autograd) or finite differences, chosen so
that a dropped term, a wrong sign/index/scale or a transposed operand fails at least one.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import sattn_oracle as orc

RNG = np.random.default_rng(20240904)
GOLD = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


def _golden():
    out = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=", 1)
            out[k.strip()] = v.strip()
    return out


def _rand(B, H, N, d, scale=1.0):
    return RNG.standard_normal((B, H, N, d)) * scale


def _alibi_slopes(H):
    return np.array([2.0 ** (-8.0 * (h + 1) / H) for h in range(H)])


# ------------------------------------------------------------------ closed forms

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [3, 16])
def test_zero_logits_give_sigma_b_times_sum_of_visible_v(causal, d):
    # Q = 0 => every logit is b, whatever d: O_i = sigma(b) * sum_{j visible} V_j
    B, H, N = 2, 3, 11
    v = _rand(B, H, N, d)
    k = _rand(B, H, N, d)
    q = np.zeros_like(v)
    for b in (0.0, -math.log(N), -math.log(N - 1), 1.7):
        o = orc.sigmoid_attn_fwd(q, k, v, b, causal=causal)
        sb = 1.0 / (1.0 + math.exp(-b))
        csum = np.cumsum(v, axis=2) if causal else np.broadcast_to(v.sum(2, keepdims=True), v.shape)
        np.testing.assert_allclose(o, sb * csum, rtol=1e-13, atol=1e-13)


def test_paper_bias_values():
    # Appendix E: exp(-b) = n-1 makes all weights 1/n (O = mean V); b=-log n gives 1/(n+1); b=0 gives 1/2.
    g = _golden()
    assert g["uniform_weight_bias"] == "-log(n-1)" and g["practice_bias_weight"] == "1/(n+1)"
    N, d = 37, 5
    v = _rand(1, 1, N, d)
    z = np.zeros_like(v)
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(z, z, v, -math.log(N - 1)),
                               np.broadcast_to(v.mean(2, keepdims=True), v.shape), rtol=1e-13)
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(z, z, v, -math.log(N)),
                               np.broadcast_to(v.sum(2, keepdims=True) / (N + 1), v.shape), rtol=1e-13)
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(z, z, v, 0.0),
                               np.broadcast_to(float(g["heaviside_at_zero"]) * v.sum(2, keepdims=True), v.shape),
                               rtol=1e-13)


def test_single_token_scalar_case_fixes_scale_and_bias_order():
    # N=1, d=4, q=k=(1,1,1,1): q.k/sqrt(d) = 2, so O = sigmoid(2+b) v.  A missing 1/sqrt(d)
    # (sigmoid(4)), a sqrt(d) factor (sigmoid(8)) or b scaled with the logits would all differ.
    g = _golden()
    q = np.ones((1, 1, 1, 4))
    v = np.array([[[[1.0, -2.0, 0.5, 3.0]]]])
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(q, q, v, 0.0), float(g["sigmoid(2)"]) * v, rtol=1e-15)
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(q, q, v, -3.0), float(g["sigmoid(-1)"]) * v, rtol=1e-15)
    # d=16, q.k = 2 -> 2/4 = 0.5
    q16 = np.zeros((1, 1, 1, 16)); q16[..., 0] = 2.0
    k16 = np.zeros((1, 1, 1, 16)); k16[..., 0] = 1.0
    v16 = _rand(1, 1, 1, 16)
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(q16, k16, v16, 0.0), float(g["sigmoid(0.5)"]) * v16, rtol=1e-15)


def test_two_token_hand_example_fixes_operand_roles():
    # i indexes queries, j keys: O_0 = s(q0.k0) v0 + s(q0.k1) v1.  Swapping Q and K, or using
    # V^T, changes the result.  d=1 so the logits are plain products.
    q = np.array([[[[1.0], [0.0]]]])
    k = np.array([[[[2.0], [-1.0]]]])
    v = np.array([[[[10.0], [100.0]]]])
    g = _golden()
    s2, sm1 = float(g["sigmoid(2)"]), float(g["sigmoid(-1)"])
    o = orc.sigmoid_attn_fwd(q, k, v, 0.0)
    np.testing.assert_allclose(o[0, 0, 0, 0], s2 * 10 + sm1 * 100, rtol=1e-15)
    np.testing.assert_allclose(o[0, 0, 1, 0], 0.5 * 110, rtol=1e-15)
    oc = orc.sigmoid_attn_fwd(q, k, v, 0.0, causal=True)
    np.testing.assert_allclose(oc[0, 0, 0, 0], s2 * 10, rtol=1e-15)       # key 1 hidden from query 0
    np.testing.assert_allclose(oc[0, 0, 1, 0], 0.5 * 110, rtol=1e-15)     # diagonal kept


def test_sequence_form_with_log_n_bias():
    # Section 2, sequence equation: with b = -log n, weight = exp(s)/(exp(s)+n)
    B, H, N, d = 1, 2, 19, 8
    q, k, v = _rand(B, H, N, d), _rand(B, H, N, d), _rand(B, H, N, d)
    s = np.einsum("bhid,bhjd->bhij", q, k) / math.sqrt(d)
    w = np.exp(s) / (np.exp(s) + N)
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(q, k, v, -math.log(N)), w @ v, rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ identities and limits

def test_reflection_symmetry():
    # sigma(-x) = 1 - sigma(x): O(Q,b) + O(-Q,-b) = sum_j V_j (non-causal, no ALiBi)
    B, H, N, d = 2, 2, 13, 6
    q, k, v = _rand(B, H, N, d), _rand(B, H, N, d), _rand(B, H, N, d)
    b = -0.8
    tot = orc.sigmoid_attn_fwd(q, k, v, b) + orc.sigmoid_attn_fwd(-q, k, v, -b)
    np.testing.assert_allclose(tot, np.broadcast_to(v.sum(2, keepdims=True), v.shape), rtol=1e-12, atol=1e-12)


def test_heaviside_limit():
    # Appendix C: sigmoid(lambda x) -> H(x).  Large lambda, b=0: O_i -> sum_{j: s_ij>0} V_j
    B, H, N, d = 1, 1, 9, 4
    q, k, v = _rand(B, H, N, d), _rand(B, H, N, d), _rand(B, H, N, d)
    s = np.einsum("bhid,bhjd->bhij", q, k)
    assert np.abs(s).min() > 1e-3
    o = orc.sigmoid_attn_fwd(1e6 * q, k, v, 0.0)
    np.testing.assert_allclose(o, (s > 0).astype(float) @ v, rtol=1e-12, atol=1e-12)
    assert np.isfinite(o).all()


def test_additive_over_key_halves_and_linear_in_v():
    B, H, N, d = 1, 2, 16, 5
    q, k, v = _rand(B, H, N, d), _rand(B, H, N, d), _rand(B, H, N, d)
    b = -math.log(N)
    full = orc.sigmoid_attn_fwd(q, k, v, b)
    # no normaliser: zeroing V on one half of the keys and adding the two results gives the full one
    v1, v2 = v.copy(), v.copy()
    v1[:, :, N // 2:] = 0
    v2[:, :, :N // 2] = 0
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(q, k, v1, b) + orc.sigmoid_attn_fwd(q, k, v2, b), full,
                               rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(q, k, 3.0 * v, b), 3.0 * full, rtol=1e-12, atol=1e-14)


def test_permutation_equivariance():
    B, H, N, d = 1, 1, 12, 4
    q, k, v = _rand(B, H, N, d), _rand(B, H, N, d), _rand(B, H, N, d)
    perm = RNG.permutation(N)
    o = orc.sigmoid_attn_fwd(q, k, v, -1.0)
    op = orc.sigmoid_attn_fwd(q[:, :, perm], k[:, :, perm], v[:, :, perm], -1.0)
    np.testing.assert_allclose(op, o[:, :, perm], rtol=1e-12, atol=1e-13)


def test_alibi_closed_form_and_zero_slope():
    # Q=0, causal: O_i = sum_{j<=i} sigma(b - m (i-j)) V_j  -- a 1-D correlation
    B, H, N, d = 1, 3, 10, 4
    v = _rand(B, H, N, d)
    z = np.zeros_like(v)
    slopes = _alibi_slopes(H)
    b = -0.3
    o = orc.sigmoid_attn_fwd(z, z, v, b, causal=True, alibi_slopes=slopes)
    for h in range(H):
        w = 1.0 / (1.0 + np.exp(-(b - slopes[h] * np.arange(N))))   # weight as a function of i-j
        for i in range(N):
            ref = sum(w[i - j] * v[0, h, j] for j in range(i + 1))
            np.testing.assert_allclose(o[0, h, i], ref, rtol=1e-12)
    # non-causal uses |i-j| (symmetric)
    o2 = orc.sigmoid_attn_fwd(z, z, v, b, causal=False, alibi_slopes=slopes)
    for h in range(H):
        w = 1.0 / (1.0 + np.exp(-(b - slopes[h] * np.arange(N))))
        ref = sum(w[abs(4 - j)] * v[0, h, j] for j in range(N))
        np.testing.assert_allclose(o2[0, h, 4], ref, rtol=1e-12)
    # slope 0 is bit-identical to no ALiBi
    q, k = _rand(B, H, N, d), _rand(B, H, N, d)
    assert np.array_equal(orc.sigmoid_attn_fwd(q, k, v, b, alibi_slopes=np.zeros(H)),
                          orc.sigmoid_attn_fwd(q, k, v, b))


# ------------------------------------------------------------------ library routine (torch fp64 + autograd)

def _torch_ref(q, k, v, dout, bias, causal, slopes):
    q, k, v, dout = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v, dout))
    B, H, N, d = q.shape
    s = q @ k.transpose(-1, -2) / math.sqrt(d) + bias
    idx = torch.arange(N)
    if slopes is not None:
        dist = (idx[:, None] - idx[None, :]).abs().double()
        s = s - torch.tensor(slopes, dtype=torch.float64)[None, :, None, None] * dist
    p = torch.sigmoid(s)
    if causal:
        p = p * (idx[None, :] <= idx[:, None]).double()
    o = p @ v
    (o * dout).sum().backward()
    return o.detach().numpy(), q.grad.numpy(), k.grad.numpy(), v.grad.numpy()


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("alibi", [False, True])
@pytest.mark.parametrize("shape", [(1, 2, 33, 8), (2, 3, 64, 16), (1, 1, 257, 64)])
def test_against_torch_fp64_autograd(causal, alibi, shape):
    B, H, N, d = shape
    q, k, v, dout = (_rand(B, H, N, d) for _ in range(4))
    slopes = _alibi_slopes(H) if alibi else None
    bias = -math.log(N)
    o, dq, dk, dv = _torch_ref(q, k, v, dout, bias, causal, slopes)
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(q, k, v, bias, causal, slopes), o, rtol=1e-11, atol=1e-13)
    gq, gk, gv = orc.sigmoid_attn_bwd(q, k, v, dout, bias, causal, slopes)
    np.testing.assert_allclose(gq, dq, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(gk, dk, rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(gv, dv, rtol=1e-10, atol=1e-13)


# ------------------------------------------------------------------ finite differences

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("alibi", [False, True])
def test_backward_by_central_finite_differences(causal, alibi):
    # L = sum(O * dO); dL/dx by central differences on every input element (N=5, d=3).
    B, H, N, d = 1, 2, 5, 3
    q, k, v, dout = (_rand(B, H, N, d) for _ in range(4))
    slopes = _alibi_slopes(H) if alibi else None
    bias = -0.4

    def loss(q_, k_, v_):
        return float((orc.sigmoid_attn_fwd(q_, k_, v_, bias, causal, slopes) * dout).sum())

    dq, dk, dv = orc.sigmoid_attn_bwd(q, k, v, dout, bias, causal, slopes)
    eps = 1e-5
    for name, x, g in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(x)
        it = np.nditer(x, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            xp, xm = x.copy(), x.copy()
            xp[idx] += eps
            xm[idx] -= eps
            args_p = {"q": (xp, k, v), "k": (q, xp, v), "v": (q, k, xp)}[name]
            args_m = {"q": (xm, k, v), "k": (q, xm, v), "v": (q, k, xm)}[name]
            num[idx] = (loss(*args_p) - loss(*args_m)) / (2 * eps)
        np.testing.assert_allclose(g, num, rtol=2e-7, atol=1e-9, err_msg=name)


def test_zero_logit_gradients_closed_form():
    # Q=0: dV_j = sigma(b) sum_i dO_i ;  dQ_i = sigma(b)(1-sigma(b))/sqrt(d) sum_j (dO_i.V_j) K_j
    B, H, N, d = 1, 1, 7, 4
    k, v, dout = _rand(B, H, N, d), _rand(B, H, N, d), _rand(B, H, N, d)
    q = np.zeros_like(k)
    b = -1.2
    sb = 1 / (1 + math.exp(-b))
    dq, dk, dv = orc.sigmoid_attn_bwd(q, k, v, dout, b)
    np.testing.assert_allclose(dv, np.broadcast_to(sb * dout.sum(2, keepdims=True), v.shape), rtol=1e-13)
    dp = np.einsum("bhid,bhjd->bhij", dout, v)
    np.testing.assert_allclose(dq, sb * (1 - sb) / math.sqrt(d) * (dp @ k), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dk, 0.0, atol=1e-15)   # dK = dS^T Q / sqrt(d) and Q = 0


# ------------------------------------------------------------------ bias gradient (row sums of dS)

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("alibi", [False, True])
def test_bias_gradient_by_central_differences_in_b(causal, alibi):
    # Row i of O depends on b only through row i of T, so d/db of sum_t O_it dO_it is the
    # gradient of a bias on row i alone: the row sum of dS.  The forward oracle gives it by
    # central differences without any backward formula.
    B, H, N, d = 2, 2, 9, 4
    q, k, v, dout = (_rand(B, H, N, d) for _ in range(4))
    slopes = _alibi_slopes(H) if alibi else None
    bias, eps = -0.7, 1e-5
    lp = (orc.sigmoid_attn_fwd(q, k, v, bias + eps, causal, slopes) * dout).sum(-1)
    lm = (orc.sigmoid_attn_fwd(q, k, v, bias - eps, causal, slopes) * dout).sum(-1)
    db = orc.sigmoid_attn_bias_grad(q, k, v, dout, bias, causal, slopes)
    assert db.shape == (B, H, N)
    np.testing.assert_allclose(db, (lp - lm) / (2 * eps), rtol=2e-7, atol=1e-9)


def test_bias_gradient_against_torch_autograd_and_closed_form():
    B, H, N, d = 1, 3, 40, 8
    q, k, v, dout = (_rand(B, H, N, d) for _ in range(4))
    slopes = _alibi_slopes(H)
    b = torch.tensor(-math.log(N), dtype=torch.float64, requires_grad=True)
    tq, tk, tv, tdo = (torch.tensor(x, dtype=torch.float64) for x in (q, k, v, dout))
    idx = torch.arange(N)
    t = tq @ tk.transpose(-1, -2) / math.sqrt(d) + b \
        - torch.tensor(slopes)[None, :, None, None] * (idx[:, None] - idx[None, :]).abs().double()
    p = torch.sigmoid(t) * (idx[None, :] <= idx[:, None]).double()
    ((p @ tv) * tdo).sum().backward()
    db = orc.sigmoid_attn_bias_grad(q, k, v, dout, -math.log(N), True, slopes)
    np.testing.assert_allclose(db.sum(), b.grad.item(), rtol=1e-11)
    # Q = 0, no ALiBi: every P is sigma(b), so db_i = sigma(b)(1 - sigma(b)) dO_i . sum_{j visible} V_j
    z = np.zeros_like(q)
    sb = 1 / (1 + math.exp(0.9))
    got = orc.sigmoid_attn_bias_grad(z, k, v, dout, -0.9, True)
    ref = sb * (1 - sb) * np.einsum("bhid,bhid->bhi", dout, np.cumsum(v, axis=2))
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-14)
    # consistent with the backward pass: dQ_i = (1/sqrt d) sum_j dS_ij K_j, so with every K_j = c
    # (the same vector), dQ_i = db_i c / sqrt(d)
    c = RNG.standard_normal(d)
    kc = np.broadcast_to(c, k.shape).copy()
    dq, _, _ = orc.sigmoid_attn_bwd(q, kc, v, dout, -0.3, False)
    dbc = orc.sigmoid_attn_bias_grad(q, kc, v, dout, -0.3, False)
    np.testing.assert_allclose(dq, dbc[..., None] * c / math.sqrt(d), rtol=1e-11, atol=1e-14)


# ------------------------------------------------------------------ shared key/value heads

@pytest.mark.parametrize("Hkv", [1, 2, 4])
def test_shared_kv_heads_against_torch_autograd(Hkv):
    B, H, N, d = 2, 4, 19, 8
    q, dout = _rand(B, H, N, d), _rand(B, H, N, d)
    k, v = _rand(B, Hkv, N, d), _rand(B, Hkv, N, d)
    slopes = _alibi_slopes(H)
    bias = -math.log(N)
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    idx = torch.arange(N)
    g = H // Hkv
    # head h of Q against head h // g of K, V, written with an explicit index (no repeat)
    kv_of = torch.arange(H) // g
    t = torch.einsum("bhid,bhjd->bhij", tq, tk[:, kv_of]) / math.sqrt(d) + bias \
        - torch.tensor(slopes)[None, :, None, None] * (idx[:, None] - idx[None, :]).abs().double()
    p = torch.sigmoid(t) * (idx[None, :] <= idx[:, None]).double()
    o = torch.einsum("bhij,bhjd->bhid", p, tv[:, kv_of])
    (o * torch.tensor(dout)).sum().backward()
    np.testing.assert_allclose(orc.sigmoid_attn_mqa_fwd(q, k, v, bias, True, slopes), o.detach().numpy(),
                               rtol=1e-11, atol=1e-13)
    dq, dk, dv = orc.sigmoid_attn_mqa_bwd(q, k, v, dout, bias, True, slopes)
    assert dk.shape == k.shape and dv.shape == v.shape
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-13)
    if Hkv == H:   # one K/V head per query head is plain attention
        assert np.array_equal(orc.sigmoid_attn_mqa_fwd(q, k, v, bias, True, slopes),
                              orc.sigmoid_attn_fwd(q, k, v, bias, True, slopes))


def test_multi_query_zero_logit_closed_form():
    # Q = 0, one K/V head: every query head outputs sigma(b) * sum_j V_j, and dV_j collects
    # sigma(b) * dO_i over every query head and row
    B, H, N, d = 1, 3, 6, 4
    k, v, dout = _rand(B, 1, N, d), _rand(B, 1, N, d), _rand(B, H, N, d)
    q = np.zeros((B, H, N, d))
    sb = 1 / (1 + math.exp(0.8))
    o = orc.sigmoid_attn_mqa_fwd(q, k, v, -0.8)
    np.testing.assert_allclose(o, np.broadcast_to(sb * v.sum(2, keepdims=True), o.shape), rtol=1e-13)
    _, _, dv = orc.sigmoid_attn_mqa_bwd(q, k, v, dout, -0.8)
    np.testing.assert_allclose(dv, np.broadcast_to(sb * dout.sum((1, 2), keepdims=True), dv.shape), rtol=1e-12)


# ------------------------------------------------------------------ different numbers of queries and keys

def test_cross_attention_pins():
    B, H, Nq, Nk, d = 2, 2, 7, 12, 8
    q, dout = _rand(B, H, Nq, d), _rand(B, H, Nq, d)
    k, v = _rand(B, H, Nk, d), _rand(B, H, Nk, d)
    b = -math.log(Nk)
    o = orc.sigmoid_attn_cross_fwd(q, k, v, b)
    dq, dk, dv = orc.sigmoid_attn_cross_bwd(q, k, v, dout, b)
    # (1) square attention (the C oracle) on inputs padded to 12 rows: queries beyond the 7th do
    # not influence the first 7 outputs, and with zero upstream gradient they add nothing to dK, dV
    pad = lambda x: np.concatenate([x, np.zeros((B, H, Nk - Nq, d))], axis=2)
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(pad(q), k, v, b)[:, :, :Nq], o, rtol=1e-12, atol=1e-14)
    sq, sk, sv = orc.sigmoid_attn_bwd(pad(q), k, v, pad(dout), b)
    np.testing.assert_allclose(sq[:, :, :Nq], dq, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(sk, dk, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(sv, dv, rtol=1e-11, atol=1e-14)
    # (2) more queries than keys: pad the keys with V = 0 rows, which contribute sigma(.) * 0
    q2, d2 = _rand(B, H, Nk, d), _rand(B, H, Nk, d)
    k2, v2 = _rand(B, H, Nq, d), _rand(B, H, Nq, d)
    np.testing.assert_allclose(orc.sigmoid_attn_fwd(q2, pad(k2), pad(v2), b),
                               orc.sigmoid_attn_cross_fwd(q2, k2, v2, b), rtol=1e-12, atol=1e-14)
    # (3) torch autograd
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    to = torch.sigmoid(tq @ tk.transpose(-1, -2) / math.sqrt(d) + b) @ tv
    (to * torch.tensor(dout)).sum().backward()
    np.testing.assert_allclose(o, to.detach().numpy(), rtol=1e-12, atol=1e-14)
    for got, ref in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        np.testing.assert_allclose(got, ref.numpy(), rtol=1e-10, atol=1e-13)
    # (4) Q = 0: O_i = sigma(b) * sum of all Nk values
    z = np.zeros_like(q)
    np.testing.assert_allclose(orc.sigmoid_attn_cross_fwd(z, k, v, -0.4),
                               np.broadcast_to(v.sum(2, keepdims=True) / (1 + math.exp(0.4)), o.shape), rtol=1e-13)


@pytest.mark.parametrize("Nq,Nk", [(5, 12), (12, 12), (1, 9), (9, 4)])
@pytest.mark.parametrize("alibi", [False, True])
def test_cross_attention_with_end_aligned_causal_mask_pins(Nq, Nk, alibi):
    """The reading for n_q != n_k: the queries are the last n_q positions of the key sequence."""
    B, H, d = 2, 3, 8
    q, dout = _rand(B, H, Nq, d), _rand(B, H, Nq, d)
    k, v = _rand(B, H, Nk, d), _rand(B, H, Nk, d)
    slopes = np.array([0.5, 0.25, 0.0625]) if alibi else None
    b = -0.7
    o = orc.sigmoid_attn_cross_fwd(q, k, v, b, True, slopes)
    dq, dk, dv = orc.sigmoid_attn_cross_bwd(q, k, v, dout, b, True, slopes)
    if Nk >= Nq:
        # (1) the square causal attention (the pinned C oracle) over all n_k positions, whose last
        # n_q queries are ours: its last n_q output rows are our output; with zero upstream
        # gradient on the earlier rows its dK, dV are ours and the last rows of its dQ are our dQ
        qf = np.concatenate([_rand(B, H, Nk - Nq, d), q], axis=2)
        df = np.concatenate([np.zeros((B, H, Nk - Nq, d)), dout], axis=2)
        np.testing.assert_allclose(orc.sigmoid_attn_fwd(qf, k, v, b, True, slopes)[:, :, Nk - Nq:], o, rtol=1e-12, atol=1e-14)
        sq, sk, sv = orc.sigmoid_attn_bwd(qf, k, v, df, b, True, slopes)
        np.testing.assert_allclose(sq[:, :, Nk - Nq:], dq, rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(sk, dk, rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(sv, dv, rtol=1e-11, atol=1e-14)
    else:
        # (2) more queries than keys: the first n_q - n_k queries sit before every key and see
        # nothing; the rest is the square causal attention of the last n_k queries
        cut = Nq - Nk
        assert np.all(o[:, :, :cut] == 0) and np.all(dq[:, :, :cut] == 0)
        np.testing.assert_allclose(orc.sigmoid_attn_fwd(q[:, :, cut:], k, v, b, True, slopes), o[:, :, cut:], rtol=1e-12, atol=1e-14)
        sq, sk, sv = orc.sigmoid_attn_bwd(q[:, :, cut:], k, v, dout[:, :, cut:], b, True, slopes)
        np.testing.assert_allclose(sq, dq[:, :, cut:], rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(sk, dk, rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(sv, dv, rtol=1e-11, atol=1e-14)
    # (3) brute force over pairs, straight from the definition
    ref = np.zeros_like(o)
    for bb in range(B):
        for h in range(H):
            for i in range(Nq):
                for j in range(Nk):
                    pi = i + Nk - Nq
                    if j > pi:
                        continue
                    t = q[bb, h, i] @ k[bb, h, j] / math.sqrt(d) + b - (slopes[h] * abs(pi - j) if alibi else 0.0)
                    ref[bb, h, i] += v[bb, h, j] / (1.0 + math.exp(-t))
    np.testing.assert_allclose(o, ref, rtol=1e-12, atol=1e-14)
    # (4) torch autograd with an explicit mask
    tq, tk, tv = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (q, k, v))
    pos_q = torch.arange(Nq)[:, None] + (Nk - Nq)
    pos_k = torch.arange(Nk)[None, :]
    t = tq @ tk.transpose(-1, -2) / math.sqrt(d) + b
    if alibi:
        t = t - torch.tensor(slopes).reshape(1, H, 1, 1) * (pos_q - pos_k).abs()
    to = (torch.sigmoid(t) * (pos_k <= pos_q)) @ tv
    (to * torch.tensor(dout)).sum().backward()
    np.testing.assert_allclose(o, to.detach().numpy(), rtol=1e-12, atol=1e-14)
    for got, ref_g in ((dq, tq.grad), (dk, tk.grad), (dv, tv.grad)):
        np.testing.assert_allclose(got, ref_g.numpy(), rtol=1e-10, atol=1e-13)
    # (5) without the mask and slopes the extended functions are the plain ones
    np.testing.assert_array_equal(orc.sigmoid_attn_cross_fwd(q, k, v, b), orc.sigmoid_attn_cross_fwd(q, k, v, b, False, None))


# ------------------------------------------------------------------ hybrid-norm

@pytest.mark.parametrize("kind", ["layer", "rms"])
def test_headconcat_norm_against_torch_and_invariants(kind):
    B, H, N, d = 2, 3, 7, 8
    x, dy = _rand(B, H, N, d) * 3 + 0.7, _rand(B, H, N, d)
    eps = 1e-5
    y, mean, rstd = orc.headconcat_norm_fwd(x, kind, eps)
    # library routine on the token-major layout [B, N, H*d]
    t = torch.tensor(x.transpose(0, 2, 1, 3).reshape(B, N, H * d), dtype=torch.float64, requires_grad=True)
    if kind == "layer":
        ref = torch.nn.functional.layer_norm(t, (H * d,), eps=eps)
    else:
        ref = t * torch.rsqrt(t.pow(2).mean(-1, keepdim=True) + eps)
    back = lambda a: a.reshape(B, N, H, d).transpose(0, 2, 1, 3)
    np.testing.assert_allclose(y, back(ref.detach().numpy()), rtol=1e-12, atol=1e-13)
    (ref * torch.tensor(dy.transpose(0, 2, 1, 3).reshape(B, N, H * d))).sum().backward()
    np.testing.assert_allclose(orc.headconcat_norm_bwd(x, dy, kind, eps), back(t.grad.numpy()), rtol=1e-10, atol=1e-12)
    # invariants: unit second moment per token (up to eps), zero mean for LayerNorm, scale invariance
    tok = y.transpose(0, 2, 1, 3).reshape(B, N, -1)
    np.testing.assert_allclose((tok ** 2).mean(-1), 1.0, rtol=1e-4)
    if kind == "layer":
        np.testing.assert_allclose(tok.mean(-1), 0.0, atol=1e-13)
        assert np.abs(mean).max() > 0.1
    else:
        assert np.all(mean == 0.0)
    # exact only without the eps term: scale invariance, and a gradient orthogonal to y
    y0, _, _ = orc.headconcat_norm_fwd(x, kind, 0.0)
    y2, _, _ = orc.headconcat_norm_fwd(1000.0 * x, kind, 0.0)
    np.testing.assert_allclose(y2, y0, rtol=1e-12)
    dx = orc.headconcat_norm_bwd(x, dy, kind, 0.0)
    np.testing.assert_allclose((dx * y0).sum(axis=(1, 3)), 0.0, atol=1e-12)
    if kind == "layer":
        np.testing.assert_allclose(dx.sum(axis=(1, 3)), 0.0, atol=1e-12)


# ------------------------------------------------------------------ sampled-row entry points

@pytest.mark.parametrize("causal", [False, True])
def test_row_sampling_entry_points_match_full_pass(causal):
    B, H, N, d = 1, 2, 50, 8
    q, k, v, dout = (_rand(B, H, N, d) for _ in range(4))
    slopes = _alibi_slopes(H)
    bias = -math.log(N)
    o = orc.sigmoid_attn_fwd(q, k, v, bias, causal, slopes)
    dq, dk, dv = orc.sigmoid_attn_bwd(q, k, v, dout, bias, causal, slopes)
    rows = [0, 1, 17, 49]
    for h in range(H):
        a = (q[0, h], k[0, h], v[0, h])
        np.testing.assert_allclose(orc.sigmoid_attn_fwd_rows(*a, bias, causal, slopes[h], rows), o[0, h, rows],
                                   rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(orc.sigmoid_attn_dq_rows(*a, dout[0, h], bias, causal, slopes[h], rows),
                                   dq[0, h, rows], rtol=1e-12, atol=1e-15)
        rk, rv = orc.sigmoid_attn_dkdv_rows(*a, dout[0, h], bias, causal, slopes[h], rows)
        np.testing.assert_allclose(rk, dk[0, h, rows], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(rv, dv[0, h, rows], rtol=1e-12, atol=1e-15)


# ------------------------------------------------------------------ the pins catch planted mistakes

def _mutant(kind):
    """A numpy sigmoid attention (forward, backward) with one deliberate mistake `kind`
    (None: no mistake).  Lives here, on the CPU, only to show that the pins above fail on it."""

    def probs(q, k, bias, causal, slopes):
        B, H, N, d = q.shape
        scale = 1.0 if kind == "dropped_scale" else math.sqrt(d) if kind == "sqrt_d_scale" else 1.0 / math.sqrt(d)
        s = np.einsum("bhid,bhjd->bhij", q, k)
        if kind == "qk_swapped":
            s = s.transpose(0, 1, 3, 2)
        t = (s + bias) * scale if kind == "bias_before_scale" else s * scale + bias
        idx = np.arange(N)
        if slopes is not None:
            dist = np.abs(idx[:, None] - idx[None, :]).astype(np.float64)
            sgn = 1.0 if kind == "alibi_sign" else -1.0
            t = t + sgn * np.asarray(slopes, dtype=np.float64)[None, :, None, None] * dist
        p = 1.0 / (1.0 + np.exp(-t))
        if causal:
            keep = idx[None, :] < idx[:, None] if kind == "diagonal_masked" else idx[None, :] <= idx[:, None]
            if kind == "mask_flipped":
                keep = idx[None, :] >= idx[:, None]
            p = p * keep
        return p

    def fwd(q, k, v, bias, causal=False, alibi_slopes=None):
        q, k, v = (np.asarray(x, dtype=np.float64) for x in (q, k, v))
        return probs(q, k, bias, causal, alibi_slopes) @ v

    def bwd(q, k, v, dout, bias, causal=False, alibi_slopes=None):
        q, k, v, dout = (np.asarray(x, dtype=np.float64) for x in (q, k, v, dout))
        d = q.shape[-1]
        p = probs(q, k, bias, causal, alibi_slopes)
        dv = np.einsum("bhij,bhid->bhjd", p, dout)
        if kind == "dv_not_transposed":
            dv = np.einsum("bhij,bhjd->bhid", p, dout)
        dp = np.einsum("bhid,bhjd->bhij", dout, v)
        ds = p * dp if kind == "dropped_one_minus_p" else p * (1.0 - p) * dp
        g = math.sqrt(d) if kind == "bwd_sqrt_d" else 1.0 / math.sqrt(d)   # the factor the paper's table prints
        dq = np.einsum("bhij,bhjd->bhid", ds, k) * g
        dk = np.einsum("bhij,bhid->bhjd", ds, q) * g
        if kind == "dq_dk_swapped":
            dq, dk = dk, dq
        return dq, dk, dv

    return fwd, bwd


_FWD_PINS = [
    lambda: test_zero_logits_give_sigma_b_times_sum_of_visible_v(True, 3),
    test_paper_bias_values,
    test_single_token_scalar_case_fixes_scale_and_bias_order,
    test_two_token_hand_example_fixes_operand_roles,
    test_sequence_form_with_log_n_bias,
    test_reflection_symmetry,
    test_alibi_closed_form_and_zero_slope,
]
_BWD_PINS = [
    lambda: test_backward_by_central_finite_differences(True, True),
    test_zero_logit_gradients_closed_form,
    lambda: test_against_torch_fp64_autograd(True, True, (1, 2, 33, 8)),
]


def _failing_pins(pins):
    failed = 0
    for pin in pins:
        try:
            pin()
        except AssertionError:
            failed += 1
    return failed


def test_the_unmutated_twin_passes_every_pin(monkeypatch):
    # the harness itself: without a planted mistake the numpy twin satisfies all the pins, so a
    # failure below is caused by the mistake and not by the twin
    fwd, bwd = _mutant(None)
    monkeypatch.setattr(orc, "sigmoid_attn_fwd", fwd)
    monkeypatch.setattr(orc, "sigmoid_attn_bwd", bwd)
    assert _failing_pins(_FWD_PINS + _BWD_PINS) == 0


@pytest.mark.parametrize("kind,pins", [
    ("dropped_scale", _FWD_PINS), ("sqrt_d_scale", _FWD_PINS), ("bias_before_scale", _FWD_PINS),
    ("qk_swapped", _FWD_PINS), ("alibi_sign", _FWD_PINS), ("diagonal_masked", _FWD_PINS),
    ("mask_flipped", _FWD_PINS),
    ("dv_not_transposed", _BWD_PINS), ("dropped_one_minus_p", _BWD_PINS), ("bwd_sqrt_d", _BWD_PINS),
    ("dq_dk_swapped", _BWD_PINS),
])
def test_planted_mistakes_are_caught_by_the_pins(monkeypatch, kind, pins):
    """Run the pins themselves against an implementation with one planted mistake: at least one
    pin of the relevant group must fail (backward mistakes leave the forward pins green)."""
    fwd, bwd = _mutant(kind)
    monkeypatch.setattr(orc, "sigmoid_attn_fwd", fwd)
    monkeypatch.setattr(orc, "sigmoid_attn_bwd", bwd)
    assert _failing_pins(pins) >= 1, f"no pin notices the mistake '{kind}'"
