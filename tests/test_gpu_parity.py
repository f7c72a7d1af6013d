"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by
element on the same seeded inputs.

Error measures (both sides in their own precision; the oracle consumes the bf16-rounded
inputs exactly).  `nerr`: for each output tensor X, max|X - X_ref| / max|X_ref|.  `row_err`:
the same ratio taken per token row (max over the row's d features of the difference, over the
row's own max|X_ref|), worst row reported -- under a causal mask early rows are far smaller
than the tensor's maximum (row i of O sums i+1 weights of size ~1/N), so only a per-row
measure notices a wrong early row.  Bars: 2e-2 for the bf16 path, 1e-5 for the fp32 path, for
both measures.
"""
import math

import numpy as np
import pytest
import torch

import paper_2409_04431_amd as sa
from oracle import sattn_oracle as orc
from paper_2409_04431_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
TOL_F32 = 1e-5


def nerr(x, ref):
    """max|x - ref| / max|ref|; an all-zero reference demands an all-zero result."""
    x = x.detach().float().cpu().numpy().astype(np.float64) if hasattr(x, "detach") else x
    den = np.abs(ref).max()
    if den == 0.0:
        return 0.0 if np.abs(x).max() == 0.0 else float("inf")
    return float(np.abs(x - ref).max() / den)


def row_err(x, ref, floor=1e-3):
    """Worst token row of max_c|x - ref| / max(max_c|ref|, floor * max|ref|) (last axis = the
    features of one row).  The floor, a thousandth of the tensor's largest entry, only matters
    for rows whose reference vanishes by cancellation (softmax dQ of the first causal row is
    exactly zero: P_00 = 1 and dP_00 = D_0); the early causal rows this measure exists for are
    ~N^-1/2 of the maximum, far above it."""
    x = x.detach().float().cpu().numpy().astype(np.float64) if hasattr(x, "detach") else x
    x = x.reshape(-1, x.shape[-1])
    ref = np.asarray(ref).reshape(-1, x.shape[-1])
    if x.shape[0] == 0:
        return 0.0
    top = np.abs(ref).max()
    if top == 0.0:
        return 0.0 if np.abs(x).max() == 0.0 else float("inf")
    num = np.abs(x - ref).max(axis=1)
    den = np.maximum(np.abs(ref).max(axis=1), floor * top)
    return float((num / den).max())


def _dev(x):
    return x.cuda()


def _guarded(shape, dtype=torch.bfloat16, pad=256, fill=777.0):
    """An output tensor of `shape` (NaN-filled) inside a larger buffer with sentinel values on
    both sides, and a function that checks the sentinels are untouched."""
    n = int(np.prod(shape))
    buf = torch.full((n + 2 * pad,), fill, dtype=dtype, device="cuda")
    out = buf[pad:pad + n].view(*shape)
    out.fill_(float("nan"))

    def check():
        assert bool((buf[:pad] == fill).all()) and bool((buf[pad + n:] == fill).all()), "write outside the output tensor"
    return out, check


def _run_fwd_bwd(inp, bias, causal, slopes, backward=True):
    q, k, v = (_dev(inp[n]) for n in ("q", "k", "v"))
    sl = _dev(slopes) if slopes is not None else None
    o = torch.full_like(q, float("nan"))
    sa.sigmoid_attn_fwd(q, k, v, o, bias, causal, sl)
    res = {"o": o}
    if backward:
        do = _dev(inp["dout"])
        dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(3))
        sa.sigmoid_attn_bwd(q, k, v, do, dq, dk, dv, bias, causal, sl)
        res.update(dq=dq, dk=dk, dv=dv)
    torch.cuda.synchronize()
    return res


def _rand_inputs(B, H, N, d, seed, dtype=torch.bfloat16, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return {n: (torch.randn(B, H, N, d, generator=g) * scale).to(dtype) for n in ("q", "k", "v", "dout")}


# ------------------------------------------------------------------ small shapes, full oracle

SMALL = [
    # B, H, N, d, causal, alibi   (several tiles + ragged tails; N=1 and N<32 degenerate cases)
    (1, 1, 128, 128, False, False),
    (1, 2, 256, 128, True, False),
    (2, 2, 200, 128, True, True),
    (1, 2, 333, 128, False, True),
    (1, 2, 256, 64, False, False),
    (2, 3, 100, 64, True, True),
    (1, 1, 1, 64, False, False),
    (1, 1, 17, 128, True, False),
    (1, 2, 1000, 64, False, False),
    (1, 1, 513, 128, True, False),
    (1, 3, 385, 64, True, False),
]


@pytest.mark.parametrize("B,H,N,d,causal,alibi", SMALL)
def test_bf16_forward_backward_match_oracle(B, H, N, d, causal, alibi):
    inp = _rand_inputs(B, H, N, d, seed=N * 7 + d)
    slopes = W.alibi_slopes(H) if alibi else None
    bias = -math.log(N)
    got = _run_fwd_bwd(inp, bias, causal, slopes)
    sl = slopes.numpy() if alibi else None
    ro = orc.sigmoid_attn_fwd(inp["q"], inp["k"], inp["v"], bias, causal, sl)
    rq, rk, rv = orc.sigmoid_attn_bwd(inp["q"], inp["k"], inp["v"], inp["dout"], bias, causal, sl)
    for name, ref in (("o", ro), ("dq", rq), ("dk", rk), ("dv", rv)):
        assert not torch.isnan(got[name]).any(), f"{name} has unwritten elements"
        e, er = nerr(got[name], ref), row_err(got[name], ref)
        assert e <= TOL_BF16 and er <= TOL_BF16, f"{name}: {e:.3e} (worst row {er:.3e})"


def test_config2_full_tensor():
    # B4 H12 N1024 d64 bf16 non-causal, inputs scaled by 1/sqrt(d): full oracle pass
    c = W.CONFIGS[2]
    inp = W.make_inputs(c)
    got = _run_fwd_bwd(inp, c.bias, c.causal, None)
    ro = orc.sigmoid_attn_fwd(inp["q"], inp["k"], inp["v"], c.bias, c.causal)
    rq, rk, rv = orc.sigmoid_attn_bwd(inp["q"], inp["k"], inp["v"], inp["dout"], c.bias, c.causal)
    for name, ref in (("o", ro), ("dq", rq), ("dk", rk), ("dv", rv)):
        assert nerr(got[name], ref) <= TOL_BF16, name
        assert row_err(got[name], ref) <= TOL_BF16, name


def test_zero_logits_closed_form_and_bias_values():
    # Q = 0: O_i = sigmoid(b) * sum_j V_j exactly representable structure; b = 0 gives 0.5*sum V
    B, H, N, d = 1, 2, 300, 128
    inp = _rand_inputs(B, H, N, d, seed=5)
    inp["q"] = torch.zeros_like(inp["q"])
    for b in (0.0, -math.log(N)):
        got = _run_fwd_bwd(inp, b, False, None, backward=False)
        ref = (1 / (1 + math.exp(-b))) * inp["v"].double().sum(2, keepdim=True).expand(B, H, N, d).numpy()
        assert nerr(got["o"], ref) <= TOL_BF16


def test_saturation_large_logits_stay_finite():
    # sigmoid(lambda x) -> Heaviside: huge |logits| must saturate to 0/1 without inf/nan
    B, H, N, d = 1, 1, 160, 64
    inp = _rand_inputs(B, H, N, d, seed=11)
    inp["q"] = (inp["q"].float() * 300).bfloat16()
    got = _run_fwd_bwd(inp, 0.0, False, None)
    for t in got.values():
        assert torch.isfinite(t.float()).all()
    ref = orc.sigmoid_attn_fwd(inp["q"], inp["k"], inp["v"], 0.0)
    assert nerr(got["o"], ref) <= TOL_BF16


def test_repeat_runs_are_bit_identical():
    inp = _rand_inputs(2, 2, 384, 128, seed=3)
    a = _run_fwd_bwd(inp, -math.log(384), True, None)
    b = _run_fwd_bwd(inp, -math.log(384), True, None)
    for n in a:
        assert torch.equal(a[n], b[n]), n


def test_strided_bnhd_layout_and_no_out_of_bounds_writes():
    # tensors stored [B, N, H, d] (the paper's benchmark layout) viewed as [B, H, N, d];
    # outputs live inside larger buffers with sentinels around them
    B, H, N, d = 2, 3, 150, 64
    inp = _rand_inputs(B, H, N, d, seed=21)
    bias = -math.log(N)

    def bnhd(x):
        return x.permute(0, 2, 1, 3).contiguous().cuda().permute(0, 2, 1, 3)

    q, k, v, do = (bnhd(inp[n]) for n in ("q", "k", "v", "dout"))
    assert not q.is_contiguous()
    pad = 64
    bufs = [torch.full((B * N * H * d + 2 * pad,), 777.0, dtype=torch.bfloat16, device="cuda") for _ in range(4)]
    outs = [b[pad:-pad].view(B, N, H, d).permute(0, 2, 1, 3) for b in bufs]
    o, dq, dk, dv = outs
    sa.sigmoid_attn_fwd(q, k, v, o, bias, True)
    sa.sigmoid_attn_bwd(q, k, v, do, dq, dk, dv, bias, True)
    torch.cuda.synchronize()
    for b in bufs:
        assert (b[:pad] == 777.0).all() and (b[-pad:] == 777.0).all()
    ro = orc.sigmoid_attn_fwd(inp["q"], inp["k"], inp["v"], bias, True)
    rq, rk, rv = orc.sigmoid_attn_bwd(inp["q"], inp["k"], inp["v"], inp["dout"], bias, True)
    for x, r in zip(outs, (ro, rq, rk, rv)):
        assert nerr(x, r) <= TOL_BF16


def test_split_backward_entry_points_equal_the_fused_call():
    inp = _rand_inputs(1, 2, 200, 128, seed=8)
    q, k, v, do = (_dev(inp[n]) for n in ("q", "k", "v", "dout"))
    b = -math.log(200)
    dq, dk, dv = (torch.empty_like(q) for _ in range(3))
    dq2, dk2, dv2 = (torch.empty_like(q) for _ in range(3))
    sa.sigmoid_attn_bwd(q, k, v, do, dq, dk, dv, b, True)
    sa.sigmoid_attn_bwd_dkdv(q, k, v, do, dk2, dv2, b, True)
    sa.sigmoid_attn_bwd_dq(q, k, v, do, dq2, b, True)
    torch.cuda.synchronize()
    assert torch.equal(dq, dq2) and torch.equal(dk, dk2) and torch.equal(dv, dv2)


# ------------------------------------------------------------------ fp32 path

def test_config1_fp32_full_tensor():
    # B1 H2 N256 d64 fp32 non-causal b=-ln 256: everything fp32, bar 1e-5
    c = W.CONFIGS[1]
    inp = W.make_inputs(c)
    got = _run_fwd_bwd(inp, c.bias, c.causal, None)
    ro = orc.sigmoid_attn_fwd(inp["q"], inp["k"], inp["v"], c.bias, c.causal)
    rq, rk, rv = orc.sigmoid_attn_bwd(inp["q"], inp["k"], inp["v"], inp["dout"], c.bias, c.causal)
    for name, ref in (("o", ro), ("dq", rq), ("dk", rk), ("dv", rv)):
        e, er = nerr(got[name], ref), row_err(got[name], ref)
        assert e <= TOL_F32 and er <= TOL_F32, f"{name}: {e:.3e} (worst row {er:.3e})"


@pytest.mark.parametrize("B,H,N,d,causal,alibi", [
    (1, 2, 256, 64, True, True), (2, 2, 200, 128, True, False), (1, 1, 77, 128, False, True),
    (1, 1, 1, 64, False, False), (1, 3, 300, 64, True, False), (1, 1, 129, 128, False, False),
])
def test_fp32_forward_backward_match_oracle(B, H, N, d, causal, alibi):
    inp = _rand_inputs(B, H, N, d, seed=N + d, dtype=torch.float32)
    slopes = W.alibi_slopes(H) if alibi else None
    bias = -math.log(N)
    got = _run_fwd_bwd(inp, bias, causal, slopes)
    sl = slopes.numpy() if alibi else None
    ro = orc.sigmoid_attn_fwd(inp["q"], inp["k"], inp["v"], bias, causal, sl)
    rq, rk, rv = orc.sigmoid_attn_bwd(inp["q"], inp["k"], inp["v"], inp["dout"], bias, causal, sl)
    for name, ref in (("o", ro), ("dq", rq), ("dk", rk), ("dv", rv)):
        assert not torch.isnan(got[name]).any()
        e = nerr(got[name], ref)
        assert e <= TOL_F32, f"{name}: {e:.3e}"


# ------------------------------------------------------------------ softmax comparison kernels

def _run_softmax(inp, causal, slopes):
    q, k, v, do = (_dev(inp[n]) for n in ("q", "k", "v", "dout"))
    sl = _dev(slopes) if slopes is not None else None
    B, H, N, d = q.shape
    (o, g0), (dq, g1), (dk, g2), (dv, g3) = (_guarded(q.shape) for _ in range(4))
    lse, g4 = _guarded((B, H, N), torch.float32)
    sa.softmax_attn_fwd(q, k, v, o, lse, causal, sl)
    sa.softmax_attn_bwd(q, k, v, o, lse, do, dq, dk, dv, causal, sl)
    torch.cuda.synchronize()
    for g in (g0, g1, g2, g3, g4):   # nothing written outside the outputs
        g()
    return dict(o=o, lse=lse, dq=dq, dk=dk, dv=dv)


@pytest.mark.parametrize("B,H,N,d,causal,alibi", [
    (1, 2, 256, 128, False, False), (1, 2, 256, 128, True, False), (2, 2, 200, 128, True, True),
    (1, 2, 333, 64, False, True), (1, 1, 1, 64, False, False), (1, 2, 1000, 64, True, False),
    (1, 1, 17, 128, True, False), (1, 1, 513, 128, True, False),
])
def test_softmax_comparison_kernels_match_oracle(B, H, N, d, causal, alibi):
    inp = _rand_inputs(B, H, N, d, seed=N + 1)
    slopes = W.alibi_slopes(H) if alibi else None
    got = _run_softmax(inp, causal, slopes)
    sl = slopes.numpy() if alibi else None
    ro, rl = orc.softmax_attn_fwd(inp["q"], inp["k"], inp["v"], causal, sl)
    rq, rk, rv = orc.softmax_attn_bwd(inp["q"], inp["k"], inp["v"], inp["dout"], causal, sl)
    assert float(np.abs(got["lse"].cpu().numpy() - rl).max()) <= 1e-3
    for name, ref in (("o", ro), ("dq", rq), ("dk", rk), ("dv", rv)):
        assert not torch.isnan(got[name]).any()
        e = nerr(got[name], ref)
        assert e <= TOL_BF16, f"{name}: {e:.3e}"
    # rows of P sum to one: with V = 1 the output is 1
    ones = {**inp, "v": torch.ones_like(inp["v"])}
    o1 = _run_softmax(ones, causal, slopes)["o"].float()
    assert float((o1 - 1).abs().max()) <= 1e-2


@pytest.mark.parametrize("B,H,N,d,causal,alibi", [
    (1, 2, 700, 128, False, False), (1, 2, 1100, 128, True, True), (2, 1, 450, 64, True, False),
    (1, 2, 333, 64, False, True),
])
def test_softmax_forward_with_moving_maxima_pinned_and_compiler_scheduled(B, H, N, d, causal, alibi):
    """Logits with a standard deviation of 4: the running maximum of a row keeps moving along
    the key loop, so the rescaling of the partial output is exercised at many steps.  Both forms
    of the forward (hand-pinned steady step, compiler-scheduled step) against the oracle."""
    inp = _rand_inputs(B, H, N, d, seed=77 + N)
    inp["q"] = (inp["q"].float() * 2).to(torch.bfloat16)
    inp["k"] = (inp["k"].float() * 2).to(torch.bfloat16)
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if alibi else None
    q, k, v = (_dev(inp[n]) for n in ("q", "k", "v"))
    ro, rl = orc.softmax_attn_fwd(inp["q"], inp["k"], inp["v"], causal, slopes.numpy() if alibi else None)
    for entry in (sa.softmax_attn_fwd, sa.softmax_attn_fwd_compiler_scheduled):
        (o, g0), (lse, g1) = _guarded(q.shape, torch.bfloat16), _guarded((B, H, N), torch.float32)
        entry(q, k, v, o, lse, causal, sl)
        torch.cuda.synchronize()
        g0(); g1()
        assert not torch.isnan(o).any() and not torch.isnan(lse).any()
        assert nerr(o, ro) <= TOL_BF16 and row_err(o, ro) <= TOL_BF16, entry.__name__
        assert float(np.abs(lse.cpu().numpy() - rl).max()) <= 2e-3, entry.__name__


def test_softmax_full_size_config3_sampled_rows():
    c = W.CONFIGS[3]
    inp = W.make_inputs(c)
    got = {n: t.cpu() for n, t in _run_softmax(inp, c.causal, None).items()}
    rng = np.random.default_rng(33)
    for (b, h) in [(0, 0), (7, 15)]:
        rows = _sample_rows(c.N, 64, rng)
        ro, rl = orc.softmax_attn_fwd_rows(inp["q"][b, h], inp["k"][b, h], inp["v"][b, h], c.causal, 0.0, rows)
        assert nerr(got["o"][b, h][rows], ro) <= TOL_BF16 and row_err(got["o"][b, h][rows], ro) <= TOL_BF16
        assert float(np.abs(got["lse"][b, h][rows].numpy() - rl).max()) <= 1e-3
    # backward at full size: one head against the full fp64 oracle pass of that head
    b, h = 3, 5
    sl = (slice(b, b + 1), slice(h, h + 1))
    rq, rk, rv = orc.softmax_attn_bwd(inp["q"][sl], inp["k"][sl], inp["v"][sl], inp["dout"][sl], c.causal)
    for name, ref in (("dq", rq), ("dk", rk), ("dv", rv)):
        e, er = nerr(got[name][sl], ref), row_err(got[name][sl], ref)
        assert e <= TOL_BF16 and er <= TOL_BF16, f"{name}: {e:.3e}, worst row {er:.3e}"


# ------------------------------------------------------------------ full benchmark sizes, sampled rows

def _sample_rows(N, n, rng, extra=()):  # noqa: E302
    """n random rows plus the rows where mistakes hide: the first rows (tiny under a causal
    mask), both sides of every tile boundary size in use (32, 64, 128, 256), and the last rows."""
    rows = set(int(r) for r in rng.integers(0, N, size=n))
    fixed = (0, 1, 2, 31, 32, 63, 64, 127, 128, 255, 256, N // 2 - 1, N // 2, N - 257, N - 129, N - 33, N - 2, N - 1)
    rows.update(r for r in fixed if 0 <= r < N)
    rows.update(extra)
    return sorted(rows)


def _check_rows(c, inp, got, b, h, rows, label):
    """O, dQ, dK, dV of head (b, h) on `rows` against the oracle, both error measures."""
    sl = inp.get("slopes")
    q, k, v = (inp[n][b, h] for n in ("q", "k", "v"))
    slope = float(sl[h]) if sl is not None else 0.0
    refs = {"o": orc.sigmoid_attn_fwd_rows(q, k, v, c.bias, c.causal, slope, rows)}
    if c.backward:
        do = inp["dout"][b, h]
        refs["dq"] = orc.sigmoid_attn_dq_rows(q, k, v, do, c.bias, c.causal, slope, rows)
        refs["dk"], refs["dv"] = orc.sigmoid_attn_dkdv_rows(q, k, v, do, c.bias, c.causal, slope, rows)
    worst = 0.0
    for name, ref in refs.items():
        x = got[name][b, h][rows]
        e, er = nerr(x, ref), row_err(x, ref)
        assert e <= TOL_BF16 and er <= TOL_BF16, f"{name} head {(b, h)} ({label}): {e:.3e}, worst row {er:.3e}"
        worst = max(worst, er)
    return worst


@pytest.mark.parametrize("cfg,full_heads,dense_heads,ndense", [
    (3, [(0, 0), (7, 15)], [(3, 6)], 1024),
    (4, [(0, 13)], [(0, 0), (0, 31)], 2048),
    (5, [], [(0, 0), (1, 7)], 1024),
])
def test_full_size_configs_on_sampled_rows(cfg, full_heads, dense_heads, ndense):
    """The benchmark configurations at full size, in the launch configuration the benchmark
    times.  Every (batch, head): 8 random rows plus the first rows and the tile-boundary rows.
    `full_heads`: every row of the head.  `dense_heads`: `ndense` random rows, and rows 0..63."""
    c = W.CONFIGS[cfg]
    inp = W.make_inputs(c)
    got = _run_fwd_bwd(inp, c.bias, c.causal, inp.get("slopes"), backward=c.backward)
    got = {n: t.cpu() for n, t in got.items()}
    for t in got.values():
        assert torch.isfinite(t.float()).all()
    rng = np.random.default_rng(cfg)
    worst = 0.0
    for b in range(c.B):
        for h in range(c.H):
            worst = max(worst, _check_rows(c, inp, got, b, h, _sample_rows(c.N, 8, rng), "every head"))
    for (b, h) in full_heads:
        worst = max(worst, _check_rows(c, inp, got, b, h, list(range(c.N)), "all rows"))
    for (b, h) in dense_heads:
        worst = max(worst, _check_rows(c, inp, got, b, h, _sample_rows(c.N, ndense, rng, extra=range(64)), "dense sample"))
    print(f"config {cfg}: worst per-row error {worst:.3e}")


def test_full_size_additivity_over_key_halves():
    # a property that holds at any size: with no normaliser, zeroing V on each half of the
    # keys and adding the two outputs reproduces the full output (up to bf16 rounding of O)
    c = W.CONFIGS[3]
    inp = W.make_inputs(c, shape=(1, 2, c.N, c.d))
    q, k, v = (_dev(inp[n]) for n in ("q", "k", "v"))
    o, o1, o2 = (torch.empty_like(q) for _ in range(3))
    v1, v2 = v.clone(), v.clone()
    v1[:, :, c.N // 2:] = 0
    v2[:, :, :c.N // 2] = 0
    sa.sigmoid_attn_fwd(q, k, v, o, c.bias, False)
    sa.sigmoid_attn_fwd(q, k, v1, o1, c.bias, False)
    sa.sigmoid_attn_fwd(q, k, v2, o2, c.bias, False)
    torch.cuda.synchronize()
    ref = o.float().cpu().numpy().astype(np.float64)
    assert nerr((o1.float() + o2.float()), ref) <= TOL_BF16


def test_matrix_rate_probe_runs_and_reports_a_plausible_rate():
    sink = torch.zeros(64 * 256, dtype=torch.float32, device="cuda")
    sa.sattn_mfma_bf16_probe(64, 100, sink)          # warm-up
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    flops = sa.sattn_mfma_bf16_probe(64, 4000, sink)
    e1.record()
    torch.cuda.synchronize()
    assert flops == 64 * 4 * 4000 * 8 * 32768
    assert torch.isfinite(sink).all()
    per_cu = flops / (e0.elapsed_time(e1) * 1e-3) / 64 / 1e12   # TFLOP/s per compute unit
    assert 2.0 < per_cu < 2.5e3 / 256 * 1.05                    # below the nominal 9.8 TFLOP/s per CU


@pytest.mark.parametrize("B,H,N,d,causal,alibi", [(1, 2, 333, 128, True, False), (2, 2, 200, 64, True, True),
                                                  (1, 1, 640, 128, False, True)])
def test_compiler_scheduled_entry_points_match_oracle(B, H, N, d, causal, alibi):
    inp = _rand_inputs(B, H, N, d, seed=77)
    slopes = W.alibi_slopes(H) if alibi else None
    bias = -float(np.log(N))
    q, k, v, do = (_dev(inp[n]) for n in ("q", "k", "v", "dout"))
    sl = _dev(slopes) if slopes is not None else None
    o, dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(4))
    sa.sigmoid_attn_fwd_compiler_scheduled(q, k, v, o, bias, causal, sl)
    sa.sigmoid_attn_bwd_compiler_scheduled(q, k, v, do, dq, dk, dv, bias, causal, sl)
    torch.cuda.synchronize()
    ro = orc.sigmoid_attn_fwd(inp["q"], inp["k"], inp["v"], bias, causal, slopes)
    rdq, rdk, rdv = orc.sigmoid_attn_bwd(inp["q"], inp["k"], inp["v"], inp["dout"], bias, causal, slopes)
    for name, got, ref in (("o", o, ro), ("dq", dq, rdq), ("dk", dk, rdk), ("dv", dv, rdv)):
        assert nerr(got, ref) <= TOL_BF16, name


# ------------------------------------------------------------------ variable-length batches

@pytest.mark.parametrize("d,causal,alibi,per_seq_bias", [(128, True, False, True), (64, False, True, True),
                                                         (128, True, True, False)])
def test_varlen_batches_match_per_sequence_calls_and_oracle(d, causal, alibi, per_seq_bias):
    H = 2
    lens = [200, 1, 0, 333, 64, 129]                      # ragged, a single token, an empty sequence
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1])
    g = torch.Generator().manual_seed(4321)
    q, k, v, do = (torch.randn(total, H, d, generator=g).bfloat16() for _ in range(4))
    slopes = W.alibi_slopes(H) if alibi else None
    biases = torch.tensor([-float(np.log(max(n, 2))) for n in lens], dtype=torch.float32)
    bias = -float(np.log(max(lens)))
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    sl = _dev(slopes) if slopes is not None else None
    (o, g0), (dq, g1), (dk, g2), (dv, g3) = (_guarded(Q.shape) for _ in range(4))
    cu_d = torch.from_numpy(cu).cuda()
    bp = biases.cuda() if per_seq_bias else None
    sa.sigmoid_attn_varlen_fwd(Q, K, V, o, cu_d, max(lens), bias, causal, sl, bp)
    sa.sigmoid_attn_varlen_bwd(Q, K, V, DO, dq, dk, dv, cu_d, max(lens), bias, causal, sl, bp)
    torch.cuda.synchronize()
    for g in (g0, g1, g2, g3):   # nothing written outside the packed outputs
        g()
    for s_, n in enumerate(lens):
        if n == 0:
            continue
        a, b_ = int(cu[s_]), int(cu[s_ + 1])
        bs = float(biases[s_]) if per_seq_bias else bias
        # dense call on this sequence alone: [1, H, n, d] views of the packed tensors
        dense = lambda t: t[a:b_].permute(1, 0, 2).unsqueeze(0)
        o1, dq1, dk1, dv1 = (torch.full((1, H, n, d), float("nan"), dtype=torch.bfloat16, device="cuda") for _ in range(4))
        sa.sigmoid_attn_fwd(dense(Q), dense(K), dense(V), o1, bs, causal, sl)
        sa.sigmoid_attn_bwd(dense(Q), dense(K), dense(V), dense(DO), dq1, dk1, dv1, bs, causal, sl)
        torch.cuda.synchronize()
        for name, packed, alone in (("o", o, o1), ("dq", dq, dq1), ("dk", dk, dk1), ("dv", dv, dv1)):
            assert torch.equal(dense(packed), alone), f"{name} of sequence {s_} differs from the dense call"
        qs, ks, vs, ds = (t[a:b_].permute(1, 0, 2).unsqueeze(0) for t in (q, k, v, do))
        ro = orc.sigmoid_attn_fwd(qs, ks, vs, bs, causal, slopes)
        rdq, rdk, rdv = orc.sigmoid_attn_bwd(qs, ks, vs, ds, bs, causal, slopes)
        for name, got, ref in (("o", o1, ro), ("dq", dq1, rdq), ("dk", dk1, rdk), ("dv", dv1, rdv)):
            assert nerr(got, ref) <= TOL_BF16, f"{name} of sequence {s_}"


# ------------------------------------------------------------------ learnable-bias gradient

@pytest.mark.parametrize("B,H,N,d,causal,alibi,dtype", [
    (1, 2, 1024, 128, True, False, torch.bfloat16),     # steady-state loop, diagonal, fill and drain
    (2, 2, 1000, 128, False, True, torch.bfloat16),     # ragged last chunk
    (1, 3, 333, 64, True, True, torch.bfloat16),
    (2, 1, 1, 64, False, False, torch.bfloat16),
    (1, 2, 200, 128, True, True, torch.float32),
    (1, 2, 130, 64, False, False, torch.float32),
])
def test_bias_gradient_rows_match_oracle_and_leave_the_other_gradients_unchanged(B, H, N, d, causal, alibi, dtype):
    inp = _rand_inputs(B, H, N, d, seed=977 + N, dtype=dtype)
    slopes = W.alibi_slopes(H) if alibi else None
    bias = -math.log(max(N, 2))
    q, k, v, do = (_dev(inp[n]) for n in ("q", "k", "v", "dout"))
    sl = _dev(slopes) if slopes is not None else None
    dq, dk, dv, dq0, dk0, dv0 = (torch.full_like(q, float("nan")) for _ in range(6))
    rows = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    db = torch.full((B, H), float("nan"), dtype=torch.float32, device="cuda")
    sa.sigmoid_attn_bwd_bias_grad(q, k, v, do, dq, dk, dv, rows, bias, causal, sl, db=db)
    sa.sigmoid_attn_bwd(q, k, v, do, dq0, dk0, dv0, bias, causal, sl)
    torch.cuda.synchronize()
    # the same arithmetic produces dQ, dK, dV with or without the row sums
    assert torch.equal(dq, dq0) and torch.equal(dk, dk0) and torch.equal(dv, dv0)
    f = lambda t: inp[t].double().numpy()
    ref = orc.sigmoid_attn_bias_grad(f("q"), f("k"), f("v"), f("dout"), bias, causal, slopes)
    # dS is formed in fp32 from exact products of the stored inputs and summed in fp32 in both
    # paths, so the row sums carry fp32-level error, far below the bf16 bar of the outputs
    tol = 2e-4 if dtype == torch.bfloat16 else TOL_F32
    assert nerr(rows, ref) <= tol
    assert nerr(db, ref.sum(-1)) <= tol
    np.testing.assert_allclose(db.cpu().numpy(), rows.double().sum(-1).cpu().numpy(), rtol=1e-5, atol=1e-6 * np.abs(ref).max() * N)
    # without db only the rows are written
    rows2 = torch.full_like(rows, float("nan"))
    sa.sigmoid_attn_bwd_bias_grad(q, k, v, do, dq, dk, dv, rows2, bias, causal, sl)
    torch.cuda.synchronize()
    assert torch.equal(rows2, rows)


@pytest.mark.parametrize("d,causal,alibi", [(128, True, False), (64, False, True)])
def test_varlen_bias_gradient_matches_per_sequence_calls_and_oracle(d, causal, alibi):
    # the packed entry point with the row sums of dS: per sequence bit-identical to the dense bias-gradient
    # call on that sequence alone, and within the oracle's bar; db[b, h] = the sum over the sequence's rows
    H = 2
    lens = [300, 1, 0, 129, 64]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1])
    g = torch.Generator().manual_seed(2468)
    q, k, v, do = (torch.randn(total, H, d, generator=g).bfloat16() for _ in range(4))
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if slopes is not None else None
    biases = torch.tensor([-float(np.log(max(n, 2))) for n in lens], dtype=torch.float32)
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    dq, dk, dv, dq0, dk0, dv0 = (torch.full_like(Q, float("nan")) for _ in range(6))
    rows, guard = _guarded((H, total), torch.float32)
    db = torch.full((len(lens), H), float("nan"), dtype=torch.float32, device="cuda")
    cu_d = torch.from_numpy(cu).cuda()
    sa.sigmoid_attn_varlen_bwd_bias_grad(Q, K, V, DO, dq, dk, dv, rows, cu_d, max(lens), 0.0, causal, sl, biases.cuda(), db=db)
    sa.sigmoid_attn_varlen_bwd(Q, K, V, DO, dq0, dk0, dv0, cu_d, max(lens), 0.0, causal, sl, biases.cuda())
    torch.cuda.synchronize()
    guard()
    for a_, b_ in ((dq, dq0), (dk, dk0), (dv, dv0)):   # the other gradients do not change
        assert torch.equal(a_, b_)
    assert not torch.isnan(rows).any()
    for s_, n in enumerate(lens):
        a, b_ = int(cu[s_]), int(cu[s_ + 1])
        if n == 0:
            assert torch.all(db[s_] == 0)
            continue
        dense = lambda t: t[a:b_].permute(1, 0, 2).unsqueeze(0)
        r1 = torch.full((1, H, n), float("nan"), dtype=torch.float32, device="cuda")
        o1, o2, o3 = (torch.empty(1, H, n, d, dtype=torch.bfloat16, device="cuda") for _ in range(3))
        sa.sigmoid_attn_bwd_bias_grad(dense(Q), dense(K), dense(V), dense(DO), o1, o2, o3, r1, float(biases[s_]), causal, sl)
        torch.cuda.synchronize()
        assert torch.equal(rows[:, a:b_], r1[0])
        f = lambda t: t[a:b_].permute(1, 0, 2).unsqueeze(0).double().numpy()
        ref = orc.sigmoid_attn_bias_grad(f(q), f(k), f(v), f(do), float(biases[s_]), causal, slopes)
        assert nerr(rows[:, a:b_], ref[0]) <= 2e-4
        np.testing.assert_allclose(db[s_].cpu().numpy(), ref[0].sum(-1), rtol=2e-4, atol=2e-4 * np.abs(ref).max() * n)


# ------------------------------------------------------------------ fp32 forms of the extended entry points

def test_fp32_variable_length_with_bias_gradient_matches_oracle():
    H, d, causal = 2, 64, True
    lens = [70, 1, 0, 200, 129]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1])
    g = torch.Generator().manual_seed(99)
    q, k, v, do = (torch.randn(total, H, d, generator=g) for _ in range(4))
    slopes = W.alibi_slopes(H)
    biases = torch.tensor([-float(np.log(max(n, 2))) for n in lens], dtype=torch.float32)
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    outs = [_guarded(Q.shape, torch.float32) for _ in range(4)]
    (o, _), (dq, _), (dk, _), (dv, _) = outs
    db_rows = torch.full((H, total), float("nan"), dtype=torch.float32, device="cuda")
    db = torch.full((len(lens), H), float("nan"), dtype=torch.float32, device="cuda")
    cu_d = torch.from_numpy(cu).cuda()
    sa.sigmoid_attn_varlen_fwd(Q, K, V, o, cu_d, max(lens), 0.0, causal, _dev(slopes), biases.cuda())
    sa.sigmoid_attn_varlen_bwd_bias_grad(Q, K, V, DO, dq, dk, dv, db_rows, cu_d, max(lens), 0.0, causal, _dev(slopes),
                                         biases.cuda(), db)
    torch.cuda.synchronize()
    for _, guard in outs:
        guard()
    for s_, n in enumerate(lens):
        a, b_ = int(cu[s_]), int(cu[s_ + 1])
        if n == 0:
            assert bool((db[s_] == 0).all())
            continue
        bs = float(biases[s_])
        dense = lambda t: t[a:b_].permute(1, 0, 2).unsqueeze(0).double().numpy()
        ro = orc.sigmoid_attn_fwd(dense(q), dense(k), dense(v), bs, causal, slopes)
        rq, rk, rv = orc.sigmoid_attn_bwd(dense(q), dense(k), dense(v), dense(do), bs, causal, slopes)
        rrows = orc.sigmoid_attn_bias_grad(dense(q), dense(k), dense(v), dense(do), bs, causal, slopes)
        rdb = rrows.sum(-1)
        for name, got, ref in (("o", o, ro), ("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
            e = nerr(got[a:b_].permute(1, 0, 2).unsqueeze(0).contiguous(), ref)
            assert e <= TOL_F32, f"{name} of sequence {s_}: {e:.3e}"
        assert nerr(db_rows[:, a:b_].unsqueeze(0).contiguous(), rrows) <= TOL_F32
        assert nerr(db[s_:s_ + 1], rdb) <= TOL_F32


@pytest.mark.parametrize("B,H,Hkv,N,d,causal,alibi", [(1, 4, 2, 150, 64, True, True), (2, 4, 1, 257, 128, False, False)])
def test_fp32_shared_kv_heads_match_oracle(B, H, Hkv, N, d, causal, alibi):
    g = torch.Generator().manual_seed(31 + N)
    q, do = (torch.randn(B, H, N, d, generator=g) for _ in range(2))
    k, v = (torch.randn(B, Hkv, N, d, generator=g) for _ in range(2))
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if alibi else None
    bias = -math.log(N)
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    (o, g0), (dq, g1) = (_guarded(Q.shape, torch.float32) for _ in range(2))
    (dk, g2), (dv, g3) = (_guarded(K.shape, torch.float32) for _ in range(2))
    sa.sigmoid_attn_mqa_fwd(Q, K, V, o, bias, causal, sl)
    sa.sigmoid_attn_mqa_bwd(Q, K, V, DO, dq, dk, dv, bias, causal, sl)
    torch.cuda.synchronize()
    for guard in (g0, g1, g2, g3):
        guard()
    f = lambda t: t.double().numpy()
    ro = orc.sigmoid_attn_mqa_fwd(f(q), f(k), f(v), bias, causal, slopes)
    rdq, rdk, rdv = orc.sigmoid_attn_mqa_bwd(f(q), f(k), f(v), f(do), bias, causal, slopes)
    for name, got, ref in (("o", o, ro), ("dq", dq, rdq), ("dk", dk, rdk), ("dv", dv, rdv)):
        assert nerr(got, ref) <= TOL_F32, f"{name}: {nerr(got, ref):.3e}"


@pytest.mark.parametrize("B,H,Nq,Nk,d", [(1, 2, 100, 333, 64), (1, 1, 257, 64, 128), (2, 1, 1, 130, 64)])
def test_fp32_cross_attention_matches_oracle(B, H, Nq, Nk, d):
    g = torch.Generator().manual_seed(700 + Nq + Nk)
    q, do = (torch.randn(B, H, Nq, d, generator=g) for _ in range(2))
    k, v = (torch.randn(B, H, Nk, d, generator=g) for _ in range(2))
    bias = -math.log(max(Nk, 2))
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    (o, g0), (dq, g1) = (_guarded(Q.shape, torch.float32) for _ in range(2))
    (dk, g2), (dv, g3) = (_guarded(K.shape, torch.float32) for _ in range(2))
    sa.sigmoid_attn_cross_fwd(Q, K, V, o, bias)
    sa.sigmoid_attn_cross_bwd(Q, K, V, DO, dq, dk, dv, bias)
    torch.cuda.synchronize()
    for guard in (g0, g1, g2, g3):
        guard()
    f = lambda t: t.double().numpy()
    ro = orc.sigmoid_attn_cross_fwd(f(q), f(k), f(v), bias)
    rdq, rdk, rdv = orc.sigmoid_attn_cross_bwd(f(q), f(k), f(v), f(do), bias)
    for name, got, ref in (("o", o, ro), ("dq", dq, rdq), ("dk", dk, rdk), ("dv", dv, rdv)):
        assert nerr(got, ref) <= TOL_F32, f"{name}: {nerr(got, ref):.3e}"


# ------------------------------------------------------------------ measurement aids

def test_clock_probe_records_per_workgroup_and_respects_its_capacity():
    B, H, N, d = 2, 3, 1024, 128
    inp = _rand_inputs(B, H, N, d, seed=5)
    q, k, v, do = (_dev(inp[n]) for n in ("q", "k", "v", "dout"))
    o, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
    bias = -math.log(N)
    ref = torch.empty_like(q)
    sa.sigmoid_attn_fwd(q, k, v, ref, bias, True)
    n_wg = B * H * (N // 128)            # workgroups of each backward pass
    cap = n_wg - 5                        # fewer slots than workgroups: the rest must not write
    for name, fn in (("fwd", lambda: sa.sigmoid_attn_fwd(q, k, v, o, bias, True)),
                     ("dkdv", lambda: sa.sigmoid_attn_bwd_dkdv(q, k, v, do, dk, dv, bias, True)),
                     ("dq", lambda: sa.sigmoid_attn_bwd_dq(q, k, v, do, dq, bias, True))):
        buf = torch.zeros(8 * cap + 64, dtype=torch.int64, device="cuda")
        buf[8 * cap:] = -7
        sa.sattn_set_clock_probe(buf[:8 * cap])
        try:
            fn()
            torch.cuda.synchronize()
        finally:
            sa.sattn_set_clock_probe(None)
        assert bool((buf[8 * cap:] == -7).all()), name
        c = buf[:8 * cap].view(-1, 8).cpu()
        ran = c[c[:, 1] > 0]
        assert ran.shape[0] > 0, name
        assert bool((ran[:, 0] > 0).all())                       # core cycles
        m = ran[:, 2:6]                                           # stamps in order, all before the end
        assert bool((m[:, 0] > 0).all()) and bool((m[:, 1:] >= m[:, :-1]).all()) and bool((m[:, 3] <= ran[:, 1]).all()), name
        assert bool((ran[:, 6] <= ran[:, 7]).all()) and bool((ran[:, 7] >= 1).all()) and bool((ran[:, 7] <= N // 64 + 1).all()), name
    assert torch.equal(o, ref)   # the probe does not change results


# ------------------------------------------------------------------ seeded random shapes and launch forms

def _random_cases(n, seed=2024):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        d = int(rng.choice([64, 128]))
        B, H = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        kind = i % 3
        if kind == 0:      # around a tile boundary
            N = max(1, int(rng.integers(1, 22)) * 64 + int(rng.integers(-2, 3)))
        elif kind == 1:    # exact multiples of the 128-row block
            N = int(rng.integers(1, 11)) * 128
        else:
            N = int(rng.integers(1, 1400))
        cases.append(dict(B=B, H=H, N=N, d=d, causal=bool(rng.integers(0, 2)), alibi=bool(rng.integers(0, 2)),
                          layout=str(rng.choice(["bhnd", "bnhd"])), waves=int(rng.choice([0, 4, 8, 64])),
                          vslots=int(rng.choice([0, 2, 3])), merged=int(rng.integers(0, 3)),
                          bias=float(rng.uniform(-8.0, 1.0)), scale=float(rng.choice([0.5, 1.0, 2.0])), seed=1000 + i))
    return cases


@pytest.mark.parametrize("c", _random_cases(72), ids=lambda c: "B{B}H{H}N{N}d{d}{causal:d}{alibi:d}{layout}w{waves}v{vslots}m{merged}".format(**c))
def test_seeded_random_shapes_layouts_and_launch_forms_match_oracle(c):
    """Shapes, flags, memory layouts ([B,H,N,d] or a [B,N,H,d] buffer seen through strides),
    forward tile shapes and the one-grid / two-launch forms of the backward drawn from a seeded
    generator: every output against the oracle, with sentinels around the output buffers."""
    B, H, N, d = c["B"], c["H"], c["N"], c["d"]
    inp = _rand_inputs(B, H, N, d, seed=c["seed"], scale=c["scale"])
    inp["dout"] = (inp["dout"].float() / c["scale"]).to(torch.bfloat16)
    slopes = W.alibi_slopes(H) if c["alibi"] else None
    sl = _dev(slopes) if c["alibi"] else None

    def place(t):   # the logical [B,H,N,d] tensor, possibly living in a [B,N,H,d] buffer
        t = _dev(t)
        return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) if c["layout"] == "bnhd" else t

    def out():
        buf, guard = _guarded((B, N, H, d) if c["layout"] == "bnhd" else (B, H, N, d))
        return (buf.permute(0, 2, 1, 3) if c["layout"] == "bnhd" else buf), guard
    q, k, v, do = (place(inp[n]) for n in ("q", "k", "v", "dout"))
    (o, g0), (dq, g1), (dk, g2), (dv, g3) = out(), out(), out(), out()
    if c["waves"] == 64 and c["alibi"] and not c["causal"]:
        c = dict(c, waves=0)   # the 64-row kernel has ALiBi only in its causal form; forcing it is an error
    try:
        sa.sattn_set_fwd_waves(c["waves"])
        sa.sattn_set_fwd_v_slots(c["vslots"])
        sa.sattn_set_bwd_merged(c["merged"])
        sa.sigmoid_attn_fwd(q, k, v, o, c["bias"], c["causal"], sl)
        sa.sigmoid_attn_bwd(q, k, v, do, dq, dk, dv, c["bias"], c["causal"], sl)
        torch.cuda.synchronize()
    finally:
        sa.sattn_set_fwd_waves(0)
        sa.sattn_set_fwd_v_slots(0)
        sa.sattn_set_bwd_merged(0)
    for g in (g0, g1, g2, g3):
        g()
    f = lambda n: inp[n].double().numpy()
    ro = orc.sigmoid_attn_fwd(f("q"), f("k"), f("v"), c["bias"], c["causal"], slopes)
    rq, rk, rv = orc.sigmoid_attn_bwd(f("q"), f("k"), f("v"), f("dout"), c["bias"], c["causal"], slopes)
    for name, got, ref in (("o", o, ro), ("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
        got = got.contiguous()
        assert not torch.isnan(got).any(), name
        e, er = nerr(got, ref), row_err(got, ref)
        assert e <= TOL_BF16 and er <= TOL_BF16, f"{name}: {e:.3e}, worst row {er:.3e}"


# ------------------------------------------------------------------ backward as one grid

@pytest.mark.parametrize("B,H,N,d,causal,alibi", [(1, 2, 700, 128, True, True), (2, 3, 333, 64, False, True),
                                                  (1, 1, 1025, 128, False, False), (3, 2, 96, 64, True, False),
                                                  (2, 2, 512, 128, True, False)])
def test_backward_in_one_grid_equals_the_two_launches_and_the_oracle(B, H, N, d, causal, alibi):
    inp = _rand_inputs(B, H, N, d, seed=57 + N)
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if alibi else None
    bias = -math.log(N)
    q, k, v, do = (_dev(inp[n]) for n in ("q", "k", "v", "dout"))
    res = {}
    try:
        for mode in (1, 2):     # 1: both passes in one launch; 2: one launch per pass
            sa.sattn_set_bwd_merged(mode)
            outs = [_guarded(q.shape) for _ in range(3)]
            sa.sigmoid_attn_bwd(q, k, v, do, outs[0][0], outs[1][0], outs[2][0], bias, causal, sl)
            torch.cuda.synchronize()
            for _, g in outs:
                g()
            res[mode] = [o for o, _ in outs]
    finally:
        sa.sattn_set_bwd_merged(0)
    for a, b in zip(res[1], res[2]):
        assert not torch.isnan(a).any() and torch.equal(a, b)
    f = lambda t: inp[t].double().numpy()
    ref = orc.sigmoid_attn_bwd(f("q"), f("k"), f("v"), f("dout"), bias, causal, slopes)
    for name, got, r in zip(("dq", "dk", "dv"), res[1], ref):
        assert nerr(got, r) <= TOL_BF16, name


# ------------------------------------------------------------------ forward tile shape

@pytest.mark.parametrize("B,H,N,d,causal,alibi", [(1, 2, 700, 128, True, True), (2, 2, 333, 64, False, True),
                                                  (1, 1, 1025, 128, False, False), (1, 3, 96, 64, True, False)])
def test_forward_tile_shapes_agree_bit_for_bit_and_with_the_oracle(B, H, N, d, causal, alibi):
    inp = _rand_inputs(B, H, N, d, seed=31 + N)
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if slopes is not None else None
    bias = -math.log(N)
    q, k, v = (_dev(inp[n]) for n in ("q", "k", "v"))
    outs, souts = {}, {}
    try:
        for waves, vs in ((4, 3), (8, 3), (42, 2)):     # 42: 4 waves with the two-slot V ring
            sa.sattn_set_fwd_waves(4 if waves == 42 else waves)
            sa.sattn_set_fwd_v_slots(vs)
            o = torch.full_like(q, float("nan"))
            so = torch.full_like(q, float("nan"))
            lse = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
            sa.sigmoid_attn_fwd(q, k, v, o, bias, causal, sl)
            sa.softmax_attn_fwd(q, k, v, so, lse, causal, sl)
            torch.cuda.synchronize()
            outs[waves], souts[waves] = o, (so, lse)
    finally:
        sa.sattn_set_fwd_waves(0)
        sa.sattn_set_fwd_v_slots(0)
    for other in (8, 42):
        assert torch.equal(outs[4], outs[other])
        assert torch.equal(souts[4][0], souts[other][0]) and torch.equal(souts[4][1], souts[other][1])
    f = lambda t: inp[t].double().numpy()
    assert nerr(outs[4], orc.sigmoid_attn_fwd(f("q"), f("k"), f("v"), bias, causal, slopes)) <= TOL_BF16
    ro, rl = orc.softmax_attn_fwd(f("q"), f("k"), f("v"), causal, slopes)
    assert nerr(souts[4][0], ro) <= TOL_BF16
    assert np.abs(souts[4][1].cpu().numpy() - rl).max() <= 1e-3


@pytest.mark.parametrize("B,H,N,d,causal,alibi", [
    (1, 2, 700, 128, True, True), (2, 1, 1025, 128, False, False), (1, 2, 2048, 128, True, False),
    (1, 1, 1536, 128, False, False), (1, 3, 96, 128, True, False), (1, 1, 1, 128, False, False),
    (2, 2, 333, 128, True, True), (1, 1, 4096, 128, True, True), (1, 2, 257, 128, False, False),
])
def test_forward_with_64_row_waves(B, H, N, d, causal, alibi):
    """The forward shape with four waves of 64 query rows (head dimension 128).  Forced shape
    64 keeps the arithmetic of the 32-row kernels (bit-identical outputs); 65 multiplies Q by
    the logit scale once and rounds it to bf16 (one more operand rounding), so it is held to the
    oracle's bar only.  N = 1 ... 4096 covers: no steady-state tile at all, ragged last chunks,
    the diagonal steps of every wave, and long pinned loops."""
    inp = _rand_inputs(B, H, N, d, seed=64 + N)
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if slopes is not None else None
    bias = -math.log(max(N, 2))
    q, k, v = (_dev(inp[n]) for n in ("q", "k", "v"))
    outs = {}
    try:
        for shape in (8, 64, 65):
            sa.sattn_set_fwd_waves(shape)
            o = torch.full_like(q, float("nan"))
            sa.sigmoid_attn_fwd(q, k, v, o, bias, causal, sl)
            torch.cuda.synchronize()
            outs[shape] = o
    finally:
        sa.sattn_set_fwd_waves(0)
    assert torch.equal(outs[64], outs[8])
    ref = orc.sigmoid_attn_fwd(inp["q"], inp["k"], inp["v"], bias, causal, slopes)
    for shape in (64, 65):
        assert not torch.isnan(outs[shape]).any()
        e, er = nerr(outs[shape], ref), row_err(outs[shape], ref)
        print(f"shape {shape}: {e:.3e}, worst row {er:.3e}")
        assert e <= TOL_BF16 and er <= TOL_BF16, f"shape {shape}: {e:.3e}, worst row {er:.3e}"


@pytest.mark.parametrize("B,H,N,alibi", [(16, 16, 4096, False), (8, 32, 4100, True), (2, 64, 7600, True)])
def test_forward_with_paired_causal_blocks(B, H, N, alibi):
    """Causal launches of the 64-row forward deal a head's blocks out in pairs (longest with
    shortest) when there are at least 16 of them and a pair per compute unit: same numbers as
    single blocks (forced shape 66), bit for bit; sampled rows against the oracle; and the clock
    probe still gets one record per block.  N = 4100 has 17 blocks (odd: not paired)."""
    d = 128
    g = torch.Generator().manual_seed(6600 + N)
    q, k, v = (torch.randn(B, H, N, d, generator=g).bfloat16() for _ in range(3))
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if slopes is not None else None
    bias = -math.log(N)
    Q, K, V = (_dev(t) for t in (q, k, v))
    outs = {}
    n_blocks = B * H * ((N + 255) // 256)
    buf = torch.zeros(8 * n_blocks + 64, dtype=torch.int64, device="cuda")
    buf[8 * n_blocks:] = -7
    try:
        for shape in (66, 64):
            sa.sattn_set_fwd_waves(shape)
            o, guard = _guarded(Q.shape)
            if shape == 64:
                sa.sattn_set_clock_probe(buf[:8 * n_blocks])
            sa.sigmoid_attn_fwd(Q, K, V, o, bias, True, sl)
            torch.cuda.synchronize()
            guard()
            outs[shape] = o
    finally:
        sa.sattn_set_clock_probe(None)
        sa.sattn_set_fwd_waves(0)
    assert not torch.isnan(outs[64]).any() and torch.equal(outs[64], outs[66])
    rec = buf[:8 * n_blocks].view(-1, 8).cpu()
    assert bool((buf[8 * n_blocks:] == -7).all()) and bool((rec[:, 1] > 0).all())   # every block left its record
    assert int(rec[:, 7].sum()) == B * H * sum(min((256 * (b + 1) + 63) // 64, (N + 63) // 64) for b in range((N + 255) // 256))
    rows = np.array(sorted({0, 31, 255, 256, N // 2, N - 257, N - 1}))
    f = lambda t: t.double().numpy()
    for (b, h) in ((0, 0), (B - 1, H - 1), (B // 2, 3)):
        ref = orc.sigmoid_attn_fwd_rows(f(q[b, h]), f(k[b, h]), f(v[b, h]), bias, True,
                                        0.0 if slopes is None else float(slopes[h]), rows)
        got = outs[64][b, h][torch.as_tensor(rows, device="cuda")]
        assert row_err(got, ref) <= TOL_BF16, f"{(b, h)}: {row_err(got, ref):.3e}"


@pytest.mark.parametrize("B,H,N,d,alibi", [(8, 8, 2048, 128, True), (4, 16, 2100, 64, False), (16, 4, 4096, 64, True),
                                           (4, 4, 4000, 128, True), (8, 8, 1000, 64, False)])   # the last two: ragged last block
def test_backward_with_paired_causal_blocks(B, H, N, d, alibi):
    """The causal backward passes deal a head's 128-row blocks out in pairs (longest with
    shortest) when there is an even number of them (at least 4) and a pair per compute unit:
    same numbers as single blocks (mode 3 of the one-grid setter), bit for bit; sampled rows
    against the oracle; one clock-probe record per block.  N = 2100 has 17 blocks (not paired)."""
    g = torch.Generator().manual_seed(6700 + N + d)
    q, k, v, do = (torch.randn(B, H, N, d, generator=g).bfloat16() for _ in range(4))
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if slopes is not None else None
    bias = -math.log(N)
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    n_blocks = B * H * ((N + 127) // 128)
    outs = {}
    try:
        for mode in (3, 2):
            sa.sattn_set_bwd_merged(mode)
            (dq, g0), (dk, g1), (dv, g2) = (_guarded(Q.shape) for _ in range(3))
            sa.sigmoid_attn_bwd(Q, K, V, DO, dq, dk, dv, bias, True, sl)
            torch.cuda.synchronize()
            for guard in (g0, g1, g2):
                guard()
            outs[mode] = (dq, dk, dv)
        for fn in (lambda: sa.sigmoid_attn_bwd_dkdv(Q, K, V, DO, dk, dv, bias, True, sl),
                   lambda: sa.sigmoid_attn_bwd_dq(Q, K, V, DO, dq, bias, True, sl)):
            buf = torch.zeros(8 * n_blocks + 64, dtype=torch.int64, device="cuda")
            buf[8 * n_blocks:] = -7
            sa.sattn_set_clock_probe(buf[:8 * n_blocks])
            fn()
            torch.cuda.synchronize()
            sa.sattn_set_clock_probe(None)
            rec = buf[:8 * n_blocks].view(-1, 8).cpu()
            assert bool((buf[8 * n_blocks:] == -7).all()) and bool((rec[:, 1] > 0).all())
    finally:
        sa.sattn_set_clock_probe(None)
        sa.sattn_set_bwd_merged(0)
    for a, b_ in zip(outs[2], outs[3]):
        assert not torch.isnan(a).any() and torch.equal(a, b_)
    rows = np.array(sorted({0, 31, 127, 128, N // 2, N - 129, N - 1}))
    ridx = torch.as_tensor(rows, device="cuda")
    f = lambda t: t.double().numpy()
    dq, dk, dv = outs[2]
    for (b, h) in ((0, 0), (B - 1, H - 1), (B // 2, 1)):
        slope = 0.0 if slopes is None else float(slopes[h])
        rq = orc.sigmoid_attn_dq_rows(f(q[b, h]), f(k[b, h]), f(v[b, h]), f(do[b, h]), bias, True, slope, rows)
        rk, rv = orc.sigmoid_attn_dkdv_rows(f(q[b, h]), f(k[b, h]), f(v[b, h]), f(do[b, h]), bias, True, slope, rows)
        for name, got, ref in (("dq", dq, rq), ("dk", dk, rk), ("dv", dv, rv)):
            e = row_err(got[b, h][ridx], ref)
            assert e <= TOL_BF16, f"{name} {(b, h)}: {e:.3e}"


@pytest.mark.parametrize("B,H,Hkv,N,d,alibi", [(8, 16, 4, 2048, 128, True), (8, 8, 2, 4096, 64, False), (16, 16, 16, 1024, 128, False)])
def test_shared_kv_heads_with_paired_causal_blocks(B, H, Hkv, N, d, alibi):
    """The grouped dK/dV pass deals key blocks out in pairs as the dense one does: bit-equal to
    single blocks (whose results the other shared-head tests hold to the oracle), and dK, dV of
    sampled key rows against the oracle summed over the group's query heads."""
    g = torch.Generator().manual_seed(6800 + N + Hkv)
    q, do = (torch.randn(B, H, N, d, generator=g).bfloat16() for _ in range(2))
    k, v = (torch.randn(B, Hkv, N, d, generator=g).bfloat16() for _ in range(2))
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if slopes is not None else None
    bias = -math.log(N)
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    outs = {}
    try:
        for mode in (3, 0):
            sa.sattn_set_bwd_merged(mode)
            (dq, g0) = _guarded(Q.shape)
            (dk, g1), (dv, g2) = (_guarded(K.shape) for _ in range(2))
            sa.sigmoid_attn_mqa_bwd(Q, K, V, DO, dq, dk, dv, bias, True, sl)
            torch.cuda.synchronize()
            for guard in (g0, g1, g2):
                guard()
            outs[mode] = (dq, dk, dv)
    finally:
        sa.sattn_set_bwd_merged(0)
    for a, b_ in zip(outs[0], outs[3]):
        assert not torch.isnan(a).any() and torch.equal(a, b_)
    rows = np.array(sorted({0, 127, 128, N // 2 + 5, N - 129, N - 1}))
    ridx = torch.as_tensor(rows, device="cuda")
    f = lambda t: t.double().numpy()
    G = H // Hkv
    for (b, gk) in ((0, 0), (B - 1, Hkv - 1)):
        rk, rv = np.zeros((len(rows), d)), np.zeros((len(rows), d))
        for h in range(gk * G, (gk + 1) * G):
            a, b2 = orc.sigmoid_attn_dkdv_rows(f(q[b, h]), f(k[b, gk]), f(v[b, gk]), f(do[b, h]), bias, True,
                                               0.0 if slopes is None else float(slopes[h]), rows)
            rk += a
            rv += b2
        for name, got, ref in (("dk", outs[0][1][b, gk][ridx], rk), ("dv", outs[0][2][b, gk][ridx], rv)):
            e = row_err(got, ref)
            assert e <= TOL_BF16, f"{name} {(b, gk)}: {e:.3e}"


@pytest.mark.parametrize("B,H,Hkv,N,d,causal,alibi", [
    (1, 8, 1, 700, 128, True, True),        # one K/V head: the group split over up to 8 workgroups
    (2, 4, 1, 333, 64, False, False),       # ragged, no mask
    (1, 6, 2, 520, 128, True, False),       # groups of three: cannot be split (stays one workgroup per group)
    (1, 16, 2, 1024, 64, True, True),
])
def test_shared_kv_heads_with_split_groups_match_oracle(B, H, Hkv, N, d, causal, alibi):
    g = torch.Generator().manual_seed(6900 + N + H)
    q, do = (torch.randn(B, H, N, d, generator=g).bfloat16() for _ in range(2))
    k, v = (torch.randn(B, Hkv, N, d, generator=g).bfloat16() for _ in range(2))
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if slopes is not None else None
    bias = -math.log(N)
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    need = sa.sigmoid_attn_mqa_bwd_workspace_bytes(B, H, Hkv, N, d, torch.bfloat16, causal)
    assert (need > 0) == ((H // Hkv) % 2 == 0)     # these grids are far too small not to split an even group
    buf = torch.full((need + 512,), 77, dtype=torch.uint8, device="cuda")   # workspace with sentinels on both sides
    ws = buf[256:256 + need]
    gw = lambda: bool((buf[:256] == 77).all()) and bool((buf[256 + need:] == 77).all()) or pytest.fail("write outside the workspace")
    (dq, g0) = _guarded(Q.shape)
    (dk, g1), (dv, g2) = (_guarded(K.shape) for _ in range(2))
    sa.sigmoid_attn_mqa_bwd_split(Q, K, V, DO, dq, dk, dv, bias, causal, sl, ws if need else None)
    torch.cuda.synchronize()
    for guard in (g0, g1, g2, gw):
        guard()
    f = lambda t: t.double().numpy()
    sl64 = None if slopes is None else slopes.double().numpy()
    rdq, rdk, rdv = orc.sigmoid_attn_mqa_bwd(f(q), f(k), f(v), f(do), bias, causal, sl64)
    for name, got, ref in (("dq", dq, rdq), ("dk", dk, rdk), ("dv", dv, rdv)):
        assert not torch.isnan(got).any(), name
        e, er = nerr(got, ref), row_err(got, ref)
        assert e <= TOL_BF16 and er <= TOL_BF16, f"{name}: {e:.3e}, worst row {er:.3e}"
    if need:   # too small a workspace is refused, nothing written
        with pytest.raises(sa.SattnError):
            sa.sigmoid_attn_mqa_bwd_split(Q, K, V, DO, dq, dk, dv, bias, causal, sl, ws[:need - 16])


def test_shared_kv_heads_with_split_groups_at_full_size():
    """One K/V head at the headline size (256 unequal workgroups without the split): the split
    form against the one-workgroup-per-group form, which the other tests hold to the oracle --
    they differ in the order of the fp32 sums over the query heads and in nothing else."""
    B, H, Hkv, N, d = 8, 16, 1, 4096, 128
    g = torch.Generator().manual_seed(6999)
    q, do = (torch.randn(B, H, N, d, generator=g).bfloat16() for _ in range(2))
    k, v = (torch.randn(B, Hkv, N, d, generator=g).bfloat16() for _ in range(2))
    bias = -math.log(N)
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    dq, dq2 = torch.empty_like(Q), torch.empty_like(Q)
    dk, dv, dk2, dv2 = (torch.full_like(K, float("nan")) for _ in range(4))
    assert sa.sigmoid_attn_mqa_bwd_workspace_bytes(B, H, Hkv, N, d, torch.bfloat16, True) == 2 * 2 * B * N * d * 4
    sa.sigmoid_attn_mqa_bwd(Q, K, V, DO, dq, dk, dv, bias, True)
    sa.sigmoid_attn_mqa_bwd_split(Q, K, V, DO, dq2, dk2, dv2, bias, True)
    torch.cuda.synchronize()
    assert torch.equal(dq, dq2)
    for name, a, b_ in (("dk", dk, dk2), ("dv", dv, dv2)):
        assert not torch.isnan(b_).any()
        e = row_err(b_, a.double().cpu().numpy())
        assert e <= 2 ** -7, f"{name}: {e:.3e}"       # two bf16 roundings of nearly equal fp32 sums


@pytest.mark.parametrize("B,H,N,d,alibi", [(8, 8, 2048, 128, True), (16, 8, 1000, 64, False), (4, 16, 2100, 128, False)])
def test_softmax_backward_pinned_paired_and_compiler_scheduled_forms_agree(B, H, N, d, alibi):
    """The softmax comparison backward in its three forms on a causal problem large enough for the
    paired blocks: hand-pinned with pairs (the default), hand-pinned with single blocks (bit-equal)
    and compiler-scheduled (same arithmetic, another summation order inside the MFMAs' inputs:
    equal to a bf16 rounding); sampled rows of the default against the oracle.  N = 1000 has a
    ragged last block, N = 2100 an odd number of blocks (not paired)."""
    g = torch.Generator().manual_seed(7700 + N + d)
    q, k, v, do = (torch.randn(B, H, N, d, generator=g).bfloat16() for _ in range(4))
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if slopes is not None else None
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    o = torch.empty_like(Q)
    lse = torch.empty(B, H, N, dtype=torch.float32, device="cuda")
    sa.softmax_attn_fwd(Q, K, V, o, lse, True, sl)
    outs = {}
    try:
        for name, mode, fn in (("paired", 0, sa.softmax_attn_bwd), ("single", 3, sa.softmax_attn_bwd),
                               ("cs", 0, sa.softmax_attn_bwd_compiler_scheduled)):
            sa.sattn_set_bwd_merged(mode)
            (dq, g0), (dk, g1), (dv, g2) = (_guarded(Q.shape) for _ in range(3))
            fn(Q, K, V, o, lse, DO, dq, dk, dv, True, sl)
            torch.cuda.synchronize()
            for guard in (g0, g1, g2):
                guard()
            outs[name] = (dq, dk, dv)
    finally:
        sa.sattn_set_bwd_merged(0)
    for a, b_, c in zip(outs["paired"], outs["single"], outs["cs"]):
        assert not torch.isnan(a).any() and torch.equal(a, b_)
        assert row_err(a, c.double().cpu().numpy()) <= 2 ** -7
    rows = np.array(sorted({0, 31, 127, 128, N // 2, N - 129, N - 1}))
    ridx = torch.as_tensor(rows, device="cuda")
    f = lambda t: t.double().numpy()
    for (b, h) in ((0, 0), (B - 1, H - 1)):
        sl1 = None if slopes is None else slopes[h:h + 1].double().numpy()
        one = lambda t: f(t[b:b + 1, h:h + 1])
        rq, rk, rv = orc.softmax_attn_bwd(one(q), one(k), one(v), one(do), True, sl1)
        for name, got, ref in (("dq", outs["paired"][0], rq), ("dk", outs["paired"][1], rk), ("dv", outs["paired"][2], rv)):
            e = row_err(got[b, h][ridx], ref[0, 0][rows])
            assert e <= TOL_BF16, f"{name} {(b, h)}: {e:.3e}"


def test_forward_with_64_row_waves_on_packed_shared_and_cross_inputs():
    # the entry points that reuse the forward kernels: variable-length batches, shared K/V heads,
    # different numbers of queries and keys -- each against its own 32-row result, bit for bit
    H, d = 4, 128
    g = torch.Generator().manual_seed(640)
    lens = [900, 1, 0, 333, 1500]
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
    total = sum(lens)
    q, k, v = (torch.randn(total, H, d, generator=g).bfloat16().cuda() for _ in range(3))
    bs = torch.tensor([-math.log(max(n, 2)) for n in lens], dtype=torch.float32).cuda()
    Q4, K4, V4 = (torch.randn(2, H, 1100, d, generator=g).bfloat16().cuda() for _ in range(3))
    Kg, Vg = K4[:, :2].contiguous(), V4[:, :2].contiguous()
    Kc, Vc = (torch.randn(2, H, 1700, d, generator=g).bfloat16().cuda() for _ in range(2))
    res = {}
    try:
        for shape in (8, 64):
            sa.sattn_set_fwd_waves(shape)
            o1 = torch.full_like(q, float("nan"))
            sa.sigmoid_attn_varlen_fwd(q, k, v, o1, cu, max(lens), 0.0, True, None, bs)
            o2 = torch.full_like(Q4, float("nan"))
            sa.sigmoid_attn_mqa_fwd(Q4, Kg, Vg, o2, -7.0, True)
            o3 = torch.full_like(Q4, float("nan"))
            sa.sigmoid_attn_cross_fwd(Q4, Kc, Vc, o3, -7.4)
            torch.cuda.synchronize()
            res[shape] = (o1, o2, o3)
    finally:
        sa.sattn_set_fwd_waves(0)
    for a, b_ in zip(res[8], res[64]):
        assert not torch.isnan(b_).any() and torch.equal(a, b_)


# ------------------------------------------------------------------ shared key/value heads

@pytest.mark.parametrize("B,H,Hkv,N,d,causal,alibi", [
    (1, 4, 1, 1024, 128, True, True),      # multi-query, several tiles per head, steady-state loop
    (2, 4, 2, 333, 128, False, False),     # two groups, ragged
    (1, 6, 2, 200, 64, True, False),
    (1, 3, 1, 700, 64, False, True),
    (1, 2, 2, 160, 128, True, False),      # one K/V head per query head: the plain kernels' results
])
def test_shared_kv_heads_match_oracle_and_the_expanded_dense_call(B, H, Hkv, N, d, causal, alibi):
    g = torch.Generator().manual_seed(5150 + N)
    q, do = (torch.randn(B, H, N, d, generator=g).bfloat16() for _ in range(2))
    k, v = (torch.randn(B, Hkv, N, d, generator=g).bfloat16() for _ in range(2))
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if slopes is not None else None
    bias = -math.log(N)
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    (o, g0), (dq, g1) = (_guarded(Q.shape) for _ in range(2))
    (dk, g2), (dv, g3) = (_guarded(K.shape) for _ in range(2))
    sa.sigmoid_attn_mqa_fwd(Q, K, V, o, bias, causal, sl)
    sa.sigmoid_attn_mqa_bwd(Q, K, V, DO, dq, dk, dv, bias, causal, sl)
    torch.cuda.synchronize()
    for g in (g0, g1, g2, g3):   # nothing written outside the outputs (dK/dV have fewer heads)
        g()
    f = lambda t: t.double().numpy()
    ro = orc.sigmoid_attn_mqa_fwd(f(q), f(k), f(v), bias, causal, slopes)
    rdq, rdk, rdv = orc.sigmoid_attn_mqa_bwd(f(q), f(k), f(v), f(do), bias, causal, slopes)
    for name, got, ref in (("o", o, ro), ("dq", dq, rdq), ("dk", dk, rdk), ("dv", dv, rdv)):
        assert not torch.isnan(got).any(), name
        assert nerr(got, ref) <= TOL_BF16, f"{name}: {nerr(got, ref):.3e}"
    # the query side is the dense computation on K/V heads repeated over their groups, bit for bit
    Ke, Ve = (t.repeat_interleave(H // Hkv, dim=1).contiguous() for t in (K, V))
    o2, dq2, dk2, dv2 = (torch.full_like(Q, float("nan")) for _ in range(4))
    sa.sigmoid_attn_fwd(Q, Ke, Ve, o2, bias, causal, sl)
    sa.sigmoid_attn_bwd(Q, Ke, Ve, DO, dq2, dk2, dv2, bias, causal, sl)
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(dq, dq2)
    if Hkv == H:
        assert torch.equal(dk, dk2) and torch.equal(dv, dv2)


# ------------------------------------------------------------------ hybrid-norm

@pytest.mark.parametrize("B,H,N,d,kind,bnhd", [
    (2, 16, 300, 128, "layer", False), (1, 12, 257, 64, "layer", True), (2, 3, 65, 64, "rms", False),
    (1, 32, 130, 128, "rms", True), (1, 64, 9, 128, "layer", False), (3, 1, 5, 64, "layer", False),
])
def test_headconcat_norm_matches_oracle(B, H, N, d, kind, bnhd):
    g = torch.Generator().manual_seed(88 + H)
    x = (torch.randn(B, H, N, d, generator=g) * 2.0 + 0.5).bfloat16()
    dy = torch.randn(B, H, N, d, generator=g).bfloat16()

    def dev(t):   # optionally token-major storage viewed as [B,H,N,d]
        if not bnhd:
            return t.cuda()
        return t.permute(0, 2, 1, 3).contiguous().cuda().permute(0, 2, 1, 3)
    X, DY = dev(x), dev(dy)

    def out():   # guarded output in the same storage order as the inputs
        t, g = _guarded((B, N, H, d) if bnhd else (B, H, N, d))
        return (t.permute(0, 2, 1, 3) if bnhd else t), g
    (Y, g0), (DX, g1) = out(), out()
    stats, g2 = _guarded((B, N, 2), torch.float32)
    sa.sattn_headconcat_norm_fwd(X, Y, stats, kind, 1e-5)
    sa.sattn_headconcat_norm_bwd(X, DY, stats, DX, kind)
    torch.cuda.synchronize()
    for g in (g0, g1, g2):   # nothing written outside the outputs
        g()
    ry, rmean, rrstd = orc.headconcat_norm_fwd(x.double().numpy(), kind, 1e-5)
    rdx = orc.headconcat_norm_bwd(x.double().numpy(), dy.double().numpy(), kind, 1e-5)
    # fp32 statistics of exactly representable inputs; outputs rounded once to bf16 (2^-9 relative)
    np.testing.assert_allclose(stats[..., 0].cpu().numpy(), rmean, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(stats[..., 1].cpu().numpy(), rrstd, rtol=1e-5)
    assert nerr(Y, ry) <= 4e-3 and nerr(DX, rdx) <= 4e-3


# ------------------------------------------------------------------ the added entry points at config-3 size

def test_full_size_variable_length_bias_gradient_and_shared_heads():
    c = W.CONFIGS[3]
    H, d = c.H, c.d
    g = torch.Generator().manual_seed(303)
    # variable length: eight sequences filling config 3's token count of one batch row pair
    lens = [4096, 1000, 3333, 64, 2048, 1, 4095, 1747]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    total = int(cu[-1])
    q, k, v, do = (torch.randn(total, H, d, generator=g).bfloat16().cuda() for _ in range(4))
    o, dq, dk, dv = (torch.full_like(q, float("nan")) for _ in range(4))
    cu_d = torch.from_numpy(cu).cuda()
    bs = torch.tensor([-math.log(max(n, 2)) for n in lens], dtype=torch.float32).cuda()
    sa.sigmoid_attn_varlen_fwd(q, k, v, o, cu_d, max(lens), 0.0, True, None, bs)
    sa.sigmoid_attn_varlen_bwd(q, k, v, do, dq, dk, dv, cu_d, max(lens), 0.0, True, None, bs)
    torch.cuda.synchronize()
    for t in (o, dq, dk, dv):
        assert torch.isfinite(t.float()).all()
    for s_ in (0, 2, 5, 7):
        a, b_ = int(cu[s_]), int(cu[s_ + 1])
        n = b_ - a
        dense = lambda t: t[a:b_].permute(1, 0, 2).unsqueeze(0)
        o1, dq1, dk1, dv1 = (torch.empty(1, H, n, d, dtype=torch.bfloat16, device="cuda") for _ in range(4))
        sa.sigmoid_attn_fwd(dense(q), dense(k), dense(v), o1, float(bs[s_]), True)
        sa.sigmoid_attn_bwd(dense(q), dense(k), dense(v), dense(do), dq1, dk1, dv1, float(bs[s_]), True)
        torch.cuda.synchronize()
        for packed, alone in ((o, o1), (dq, dq1), (dk, dk1), (dv, dv1)):
            assert torch.equal(dense(packed), alone)
        # and against the oracle: sampled rows of two heads of this sequence, with its own bias
        rng = np.random.default_rng(900 + s_)
        for h in (0, H - 1 - s_ % 3):
            rows = _sample_rows(n, 48, rng)
            qs, ks, vs, ds = (t[a:b_, h].cpu() for t in (q, k, v, do))
            bias_s = float(bs[s_])
            refs = {"o": orc.sigmoid_attn_fwd_rows(qs, ks, vs, bias_s, True, 0.0, rows),
                    "dq": orc.sigmoid_attn_dq_rows(qs, ks, vs, ds, bias_s, True, 0.0, rows)}
            refs["dk"], refs["dv"] = orc.sigmoid_attn_dkdv_rows(qs, ks, vs, ds, bias_s, True, 0.0, rows)
            for name, packed in (("o", o), ("dq", dq), ("dk", dk), ("dv", dv)):
                x = packed[a:b_, h].cpu()[rows]
                e, er = nerr(x, refs[name]), row_err(x, refs[name])
                assert e <= TOL_BF16 and er <= TOL_BF16, f"varlen {name} seq {s_} head {h}: {e:.3e}, row {er:.3e}"
    # bias gradient on config 3 itself: one head against the oracle, every head against dQ's twin
    inp = W.make_inputs(c)
    Q, K, V, DO = (_dev(inp[n]) for n in ("q", "k", "v", "dout"))
    dq, dk, dv, dq0, dk0, dv0 = (torch.empty_like(Q) for _ in range(6))
    rows = torch.full((c.B, c.H, c.N), float("nan"), dtype=torch.float32, device="cuda")
    db = torch.empty(c.B, c.H, dtype=torch.float32, device="cuda")
    sa.sigmoid_attn_bwd_bias_grad(Q, K, V, DO, dq, dk, dv, rows, c.bias, c.causal, None, db=db)
    sa.sigmoid_attn_bwd(Q, K, V, DO, dq0, dk0, dv0, c.bias, c.causal)
    torch.cuda.synchronize()
    assert torch.equal(dq, dq0) and torch.equal(dk, dk0) and torch.equal(dv, dv0)
    f = lambda n, b, h: inp[n][b:b + 1, h:h + 1].double().numpy()
    ref = orc.sigmoid_attn_bias_grad(f("q", 5, 9), f("k", 5, 9), f("v", 5, 9), f("dout", 5, 9), c.bias, c.causal)
    assert nerr(rows[5:6, 9:10], ref) <= 2e-4
    np.testing.assert_allclose(db.cpu().numpy(), rows.double().sum(-1).cpu().numpy(), rtol=1e-4, atol=1e-4)
    # shared K/V heads at config-3 size: the query side equals the dense call on repeated heads
    Hkv = 4
    Kg, Vg = K[:, :Hkv].contiguous(), V[:, :Hkv].contiguous()
    o, dq = torch.empty_like(Q), torch.empty_like(Q)
    dkg, dvg = torch.empty_like(Kg), torch.empty_like(Vg)
    sa.sigmoid_attn_mqa_fwd(Q, Kg, Vg, o, c.bias, c.causal)
    sa.sigmoid_attn_mqa_bwd(Q, Kg, Vg, DO, dq, dkg, dvg, c.bias, c.causal)
    Ke, Ve = (t.repeat_interleave(c.H // Hkv, dim=1).contiguous() for t in (Kg, Vg))
    o2, dq2, dk2, dv2 = (torch.empty_like(Q) for _ in range(4))
    sa.sigmoid_attn_fwd(Q, Ke, Ve, o2, c.bias, c.causal)
    sa.sigmoid_attn_bwd(Q, Ke, Ve, DO, dq2, dk2, dv2, c.bias, c.causal)
    torch.cuda.synchronize()
    assert torch.equal(o, o2) and torch.equal(dq, dq2)
    # dK/dV: fp32 sum inside one workgroup against the sum of the dense call's bf16 per-head results
    fold = lambda t: t.float().reshape(c.B, Hkv, c.H // Hkv, c.N, c.d).sum(2).cpu().numpy().astype(np.float64)
    assert nerr(dkg, fold(dk2)) <= TOL_BF16 and nerr(dvg, fold(dv2)) <= TOL_BF16
    # against the oracle: a shared head's gradient is the sum over its group's query heads
    rng = np.random.default_rng(77)
    G = c.H // Hkv
    dkg_c, dvg_c = dkg.cpu(), dvg.cpu()
    for (b, g_) in ((0, 0), (5, 3), (7, 1)):
        rows = _sample_rows(c.N, 40, rng)
        rk = np.zeros((len(rows), c.d))
        rv = np.zeros((len(rows), c.d))
        for h in range(g_ * G, (g_ + 1) * G):
            a, b2 = orc.sigmoid_attn_dkdv_rows(inp["q"][b, h], inp["k"][b, g_], inp["v"][b, g_], inp["dout"][b, h],
                                               c.bias, c.causal, 0.0, rows)
            rk += a
            rv += b2
        for name, x, ref in (("dk", dkg_c[b, g_][rows], rk), ("dv", dvg_c[b, g_][rows], rv)):
            e, er = nerr(x, ref), row_err(x, ref)
            assert e <= TOL_BF16 and er <= TOL_BF16, f"shared-head {name} {(b, g_)}: {e:.3e}, row {er:.3e}"


# ------------------------------------------------------------------ different numbers of queries and keys

@pytest.mark.parametrize("B,H,Nq,Nk,d", [
    (1, 2, 300, 1100, 128), (2, 1, 1024, 257, 128), (1, 3, 1, 700, 64), (1, 2, 640, 1, 64),
    (1, 1, 129, 2048, 64), (1, 2, 777, 777, 128),
])
def test_cross_attention_matches_oracle(B, H, Nq, Nk, d):
    g = torch.Generator().manual_seed(7000 + Nq + Nk)
    q, do = (torch.randn(B, H, Nq, d, generator=g).bfloat16() for _ in range(2))
    k, v = (torch.randn(B, H, Nk, d, generator=g).bfloat16() for _ in range(2))
    bias = -math.log(max(Nk, 2))
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    (o, g0), (dq, g1) = (_guarded(Q.shape) for _ in range(2))
    (dk, g2), (dv, g3) = (_guarded(K.shape) for _ in range(2))
    sa.sigmoid_attn_cross_fwd(Q, K, V, o, bias)
    sa.sigmoid_attn_cross_bwd(Q, K, V, DO, dq, dk, dv, bias)
    torch.cuda.synchronize()
    for g in (g0, g1, g2, g3):   # nothing written outside the outputs (two different lengths)
        g()
    f = lambda t: t.double().numpy()
    ro = orc.sigmoid_attn_cross_fwd(f(q), f(k), f(v), bias)
    rdq, rdk, rdv = orc.sigmoid_attn_cross_bwd(f(q), f(k), f(v), f(do), bias)
    for name, got, ref in (("o", o, ro), ("dq", dq, rdq), ("dk", dk, rdk), ("dv", dv, rdv)):
        assert not torch.isnan(got).any(), name
        assert nerr(got, ref) <= TOL_BF16, f"{name}: {nerr(got, ref):.3e}"
    if Nq == Nk:   # the square entry points run the same kernels
        o2, dq2, dk2, dv2 = (torch.empty_like(Q) for _ in range(4))
        sa.sigmoid_attn_fwd(Q, K, V, o2, bias)
        sa.sigmoid_attn_bwd(Q, K, V, DO, dq2, dk2, dv2, bias)
        torch.cuda.synchronize()
        assert torch.equal(o, o2) and torch.equal(dq, dq2) and torch.equal(dk, dk2) and torch.equal(dv, dv2)


def _aligned_case(B, H, Nq, Nk, d, causal, alibi, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    cast = (lambda t: t.bfloat16()) if dtype == torch.bfloat16 else (lambda t: t)
    q, do = (cast(torch.randn(B, H, Nq, d, generator=g)) for _ in range(2))
    k, v = (cast(torch.randn(B, H, Nk, d, generator=g)) for _ in range(2))
    slopes = W.alibi_slopes(H) if alibi else None
    sl = _dev(slopes) if slopes is not None else None
    bias = -math.log(max(Nk, 2))
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    (o, g0), (dq, g1) = (_guarded(Q.shape, dtype) for _ in range(2))
    (dk, g2), (dv, g3) = (_guarded(K.shape, dtype) for _ in range(2))
    sa.sigmoid_attn_cross_aligned_fwd(Q, K, V, o, bias, causal, sl)
    sa.sigmoid_attn_cross_aligned_bwd(Q, K, V, DO, dq, dk, dv, bias, causal, sl)
    torch.cuda.synchronize()
    for guard in (g0, g1, g2, g3):
        guard()
    f = lambda t: t.double().numpy()
    sl64 = None if slopes is None else slopes.double().numpy()
    ro = orc.sigmoid_attn_cross_fwd(f(q), f(k), f(v), bias, causal, sl64)
    rdq, rdk, rdv = orc.sigmoid_attn_cross_bwd(f(q), f(k), f(v), f(do), bias, causal, sl64)
    return (Q, K, V, DO, sl, bias), (o, dq, dk, dv), (ro, rdq, rdk, rdv)


# Queries placed at the end of the key sequence (a prefix of keys and values is already there):
# the causal mask and ALiBi of that placement.  bf16 offsets are multiples of 32 under the mask.
@pytest.mark.parametrize("B,H,Nq,Nk,d,causal,alibi", [
    (1, 2, 300, 1100, 128, True, False),     # a prefix of 800 keys, ragged
    (1, 2, 300, 1100, 128, True, True),
    (2, 1, 1024, 256, 128, True, True),      # fewer keys than queries: the first 768 queries see none
    (1, 3, 1, 705, 64, True, True),          # one new token
    (1, 2, 640, 32, 64, True, False),
    (1, 1, 129, 2049, 64, True, True),
    (1, 2, 1500, 3100, 128, True, True),     # steady-state loops of every kernel
    (1, 2, 1500, 3100, 64, True, False),
    (1, 2, 1100, 940, 128, True, True),      # offset -160: a 64-row wave whose first row block sees no key
    (1, 2, 300, 1001, 128, False, True),     # no mask: any offset; ALiBi measured from the shifted position
    (1, 2, 1001, 300, 64, False, True),
])
def test_end_aligned_cross_attention_matches_oracle(B, H, Nq, Nk, d, causal, alibi):
    args, got, ref = _aligned_case(B, H, Nq, Nk, d, causal, alibi, torch.bfloat16, 7100 + Nq + Nk)
    for name, x, r in zip(("o", "dq", "dk", "dv"), got, ref):
        assert not torch.isnan(x).any(), name
        assert nerr(x, r) <= TOL_BF16, f"{name}: {nerr(x, r):.3e}"
    Q, K, V, DO, sl, bias = args
    if d == 128 and (causal or not alibi):   # the 64-row forward shape (no ALiBi without the mask) computes the same numbers
        try:
            sa.sattn_set_fwd_waves(64)
            o64 = torch.full_like(Q, float("nan"))
            sa.sigmoid_attn_cross_aligned_fwd(Q, K, V, o64, bias, causal, sl)
            torch.cuda.synchronize()
        finally:
            sa.sattn_set_fwd_waves(0)
        assert torch.equal(o64, got[0])


def test_end_aligned_cross_attention_with_paired_blocks():
    """Enough heads and blocks that the causal kernels deal the blocks out in pairs, with the
    queries at the end of a longer key sequence: bit-equal to single blocks, and sampled rows
    against the square causal oracle on the whole sequence (queries and output gradients of the
    prefix positions padded with zeros, which changes nothing for the sampled outputs)."""
    B, H, Nq, Nk, d = 2, 16, 4096, 5120, 128
    off = Nk - Nq
    g = torch.Generator().manual_seed(7400)
    q, do = (torch.randn(B, H, Nq, d, generator=g).bfloat16() for _ in range(2))
    k, v = (torch.randn(B, H, Nk, d, generator=g).bfloat16() for _ in range(2))
    slopes = W.alibi_slopes(H)
    sl = _dev(slopes)
    bias = -math.log(Nk)
    Q, K, V, DO = (_dev(t) for t in (q, k, v, do))
    outs = {}
    try:
        for waves, mode in ((66, 3), (0, 0)):
            sa.sattn_set_fwd_waves(waves)
            sa.sattn_set_bwd_merged(mode)
            (o, g0), (dq, g1) = (_guarded(Q.shape) for _ in range(2))
            (dk, g2), (dv, g3) = (_guarded(K.shape) for _ in range(2))
            sa.sigmoid_attn_cross_aligned_fwd(Q, K, V, o, bias, True, sl)
            sa.sigmoid_attn_cross_aligned_bwd(Q, K, V, DO, dq, dk, dv, bias, True, sl)
            torch.cuda.synchronize()
            for guard in (g0, g1, g2, g3):
                guard()
            outs[waves] = (o, dq, dk, dv)
    finally:
        sa.sattn_set_fwd_waves(0)
        sa.sattn_set_bwd_merged(0)
    for a, b_ in zip(outs[0], outs[66]):
        assert not torch.isnan(a).any() and torch.equal(a, b_)
    o, dq, dk, dv = outs[0]
    f = lambda t: t.double().numpy()
    qrows = np.array(sorted({0, 31, 255, 256, Nq // 2, Nq - 257, Nq - 1}))
    krows = np.array(sorted({0, 127, off - 1, off, off + 130, Nk // 2, Nk - 129, Nk - 1}))
    for (b, h) in ((0, 0), (1, 15), (1, 6)):
        qp, dop = np.zeros((Nk, d)), np.zeros((Nk, d))
        qp[off:], dop[off:] = f(q[b, h]), f(do[b, h])
        kk, vv, slope = f(k[b, h]), f(v[b, h]), float(slopes[h])
        ro = orc.sigmoid_attn_fwd_rows(qp, kk, vv, bias, True, slope, qrows + off)
        rq = orc.sigmoid_attn_dq_rows(qp, kk, vv, dop, bias, True, slope, qrows + off)
        rk, rv = orc.sigmoid_attn_dkdv_rows(qp, kk, vv, dop, bias, True, slope, krows)
        qi, ki = torch.as_tensor(qrows, device="cuda"), torch.as_tensor(krows, device="cuda")
        for name, got, ref in (("o", o[b, h][qi], ro), ("dq", dq[b, h][qi], rq), ("dk", dk[b, h][ki], rk),
                               ("dv", dv[b, h][ki], rv)):
            e = row_err(got, ref)
            assert e <= TOL_BF16, f"{name} {(b, h)}: {e:.3e}"


def test_end_aligned_cross_attention_with_equal_counts_is_self_attention():
    B, H, N, d = 1, 2, 777, 128
    args, got, _ = _aligned_case(B, H, N, N, d, True, True, torch.bfloat16, 7177)
    Q, K, V, DO, sl, bias = args
    o2, dq2, dk2, dv2 = (torch.empty_like(Q) for _ in range(4))
    sa.sigmoid_attn_fwd(Q, K, V, o2, bias, True, sl)
    sa.sigmoid_attn_bwd(Q, K, V, DO, dq2, dk2, dv2, bias, True, sl)
    torch.cuda.synchronize()
    for a, b_ in zip(got, (o2, dq2, dk2, dv2)):
        assert torch.equal(a, b_)


def test_end_aligned_cross_attention_rejects_unaligned_offsets_in_bf16():
    q = torch.zeros(1, 1, 64, 64, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(1, 1, 100, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sa.SattnError):
        sa.sigmoid_attn_cross_aligned_fwd(q, k, k, torch.empty_like(q), 0.0, True)


@pytest.mark.parametrize("B,H,Nq,Nk,d,causal,alibi", [
    (1, 2, 100, 333, 64, True, True),        # any offset in fp32
    (1, 1, 333, 100, 128, True, False),
    (2, 2, 65, 64, 64, True, True),
    (1, 2, 50, 1000, 128, False, True),
    (1, 1, 257, 290, 128, True, True),
])
def test_fp32_end_aligned_cross_attention_matches_oracle(B, H, Nq, Nk, d, causal, alibi):
    _, got, ref = _aligned_case(B, H, Nq, Nk, d, causal, alibi, torch.float32, 7300 + Nq + Nk)
    for name, x, r in zip(("o", "dq", "dk", "dv"), got, ref):
        assert nerr(x, r) <= TOL_F32, f"{name}: {nerr(x, r):.3e}"
