"""ctypes front end of the fp64 CPU oracle (sattn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the cpu_baseline
leg of the benchmark.  It shares nothing with the HIP path and the product never calls it.

Every function takes numpy arrays (any float dtype; converted exactly to float64) laid out
[B, H, N, d], and returns float64 numpy arrays.  `bias` is the scalar b of the boxed
sigmoid-attention equation in Section 2; `alibi_slopes` is an optional length-H array m_h;
`causal` keeps keys j <= i.
"""
import ctypes
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sattn_oracle.c")
_LIB = os.path.join(_HERE, "libsattn_oracle.so")

_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int)


def build(force=False):
    """Compile the C oracle with gcc (OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def _f64(x):
    if hasattr(x, "detach"):  # torch tensor (bf16 has no numpy dtype: widen first, exactly)
        x = x.detach().cpu().double().numpy()
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _ptr(a):
    return a.ctypes.data_as(_dp)


def _slopes(alibi_slopes, H):
    if alibi_slopes is None:
        return None, None
    s = _f64(alibi_slopes).reshape(-1)
    assert s.shape[0] == H
    return s, _ptr(s)


def sigmoid_attn_fwd(q, k, v, bias, causal=False, alibi_slopes=None):
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, H, N, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape
    o = np.empty_like(q)
    s, sp = _slopes(alibi_slopes, H)
    _load().oracle_sigmoid_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), B, H, N, d, ctypes.c_double(bias),
                                    int(bool(causal)), sp)
    return o


def sigmoid_attn_bwd(q, k, v, dout, bias, causal=False, alibi_slopes=None):
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    B, H, N, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape and dout.shape == q.shape
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    s, sp = _slopes(alibi_slopes, H)
    _load().oracle_sigmoid_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), B, H, N,
                                    d, ctypes.c_double(bias), int(bool(causal)), sp)
    return dq, dk, dv


def sigmoid_attn_bias_grad(q, k, v, dout, bias, causal=False, alibi_slopes=None):
    """Row sums of dS, [B, H, N]: the gradient of a bias added to each query row's logits."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    B, H, N, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape and dout.shape == q.shape
    db = np.empty((B, H, N), dtype=np.float64)
    s, sp = _slopes(alibi_slopes, H)
    _load().oracle_sigmoid_attn_bias_grad(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(db), B, H, N, d,
                                          ctypes.c_double(bias), int(bool(causal)), sp)
    return db


# ---- shared key/value heads (multi-query attention, Section 5.1: one K/V head for all query
# heads; grouped in general).  Query head h reads K/V head h // (H / Hkv).  By definition this
# is dense attention on the K/V heads repeated over their groups, and a shared head's gradient
# is the sum of the gradients of its copies.

def _expand_kv(x, H):
    x = _f64(x)
    Hkv = x.shape[1]
    assert H % Hkv == 0
    return np.ascontiguousarray(np.repeat(x, H // Hkv, axis=1)), Hkv


def sigmoid_attn_mqa_fwd(q, k, v, bias, causal=False, alibi_slopes=None):
    H = np.shape(q)[1]
    ke, _ = _expand_kv(k, H)
    ve, _ = _expand_kv(v, H)
    return sigmoid_attn_fwd(q, ke, ve, bias, causal, alibi_slopes)


def sigmoid_attn_mqa_bwd(q, k, v, dout, bias, causal=False, alibi_slopes=None):
    B, H, N, d = np.shape(q)
    ke, Hkv = _expand_kv(k, H)
    ve, _ = _expand_kv(v, H)
    dq, dke, dve = sigmoid_attn_bwd(q, ke, ve, dout, bias, causal, alibi_slopes)
    fold = lambda g: g.reshape(B, Hkv, H // Hkv, N, d).sum(axis=2)
    return dq, fold(dke), fold(dve)


def softmax_attn_fwd(q, k, v, causal=False, alibi_slopes=None):
    """Returns (O, LSE) with LSE [B,H,N] in natural-log units."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, H, N, d = q.shape
    o = np.empty_like(q)
    lse = np.empty((B, H, N), dtype=np.float64)
    s, sp = _slopes(alibi_slopes, H)
    _load().oracle_softmax_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), B, H, N, d, int(bool(causal)),
                                    sp)
    return o, lse


def softmax_attn_bwd(q, k, v, dout, causal=False, alibi_slopes=None):
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    B, H, N, d = q.shape
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    s, sp = _slopes(alibi_slopes, H)
    _load().oracle_softmax_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), _ptr(dq), _ptr(dk), _ptr(dv), B, H, N,
                                    d, int(bool(causal)), sp)
    return dq, dk, dv


# ---- sampled rows of ONE head: q,k,v,dout are [N, d]; rows is a list of indices -------------

def _rows(rows):
    r = np.ascontiguousarray(np.asarray(rows, dtype=np.int32))
    return r, r.ctypes.data_as(_ip)


def sigmoid_attn_fwd_rows(q, k, v, bias, causal, slope, rows):
    q, k, v = _f64(q), _f64(k), _f64(v)
    N, d = q.shape
    r, rp = _rows(rows)
    out = np.empty((len(r), d), dtype=np.float64)
    _load().oracle_sigmoid_attn_fwd_rows(_ptr(q), _ptr(k), _ptr(v), N, d, ctypes.c_double(bias), int(bool(causal)),
                                         ctypes.c_double(slope), rp, len(r), _ptr(out))
    return out


def sigmoid_attn_dq_rows(q, k, v, dout, bias, causal, slope, rows):
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    N, d = q.shape
    r, rp = _rows(rows)
    out = np.empty((len(r), d), dtype=np.float64)
    _load().oracle_sigmoid_attn_dq_rows(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), N, d, ctypes.c_double(bias),
                                        int(bool(causal)), ctypes.c_double(slope), rp, len(r), _ptr(out))
    return out


def sigmoid_attn_dkdv_rows(q, k, v, dout, bias, causal, slope, rows):
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    N, d = q.shape
    r, rp = _rows(rows)
    dk = np.empty((len(r), d), dtype=np.float64)
    dv = np.empty((len(r), d), dtype=np.float64)
    _load().oracle_sigmoid_attn_dkdv_rows(_ptr(q), _ptr(k), _ptr(v), _ptr(dout), N, d, ctypes.c_double(bias),
                                          int(bool(causal)), ctypes.c_double(slope), rp, len(r), _ptr(dk), _ptr(dv))
    return dk, dv


def softmax_attn_fwd_rows(q, k, v, causal, slope, rows):
    q, k, v = _f64(q), _f64(k), _f64(v)
    N, d = q.shape
    r, rp = _rows(rows)
    out = np.empty((len(r), d), dtype=np.float64)
    lse = np.empty((len(r),), dtype=np.float64)
    _load().oracle_softmax_attn_fwd_rows(_ptr(q), _ptr(k), _ptr(v), N, d, int(bool(causal)), ctypes.c_double(slope),
                                         rp, len(r), _ptr(out), _ptr(lse))
    return out, lse


# ---- hybrid-norm: normalisation of the attention output over the concatenated heads
# (Section 5.5 and Appendix G.6: x + norm(sigmoid-attention), LayerNorm without learnable
# affine parameters; RMSNorm is the other norm the paper's models use).  o is [B, H, N, d];
# token (b, n) is normalised over its H*d features.  LayerNorm: (x - mean) / sqrt(var + eps)
# with the population variance; RMSNorm: x / sqrt(mean(x^2) + eps).

def headconcat_norm_fwd(o, kind="layer", eps=1e-5):
    """Returns (y [B,H,N,d], mean [B,N], rstd [B,N]); mean is zero for kind == 'rms'."""
    x = _f64(o)
    B, H, N, d = x.shape
    F = H * d
    mean = np.zeros((B, N))
    if kind == "layer":
        for h in range(H):
            mean += x[:, h].sum(axis=-1)
        mean /= F
    else:
        assert kind == "rms"
    var = np.zeros((B, N))
    for h in range(H):
        var += ((x[:, h] - mean[..., None]) ** 2).sum(axis=-1)
    var /= F
    rstd = 1.0 / np.sqrt(var + eps)
    y = (x - mean[:, None, :, None]) * rstd[:, None, :, None]
    return y, mean, rstd


def headconcat_norm_bwd(o, dy, kind="layer", eps=1e-5):
    """dL/do for L = sum(y * dy), from the chain rule through mean and variance."""
    x, g = _f64(o), _f64(dy)
    B, H, N, d = x.shape
    F = H * d
    y, mean, rstd = headconcat_norm_fwd(x, kind, eps)
    gy = (g * y).sum(axis=(1, 3)) / F            # mean over features of dy * y
    dx = g - y * gy[:, None, :, None]
    if kind == "layer":
        dx = dx - (g.sum(axis=(1, 3)) / F)[:, None, :, None]
    return dx * rstd[:, None, :, None]


# ---- different numbers of queries and keys: the definition of Section 2 with Q of n_q rows and
# K, V of n_k rows, written with fp64 matrix products.
#   P = sigmoid(Q K^T / sqrt(d) + b)  [n_q x n_k],  O = P V
#   dV = P^T dO,  dP = dO V^T,  dS = P (1 - P) dP,  dQ = dS K / sqrt(d),  dK = dS^T Q / sqrt(d)
# The paper's models only use n_q = n_k, so where the causal mask (Appendix E.1's decoder
# setting) and ALiBi (Section 5.3) sit when the two differ is a reading: the queries are taken
# to be the LAST n_q positions of the key sequence (query i sits at position i + n_k - n_q, as
# when a prefix's keys and values are already there and new tokens attend to them): key j is
# visible to query i iff j <= i + n_k - n_q, and the ALiBi distance is |i + n_k - n_q - j|.
# With n_q = n_k both reduce to the square definitions.

def _cross_probs(q, k, bias, causal=False, alibi_slopes=None):
    d = q.shape[-1]
    H, nq, nk = q.shape[1], q.shape[2], k.shape[2]
    t = np.einsum("bhid,bhjd->bhij", q, k) / math.sqrt(d) + bias
    pos_q = np.arange(nq)[:, None] + (nk - nq)
    pos_k = np.arange(nk)[None, :]
    if alibi_slopes is not None:
        m = np.asarray(alibi_slopes, dtype=np.float64).reshape(1, H, 1, 1)
        t = t - m * np.abs(pos_q - pos_k)[None, None]
    e = np.exp(-np.abs(t))
    p = np.where(t >= 0, 1.0 / (1.0 + e), e / (1.0 + e))
    if causal:
        p = p * (pos_k <= pos_q)[None, None]
    return p


def sigmoid_attn_cross_fwd(q, k, v, bias, causal=False, alibi_slopes=None):
    q, k, v = _f64(q), _f64(k), _f64(v)
    return np.einsum("bhij,bhjd->bhid", _cross_probs(q, k, bias, causal, alibi_slopes), v)


def sigmoid_attn_cross_bwd(q, k, v, dout, bias, causal=False, alibi_slopes=None):
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    inv = 1.0 / math.sqrt(q.shape[-1])
    p = _cross_probs(q, k, bias, causal, alibi_slopes)
    dv = np.einsum("bhij,bhid->bhjd", p, dout)
    ds = p * (1.0 - p) * np.einsum("bhid,bhjd->bhij", dout, v)   # masked pairs: p = 0, so dS = 0
    return np.einsum("bhij,bhjd->bhid", ds, k) * inv, np.einsum("bhij,bhid->bhjd", ds, q) * inv, dv
