"""ctypes binding of libsattn.so: argument marshalling only.

Every function mirrors the C entry point of the same name in include/sattn.h.  Tensors are
torch CUDA tensors of shape [B, H, N, d] (any strides with a contiguous last dimension);
PyTorch is used for device memory and the current stream, nothing else.  There is no CPU
fallback: if the library cannot be loaded the call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsattn.so")
_lib = None

SATTN_BF16, SATTN_F32 = 0, 1


class SattnError(RuntimeError):
    pass


class _Strides(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int64), ("head", ctypes.c_int64), ("seq", ctypes.c_int64)]


_SP = ctypes.POINTER(_Strides)
_vp = ctypes.c_void_p


def library_path():
    return _LIB_PATH


def load_library():
    """Load libsattn.so (built by paper_2409_04431_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise SattnError(f"{_LIB_PATH} is missing: build it first (python -m paper_2409_04431_amd.build)")
    lib = ctypes.CDLL(_LIB_PATH)
    i, f, sz = ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.sigmoid_attn_fwd.argtypes = [_vp, _vp, _vp, _vp, i, i, i, i, i, f, i, _vp, _SP, _SP, _SP, _SP, _vp]
    lib.sigmoid_attn_fwd.restype = i
    lib.sigmoid_attn_bwd.argtypes = [_vp] * 7 + [i, i, i, i, i, f, i, _vp] + [_SP] * 7 + [_vp, sz, _vp]
    lib.sigmoid_attn_bwd.restype = i
    lib.sigmoid_attn_fwd_compiler_scheduled.argtypes = lib.sigmoid_attn_fwd.argtypes
    lib.sigmoid_attn_fwd_compiler_scheduled.restype = i
    lib.sigmoid_attn_bwd_compiler_scheduled.argtypes = lib.sigmoid_attn_bwd.argtypes
    lib.sigmoid_attn_bwd_compiler_scheduled.restype = i
    lib.sigmoid_attn_mqa_fwd.argtypes = [_vp, _vp, _vp, _vp, i, i, i, i, i, i, f, i, _vp, _SP, _SP, _SP, _SP, _vp]
    lib.sigmoid_attn_mqa_fwd.restype = i
    lib.sigmoid_attn_mqa_bwd.argtypes = [_vp] * 7 + [i, i, i, i, i, i, f, i, _vp] + [_SP] * 7 + [_vp]
    lib.sigmoid_attn_mqa_bwd.restype = i
    lib.sigmoid_attn_mqa_bwd_split.argtypes = [_vp] * 7 + [i, i, i, i, i, i, f, i, _vp] + [_SP] * 7 + [_vp, sz, _vp]
    lib.sigmoid_attn_mqa_bwd_split.restype = i
    lib.sigmoid_attn_mqa_bwd_workspace_bytes.argtypes = [i, i, i, i, i, i, i]
    lib.sigmoid_attn_mqa_bwd_workspace_bytes.restype = sz
    lib.sigmoid_attn_cross_fwd.argtypes = [_vp, _vp, _vp, _vp, i, i, i, i, i, i, f, _SP, _SP, _SP, _SP, _vp]
    lib.sigmoid_attn_cross_fwd.restype = i
    lib.sigmoid_attn_cross_bwd.argtypes = [_vp] * 7 + [i, i, i, i, i, i, f] + [_SP] * 7 + [_vp]
    lib.sigmoid_attn_cross_bwd.restype = i
    lib.sigmoid_attn_cross_aligned_fwd.argtypes = [_vp, _vp, _vp, _vp, i, i, i, i, i, i, f, i, _vp, _SP, _SP, _SP, _SP, _vp]
    lib.sigmoid_attn_cross_aligned_fwd.restype = i
    lib.sigmoid_attn_cross_aligned_bwd.argtypes = [_vp] * 7 + [i, i, i, i, i, i, f, i, _vp] + [_SP] * 7 + [_vp]
    lib.sigmoid_attn_cross_aligned_bwd.restype = i
    lib.sigmoid_attn_bwd_bias_grad.argtypes = [_vp] * 9 + [i, i, i, i, i, f, i, _vp] + [_SP] * 7 + [_vp]
    lib.sigmoid_attn_bwd_bias_grad.restype = i
    ip = ctypes.c_void_p
    lib.sigmoid_attn_varlen_fwd.argtypes = [_vp, _vp, _vp, _vp, ip, _vp, i, i, i, i, i, f, i, _vp, _SP, _SP, _SP, _SP, _vp]
    lib.sigmoid_attn_varlen_fwd.restype = i
    lib.sigmoid_attn_varlen_bwd.argtypes = [_vp] * 7 + [ip, _vp, i, i, i, i, i, f, i, _vp] + [_SP] * 7 + [_vp]
    lib.sigmoid_attn_varlen_bwd.restype = i
    lib.sigmoid_attn_varlen_bwd_bias_grad.argtypes = [_vp] * 9 + [ip, _vp, i, i, i, ctypes.c_int64, i, i, f, i, _vp] + [_SP] * 7 + [_vp]
    lib.sigmoid_attn_varlen_bwd_bias_grad.restype = i
    lib.sigmoid_attn_bwd_dkdv.argtypes = [_vp] * 6 + [i, i, i, i, i, f, i, _vp] + [_SP] * 6 + [_vp]
    lib.sigmoid_attn_bwd_dkdv.restype = i
    lib.sigmoid_attn_bwd_dq.argtypes = [_vp] * 5 + [i, i, i, i, i, f, i, _vp] + [_SP] * 5 + [_vp]
    lib.sigmoid_attn_bwd_dq.restype = i
    lib.sigmoid_attn_bwd_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.sigmoid_attn_bwd_workspace_bytes.restype = sz
    lib.softmax_attn_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp, i, i, i, i, i, i, _vp, _SP, _SP, _SP, _SP, _vp]
    lib.softmax_attn_fwd.restype = i
    lib.softmax_attn_fwd_compiler_scheduled.argtypes = lib.softmax_attn_fwd.argtypes
    lib.softmax_attn_fwd_compiler_scheduled.restype = i
    lib.softmax_attn_bwd.argtypes = [_vp] * 9 + [i, i, i, i, i, i, _vp] + [_SP] * 8 + [_vp, sz, _vp]
    lib.softmax_attn_bwd.restype = i
    lib.softmax_attn_bwd_compiler_scheduled.argtypes = lib.softmax_attn_bwd.argtypes
    lib.softmax_attn_bwd_compiler_scheduled.restype = i
    lib.softmax_attn_bwd_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.softmax_attn_bwd_workspace_bytes.restype = sz
    lib.softmax_attn_bwd_noalloc.argtypes = [_vp] * 9 + [i, i, i, i, i, i, _vp] + [_SP] * 8 + [_vp]
    lib.softmax_attn_bwd_noalloc.restype = i
    lib.softmax_attn_bwd_noalloc_max_rows.argtypes = []
    lib.softmax_attn_bwd_noalloc_max_rows.restype = sz
    lib.sattn_strerror.argtypes = [i]
    lib.sattn_strerror.restype = ctypes.c_char_p
    lib.sattn_mfma_bf16_probe.argtypes = [i, i, _vp, _vp]
    lib.sattn_mfma_bf16_probe.restype = i
    lib.sattn_headconcat_norm_fwd.argtypes = [_vp, _vp, _vp, i, i, i, i, i, i, f, _SP, _SP, _vp]
    lib.sattn_headconcat_norm_fwd.restype = i
    lib.sattn_headconcat_norm_bwd.argtypes = [_vp, _vp, _vp, _vp, i, i, i, i, i, i, _SP, _SP, _SP, _vp]
    lib.sattn_headconcat_norm_bwd.restype = i
    lib.sattn_fwd_waves.argtypes = [i, i, i, i, i]
    lib.sattn_fwd_waves.restype = i
    lib.sattn_set_fwd_waves.argtypes = [i]
    lib.sattn_set_fwd_waves.restype = i
    lib.sattn_fwd_v_slots.argtypes = [i, i, i, i, i]
    lib.sattn_fwd_v_slots.restype = i
    lib.sattn_set_fwd_v_slots.argtypes = [i]
    lib.sattn_set_fwd_v_slots.restype = i
    lib.sattn_set_bwd_merged.argtypes = [i]
    lib.sattn_set_bwd_merged.restype = i
    lib.sattn_bwd_merged.argtypes = [i, i, i, i]
    lib.sattn_bwd_merged.restype = i
    lib.sattn_set_clock_probe.argtypes = [_vp, i]
    lib.sattn_set_clock_probe.restype = i
    lib.sattn_wall_clock_khz.argtypes = []
    lib.sattn_wall_clock_khz.restype = i
    lib.sattn_device_info.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    lib.sattn_device_info.restype = i
    lib.sattn_version.argtypes = []
    lib.sattn_version.restype = i
    _lib = lib
    return lib


def sattn_strerror(code):
    return load_library().sattn_strerror(int(code)).decode()


def _check_varlen(cu_seqlens, bias_per_seq, *ts):
    t0 = ts[0]
    for t in ts:
        if (not t.is_cuda or t.dim() != 3 or t.shape != t0.shape or t.dtype != t0.dtype
                or t.dtype not in (torch.bfloat16, torch.float32) or t.stride(2) != 1):
            raise SattnError("varlen tensors must be CUDA bf16 or fp32 [tokens, H, d] of one dtype with a contiguous last dimension")
    if not cu_seqlens.is_cuda or cu_seqlens.dtype != torch.int32 or cu_seqlens.dim() != 1 or not cu_seqlens.is_contiguous():
        raise SattnError("cu_seqlens must be a contiguous CUDA int32 vector of B+1 offsets")
    B = cu_seqlens.numel() - 1
    if bias_per_seq is not None and (not bias_per_seq.is_cuda or bias_per_seq.dtype != torch.float32
                                     or bias_per_seq.numel() != B or not bias_per_seq.is_contiguous()):
        raise SattnError("bias_per_seq must be a contiguous CUDA float32 vector of B elements")
    return B


def _st3(t):
    return ctypes.byref(_Strides(0, t.stride(1), t.stride(0)))


def sigmoid_attn_varlen_fwd(q, k, v, o, cu_seqlens, max_seqlen, bias, causal=False, alibi_slopes=None,
                            bias_per_seq=None):
    """Forward over B packed sequences ([tokens, H, d] tensors, offsets in cu_seqlens)."""
    lib = load_library()
    B = _check_varlen(cu_seqlens, bias_per_seq, q, k, v, o)
    _, H, d = q.shape
    bp = _vp(bias_per_seq.data_ptr()) if bias_per_seq is not None else None
    rc = lib.sigmoid_attn_varlen_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(),
                                     _vp(cu_seqlens.data_ptr()), bp, B, H, int(max_seqlen), d, _dtype_code(q),
                                     float(bias), int(bool(causal)), _slopes_ptr(alibi_slopes, H),
                                     _st3(q), _st3(k), _st3(v), _st3(o), _stream())
    _raise(rc, "sigmoid_attn_varlen_fwd")
    return o


def sigmoid_attn_varlen_bwd(q, k, v, dout, dq, dk, dv, cu_seqlens, max_seqlen, bias, causal=False,
                            alibi_slopes=None, bias_per_seq=None):
    """Backward over B packed sequences ([tokens, H, d] tensors, offsets in cu_seqlens)."""
    lib = load_library()
    B = _check_varlen(cu_seqlens, bias_per_seq, q, k, v, dout, dq, dk, dv)
    _, H, d = q.shape
    bp = _vp(bias_per_seq.data_ptr()) if bias_per_seq is not None else None
    rc = lib.sigmoid_attn_varlen_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                                     dk.data_ptr(), dv.data_ptr(), _vp(cu_seqlens.data_ptr()), bp, B, H,
                                     int(max_seqlen), d, _dtype_code(q), float(bias), int(bool(causal)),
                                     _slopes_ptr(alibi_slopes, H), _st3(q), _st3(k), _st3(v), _st3(dout),
                                     _st3(dq), _st3(dk), _st3(dv), _stream())
    _raise(rc, "sigmoid_attn_varlen_bwd")
    return dq, dk, dv


def sigmoid_attn_varlen_bwd_bias_grad(q, k, v, dout, dq, dk, dv, db_rows, cu_seqlens, max_seqlen, bias, causal=False,
                                      alibi_slopes=None, bias_per_seq=None, db=None):
    """sigmoid_attn_varlen_bwd plus db_rows[h, t] = sum_j dS_tj (fp32 [H, tokens]) and, if given, db[b, h]."""
    lib = load_library()
    B = _check_varlen(cu_seqlens, bias_per_seq, q, k, v, dout, dq, dk, dv)
    total, H, d = q.shape
    for t, shape, what in ((db_rows, (H, total), "db_rows"), (db, (B, H), "db")):
        if t is None and what == "db":
            continue
        if t is None or not t.is_cuda or t.dtype != torch.float32 or tuple(t.shape) != shape or not t.is_contiguous():
            raise SattnError(f"{what} must be a contiguous CUDA float32 tensor of shape {shape}")
    bp = _vp(bias_per_seq.data_ptr()) if bias_per_seq is not None else None
    rc = lib.sigmoid_attn_varlen_bwd_bias_grad(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                                               dk.data_ptr(), dv.data_ptr(), _vp(db_rows.data_ptr()),
                                               _vp(db.data_ptr()) if db is not None else None,
                                               _vp(cu_seqlens.data_ptr()), bp, B, H, int(max_seqlen), int(total), d,
                                               _dtype_code(q), float(bias), int(bool(causal)), _slopes_ptr(alibi_slopes, H),
                                               _st3(q), _st3(k), _st3(v), _st3(dout), _st3(dq), _st3(dk), _st3(dv),
                                               _stream())
    _raise(rc, "sigmoid_attn_varlen_bwd_bias_grad")
    return dq, dk, dv, db_rows, db


def _check_mqa(q, kv, *qlike):
    _check(q, *qlike)
    _check(*kv)
    B, H, N, d = q.shape
    Bk, Hkv, Nk, dk = kv[0].shape
    if (Bk, Nk, dk) != (B, N, d) or Hkv <= 0 or H % Hkv:
        raise SattnError(f"K/V shape {tuple(kv[0].shape)} does not match Q {tuple(q.shape)} with shared heads")
    return B, H, Hkv, N, d


def sigmoid_attn_mqa_fwd(q, k, v, o, bias, causal=False, alibi_slopes=None):
    """Forward with shared K/V heads: q, o [B,H,N,d]; k, v [B,Hkv,N,d], Hkv divides H."""
    lib = load_library()
    B, H, Hkv, N, d = _check_mqa(q, (k, v), o)
    rc = lib.sigmoid_attn_mqa_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), B, H, Hkv, N, d,
                                  _dtype_code(q), float(bias), int(bool(causal)), _slopes_ptr(alibi_slopes, H),
                                  _st(q), _st(k), _st(v), _st(o), _stream())
    _raise(rc, "sigmoid_attn_mqa_fwd")
    return o


def sigmoid_attn_mqa_bwd(q, k, v, dout, dq, dk, dv, bias, causal=False, alibi_slopes=None):
    """Backward with shared K/V heads: dk, dv [B,Hkv,N,d] are summed over each head's query group."""
    lib = load_library()
    B, H, Hkv, N, d = _check_mqa(q, (k, v, dk, dv), dout, dq)
    rc = lib.sigmoid_attn_mqa_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                                  dk.data_ptr(), dv.data_ptr(), B, H, Hkv, N, d, _dtype_code(q), float(bias),
                                  int(bool(causal)), _slopes_ptr(alibi_slopes, H), _st(q), _st(k), _st(v),
                                  _st(dout), _st(dq), _st(dk), _st(dv), _stream())
    _raise(rc, "sigmoid_attn_mqa_bwd")
    return dq, dk, dv


def sigmoid_attn_mqa_bwd_workspace_bytes(B, H, Hkv, N, d, dtype=torch.bfloat16, causal=False):
    """Bytes of workspace sigmoid_attn_mqa_bwd_split wants for this problem (0: it would not split)."""
    code = SATTN_BF16 if dtype == torch.bfloat16 else SATTN_F32
    return int(load_library().sigmoid_attn_mqa_bwd_workspace_bytes(B, H, Hkv, N, d, code, int(bool(causal))))


def sigmoid_attn_mqa_bwd_split(q, k, v, dout, dq, dk, dv, bias, causal=False, alibi_slopes=None, workspace=None):
    """sigmoid_attn_mqa_bwd with a group's query heads split over several workgroups where K/V heads are
    few (fp32 partial sums in `workspace`, allocated here when not given)."""
    lib = load_library()
    B, H, Hkv, N, d = _check_mqa(q, (k, v, dk, dv), dout, dq)
    need = sigmoid_attn_mqa_bwd_workspace_bytes(B, H, Hkv, N, d, q.dtype, causal)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    wp = _vp(workspace.data_ptr()) if workspace is not None else None
    wb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib.sigmoid_attn_mqa_bwd_split(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                                        dk.data_ptr(), dv.data_ptr(), B, H, Hkv, N, d, _dtype_code(q), float(bias),
                                        int(bool(causal)), _slopes_ptr(alibi_slopes, H), _st(q), _st(k), _st(v),
                                        _st(dout), _st(dq), _st(dk), _st(dv), wp, wb, _stream())
    _raise(rc, "sigmoid_attn_mqa_bwd_split")
    return dq, dk, dv


_NORM_KINDS = {"layer": 0, "rms": 1}


def _check_stats(stats, B, N):
    if not stats.is_cuda or stats.dtype != torch.float32 or tuple(stats.shape) != (B, N, 2) or not stats.is_contiguous():
        raise SattnError(f"stats must be a contiguous CUDA float32 tensor of shape {(B, N, 2)}")


def sattn_headconcat_norm_fwd(x, y, stats, kind="layer", eps=1e-5):
    """LayerNorm / RMSNorm of a [B,H,N,d] bf16 tensor over each token's H*d features; fills stats [B,N,2]."""
    lib = load_library()
    _check(x, y)
    B, H, N, d = x.shape
    _check_stats(stats, B, N)
    rc = lib.sattn_headconcat_norm_fwd(x.data_ptr(), y.data_ptr(), _vp(stats.data_ptr()), B, H, N, d, _dtype_code(x),
                                       _NORM_KINDS[kind], float(eps), _st(x), _st(y), _stream())
    _raise(rc, "sattn_headconcat_norm_fwd")
    return y, stats


def sattn_headconcat_norm_bwd(x, dy, stats, dx, kind="layer"):
    """Gradient of sattn_headconcat_norm_fwd with respect to x, from x, dy and the forward statistics."""
    lib = load_library()
    _check(x, dy, dx)
    B, H, N, d = x.shape
    _check_stats(stats, B, N)
    rc = lib.sattn_headconcat_norm_bwd(x.data_ptr(), dy.data_ptr(), _vp(stats.data_ptr()), dx.data_ptr(), B, H, N, d,
                                       _dtype_code(x), _NORM_KINDS[kind], _st(x), _st(dy), _st(dx), _stream())
    _raise(rc, "sattn_headconcat_norm_bwd")
    return dx


def _check_cross(q, kv, *qlike):
    _check(q, *qlike)
    _check(*kv)
    B, H, Nq, d = q.shape
    Bk, Hk, Nk, dk = kv[0].shape
    if (Bk, Hk, dk) != (B, H, d) or Nk <= 0:
        raise SattnError(f"K/V shape {tuple(kv[0].shape)} does not match Q {tuple(q.shape)}")
    return B, H, Nq, Nk, d


def sigmoid_attn_cross_fwd(q, k, v, o, bias):
    """Plain sigmoid attention with Nq queries and Nk keys: q, o [B,H,Nq,d]; k, v [B,H,Nk,d]."""
    lib = load_library()
    B, H, Nq, Nk, d = _check_cross(q, (k, v), o)
    rc = lib.sigmoid_attn_cross_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), B, H, Nq, Nk, d,
                                    _dtype_code(q), float(bias), _st(q), _st(k), _st(v), _st(o), _stream())
    _raise(rc, "sigmoid_attn_cross_fwd")
    return o


def sigmoid_attn_cross_bwd(q, k, v, dout, dq, dk, dv, bias):
    """Backward of sigmoid_attn_cross_fwd: dq [B,H,Nq,d]; dk, dv [B,H,Nk,d]."""
    lib = load_library()
    B, H, Nq, Nk, d = _check_cross(q, (k, v, dk, dv), dout, dq)
    rc = lib.sigmoid_attn_cross_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                                    dk.data_ptr(), dv.data_ptr(), B, H, Nq, Nk, d, _dtype_code(q), float(bias),
                                    _st(q), _st(k), _st(v), _st(dout), _st(dq), _st(dk), _st(dv), _stream())
    _raise(rc, "sigmoid_attn_cross_bwd")
    return dq, dk, dv


def sigmoid_attn_cross_aligned_fwd(q, k, v, o, bias, causal=False, alibi_slopes=None):
    """Sigmoid attention of Nq queries placed at the end of an Nk-key sequence (query i at position
    i + Nk - Nq), with the causal mask and ALiBi of that placement: q, o [B,H,Nq,d]; k, v [B,H,Nk,d]."""
    lib = load_library()
    B, H, Nq, Nk, d = _check_cross(q, (k, v), o)
    rc = lib.sigmoid_attn_cross_aligned_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), B, H, Nq, Nk, d,
                                            _dtype_code(q), float(bias), int(bool(causal)), _slopes_ptr(alibi_slopes, H),
                                            _st(q), _st(k), _st(v), _st(o), _stream())
    _raise(rc, "sigmoid_attn_cross_aligned_fwd")
    return o


def sigmoid_attn_cross_aligned_bwd(q, k, v, dout, dq, dk, dv, bias, causal=False, alibi_slopes=None):
    """Backward of sigmoid_attn_cross_aligned_fwd: dq [B,H,Nq,d]; dk, dv [B,H,Nk,d]."""
    lib = load_library()
    B, H, Nq, Nk, d = _check_cross(q, (k, v, dk, dv), dout, dq)
    rc = lib.sigmoid_attn_cross_aligned_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                                            dk.data_ptr(), dv.data_ptr(), B, H, Nq, Nk, d, _dtype_code(q), float(bias),
                                            int(bool(causal)), _slopes_ptr(alibi_slopes, H), _st(q), _st(k), _st(v),
                                            _st(dout), _st(dq), _st(dk), _st(dv), _stream())
    _raise(rc, "sigmoid_attn_cross_aligned_bwd")
    return dq, dk, dv


def sattn_fwd_waves(B, H, N, d, causal=False):
    """Waves (32 query rows each) per workgroup the bf16 forward kernels use for this problem."""
    rc = load_library().sattn_fwd_waves(B, H, N, d, int(bool(causal)))
    if rc < 0:
        _raise(rc, "sattn_fwd_waves")
    return rc


def sattn_fwd_v_slots(B, H, N, d, causal=False):
    """Depth of the V ring (2 or 3 tiles) the bf16 forward kernels use for this problem."""
    rc = load_library().sattn_fwd_v_slots(B, H, N, d, int(bool(causal)))
    if rc < 0:
        _raise(rc, "sattn_fwd_v_slots")
    return rc


def sattn_set_fwd_v_slots(v_slots):
    """Force a V ring of 2 or 3 tiles where that shape exists (4 waves, d = 128); 0 = automatic."""
    _raise(load_library().sattn_set_fwd_v_slots(int(v_slots)), "sattn_set_fwd_v_slots")


def sattn_bwd_merged(B, H, N, causal=False):
    """True if sigmoid_attn_bwd runs both passes of this bf16 self-attention problem as one grid."""
    rc = load_library().sattn_bwd_merged(int(B), int(H), int(N), int(bool(causal)))
    _raise(min(rc, 0), "sattn_bwd_merged")
    return bool(rc)


def sattn_set_bwd_merged(mode):
    """1 forces, 2 forbids the one-grid form of the sigmoid backward (3: forbids it and the pairing of
    causal blocks as well); 0 restores the automatic choice."""
    _raise(load_library().sattn_set_bwd_merged(int(mode)), "sattn_set_bwd_merged")


def sattn_set_fwd_waves(waves):
    """Force the forward tile shape for measurements (4, 8, 64, 65, 66; 32 = automatic among the 32-row
    shapes); 0 restores the automatic choice."""
    _raise(load_library().sattn_set_fwd_waves(int(waves)), "sattn_set_fwd_waves")


def sattn_mfma_bf16_probe(blocks, iters, sink):
    """Launch the register-resident MFMA loop on torch's current stream; returns its flop count."""
    assert sink.is_cuda and sink.dtype == torch.float32 and sink.numel() >= blocks * 256
    rc = load_library().sattn_mfma_bf16_probe(int(blocks), int(iters), _vp(sink.data_ptr()), _stream())
    _raise(rc, "sattn_mfma_bf16_probe")
    return blocks * 4 * iters * 8 * 32768


def sattn_device_info():
    """(compute units, nominal peak engine clock in kHz) of the current device."""
    cus, khz = ctypes.c_int(0), ctypes.c_int(0)
    _raise(load_library().sattn_device_info(ctypes.byref(cus), ctypes.byref(khz)), "sattn_device_info")
    return cus.value, khz.value


def sattn_version():
    return int(load_library().sattn_version())


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return SATTN_BF16
    if t.dtype == torch.float32:
        return SATTN_F32
    raise SattnError(f"unsupported dtype {t.dtype}")


def _check(*ts):
    t0 = ts[0]
    for t in ts:
        if not t.is_cuda:
            raise SattnError("tensors must live on the GPU")
        if t.dim() != 4 or t.shape != t0.shape or t.dtype != t0.dtype:
            raise SattnError("tensors must share one [B,H,N,d] shape and dtype")
        if t.stride(3) != 1:
            raise SattnError("the last dimension must be contiguous")


def _st(t):
    return ctypes.byref(_Strides(t.stride(0), t.stride(1), t.stride(2)))


def _stream():
    return _vp(torch.cuda.current_stream().cuda_stream)


def _slopes_ptr(alibi_slopes, H):
    if alibi_slopes is None:
        return None
    if alibi_slopes.dtype != torch.float32 or not alibi_slopes.is_cuda or alibi_slopes.numel() != H \
            or not alibi_slopes.is_contiguous():
        raise SattnError("alibi_slopes must be a contiguous CUDA float32 tensor of H elements")
    return _vp(alibi_slopes.data_ptr())


def _raise(rc, what):
    if rc != 0:
        raise SattnError(f"{what} failed: {sattn_strerror(rc)} ({rc})")


def sigmoid_attn_fwd(q, k, v, o, bias, causal=False, alibi_slopes=None, _entry="sigmoid_attn_fwd"):
    """O = sigmoid(Q K^T/sqrt(d) + bias [- slope|i-j|], causal mask) V, written into `o`."""
    lib = load_library()
    _check(q, k, v, o)
    B, H, N, d = q.shape
    rc = getattr(lib, _entry)(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), B, H, N, d, _dtype_code(q),
                              float(bias), int(bool(causal)), _slopes_ptr(alibi_slopes, H),
                              _st(q), _st(k), _st(v), _st(o), _stream())
    _raise(rc, _entry)
    return o


def sigmoid_attn_fwd_compiler_scheduled(q, k, v, o, bias, causal=False, alibi_slopes=None):
    """Same result as sigmoid_attn_fwd from the compiler-scheduled pipeline step (comparison aid)."""
    return sigmoid_attn_fwd(q, k, v, o, bias, causal, alibi_slopes, _entry="sigmoid_attn_fwd_compiler_scheduled")


def sigmoid_attn_bwd_workspace_bytes(B, H, N, d, dtype=torch.bfloat16):
    code = SATTN_BF16 if dtype == torch.bfloat16 else SATTN_F32
    return int(load_library().sigmoid_attn_bwd_workspace_bytes(B, H, N, d, code))


def sigmoid_attn_bwd(q, k, v, dout, dq, dk, dv, bias, causal=False, alibi_slopes=None, workspace=None,
                     _entry="sigmoid_attn_bwd"):
    """dQ, dK, dV of sigmoid attention from Q, K, V, dO (P is recomputed), written in place."""
    lib = load_library()
    _check(q, k, v, dout, dq, dk, dv)
    B, H, N, d = q.shape
    need = sigmoid_attn_bwd_workspace_bytes(B, H, N, d, q.dtype)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    wp = _vp(workspace.data_ptr()) if workspace is not None else None
    wb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = getattr(lib, _entry)(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                              dk.data_ptr(), dv.data_ptr(), B, H, N, d, _dtype_code(q), float(bias),
                              int(bool(causal)), _slopes_ptr(alibi_slopes, H), _st(q), _st(k), _st(v), _st(dout),
                              _st(dq), _st(dk), _st(dv), wp, wb, _stream())
    _raise(rc, _entry)
    return dq, dk, dv


def sigmoid_attn_bwd_bias_grad(q, k, v, dout, dq, dk, dv, db_rows, bias, causal=False, alibi_slopes=None, db=None):
    """sigmoid_attn_bwd plus db_rows[b,h,i] = sum_j dS_ij (fp32 [B,H,N]) and, if given, db[b,h] = sum_i db_rows."""
    lib = load_library()
    _check(q, k, v, dout, dq, dk, dv)
    B, H, N, d = q.shape
    for t, shape, what in ((db_rows, (B, H, N), "db_rows"), (db, (B, H), "db")):
        if t is None and what == "db":
            continue
        if t is None or not t.is_cuda or t.dtype != torch.float32 or tuple(t.shape) != shape or not t.is_contiguous():
            raise SattnError(f"{what} must be a contiguous CUDA float32 tensor of shape {shape}")
    rc = lib.sigmoid_attn_bwd_bias_grad(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(), dq.data_ptr(),
                                        dk.data_ptr(), dv.data_ptr(), _vp(db_rows.data_ptr()),
                                        _vp(db.data_ptr()) if db is not None else None, B, H, N, d, _dtype_code(q),
                                        float(bias), int(bool(causal)), _slopes_ptr(alibi_slopes, H), _st(q), _st(k),
                                        _st(v), _st(dout), _st(dq), _st(dk), _st(dv), _stream())
    _raise(rc, "sigmoid_attn_bwd_bias_grad")
    return dq, dk, dv, db_rows, db


def sigmoid_attn_bwd_compiler_scheduled(q, k, v, dout, dq, dk, dv, bias, causal=False, alibi_slopes=None):
    """Same result as sigmoid_attn_bwd from the compiler-scheduled pipeline step (comparison aid)."""
    return sigmoid_attn_bwd(q, k, v, dout, dq, dk, dv, bias, causal, alibi_slopes,
                            _entry="sigmoid_attn_bwd_compiler_scheduled")


def sigmoid_attn_bwd_dkdv(q, k, v, dout, dk, dv, bias, causal=False, alibi_slopes=None):
    """Key-block-stationary half of the backward: dK and dV only."""
    lib = load_library()
    _check(q, k, v, dout, dk, dv)
    B, H, N, d = q.shape
    rc = lib.sigmoid_attn_bwd_dkdv(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(), dk.data_ptr(),
                                   dv.data_ptr(), B, H, N, d, _dtype_code(q), float(bias), int(bool(causal)),
                                   _slopes_ptr(alibi_slopes, H), _st(q), _st(k), _st(v), _st(dout), _st(dk),
                                   _st(dv), _stream())
    _raise(rc, "sigmoid_attn_bwd_dkdv")
    return dk, dv


def sigmoid_attn_bwd_dq(q, k, v, dout, dq, bias, causal=False, alibi_slopes=None):
    """Query-block-stationary half of the backward: dQ only."""
    lib = load_library()
    _check(q, k, v, dout, dq)
    B, H, N, d = q.shape
    rc = lib.sigmoid_attn_bwd_dq(q.data_ptr(), k.data_ptr(), v.data_ptr(), dout.data_ptr(), dq.data_ptr(), B, H, N,
                                 d, _dtype_code(q), float(bias), int(bool(causal)), _slopes_ptr(alibi_slopes, H),
                                 _st(q), _st(k), _st(v), _st(dout), _st(dq), _stream())
    _raise(rc, "sigmoid_attn_bwd_dq")
    return dq


def softmax_attn_fwd(q, k, v, o, lse, causal=False, alibi_slopes=None, _entry="softmax_attn_fwd"):
    """Softmax flash attention forward (comparison kernel); lse is [B,H,N] float32."""
    lib = load_library()
    _check(q, k, v, o)
    B, H, N, d = q.shape
    if lse.dtype != torch.float32 or not lse.is_cuda or tuple(lse.shape) != (B, H, N) or not lse.is_contiguous():
        raise SattnError("lse must be a contiguous CUDA float32 tensor [B,H,N]")
    rc = getattr(lib, _entry)(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, N, d,
                              _dtype_code(q), int(bool(causal)), _slopes_ptr(alibi_slopes, H),
                              _st(q), _st(k), _st(v), _st(o), _stream())
    _raise(rc, _entry)
    return o, lse


def softmax_attn_fwd_compiler_scheduled(q, k, v, o, lse, causal=False, alibi_slopes=None):
    """softmax_attn_fwd with every step in the compiler-scheduled form (comparison aid)."""
    return softmax_attn_fwd(q, k, v, o, lse, causal, alibi_slopes, _entry="softmax_attn_fwd_compiler_scheduled")


def softmax_attn_bwd_workspace_bytes(B, H, N, d, dtype=torch.bfloat16):
    code = SATTN_BF16 if dtype == torch.bfloat16 else SATTN_F32
    return int(load_library().softmax_attn_bwd_workspace_bytes(B, H, N, d, code))


def softmax_attn_bwd(q, k, v, o, lse, dout, dq, dk, dv, causal=False, alibi_slopes=None, workspace=None):
    lib = load_library()
    _check(q, k, v, o, dout, dq, dk, dv)
    B, H, N, d = q.shape
    need = softmax_attn_bwd_workspace_bytes(B, H, N, d, q.dtype)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    wp = _vp(workspace.data_ptr()) if workspace is not None else None
    wb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib.softmax_attn_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                              dout.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), B, H, N, d,
                              _dtype_code(q), int(bool(causal)), _slopes_ptr(alibi_slopes, H),
                              _st(q), _st(k), _st(v), _st(o), _st(dout), _st(dq), _st(dk), _st(dv), wp, wb, _stream())
    _raise(rc, "softmax_attn_bwd")
    return dq, dk, dv


def softmax_attn_bwd_compiler_scheduled(q, k, v, o, lse, dout, dq, dk, dv, causal=False, alibi_slopes=None, workspace=None):
    """softmax_attn_bwd with both passes in the compiler-scheduled form (measurement aid)."""
    lib = load_library()
    _check(q, k, v, o, dout, dq, dk, dv)
    B, H, N, d = q.shape
    need = softmax_attn_bwd_workspace_bytes(B, H, N, d, q.dtype)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    wp = _vp(workspace.data_ptr()) if workspace is not None else None
    wb = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = lib.softmax_attn_bwd_compiler_scheduled(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                                 dout.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), B, H, N, d,
                                                 _dtype_code(q), int(bool(causal)), _slopes_ptr(alibi_slopes, H),
                                                 _st(q), _st(k), _st(v), _st(o), _st(dout), _st(dq), _st(dk), _st(dv),
                                                 wp, wb, _stream())
    _raise(rc, "softmax_attn_bwd_compiler_scheduled")
    return dq, dk, dv


def softmax_attn_bwd_noalloc_max_rows():
    return int(load_library().softmax_attn_bwd_noalloc_max_rows())


def softmax_attn_bwd_noalloc(q, k, v, o, lse, dout, dq, dk, dv, causal=False, alibi_slopes=None):
    """softmax_attn_bwd on the library's own fixed scratch: no workspace, no allocation."""
    lib = load_library()
    _check(q, k, v, o, dout, dq, dk, dv)
    B, H, N, d = q.shape
    rc = lib.softmax_attn_bwd_noalloc(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(),
                                      dout.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), B, H, N, d,
                                      _dtype_code(q), int(bool(causal)), _slopes_ptr(alibi_slopes, H),
                                      _st(q), _st(k), _st(v), _st(o), _st(dout), _st(dq), _st(dk), _st(dv), _stream())
    _raise(rc, "softmax_attn_bwd_noalloc")
    return dq, dk, dv


def sattn_set_clock_probe(buf):
    """buf: a zeroed CUDA int64 tensor of 8 * capacity elements (eight values per workgroup), or
    None to switch the probe off."""
    lib = load_library()
    if buf is None:
        _raise(lib.sattn_set_clock_probe(None, 0), "sattn_set_clock_probe")
        return
    if not buf.is_cuda or buf.dtype != torch.int64 or not buf.is_contiguous():
        raise SattnError("the clock buffer must be a contiguous CUDA int64 tensor")
    _raise(lib.sattn_set_clock_probe(buf.data_ptr(), buf.numel() // 8), "sattn_set_clock_probe")


def sattn_wall_clock_khz():
    rc = load_library().sattn_wall_clock_khz()
    if rc <= 0:
        _raise(rc, "sattn_wall_clock_khz")
    return rc
