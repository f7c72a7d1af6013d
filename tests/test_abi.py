"""Host-side checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2409_04431_amd as sa
from paper_2409_04431_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in sorted(os.listdir(os.path.join(ROOT, "include"))) if n.endswith(".h")]


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sa.library_path()):
        from paper_2409_04431_amd.build import build_library
        build_library()
    return sa.load_library()


def _declared_functions():
    text = "\n".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:sigmoid|softmax)_attn_\w+|sattn_\w+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = _declared_functions()
    assert {"sigmoid_attn_fwd", "sigmoid_attn_bwd", "softmax_attn_fwd", "softmax_attn_bwd", "sattn_strerror",
            "sattn_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/*.h but not exported"


def test_headers_are_plain_c(tmp_path):
    """The boundary is a C ABI: both headers compile as C99 and as C++11 on their own."""
    import shutil
    import subprocess
    for cc, std, ext in (("gcc", "-std=c99", "c"), ("g++", "-std=c++11", "cpp")):
        if shutil.which(cc) is None:
            pytest.skip(f"{cc} not installed")
        src = tmp_path / f"hdr.{ext}"
        src.write_text("".join(f'#include "{h}"\n' for h in HEADERS) + "int main(void) { return 0; }\n")
        res = subprocess.run([cc, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-c", str(src), "-o", str(tmp_path / "hdr.o")],
                             capture_output=True, text=True)
        assert res.returncode == 0, res.stderr


def test_version_and_error_strings(lib):
    assert sa.sattn_version() >= 100
    for code in range(0, -8, -1):
        assert sa.sattn_strerror(code) and "unknown" not in sa.sattn_strerror(code)
    assert "unknown" in sa.sattn_strerror(-99)


def _fwd(lib, q=0x1000, k=0x2000, v=0x3000, o=0x4000, B=1, H=1, N=16, d=64, dtype=0, strides=None):
    sp = ctypes.byref(binding._Strides(*strides)) if strides else None
    return lib.sigmoid_attn_fwd(q, k, v, o, B, H, N, d, dtype, 0.0, 0, None, sp, None, None, None, None)


def test_bad_arguments_are_rejected_without_launch(lib):
    # the pointers are fake: every call must fail validation before touching the device
    assert _fwd(lib, q=None) == -1                      # SATTN_ERR_NULL
    assert _fwd(lib, o=None) == -1
    assert _fwd(lib, N=0) == -2                         # SATTN_ERR_SHAPE
    assert _fwd(lib, B=-1) == -2
    assert _fwd(lib, d=96) == -3                        # SATTN_ERR_UNSUPPORTED
    assert _fwd(lib, dtype=7) == -3
    assert _fwd(lib, q=0x1004) == -4                    # SATTN_ERR_ALIGN (pointer)
    assert _fwd(lib, strides=(1024, 1024, 60)) == -4    # seq stride < d
    assert _fwd(lib, strides=(1027, 1024, 64)) == -4    # rows not 16-byte aligned
    assert _fwd(lib, N=(1 << 24) + 1) == -2
    # one (batch, head) slice must span < 4 GiB: its rows are addressed with 32-bit byte offsets
    assert _fwd(lib, N=1 << 20, d=64, strides=(1 << 40, 1 << 40, 4096)) == -2
    assert lib.sattn_mfma_bf16_probe(0, 10, ctypes.c_void_p(0x1000), None) == -2
    assert lib.sattn_mfma_bf16_probe(4, 10, None, None) == -1


def test_backward_rejects_bad_arguments(lib):
    args = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, None]      # dv NULL
    rc = lib.sigmoid_attn_bwd(*args, 1, 1, 16, 64, 0, 0.0, 0, None, *([None] * 7), None, 0, None)
    assert rc == -1
    args[6] = 0x7000
    rc = lib.sigmoid_attn_bwd(*args, 1, 1, 16, 100, 0, 0.0, 0, None, *([None] * 7), None, 0, None)
    assert rc == -3
    assert sa.sigmoid_attn_bwd_workspace_bytes(8, 16, 4096, 128) == 0


def test_varlen_entry_points_reject_bad_arguments(lib):
    ptrs = [0x1000, 0x2000, 0x3000, 0x4000]
    tail = [2, 4, 512, 128, 0, 0.0, 1, None, None, None, None, None, None]       # B H max_seqlen d dtype bias causal ...
    assert lib.sigmoid_attn_varlen_fwd(*ptrs, None, None, *tail) == -1          # cu_seqlens NULL
    assert lib.sigmoid_attn_varlen_fwd(*ptrs, 0x5000, None, 2, 4, 512, 128, 2, 0.0, 1, None, None, None, None,
                                       None, None) == -3                        # no such dtype
    assert lib.sigmoid_attn_varlen_fwd(*ptrs, 0x5000, None, 2, 4, 512, 96, 0, 0.0, 1, None, None, None, None,
                                       None, None) == -3                        # head dimension
    assert lib.sigmoid_attn_varlen_fwd(*ptrs, 0x5000, None, 2, 4, 0, 128, 0, 0.0, 1, None, None, None, None,
                                       None, None) == -2                        # max_seqlen
    bptrs = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000]
    assert lib.sigmoid_attn_varlen_bwd(*bptrs, None, None, 2, 4, 512, 128, 0, 0.0, 1, None, *([None] * 7), None) == -1
    assert lib.sigmoid_attn_varlen_bwd(*bptrs, 0x8000, None, 2, 4, 512, 128, 2, 0.0, 1, None, *([None] * 7), None) == -3


def test_bias_gradient_entry_point_rejects_bad_arguments(lib):
    ptrs = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000]
    tail = [1, 1, 16, 64, 0, 0.0, 0, None, *([None] * 7), None]
    assert lib.sigmoid_attn_bwd_bias_grad(*ptrs, None, None, *tail) == -1            # db_rows is required
    assert lib.sigmoid_attn_bwd_bias_grad(*ptrs, 0x8002, None, *tail) == -4          # fp32 alignment
    assert lib.sigmoid_attn_bwd_bias_grad(*ptrs, 0x8000, 0x9001, *tail) == -4
    tail[3] = 100
    assert lib.sigmoid_attn_bwd_bias_grad(*ptrs, 0x8000, None, *tail) == -3          # head dimension


def test_varlen_bias_gradient_entry_point_rejects_bad_arguments(lib):
    ptrs = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000]
    tail = lambda total=900, d=128, dtype=0: [2, 4, 512, total, d, dtype, 0.0, 1, None, *([None] * 7), None]
    f = lib.sigmoid_attn_varlen_bwd_bias_grad
    assert f(*ptrs, None, None, 0x9000, None, *tail()) == -1            # db_rows is required
    assert f(*ptrs, 0x8000, None, None, None, *tail()) == -1            # cu_seqlens is required
    assert f(*ptrs, 0x8002, None, 0x9000, None, *tail()) == -4          # fp32 alignment
    assert f(*ptrs, 0x8000, None, 0x9000, None, *tail(total=0)) == -2
    assert f(*ptrs, 0x8000, None, 0x9000, None, *tail(d=96)) == -3
    assert f(*ptrs, 0x8000, None, 0x9000, None, *tail(dtype=2)) == -3   # no such dtype (bf16 and fp32 exist)


def test_backward_one_grid_choice(lib):
    # small or uneven (causal) grids run both passes of the backward in one launch
    assert sa.sattn_bwd_merged(4, 12, 1024) and sa.sattn_bwd_merged(1, 16, 2048, True)
    assert not sa.sattn_bwd_merged(8, 16, 4096, True) and not sa.sattn_bwd_merged(8, 16, 1024)
    assert not sa.sattn_bwd_merged(2, 16, 2048, True)
    assert lib.sattn_bwd_merged(0, 1, 16, 0) == -2 and lib.sattn_set_bwd_merged(4) == -3
    try:
        sa.sattn_set_bwd_merged(1)
        assert sa.sattn_bwd_merged(8, 16, 4096, True)
        for mode in (2, 3):                      # 3 also keeps one block per workgroup
            sa.sattn_set_bwd_merged(mode)
            assert not sa.sattn_bwd_merged(4, 12, 1024)
    finally:
        sa.sattn_set_bwd_merged(0)
    assert sa.sattn_bwd_merged(4, 12, 1024)


def test_forward_shape_choice(lib):
    # d = 64 always takes 4-wave workgroups; d = 128 while the grid is small (one per compute unit,
    # three-slot V ring) or the key loop short (two per compute unit, two-slot V ring)
    assert sa.sattn_fwd_waves(32, 12, 4096, 64) == 4 and sa.sattn_fwd_v_slots(32, 12, 4096, 64) == 3
    assert (sa.sattn_fwd_waves(8, 16, 4096, 128, True), sa.sattn_fwd_v_slots(8, 16, 4096, 128, True)) == (64, 3)
    # 64-row waves from 2048 tokens with the causal mask, 1536 without, given a 256-row workgroup per compute unit
    assert sa.sattn_fwd_waves(8, 16, 2048, 128, True) == 64 and sa.sattn_fwd_waves(2, 16, 4096, 128, True) == 64
    assert (sa.sattn_fwd_waves(8, 16, 1536, 128, True), sa.sattn_fwd_v_slots(8, 16, 1536, 128, True)) == (4, 2)
    assert (sa.sattn_fwd_waves(1, 16, 2048, 128, True), sa.sattn_fwd_v_slots(1, 16, 2048, 128, True)) == (4, 3)
    assert sa.sattn_fwd_waves(8, 16, 1536, 128) == 64 and sa.sattn_fwd_waves(8, 16, 1024, 128) == 4
    # long key loops with a workgroup for every compute unit: four waves of 64 query rows
    assert (sa.sattn_fwd_waves(1, 32, 16384, 128, True), sa.sattn_fwd_v_slots(1, 32, 16384, 128, True)) == (64, 3)
    assert sa.sattn_fwd_waves(2, 16, 8192, 128) == 64 and sa.sattn_fwd_waves(8, 16, 4096, 128) == 64
    assert sa.sattn_fwd_waves(1, 4, 8192, 128) == 4 and sa.sattn_fwd_waves(1, 6, 8192, 128) == 8   # too few workgroups for 256-row blocks
    assert sa.sattn_fwd_waves(2, 8, 65536, 64) == 4          # d = 64 has no 64-row shape
    assert (sa.sattn_fwd_waves(1, 2, 512, 128), sa.sattn_fwd_v_slots(1, 2, 512, 128)) == (4, 3)
    assert lib.sattn_fwd_waves(1, 1, 16, 100, 0) == -3 and lib.sattn_fwd_v_slots(1, 1, 16, 100, 0) == -3
    assert lib.sattn_fwd_waves(0, 1, 16, 64, 0) == -2
    assert lib.sattn_set_fwd_waves(3) == -3 and lib.sattn_set_fwd_v_slots(4) == -3
    try:
        sa.sattn_set_fwd_waves(8)
        assert sa.sattn_fwd_waves(1, 2, 512, 128) == 8 and sa.sattn_fwd_waves(1, 2, 512, 64) == 8
        assert sa.sattn_fwd_v_slots(8, 16, 4096, 128, True) == 3      # no two-slot ring with 8 waves
        sa.sattn_set_fwd_waves(32)   # the automatic choice held to the 32-row shapes
        assert (sa.sattn_fwd_waves(8, 16, 4096, 128, True), sa.sattn_fwd_v_slots(8, 16, 4096, 128, True)) == (8, 3)
        assert (sa.sattn_fwd_waves(8, 16, 1024, 128, True), sa.sattn_fwd_v_slots(8, 16, 1024, 128, True)) == (4, 2)
        assert sa.sattn_fwd_waves(1, 6, 8192, 128) == 8 and sa.sattn_fwd_waves(32, 12, 4096, 64) == 4
        sa.sattn_set_fwd_waves(64)
        assert sa.sattn_fwd_waves(1, 2, 512, 128) == 64 and sa.sattn_fwd_waves(1, 2, 512, 64) == 4
        sa.sattn_set_fwd_waves(4)
        sa.sattn_set_fwd_v_slots(2)
        assert sa.sattn_fwd_v_slots(1, 32, 16384, 128, True) == 2 and sa.sattn_fwd_v_slots(1, 2, 512, 64) == 3
    finally:
        sa.sattn_set_fwd_waves(0)
        sa.sattn_set_fwd_v_slots(0)
    assert sa.sattn_fwd_waves(1, 2, 512, 64) == 4


def test_shared_kv_head_entry_points_reject_bad_arguments(lib):
    ptrs = [0x1000, 0x2000, 0x3000, 0x4000]
    args = lambda H, Hkv, dtype=0: [*ptrs, 1, H, Hkv, 64, 64, dtype, 0.0, 0, None, None, None, None, None, None]
    assert lib.sigmoid_attn_mqa_fwd(*args(6, 4)) == -2          # Hkv must divide H
    assert lib.sigmoid_attn_mqa_fwd(*args(6, 0)) == -2
    assert lib.sigmoid_attn_mqa_fwd(*args(6, 2, 2)) == -3       # no such dtype (bf16 and fp32 exist)
    bptrs = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000]
    bargs = lambda H, Hkv, dtype=0: [*bptrs, 1, H, Hkv, 64, 64, dtype, 0.0, 0, None, *([None] * 7), None]
    assert lib.sigmoid_attn_mqa_bwd(*bargs(8, 3)) == -2
    assert lib.sigmoid_attn_mqa_bwd(*bargs(8, 2, 2)) == -3
    bptrs[5] = None
    assert lib.sigmoid_attn_mqa_bwd(*bargs(8, 2)) == -1         # dk NULL


def test_norm_entry_points_reject_bad_arguments(lib):
    fwd = lambda H=16, d=128, dtype=0, kind=0, stats=0x3000, eps=1e-5: lib.sattn_headconcat_norm_fwd(
        0x1000, 0x2000, stats, 1, H, 32, d, dtype, kind, eps, None, None, None)
    assert fwd(stats=None) == -1
    assert fwd(stats=0x3004) == -4
    assert fwd(dtype=1) == -3 and fwd(kind=2) == -3
    assert fwd(H=128) == -2                       # H*d beyond what one wave holds
    assert fwd(eps=-1.0) == -2
    assert lib.sattn_headconcat_norm_bwd(0x1000, None, 0x3000, 0x4000, 1, 16, 32, 128, 0, 0, None, None, None, None) == -1


def test_cross_attention_entry_points_reject_bad_arguments(lib):
    ptrs = [0x1000, 0x2000, 0x3000, 0x4000]
    f = lambda Nq=64, Nk=96, d=64, dtype=0: lib.sigmoid_attn_cross_fwd(*ptrs, 1, 2, Nq, Nk, d, dtype, 0.0,
                                                                       None, None, None, None, None)
    assert f(Nk=0) == -2 and f(Nq=0) == -2
    assert f(dtype=2) == -3                         # no such dtype (bf16 and fp32 exist)
    assert f(d=96) == -3
    bptrs = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, None, 0x7000]
    assert lib.sigmoid_attn_cross_bwd(*bptrs, 1, 2, 64, 96, 64, 0, 0.0, *([None] * 7), None) == -1


def test_end_aligned_cross_attention_entry_points_reject_bad_arguments(lib):
    ptrs = [0x1000, 0x2000, 0x3000, 0x4000]
    f = lambda Nq=64, Nk=96, d=64, dtype=0, causal=1, q=0x1000: lib.sigmoid_attn_cross_aligned_fwd(
        q, *ptrs[1:], 1, 2, Nq, Nk, d, dtype, 0.0, causal, None, None, None, None, None, None)
    assert f(Nk=0) == -2 and f(Nq=0) == -2
    assert f(dtype=2) == -3 and f(d=96) == -3
    assert f(Nq=64, Nk=100) == -3                   # bf16 + causal: the offset must be a multiple of 32
    assert f(Nq=100, Nk=64) == -3
    assert f(q=None) == -1
    bptrs = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, None, 0x7000]
    g = lambda Nq, Nk, causal: lib.sigmoid_attn_cross_aligned_bwd(*bptrs, 1, 2, Nq, Nk, 64, 0, 0.0, causal, None,
                                                                  *([None] * 7), None)
    assert g(64, 96, 1) == -1                       # dk missing
    assert g(64, 100, 1) == -3


def test_split_group_backward_workspace_size_and_rejections(lib):
    f = lambda *a: sa.sigmoid_attn_mqa_bwd_workspace_bytes(*a)
    import torch
    # (the library counts 256 compute units where it finds no device, as here)
    # one K/V head, 8 x 32 key blocks: 256 workgroups, two per compute unit wanted under the mask
    assert f(8, 16, 1, 4096, 128, torch.bfloat16, True) == 2 * 2 * 8 * 1 * 4096 * 128 * 4
    assert f(8, 16, 1, 4096, 128, torch.bfloat16, False) == 0          # one per compute unit is enough without it
    assert f(1, 16, 1, 4096, 128, torch.bfloat16, True) == 2 * 16 * 4096 * 128 * 4   # 32 blocks: split 16 ways
    assert f(1, 6, 2, 520, 128, torch.bfloat16, True) == 0             # groups of three
    assert f(8, 16, 16, 4096, 128, torch.bfloat16, True) == 0 and f(8, 16, 3, 4096, 128, torch.bfloat16, True) == 0
    assert f(8, 16, 1, 4096, 128, torch.float32, True) == 0
    ptrs = [0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 0x6000, 0x7000]
    call = lambda ws, nbytes, Hkv=1: lib.sigmoid_attn_mqa_bwd_split(*ptrs, 8, 16, Hkv, 4096, 128, 0, 0.0, 1, None,
                                                                    *([None] * 7), ws, nbytes, None)
    assert call(None, 0) == -5                                         # SATTN_ERR_WORKSPACE
    assert call(0x10000, 1024) == -5
    assert call(0x10004, 1 << 30) == -4
    assert call(None, 0, Hkv=5) == -2


def test_binding_refuses_cpu_tensors():
    import torch
    t = torch.zeros(1, 1, 8, 64, dtype=torch.bfloat16)
    with pytest.raises(sa.SattnError):
        sa.sigmoid_attn_fwd(t, t, t, t, 0.0)
