// C ABI of the sigmoid-attention library: argument validation and kernel dispatch.
// See include/sattn.h for the contract of every entry point.
#include "../../include/sattn.h"

#include <hip/hip_runtime.h>
#include <math.h>

#include "sattn_bwd.hpp"
#include "sattn_fwd.hpp"

using namespace sattn;

namespace {

int elem_size(sattn_dtype t) { return t == SATTN_BF16 ? 2 : 4; }

// Validate one tensor and turn it into a TensorRef.  Strides are in elements.
int make_ref(const void* ptr, const sattn_strides* s, int H, int N, int d, sattn_dtype dt, TensorRef* out) {
  if (!ptr) return SATTN_ERR_NULL;
  const int64_t per16 = 16 / elem_size(dt);
  int64_t sb, sh, ss;
  if (s) {
    sb = s->batch; sh = s->head; ss = s->seq;
  } else {
    ss = d; sh = (int64_t)N * d; sb = (int64_t)H * N * d;
  }
  if (((uintptr_t)ptr & 15) != 0) return SATTN_ERR_ALIGN;
  if (sb % per16 || sh % per16 || ss % per16 || ss < d) return SATTN_ERR_ALIGN;
  out->ptr = const_cast<void*>(ptr);
  out->sb = sb; out->sh = sh; out->ss = ss;
  return SATTN_OK;
}

int check_shape(int B, int H, int N, int d, sattn_dtype dt) {
  if (dt != SATTN_BF16 && dt != SATTN_F32) return SATTN_ERR_UNSUPPORTED;
  if (d != 64 && d != 128) return SATTN_ERR_UNSUPPORTED;
  if (B <= 0 || H <= 0 || N <= 0) return SATTN_ERR_SHAPE;
  if ((int64_t)N > (1 << 24)) return SATTN_ERR_SHAPE;               // key distances are formed in fp32
  if ((int64_t)B * H * ((N + 31) / 32) > 0x7fffffffLL) return SATTN_ERR_SHAPE;  // 1-D grid of workgroups
  return SATTN_OK;
}

template <typename K, typename P>
int launch(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, const P& p) {
  if (hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return SATTN_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(kernel, grid, block, lds, st, p);
  return hipGetLastError() == hipSuccess ? SATTN_OK : SATTN_ERR_LAUNCH;
}

template <int D, int BC, int NW>
int launch_sigmoid_fwd(const FwdParams& p, int causal, bool alibi, hipStream_t st) {
  constexpr size_t lds = 4 * BC * D * 2;
  dim3 grid(p.n_qblocks * p.B * p.H), block(64 * NW);
  if (causal) {
    if (alibi) return launch(sigmoid_fwd_kernel<D, BC, NW, true, true>, grid, block, lds, st, p);
    return launch(sigmoid_fwd_kernel<D, BC, NW, true, false>, grid, block, lds, st, p);
  }
  if (alibi) return launch(sigmoid_fwd_kernel<D, BC, NW, false, true>, grid, block, lds, st, p);
  return launch(sigmoid_fwd_kernel<D, BC, NW, false, false>, grid, block, lds, st, p);
}

enum BwdPart { kBwdDkDv = 1, kBwdDq = 2 };

template <int D, int BC, int NW, bool CAUSAL, bool ALIBI>
int launch_sigmoid_bwd_t(const BwdParams& p, int parts, hipStream_t st) {
  constexpr size_t lds = 4 * BC * D * 2;
  dim3 grid(p.n_blocks * p.B * p.H), block(64 * NW);
  int rc = SATTN_OK;
  if (parts & kBwdDkDv) rc = launch(sigmoid_bwd_dkdv_kernel<D, BC, NW, CAUSAL, ALIBI>, grid, block, lds, st, p);
  if (rc == SATTN_OK && (parts & kBwdDq))
    rc = launch(sigmoid_bwd_dq_kernel<D, BC, NW, CAUSAL, ALIBI>, grid, block, lds, st, p);
  return rc;
}

template <int D, int BC, int NW>
int launch_sigmoid_bwd(BwdParams p, int causal, bool alibi, int parts, hipStream_t st) {
  p.n_blocks = (p.N + 32 * NW - 1) / (32 * NW);
  if (causal) {
    if (alibi) return launch_sigmoid_bwd_t<D, BC, NW, true, true>(p, parts, st);
    return launch_sigmoid_bwd_t<D, BC, NW, true, false>(p, parts, st);
  }
  if (alibi) return launch_sigmoid_bwd_t<D, BC, NW, false, true>(p, parts, st);
  return launch_sigmoid_bwd_t<D, BC, NW, false, false>(p, parts, st);
}

int sigmoid_bwd_impl(const void* q, const void* k, const void* v, const void* dout, void* dq, void* dk, void* dv,
                     int B, int H, int N, int d, sattn_dtype dtype, float bias, int causal,
                     const float* alibi_slopes, const sattn_strides* sq, const sattn_strides* sk,
                     const sattn_strides* sv, const sattn_strides* sdout, const sattn_strides* sdq,
                     const sattn_strides* sdk, const sattn_strides* sdv, int parts, void* stream) {
  int rc = check_shape(B, H, N, d, dtype);
  if (rc) return rc;
  BwdParams p{};
  if ((rc = make_ref(q, sq, H, N, d, dtype, &p.q))) return rc;
  if ((rc = make_ref(k, sk, H, N, d, dtype, &p.k))) return rc;
  if ((rc = make_ref(v, sv, H, N, d, dtype, &p.v))) return rc;
  if ((rc = make_ref(dout, sdout, H, N, d, dtype, &p.dout))) return rc;
  if ((parts & kBwdDq) && (rc = make_ref(dq, sdq, H, N, d, dtype, &p.dq))) return rc;
  if ((parts & kBwdDkDv) && (rc = make_ref(dk, sdk, H, N, d, dtype, &p.dk))) return rc;
  if ((parts & kBwdDkDv) && (rc = make_ref(dv, sdv, H, N, d, dtype, &p.dv))) return rc;
  p.slopes = alibi_slopes;
  p.B = B; p.H = H; p.N = N;
  p.inv_sqrt_d = 1.0f / sqrtf((float)d);
  p.nscale_log2 = -kLog2e * p.inv_sqrt_d;
  p.nbias_log2 = -bias * kLog2e;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == SATTN_F32) return SATTN_ERR_UNSUPPORTED;
  if (d == 128) return launch_sigmoid_bwd<128, 64, 4>(p, causal, alibi_slopes != nullptr, parts, st);
  return launch_sigmoid_bwd<64, 64, 4>(p, causal, alibi_slopes != nullptr, parts, st);
}

}  // namespace

extern "C" {

int sigmoid_attn_fwd(const void* q, const void* k, const void* v, void* o, int B, int H, int N, int d,
                     sattn_dtype dtype, float bias, int causal, const float* alibi_slopes, const sattn_strides* sq,
                     const sattn_strides* sk, const sattn_strides* sv, const sattn_strides* so, void* stream) {
  int rc = check_shape(B, H, N, d, dtype);
  if (rc) return rc;
  FwdParams p{};
  if ((rc = make_ref(q, sq, H, N, d, dtype, &p.q))) return rc;
  if ((rc = make_ref(k, sk, H, N, d, dtype, &p.k))) return rc;
  if ((rc = make_ref(v, sv, H, N, d, dtype, &p.v))) return rc;
  if ((rc = make_ref(o, so, H, N, d, dtype, &p.o))) return rc;
  p.slopes = alibi_slopes;
  p.lse = nullptr;
  p.B = B; p.H = H; p.N = N;
  p.nscale_log2 = -kLog2e / sqrtf((float)d);
  p.nbias_log2 = -bias * kLog2e;
  hipStream_t st = (hipStream_t)stream;
  if (dtype == SATTN_F32) return SATTN_ERR_UNSUPPORTED;
  constexpr int NW = 4;
  p.n_qblocks = (N + 32 * NW - 1) / (32 * NW);
  if (d == 128) return launch_sigmoid_fwd<128, 64, NW>(p, causal, alibi_slopes != nullptr, st);
  return launch_sigmoid_fwd<64, 64, NW>(p, causal, alibi_slopes != nullptr, st);
}

int sigmoid_attn_bwd(const void* q, const void* k, const void* v, const void* dout, void* dq, void* dk, void* dv,
                     int B, int H, int N, int d, sattn_dtype dtype, float bias, int causal,
                     const float* alibi_slopes, const sattn_strides* sq, const sattn_strides* sk,
                     const sattn_strides* sv, const sattn_strides* sdout, const sattn_strides* sdq,
                     const sattn_strides* sdk, const sattn_strides* sdv, void* workspace, size_t workspace_bytes,
                     void* stream) {
  (void)workspace; (void)workspace_bytes;  // the two-kernel split needs none
  return sigmoid_bwd_impl(q, k, v, dout, dq, dk, dv, B, H, N, d, dtype, bias, causal, alibi_slopes, sq, sk, sv,
                          sdout, sdq, sdk, sdv, kBwdDkDv | kBwdDq, stream);
}

int sigmoid_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* dout, void* dk, void* dv,
                          int B, int H, int N, int d, sattn_dtype dtype, float bias, int causal,
                          const float* alibi_slopes, const sattn_strides* sq, const sattn_strides* sk,
                          const sattn_strides* sv, const sattn_strides* sdout, const sattn_strides* sdk,
                          const sattn_strides* sdv, void* stream) {
  return sigmoid_bwd_impl(q, k, v, dout, nullptr, dk, dv, B, H, N, d, dtype, bias, causal, alibi_slopes, sq, sk,
                          sv, sdout, nullptr, sdk, sdv, kBwdDkDv, stream);
}

int sigmoid_attn_bwd_dq(const void* q, const void* k, const void* v, const void* dout, void* dq, int B, int H,
                        int N, int d, sattn_dtype dtype, float bias, int causal, const float* alibi_slopes,
                        const sattn_strides* sq, const sattn_strides* sk, const sattn_strides* sv,
                        const sattn_strides* sdout, const sattn_strides* sdq, void* stream) {
  return sigmoid_bwd_impl(q, k, v, dout, dq, nullptr, nullptr, B, H, N, d, dtype, bias, causal, alibi_slopes, sq,
                          sk, sv, sdout, sdq, nullptr, nullptr, kBwdDq, stream);
}

size_t sigmoid_attn_bwd_workspace_bytes(int, int, int, int, sattn_dtype) { return 0; }

// ---- not built yet: report it instead of pretending
int softmax_attn_fwd(const void*, const void*, const void*, void*, float*, int, int, int, int, sattn_dtype, int,
                     const float*, const sattn_strides*, const sattn_strides*, const sattn_strides*,
                     const sattn_strides*, void*) { return SATTN_ERR_UNSUPPORTED; }
int softmax_attn_bwd(const void*, const void*, const void*, const void*, const float*, const void*, void*, void*,
                     void*, int, int, int, int, sattn_dtype, int, const float*, const sattn_strides*,
                     const sattn_strides*, const sattn_strides*, const sattn_strides*, const sattn_strides*,
                     const sattn_strides*, const sattn_strides*, const sattn_strides*, void*, size_t, void*) {
  return SATTN_ERR_UNSUPPORTED;
}
size_t softmax_attn_bwd_workspace_bytes(int, int, int, int, sattn_dtype) { return 0; }

const char* sattn_strerror(int code) {
  switch (code) {
    case SATTN_OK: return "success";
    case SATTN_ERR_NULL: return "a required pointer is NULL";
    case SATTN_ERR_SHAPE: return "B, H and N must be positive and within the supported range";
    case SATTN_ERR_UNSUPPORTED: return "unsupported head dimension or dtype (d must be 64 or 128)";
    case SATTN_ERR_ALIGN: return "pointers and strides must keep rows 16-byte aligned";
    case SATTN_ERR_WORKSPACE: return "workspace missing or too small";
    case SATTN_ERR_LAUNCH: return "the HIP runtime rejected the kernel launch";
    default: return "unknown error code";
  }
}

int sattn_version(void) { return 100; }

}  // extern "C"
