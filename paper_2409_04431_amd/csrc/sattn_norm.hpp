// Hybrid-norm for gfx950: LayerNorm / RMSNorm (no learnable affine parameters) of the attention
// output over the concatenated heads, forward and backward (Section 5.5, Appendix G.6:
// x + norm(sigmoid-attention); the norm alone is computed here).
//
// Token (b, n) owns H*d features spread over the H head slices of a [B,H,N,d] tensor with
// arbitrary batch/head/token strides.  The work is one read and one write of the tensor (the
// backward reads two), i.e. HBM-bound: one wave per token keeps the whole row in registers
// (CPL 16-byte chunks per lane), so statistics and normalisation need no second pass over
// memory; the variance is the two-pass one (around the mean), in fp32.  A fused epilogue in
// the attention kernel is not possible: a workgroup there owns one head, the statistics span
// all heads.
#pragma once
#include "sattn_common.hpp"

namespace sattn {

struct NormParams {
  TensorRef x, y;    // forward: input, output.  backward: x = forward input, y = dx
  TensorRef dy;      // backward only
  float* stats;      // [B, N, 2]: mean (0 for RMSNorm), 1/sqrt(var + eps); written by forward, read by backward
  int B, H, N, d;
  float eps;
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
  return v;
}

// element pointer of 16-byte chunk c (8 bf16) of token (b, n)
__device__ __forceinline__ const __bf16* chunk_ptr(const TensorRef& t, int b, int n, int c, int cpr) {
  const int h = c / cpr, o = (c % cpr) * 8;
  return (const __bf16*)t.ptr + b * t.sb + h * t.sh + (int64_t)n * t.ss + o;
}

template <int CPL, bool RMS, bool BACKWARD>
__global__ void __launch_bounds__(256)
headconcat_norm_kernel(const NormParams p) {
  const int lane = threadIdx.x & 63;
  const int64_t token = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (token >= (int64_t)p.B * p.N) return;  // whole wave
  const int b = (int)(token / p.N), n = (int)(token % p.N);
  const int cpr = p.d / 8, nchunks = p.H * cpr;
  const float inv_f = 1.0f / (float)(p.H * p.d);

  float xv[CPL][8];
#pragma unroll
  for (int i = 0; i < CPL; ++i) {
    const int c = lane + 64 * i;
    if (c < nchunks) {
      const bf16x8 v = as_bf16x8(*(const u32x4*)chunk_ptr(p.x, b, n, c, cpr));
#pragma unroll
      for (int e = 0; e < 8; ++e) xv[i][e] = (float)v[e];
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) xv[i][e] = 0.f;
    }
  }

  float mean, rstd;
  if (!BACKWARD) {
    mean = 0.f;
    if (!RMS) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < CPL; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) s += xv[i][e];
      mean = wave_sum(s) * inv_f;
    }
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < CPL; ++i)
      if (lane + 64 * i < nchunks) {
#pragma unroll
        for (int e = 0; e < 8; ++e) q = __builtin_fmaf(xv[i][e] - mean, xv[i][e] - mean, q);
      }
    // hardware reciprocal square root plus one Newton step (the statistics are kept for the
    // backward pass)
    const float a = wave_sum(q) * inv_f + p.eps;
    rstd = __builtin_amdgcn_rsqf(a);
    rstd = rstd * (1.5f - 0.5f * a * rstd * rstd);
    if (lane == 0) {
      p.stats[2 * token] = mean;
      p.stats[2 * token + 1] = rstd;
    }
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunks) {
        u32x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          w[e] = pack_bf16((xv[i][2 * e] - mean) * rstd, (xv[i][2 * e + 1] - mean) * rstd);
        *(u32x4*)const_cast<__bf16*>(chunk_ptr(p.y, b, n, c, cpr)) = w;
      }
    }
  } else {
    mean = p.stats[2 * token];
    rstd = p.stats[2 * token + 1];
    // dx = rstd * (dy - mean_f(dy) [LayerNorm only] - xhat * mean_f(dy * xhat))
    float gv[CPL][8];
    float sg = 0.f, sgy = 0.f;
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunks) {
        const bf16x8 v = as_bf16x8(*(const u32x4*)chunk_ptr(p.dy, b, n, c, cpr));
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          gv[i][e] = (float)v[e];
          xv[i][e] = (xv[i][e] - mean) * rstd;  // xhat
          sg += gv[i][e];
          sgy = __builtin_fmaf(gv[i][e], xv[i][e], sgy);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) gv[i][e] = 0.f;
      }
    }
    const float mg = RMS ? 0.f : wave_sum(sg) * inv_f;
    const float mgy = wave_sum(sgy) * inv_f;
#pragma unroll
    for (int i = 0; i < CPL; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunks) {
        u32x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float a0 = (gv[i][2 * e] - mg - xv[i][2 * e] * mgy) * rstd;
          const float a1 = (gv[i][2 * e + 1] - mg - xv[i][2 * e + 1] * mgy) * rstd;
          w[e] = pack_bf16(a0, a1);
        }
        *(u32x4*)const_cast<__bf16*>(chunk_ptr(p.y, b, n, c, cpr)) = w;
      }
    }
  }
}

}  // namespace sattn
