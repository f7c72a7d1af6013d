// fp32 sigmoid attention for gfx950: forward and the two backward kernels in one template.
// Everything (operands, logits, sigmoid, accumulation, outputs) is fp32; the matrix
// products run on the fp32 MFMA (32x32x2), exp and the division are the accurate ones.
// This is the precision path (agreement with the fp64 oracle to ~1e-6); the bf16 kernels
// are the throughput path.
//
// One workgroup = 4 waves; each wave owns 32 rows of the stationary side and keeps their
// operand fragments in registers; 32-row tiles of the streaming side pass through LDS.
//   FWD  : stationary Q          | stream K,V  : S^T = K Q^T, P^T, O^T += V^T P^T
//   DQ   : stationary Q, dO      | stream K,V  : S^T, dP^T = V dO^T, dS^T, dQ^T += K^T dS^T
//   DKDV : stationary K, V       | stream Q,dO : S = Q K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q^T dS
// (Algorithms 1 and 2 of the paper's Appendix F.1; the backward is split by output owner.)
//
// MFMA 32x32x2 fp32 fragment maps, lane l (l32 = l%32, h = l/32):
//   A (32x2): row l32, k = h;  B (2x32): col l32, k = h;  C: col l32, row 8*(r/4)+4h+r%4.
// With the streaming rows on C's rows, accumulator register r is directly the B operand
// (k-slot h <-> streaming row 8*(r/4)+4h+r%4) of the second product.
#pragma once
#include "sattn_common.hpp"

namespace sattn {

enum F32Mode { F32_FWD = 0, F32_DQ = 1, F32_DKDV = 2 };

struct F32Params {
  TensorRef q, k, v, dout;   // inputs (dout unused by FWD)
  TensorRef out0, out1;      // FWD: O ; DQ: dQ ; DKDV: dK, dV
  const float* slopes;
  int B, H, N, n_blocks;
  float scale;   // 1/sqrt(d)
  float bias;
  // DQ only, optional: row sums of dS, element (b, h, i) at b*db_sb + h*db_sh + i
  // (+ the sequence's first token in a variable-length call)
  float* db_rows;
  int64_t db_sb, db_sh;
  // The same extensions as the bf16 kernels' parameter blocks: packed sequences of different
  // lengths (cu_seqlens, optional bias per sequence), query head h reading K/V head
  // h / kv_group (>= 1; the dK/dV pass then runs per K/V head and sums over its query heads),
  // and a number of keys Nk that differs from the number of queries N (0: same; non-causal).
  const int* cu_seqlens;
  const float* bias_vec;
  int kv_group;
  int Nk;
  // position of query 0 on the key axis (Nk - N when the queries are the last N positions of the
  // key sequence, else 0; any value here): causal keeps key j for query i iff j <= i + qoff,
  // ALiBi measures |i + qoff - j|
  int qoff;
};

__device__ __forceinline__ f32x16 mfma_f32(float a, float b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

template <int D, int MODE, bool CAUSAL, bool ALIBI>
__global__ void __launch_bounds__(256, 1)
sigmoid_f32_kernel(const F32Params p) {
  constexpr int NW = 4, NT = 256, BS = 32 * NW;  // stationary rows per workgroup
  constexpr int LD = D + 2;                        // LDS row stride (floats): 32 rows -> 32 distinct even banks
  constexpr int DT = D / 32;
  constexpr bool TWO = MODE != F32_FWD;           // second stationary operand / dP product
  __shared__ float t1[32 * LD];
  __shared__ float t2[32 * LD];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  // the dK/dV pass runs one workgroup per K/V head and key block and streams the query heads of
  // that head's group one after the other; the other passes run per query head
  const int heads = MODE == F32_DKDV ? p.H / p.kv_group : p.H;
  const int bh = blockIdx.x / p.n_blocks, blk = blockIdx.x % p.n_blocks;
  const int b = bh / heads, hd = bh % heads;
  const int hkv = MODE == F32_DKDV ? hd : hd / p.kv_group;
  const int hq0 = MODE == F32_DKDV ? hd * p.kv_group : hd, n_hq = MODE == F32_DKDV ? p.kv_group : 1;
  int N = p.N;
  int64_t tok0 = 0;
  float bias = p.bias;
  if (p.cu_seqlens) {
    tok0 = p.cu_seqlens[b];
    const int len = p.cu_seqlens[b + 1] - (int)tok0;
    N = len < p.N ? len : p.N;  // never beyond the span the host checked
    if (p.bias_vec) bias = p.bias_vec[b];
    if (blk * BS >= N) return;  // this sequence has no such block (whole workgroup)
  }
  // N counts the queries, Nk the keys; Ns / Nt are the row counts of this pass's stationary /
  // streamed side
  const int Nk = p.Nk > 0 ? p.Nk : N;
  const int Ns = MODE == F32_DKDV ? Nk : N, Nt = MODE == F32_DKDV ? N : Nk;

  const float* kb = (const float*)p.k.ptr + b * p.k.sb + hkv * p.k.sh + tok0 * p.k.ss;
  const float* vb = (const float*)p.v.ptr + b * p.v.sb + hkv * p.v.sh + tok0 * p.v.ss;
  auto qhead = [&](int hq) { return (const float*)p.q.ptr + b * p.q.sb + hq * p.q.sh + tok0 * p.q.ss; };
  auto dohead = [&](int hq) {
    return TWO ? (const float*)p.dout.ptr + b * p.dout.sb + hq * p.dout.sh + tok0 * p.dout.ss : nullptr;
  };

  // stationary side: x1 (and x2); streaming side: y1, y2 (per query head in the dK/dV pass)
  const float* x1 = MODE == F32_DKDV ? kb : qhead(hq0);
  const int64_t x1s = MODE == F32_DKDV ? p.k.ss : p.q.ss;
  const float* x2 = MODE == F32_DKDV ? vb : dohead(hq0);
  const int64_t x2s = MODE == F32_DKDV ? p.v.ss : p.dout.ss;
  const int64_t y1s = MODE == F32_DKDV ? p.q.ss : p.k.ss;
  const int64_t y2s = MODE == F32_DKDV ? p.dout.ss : p.v.ss;

  const int a_wave0 = blk * BS + wave * 32;  // first stationary row of the wave
  const int ai = a_wave0 + l32;              // this lane's stationary row (query, or key for DKDV)
  const int ai_ld = ai < Ns ? ai : Ns - 1;

  float xf1[D / 2], xf2[TWO ? D / 2 : 1];
#pragma unroll
  for (int kk = 0; kk < D / 2; ++kk) {
    xf1[kk] = x1[(int64_t)ai_ld * x1s + 2 * kk + h];
    if (TWO) xf2[kk] = x2[(int64_t)ai_ld * x2s + 2 * kk + h];
  }
  f32x16 acc0[DT], acc1[MODE == F32_DKDV ? DT : 1];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      acc0[dt][r] = 0.f;
      if (MODE == F32_DKDV) acc1[dt][r] = 0.f;
    }
  float dbsum = 0.f;  // DQ: sum of this lane's dS elements

  // range of streaming tiles (32 rows each)
  const int a_hi = (blk * BS + BS < Ns ? blk * BS + BS : Ns) - 1;
  int t_lo = 0, t_hi = (Nt + 31) / 32;
  if (CAUSAL) {
    if (MODE == F32_DKDV) {  // queries before the first key's place on the query axis see nothing
      const int first = blk * BS - p.qoff;
      t_lo = (first > 0 ? first : 0) / 32;
    } else {                 // keys after the last query's place on the key axis are masked
      const int last = a_hi + p.qoff;
      t_hi = last < 0 ? 0 : (last < Nt ? last : Nt - 1) / 32 + 1;
    }
  }

  for (int hq = hq0; hq < hq0 + n_hq; ++hq) {  // one pass over the streamed side per query head
  const float* y1 = MODE == F32_DKDV ? qhead(hq) : kb;
  const float* y2 = MODE == F32_DKDV ? dohead(hq) : vb;
  const float slope = ALIBI ? p.slopes[hq] : 0.f;
  for (int t = t_lo; t < t_hi; ++t) {
    const int b0 = t * 32;  // first streaming row of the tile
    __syncthreads();        // previous tile fully consumed
    for (int idx = tid; idx < 32 * (D / 4); idx += NT) {
      int r = idx / (D / 4), c = idx % (D / 4);
      int row = b0 + r;
      row = row < Nt ? row : Nt - 1;
      f32x4 u = *(const f32x4*)(y1 + (int64_t)row * y1s + 4 * c);
      f32x4 w = *(const f32x4*)(y2 + (int64_t)row * y2s + 4 * c);
      float* d1 = &t1[r * LD + 4 * c];
      float* d2 = &t2[r * LD + 4 * c];
      d1[0] = u[0]; d1[1] = u[1]; d1[2] = u[2]; d1[3] = u[3];
      d2[0] = w[0]; d2[1] = w[1]; d2[2] = w[2]; d2[3] = w[3];
    }
    __syncthreads();

    // wave-uniform skip of tiles that are entirely masked for this wave
    bool live = a_wave0 < Ns;
    if (CAUSAL) {
      if (MODE == F32_DKDV) live = live && (b0 + 31 + p.qoff >= a_wave0);  // some query at or after some key
      else live = live && (b0 <= a_wave0 + 31 + p.qoff);                   // some key at or before some query
    }
    if (!live) continue;

    f32x16 s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
    for (int kk = 0; kk < D / 2; ++kk) {
      s = mfma_f32(t1[l32 * LD + 2 * kk + h], xf1[kk], s);
      if (MODE == F32_DQ) dp = mfma_f32(t2[l32 * LD + 2 * kk + h], xf2[kk], dp);
      if (MODE == F32_DKDV) dp = mfma_f32(t2[l32 * LD + 2 * kk + h], xf2[kk], dp);
    }
    // element (register r, this lane): streaming row bi = b0 + 8g + 4h + t, stationary row ai
    float pr[16], ds[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int bi = b0 + 8 * (r >> 2) + 4 * h + (r & 3);
      const int qrow = (MODE == F32_DKDV ? bi : ai) + p.qoff;  // the query's place on the key axis
      const int krow = MODE == F32_DKDV ? ai : bi;
      float tt = s[r] * p.scale + bias;
      if (ALIBI) tt -= slope * fabsf((float)(qrow - krow));
      float pv = 1.0f / (1.0f + expf(-tt));
      bool keep = bi < Nt && (!CAUSAL || krow <= qrow);
      pv = keep ? pv : 0.f;
      pr[r] = pv;
      if (TWO) ds[r] = pv * (1.0f - pv) * dp[r];
      if (MODE == F32_DQ) dbsum += ds[r];
    }
    // second products: acc^T[d][a] += Y^T[d][bi] * W[bi][a]
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int br = 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        if (MODE == F32_FWD) acc0[dt] = mfma_f32(t2[br * LD + 32 * dt + l32], pr[r], acc0[dt]);
        if (MODE == F32_DQ) acc0[dt] = mfma_f32(t1[br * LD + 32 * dt + l32], ds[r], acc0[dt]);
        if (MODE == F32_DKDV) {
          acc0[dt] = mfma_f32(t1[br * LD + 32 * dt + l32], ds[r], acc0[dt]);  // dK^T += Q^T dS
          acc1[dt] = mfma_f32(t2[br * LD + 32 * dt + l32], pr[r], acc1[dt]);  // dV^T += dO^T P
        }
      }
    }
  }
  }  // query heads

  if (MODE == F32_DQ) {
    // the two halves of the wave hold the sums over different keys of the same query row
    dbsum += __shfl_xor(dbsum, 32);
    if (p.db_rows && h == 0 && ai < Ns) p.db_rows[b * p.db_sb + hd * p.db_sh + tok0 + ai] = dbsum;
  }
  if (ai < Ns) {
    const float osc = MODE == F32_FWD ? 1.0f : p.scale;  // dQ, dK carry the 1/sqrt(d) of the logits
    float* o0 = (float*)p.out0.ptr + b * p.out0.sb + hd * p.out0.sh + (tok0 + ai) * p.out0.ss;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 w = {acc0[dt][4 * g] * osc, acc0[dt][4 * g + 1] * osc, acc0[dt][4 * g + 2] * osc, acc0[dt][4 * g + 3] * osc};
        *(f32x4*)(o0 + 32 * dt + 8 * g + 4 * h) = w;
      }
    if (MODE == F32_DKDV) {
      float* o1 = (float*)p.out1.ptr + b * p.out1.sb + hd * p.out1.sh + (tok0 + ai) * p.out1.ss;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 w = {acc1[dt][4 * g], acc1[dt][4 * g + 1], acc1[dt][4 * g + 2], acc1[dt][4 * g + 3]};
          *(f32x4*)(o1 + 32 * dt + 8 * g + 4 * h) = w;
        }
    }
  }
}

}  // namespace sattn
