// Fused sigmoid-attention forward for gfx950 (Algorithm 1 of the paper's Appendix F.1),
// bf16 operands, fp32 logits / sigmoid / accumulation.
//
// Work split: one workgroup = NW waves, each wave owns 32 query rows (B_r = 32*NW); the
// workgroup streams K/V tiles of BC keys through LDS (double buffered).  Per 32-key chunk
// a wave computes
//     S^T (32 keys x 32 queries) = K_chunk Q_i^T          8 (d=128) MFMA 32x32x16
//     P^T = sigmoid(S^T * 1/sqrt(d) + b [+ ALiBi])         fp32 VALU, no row max / row sum
//     O_i^T (d x 32 queries)    += V_chunk^T P^T           8 MFMA, V read with the
//                                                          transposing LDS load
// Computing the transposed products lets the S^T accumulator registers be used, after the
// bf16 round, as the B operand of the second product with no cross-lane traffic.
#pragma once
#include "sattn_common.hpp"

namespace sattn {

struct FwdParams {
  TensorRef q, k, v, o;
  const float* slopes;  // [H] or nullptr
  float* lse;           // softmax only: [B,H,N]
  int B, H, N;
  int n_qblocks;
  float nscale_log2;  // -log2(e)/sqrt(d)
  float nbias_log2;   // -b*log2(e)
};

template <int D>
struct Swz {
  static constexpr int CPR = D / 8;  // 16-byte chunks per row
  // K tile: rows are read 32-at-a-time at one logical chunk -> spread rows over chunks
  __device__ static __forceinline__ int k(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
  // V tile: the transposing read touches 4 consecutive rows x 64 contiguous bytes
  __device__ static __forceinline__ int v(int row) { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
};

// Stage one K or V tile (BC rows x D bf16) global -> registers -> LDS.
template <int D, int BC, int NT>
struct TileStager {
  static constexpr int CPR = D / 8;
  static constexpr int NCH = (BC * CPR) / NT;
  static_assert((BC * CPR) % NT == 0, "tile must split evenly over the workgroup");
  u32x4 kreg[NCH], vreg[NCH];

  __device__ __forceinline__ void load(const __bf16* kb, const __bf16* vb, int64_t kss, int64_t vss, int j0, int N,
                                       int tid) {
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      int idx = tid + n * NT;
      int r = idx / CPR, c = idx % CPR;
      int key = j0 + r;
      key = key < N ? key : N - 1;  // rows past the end are clamped here and masked in the epilogue
      kreg[n] = *(const u32x4*)(kb + (int64_t)key * kss + c * 8);
      vreg[n] = *(const u32x4*)(vb + (int64_t)key * vss + c * 8);
    }
  }
  __device__ __forceinline__ void store(uint32_t ks, uint32_t vs, int tid) const {
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      int idx = tid + n * NT;
      int r = idx / CPR, c = idx % CPR;
      lds_write_b128(ks + r * (D * 2) + ((c ^ Swz<D>::k(r)) << 4), kreg[n]);
      lds_write_b128(vs + r * (D * 2) + ((c ^ Swz<D>::v(r)) << 4), vreg[n]);
    }
  }
};

template <int D, int BC, int NW, bool CAUSAL, bool ALIBI>
__global__ void __launch_bounds__(64 * NW, (NW == 4 ? 2 : 1))
sigmoid_fwd_kernel(const FwdParams p) {
  constexpr int NT = 64 * NW;
  constexpr int BR = 32 * NW;
  constexpr int KD = D / 16;  // contraction steps of S^T
  constexpr int DT = D / 32;  // 32-row tiles of O^T
  constexpr int NCK = BC / 32;
  constexpr int TILE = BC * D * 2;  // bytes of one K or V tile

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(SATTN_LDS(char)*)smem;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, h = lane >> 5;

  const int total = p.n_qblocks * p.B * p.H;
  const int logical = xcd_remap(blockIdx.x, total);
  const int bh = logical / p.n_qblocks;
  // causal: heavy (late) query blocks first
  const int qb = CAUSAL ? (p.n_qblocks - 1 - logical % p.n_qblocks) : (logical % p.n_qblocks);
  const int b = bh / p.H, hd = bh % p.H;
  const int N = p.N;

  const __bf16* qbase = (const __bf16*)p.q.ptr + b * p.q.sb + hd * p.q.sh;
  const __bf16* kbase = (const __bf16*)p.k.ptr + b * p.k.sb + hd * p.k.sh;
  const __bf16* vbase = (const __bf16*)p.v.ptr + b * p.v.sb + hd * p.v.sh;
  __bf16* obase = (__bf16*)p.o.ptr + b * p.o.sb + hd * p.o.sh;

  const int q_wave0 = qb * BR + wave * 32;  // first query row of this wave
  const int qi = q_wave0 + l32;             // this lane's query row
  const int qi_ld = qi < N ? qi : N - 1;

  // Q fragment: B operand of S^T = K Q^T, column = query, k = d
  bf16x8 qf[KD];
#pragma unroll
  for (int kk = 0; kk < KD; ++kk) qf[kk] = as_bf16x8(*(const u32x4*)(qbase + (int64_t)qi_ld * p.q.ss + 16 * kk + 8 * h));

  f32x16 oacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;

  // per-lane LDS offsets (relative to the K / V tile of a stage, chunk 0)
  const int kap = kappa(l32);
  uint32_t koff[KD];
#pragma unroll
  for (int kk = 0; kk < KD; ++kk) koff[kk] = kap * (D * 2) + (((2 * kk + h) ^ Swz<D>::k(kap)) << 4);
  const int i16 = lane & 15, blk1 = (lane >> 4) & 1;
  uint32_t voff[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) {
    int row = 8 * h + (i16 >> 2);
    int c = 4 * dt + 2 * blk1 + ((i16 & 3) >> 1);
    voff[dt] = row * (D * 2) + ((c ^ Swz<D>::v(row)) << 4) + ((i16 & 1) << 3);
  }

  float sl2 = 0.f;
  if (ALIBI) sl2 = p.slopes[hd] * kLog2e;

  const int q_hi = (qb * BR + BR < N ? qb * BR + BR : N) - 1;  // last valid query row of the block
  const int kv_len = CAUSAL ? (q_hi + 1) : N;
  const int n_tiles = (kv_len + BC - 1) / BC;

  TileStager<D, BC, NT> st;
  st.load(kbase, vbase, p.k.ss, p.v.ss, 0, N, tid);
  st.store(lds0, lds0 + TILE, tid);
  __syncthreads();

  for (int jt = 0; jt < n_tiles; ++jt) {
    const int j0 = jt * BC;
    const uint32_t ks = lds0 + (jt & 1) * (2 * TILE), vs = ks + TILE;
    const bool more = jt + 1 < n_tiles;
    if (more) st.load(kbase, vbase, p.k.ss, p.v.ss, j0 + BC, N, tid);

#pragma unroll
    for (int ck = 0; ck < NCK; ++ck) {
      const int jc = j0 + 32 * ck;  // first key of the chunk
      if (jc >= N) break;
      if (CAUSAL && jc > q_wave0 + 31) break;  // chunk entirely above this wave's diagonal
      // ---- S^T chunk
      f32x16 s;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KD; ++kk) {
        bf16x8 a = as_bf16x8(lds_read_b128(ks + ck * 32 * (D * 2) + koff[kk]));
        s = mfma32(a, qf[kk], s);
      }
      // ---- sigmoid epilogue: p = 1 / (1 + 2^u), u = -(s/sqrt(d) + b - slope|i-j|) log2(e)
      const int jl = jc + 8 * h;  // key of register 0 for this lane half
      const bool need_mask = (jc + 31 >= N) || (CAUSAL && jc + 31 > q_wave0);
      float pr[16];
      if (ALIBI) {
        const float dist0 = (float)(qi - jl);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float dist = dist0 - (float)key_of_reg(r);
          float w = __builtin_fmaf(sl2, __builtin_fabsf(dist), p.nbias_log2);
          pr[r] = __builtin_fmaf(s[r], p.nscale_log2, w);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) pr[r] = __builtin_fmaf(s[r], p.nscale_log2, p.nbias_log2);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) pr[r] = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(pr[r]));
      if (need_mask) {
        int lim = N - 1 - jl;
        if (CAUSAL) lim = lim < qi - jl ? lim : qi - jl;
#pragma unroll
        for (int r = 0; r < 16; ++r) pr[r] = key_of_reg(r) <= lim ? pr[r] : 0.f;
      }
      // ---- O^T += V_chunk^T P^T
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2) {
        u32x4 pw;
#pragma unroll
        for (int w = 0; w < 4; ++w) pw[w] = pack_bf16(pr[8 * ks2 + 2 * w], pr[8 * ks2 + 2 * w + 1]);
        bf16x8 pb = as_bf16x8(pw);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          uint32_t a0 = vs + (ck * 32 + ks2 * 16) * (D * 2) + voff[dt];
          bf16x8 a = join_tr(lds_read_tr16(a0), lds_read_tr16(a0 + 4 * (D * 2)));
          oacc[dt] = mfma32(a, pb, oacc[dt]);
        }
      }
    }
    if (more) st.store(lds0 + ((jt + 1) & 1) * (2 * TILE), lds0 + ((jt + 1) & 1) * (2 * TILE) + TILE, tid);
    __syncthreads();
  }

  // ---- store O (bf16): register 4g+t of tile dt is O[qi][32dt + 8g + 4h + t]
  if (qi < N) {
    __bf16* orow = obase + (int64_t)qi * p.o.ss;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w;
        w[0] = pack_bf16(oacc[dt][4 * g], oacc[dt][4 * g + 1]);
        w[1] = pack_bf16(oacc[dt][4 * g + 2], oacc[dt][4 * g + 3]);
        *(u32x2*)(orow + 32 * dt + 8 * g + 4 * h) = w;
      }
  }
}

}  // namespace sattn
