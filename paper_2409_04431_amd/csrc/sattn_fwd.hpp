// Fused sigmoid-attention forward for gfx950 (Algorithm 1 of the paper's Appendix F.1),
// bf16 operands, fp32 logits / sigmoid / accumulation.
//
// Work split: one workgroup = 8 waves (two per SIMD), each wave owns 32 query rows
// (B_r = 256); the workgroup streams K/V tiles of 64 keys through a 3-slot LDS ring.
// Per 32-key chunk c a wave computes
//     S^T (32 keys x 32 queries) = K_c Q_i^T               8 (d=128) MFMA 32x32x16
//     P^T = sigmoid(S^T / sqrt(d) + b [+ ALiBi])            fp32 VALU, no row max / row sum
//     O_i^T (d x 32 queries)    += V_c^T P^T                8 MFMA, V read with the
//                                                           transposing LDS load
// Computing the transposed products lets the S^T accumulator registers be used, after the
// bf16 round, as the B operand of the second product with no cross-lane traffic.
//
// The three stages are software-pipelined inside each wave: step c issues the MFMAs of
// S^T(c+1) and of the O^T update with P^T(c-1) while the VALU evaluates sigmoid(c), so
// that matrix and vector pipes are both fed from one instruction stream.
#pragma once
#include "sattn_common.hpp"

namespace sattn {

struct FwdParams {
  TensorRef q, k, v, o;
  const float* slopes;  // [H] or nullptr
  float* lse;           // softmax only: [B,H,N]
  int B, H, N;
  int n_qblocks;
  float nscale_log2;  // -log2(e)/sqrt(d)   (softmax: +log2(e)/sqrt(d))
  float nbias_log2;   // -b*log2(e)
};

// LDS swizzles (XOR on the 16-byte chunk index within a row).
template <int D>
struct Swz {
  static constexpr int CPR = D / 8;  // 16-byte chunks per row
  // K tile: rows are read 32-at-a-time at one logical chunk -> spread rows over chunks
  __device__ static __forceinline__ int k(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
  // V tile: the transposing read touches 4 consecutive rows x 64 contiguous bytes
  __device__ static __forceinline__ int v(int row) { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
};

// Stage one tile (ROWS x D bf16) global -> registers -> LDS.
template <int D, int ROWS, int NT, bool IS_V>
struct TileStager {
  static constexpr int CPR = D / 8;
  static constexpr int NCH = (ROWS * CPR) / NT;
  static_assert((ROWS * CPR) % NT == 0, "tile must split evenly over the workgroup");
  u32x4 reg[NCH];

  __device__ __forceinline__ void load(const __bf16* base, int64_t ss, int j0, int N, int tid) {
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      int idx = tid + n * NT;
      int r = idx / CPR, c = idx % CPR;
      int key = j0 + r;
      key = key < N ? key : N - 1;  // rows past the end are clamped here and masked in the epilogue
      reg[n] = *(const u32x4*)(base + (int64_t)key * ss + c * 8);
    }
  }
  __device__ __forceinline__ void store(uint32_t lds, int tid) const {
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      int idx = tid + n * NT;
      int r = idx / CPR, c = idx % CPR;
      int sw = IS_V ? Swz<D>::v(r) : Swz<D>::k(r);
      lds_write_b128(lds + r * (D * 2) + ((c ^ sw) << 4), reg[n]);
    }
  }
};

// Per-wave constants of the forward pipeline.
template <int D>
struct FwdLane {
  static constexpr int KD = D / 16, DT = D / 32;
  uint32_t koff[KD];  // K row-wise read: row kappa(l32), chunk 2kk+h
  uint32_t voff[DT];  // V transposing read: rows 8h + i16/4, 64-byte group dt
  int qi, h;
  float nscale, nbias, sl2;
};

// Running row statistics of the softmax comparison kernel (log2 units), one query per lane.
struct SoftmaxState {
  float m;  // running maximum of the scaled logits
  float l;  // this lane half's partial sum of 2^(x - m)
};

// One pipeline step.  QK: start S^T(c+1) into s_nxt.  SIG: p_cur = bf16(sigmoid(s_cur)).
// PV: oacc += V(c-1)^T p_prv.  kbase/vbase are LDS byte addresses of the 32-key chunks.
// SOFTMAX replaces the sigmoid by the online-softmax update: row maximum (across the two
// lane halves), p = 2^(x - m), running sum, and a rescale of O^T when a maximum moved.
template <int D, bool ALIBI, bool SOFTMAX, bool QK, bool SIG, bool PV>
__device__ __forceinline__ void fwd_step(const FwdLane<D>& L, const bf16x8* qf, f32x16* oacc, f32x16& s_cur,
                                         f32x16& s_nxt, bf16x8* p_cur, const bf16x8* p_prv, uint32_t kbase,
                                         uint32_t vbase, int jc, bool mask, int N, bool causal,
                                         SoftmaxState& sm) {
  constexpr int KD = D / 16, DT = D / 32;
  bf16x8 kf[KD];
  bf16x8 vf[2 * DT];
  if (QK) {
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) kf[kk] = as_bf16x8(lds_read_b128(kbase + L.koff[kk]));
  }
  if (PV) {
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        uint32_t a0 = vbase + ks2 * 16 * (D * 2) + L.voff[dt];
        vf[ks2 * DT + dt] = join_tr(lds_read_tr16(a0), lds_read_tr16(a0 + 4 * (D * 2)));
      }
  }
  float pr[16];
  float alpha = 1.0f;
  if (SIG && SOFTMAX) {
    // x = (s/sqrt(d) - slope|i-j|) log2(e); masked keys -> -inf
    const int jl = jc + 8 * L.h;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float x = s_cur[r] * L.nscale;
      if (ALIBI) x = __builtin_fmaf(-L.sl2, __builtin_fabsf((float)(L.qi - jl) - (float)key_of_reg(r)), x);
      pr[r] = x;
    }
    if (mask) {
      int lim = N - 1 - jl;
      if (causal) lim = lim < L.qi - jl ? lim : L.qi - jl;
#pragma unroll
      for (int r = 0; r < 16; ++r) pr[r] = key_of_reg(r) <= lim ? pr[r] : -__builtin_inff();
    }
    float mx = pr[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = __builtin_fmaxf(mx, pr[r]);
    mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));  // the other half of this query's keys
    const float m_new = __builtin_fmaxf(sm.m, mx);
    alpha = __builtin_amdgcn_exp2f(sm.m - m_new);
    sm.m = m_new;
#pragma unroll
    for (int r = 0; r < 16; ++r) pr[r] -= m_new;
  }
  if (SIG && !SOFTMAX) {
    // p = 1 / (1 + 2^u), u = -(s/sqrt(d) + b - slope|i-j|) log2(e)
    const int jl = jc + 8 * L.h;  // key held by register 0 of this lane half
    if (ALIBI) {
      const float dist0 = (float)(L.qi - jl);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float dist = dist0 - (float)key_of_reg(r);
        float w = __builtin_fmaf(L.sl2, __builtin_fabsf(dist), L.nbias);
        pr[r] = __builtin_fmaf(s_cur[r], L.nscale, w);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) pr[r] = __builtin_fmaf(s_cur[r], L.nscale, L.nbias);
    }
  }
  if (QK) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s_nxt[r] = 0.f;
  }
  // interleave: one MFMA of each product, then a slice of the sigmoid
  constexpr int NM = KD > 2 * DT ? KD : 2 * DT;
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    if (QK && m < KD) s_nxt = mfma32(kf[m], qf[m], s_nxt);
    if (PV && m < 2 * DT) oacc[m % DT] = mfma32(vf[m], p_prv[m / DT], oacc[m % DT]);
    if (SIG) {
#pragma unroll
      for (int r = (16 * m) / NM; r < (16 * (m + 1)) / NM; ++r)
        pr[r] = SOFTMAX ? __builtin_amdgcn_exp2f(pr[r]) : __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(pr[r]));
    }
  }
  if (SIG && SOFTMAX) {
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += pr[r];
    sm.l = __builtin_fmaf(sm.l, alpha, sum);
    // O^T holds sums relative to the previous maximum: rescale only when some maximum moved
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
    }
  }
  if (SIG) {
    if (mask && !SOFTMAX) {
      const int jl = jc + 8 * L.h;
      int lim = N - 1 - jl;
      if (causal) lim = lim < L.qi - jl ? lim : L.qi - jl;
#pragma unroll
      for (int r = 0; r < 16; ++r) pr[r] = key_of_reg(r) <= lim ? pr[r] : 0.f;
    }
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      u32x4 pw;
#pragma unroll
      for (int w = 0; w < 4; ++w) pw[w] = pack_bf16(pr[8 * ks2 + 2 * w], pr[8 * ks2 + 2 * w + 1]);
      p_cur[ks2] = as_bf16x8(pw);
    }
  }
}

template <int D, bool CAUSAL, bool ALIBI, bool SOFTMAX>
__global__ void __launch_bounds__(512, 1)
attn_fwd_kernel(const FwdParams p) {
  constexpr int NW = 8, NT = 64 * NW, BR = 32 * NW, BC = 64;
  constexpr int KD = D / 16, DT = D / 32;
  constexpr int TILE = BC * D * 2;    // bytes of one K or V tile
  constexpr int CHUNK = 32 * D * 2;   // bytes of a 32-key chunk

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(SATTN_LDS(char)*)smem;
  const uint32_t kring = lds0, vring = lds0 + 3 * TILE;  // 3 K slots, then 3 V slots

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

  FwdLane<D> L;
  {
    const int kap = kappa(l32);
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) L.koff[kk] = kap * (D * 2) + (((2 * kk + h) ^ Swz<D>::k(kap)) << 4);
    const int i16 = lane & 15, blk1 = (lane >> 4) & 1;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      int row = 8 * h + (i16 >> 2);
      int c = 4 * dt + 2 * blk1 + ((i16 & 3) >> 1);
      L.voff[dt] = row * (D * 2) + ((c ^ Swz<D>::v(row)) << 4) + ((i16 & 1) << 3);
    }
    L.qi = qi; L.h = h;
    L.nscale = p.nscale_log2; L.nbias = p.nbias_log2;
    L.sl2 = ALIBI ? p.slopes[hd] * kLog2e : 0.f;
  }

  // keys this workgroup must visit, and chunks this wave must visit
  const int q_hi = (qb * BR + BR < N ? qb * BR + BR : N) - 1;  // last valid query row of the block
  const int kv_len = CAUSAL ? (q_hi + 1) : N;
  const int n_tiles = (kv_len + BC - 1) / BC;
  int kv_wave = N;
  if (CAUSAL) kv_wave = q_wave0 + 32 < N ? q_wave0 + 32 : N;
  const int cw = q_wave0 < N ? (kv_wave + 31) / 32 : 0;  // chunks 0..cw-1; waves past the end idle

  TileStager<D, BC, NT, false> kst;
  TileStager<D, BC, NT, true> vst;
  // prologue: K(0), V(0), K(1) visible before the first step
  kst.load(kbase, p.k.ss, 0, N, tid);
  vst.load(vbase, p.v.ss, 0, N, tid);
  kst.store(kring, tid);
  vst.store(vring, tid);
  if (n_tiles > 1) {
    kst.load(kbase, p.k.ss, BC, N, tid);
    kst.store(kring + TILE, tid);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the Q fragment is in registers before the loop starts
  __syncthreads();

  f32x16 s_cur, s_nxt;
  bf16x8 p_cur[2], p_prv[2];
#pragma unroll
  for (int r = 0; r < 16; ++r) { s_cur[r] = 0.f; s_nxt[r] = 0.f; }
  p_cur[0] = p_cur[1] = p_prv[0] = p_prv[1] = as_bf16x8(u32x4{0, 0, 0, 0});
  SoftmaxState sm{-__builtin_inff(), 0.f};

  // step -1: S^T(0)
  if (cw > 0) {
    fwd_step<D, ALIBI, SOFTMAX, true, false, false>(L, qf, oacc, s_cur, s_nxt, p_cur, p_prv, kring, 0, 0, false, N, CAUSAL, sm);
    s_cur = s_nxt;
  }

  int kslot = 0, vslot = 0;  // ring slot of tile t (K) and of tile t (V)
  for (int t = 0; t < n_tiles; ++t) {
    const bool k_more = t + 2 < n_tiles, v_more = t + 1 < n_tiles;
    if (k_more) kst.load(kbase, p.k.ss, (t + 2) * BC, N, tid);
    if (v_more) vst.load(vbase, p.v.ss, (t + 1) * BC, N, tid);
    const int kslot1 = kslot == 2 ? 0 : kslot + 1, kslot2 = kslot1 == 2 ? 0 : kslot1 + 1;
    const int vslot1 = vslot == 2 ? 0 : vslot + 1, vslotm = vslot == 0 ? 2 : vslot - 1;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = 2 * t + i;
      // K(c+1): chunk (c+1)%2 of tile (c+1)/2 ; V(c-1): chunk (c-1)%2 of tile (c-1)/2
      const uint32_t ka = kring + (i == 0 ? kslot * TILE + CHUNK : kslot1 * TILE);
      const uint32_t va = vring + (i == 0 ? vslotm * TILE + CHUNK : vslot * TILE);
      if (c + 1 < cw) {
        if (c == 0)
          fwd_step<D, ALIBI, SOFTMAX, true, true, false>(L, qf, oacc, s_cur, s_nxt, p_cur, p_prv, ka, va, 32 * c, false, N, CAUSAL, sm);
        else
          fwd_step<D, ALIBI, SOFTMAX, true, true, true>(L, qf, oacc, s_cur, s_nxt, p_cur, p_prv, ka, va, 32 * c, false, N, CAUSAL, sm);
        s_cur = s_nxt;
        p_prv[0] = p_cur[0]; p_prv[1] = p_cur[1];
      } else if (c + 1 == cw) {
        // last chunk of this wave: the only one that can touch the diagonal or the ragged end
        if (c == 0)
          fwd_step<D, ALIBI, SOFTMAX, false, true, false>(L, qf, oacc, s_cur, s_nxt, p_cur, p_prv, ka, va, 32 * c, true, N, CAUSAL, sm);
        else
          fwd_step<D, ALIBI, SOFTMAX, false, true, true>(L, qf, oacc, s_cur, s_nxt, p_cur, p_prv, ka, va, 32 * c, true, N, CAUSAL, sm);
        p_prv[0] = p_cur[0]; p_prv[1] = p_cur[1];
      } else if (c == cw) {
        fwd_step<D, ALIBI, SOFTMAX, false, false, true>(L, qf, oacc, s_cur, s_nxt, p_cur, p_prv, ka, va, 32 * c, false, N, CAUSAL, sm);
      }
    }
    if (k_more) kst.store(kring + kslot2 * TILE, tid);
    if (v_more) vst.store(vring + vslot1 * TILE, tid);
    kslot = kslot1;
    vslot = vslot1;
    __syncthreads();
  }
  // flush: O^T update of the last chunk when it fell on the last step of the loop
  if (cw == 2 * n_tiles && cw > 0) {
    const int vlast = vslot == 0 ? 2 : vslot - 1;  // slot of tile n_tiles-1
    fwd_step<D, ALIBI, SOFTMAX, false, false, true>(L, qf, oacc, s_cur, s_nxt, p_cur, p_prv, 0, vring + vlast * TILE + CHUNK, 0,
                                           false, N, CAUSAL, sm);
  }

  if (SOFTMAX) {
    // normalise by the row sum (both lane halves) and write the natural-log row log-sum-exp
    const float l_tot = sm.l + __shfl_xor(sm.l, 32);
    const float inv = 1.0f / l_tot;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[dt][r] *= inv;
    if (qi < N && h == 0) p.lse[(int64_t)bh * N + qi] = (sm.m + __builtin_amdgcn_logf(l_tot)) * kLn2;
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
