// Sigmoid-attention backward for gfx950 (Algorithm 2 of the paper's Appendix F.1), bf16
// operands, fp32 logits / sigmoid / accumulation.  P is recomputed from Q and K; nothing
// but Q, K, V, dO is read.
//
// Algorithm 2 keeps dK_j, dV_j on chip and read-modify-writes dQ_i in HBM.  Here the pass
// is split in two kernels so that every output tile has exactly one owner and no atomics or
// fp32 dQ workspace are needed (results are bit-reproducible):
//   dq kernel   : query block stationary, streams K/V tiles (S^T orientation, as forward)
//                 S^T = K Q^T, dP^T = V dO^T, dS^T = P^T(1-P^T)dP^T, dQ^T += K^T dS^T
//   dkdv kernel : key block stationary, streams Q/dO tiles (S orientation)
//                 S = Q K^T, dP = dO V^T, dS = P(1-P)dP, dV^T += dO^T P, dK^T += Q^T dS
// In both, the accumulator of the first product is, after the bf16 round, the B operand of
// the second; the A operand of the second is a transposing LDS read of a row-major tile.
#pragma once
#include "sattn_common.hpp"

namespace sattn {

struct BwdParams {
  TensorRef q, k, v, dout, dq, dk, dv;
  const float* slopes;
  const float* lse;    // softmax only: [B,H,N] natural-log row log-sum-exp from the forward
  const float* dvec;   // softmax only: [B,H,N] rowsum(dO o O)
  int B, H, N;
  int n_blocks;        // query blocks (dq kernel) or key blocks (dkdv kernel)
  float nscale_log2;   // -log2(e)/sqrt(d)
  float nbias_log2;    // -b*log2(e)
  float inv_sqrt_d;
};

// One swizzle for tiles that are read both row-wise (ds_read_b128, 32 rows at one logical
// chunk) and transposed (4 consecutive rows x 64 contiguous bytes).
template <int D>
struct SwzX {
  __device__ static __forceinline__ int f(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
  }
};

// Stage two row-major tiles (ROWS x D bf16 each) global -> registers -> LDS, both with SwzX.
template <int D, int ROWS, int NT>
struct PairStager {
  static constexpr int CPR = D / 8;
  static constexpr int NCH = (ROWS * CPR) / NT;
  static_assert((ROWS * CPR) % NT == 0, "tile must split evenly over the workgroup");
  u32x4 areg[NCH], breg[NCH];

  __device__ __forceinline__ void load(const __bf16* a, const __bf16* b, int64_t ass, int64_t bss, int r0, int N,
                                       int tid) {
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      int idx = tid + n * NT;
      int r = idx / CPR, c = idx % CPR;
      int row = r0 + r;
      row = row < N ? row : N - 1;  // clamped; the epilogue masks rows past the end
      areg[n] = *(const u32x4*)(a + (int64_t)row * ass + c * 8);
      breg[n] = *(const u32x4*)(b + (int64_t)row * bss + c * 8);
    }
  }
  __device__ __forceinline__ void store(uint32_t as, uint32_t bs, int tid) const {
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
      int idx = tid + n * NT;
      int r = idx / CPR, c = idx % CPR;
      uint32_t off = r * (D * 2) + ((c ^ SwzX<D>::f(r)) << 4);
      lds_write_b128(as + off, areg[n]);
      lds_write_b128(bs + off, breg[n]);
    }
  }
};

// Per-lane LDS byte offsets into a SwzX tile.
template <int D>
struct TileOffsets {
  static constexpr int KD = D / 16, DT = D / 32;
  uint32_t row[KD];     // row-wise A operand: row kappa(l32), chunk 2kk+h
  uint32_t tr[DT][2];   // transposing read: rows 8h + 4rd + i16/4 (+16ks +32ck), cols 32dt + ...
  __device__ __forceinline__ void init(int lane) {
    const int l32 = lane & 31, h = lane >> 5, i16 = lane & 15, blk1 = (lane >> 4) & 1;
    const int kap = kappa(l32);
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) row[kk] = kap * (D * 2) + (((2 * kk + h) ^ SwzX<D>::f(kap)) << 4);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int rd = 0; rd < 2; ++rd) {
        int r = 8 * h + 4 * rd + (i16 >> 2);
        int c = 4 * dt + 2 * blk1 + ((i16 & 3) >> 1);
        tr[dt][rd] = r * (D * 2) + ((c ^ SwzX<D>::f(r)) << 4) + ((i16 & 1) << 3);
      }
  }
};

// sigmoid(t) and t-derivative factor for 16 accumulator registers.
//   u = -(t) log2 e, e = 2^u, p = 1/(1+e)
// `dist0` / `dstep` give |i-j| for ALiBi: distance of register r is |dist0 + dstep*key_of_reg(r)|.
template <bool ALIBI>
__device__ __forceinline__ void sigmoid16(const f32x16& s, float* pr, float nscale, float nbias, float sl2, float dist0,
                                          float dstep) {
  if (ALIBI) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float dist = dist0 + dstep * (float)key_of_reg(r);
      float w = __builtin_fmaf(sl2, __builtin_fabsf(dist), nbias);
      pr[r] = __builtin_fmaf(s[r], nscale, w);
    }
  } else {
#pragma unroll
    for (int r = 0; r < 16; ++r) pr[r] = __builtin_fmaf(s[r], nscale, nbias);
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) pr[r] = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(pr[r]));
}

// softmax probabilities from saved row statistics: p = 2^(s*scale_log2 - slope|i-j|log2e - lse*log2e).
// `nlse` holds -lse*log2(e) per register (dkdv kernel) or one value for the lane (dq kernel).
template <bool ALIBI, bool PER_REG>
__device__ __forceinline__ void softmax16(const f32x16& s, float* pr, float scale_log2, float sl2, float dist0,
                                          float dstep, const float* nlse) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float w = PER_REG ? nlse[r] : nlse[0];
    if (ALIBI) {
      float dist = dist0 + dstep * (float)key_of_reg(r);
      w = __builtin_fmaf(-sl2, __builtin_fabsf(dist), w);
    }
    pr[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], scale_log2, w));
  }
}

__device__ __forceinline__ bf16x8 pack8(const float* x) {
  u32x4 w;
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = pack_bf16(x[2 * i], x[2 * i + 1]);
  return as_bf16x8(w);
}

// ------------------------------------------------------------------ dQ kernel
template <int D, int BC, int NW, bool CAUSAL, bool ALIBI, bool SOFTMAX>
__global__ void __launch_bounds__(64 * NW, 2)
attn_bwd_dq_kernel(const BwdParams p) {
  constexpr int NT = 64 * NW, BR = 32 * NW, KD = D / 16, DT = D / 32, NCK = BC / 32;
  constexpr int TILE = BC * D * 2;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(SATTN_LDS(char)*)smem;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int total = p.n_blocks * p.B * p.H;
  const int logical = xcd_remap(blockIdx.x, total);
  const int bh = logical / p.n_blocks;
  const int qb = CAUSAL ? (p.n_blocks - 1 - logical % p.n_blocks) : (logical % p.n_blocks);
  const int b = bh / p.H, hd = bh % p.H, N = p.N;

  const __bf16* qbase = (const __bf16*)p.q.ptr + b * p.q.sb + hd * p.q.sh;
  const __bf16* kbase = (const __bf16*)p.k.ptr + b * p.k.sb + hd * p.k.sh;
  const __bf16* vbase = (const __bf16*)p.v.ptr + b * p.v.sb + hd * p.v.sh;
  const __bf16* dobase = (const __bf16*)p.dout.ptr + b * p.dout.sb + hd * p.dout.sh;
  __bf16* dqbase = (__bf16*)p.dq.ptr + b * p.dq.sb + hd * p.dq.sh;

  const int q_wave0 = qb * BR + wave * 32, qi = q_wave0 + l32, qi_ld = qi < N ? qi : N - 1;
  bf16x8 qf[KD], dof[KD];
#pragma unroll
  for (int kk = 0; kk < KD; ++kk) {
    qf[kk] = as_bf16x8(*(const u32x4*)(qbase + (int64_t)qi_ld * p.q.ss + 16 * kk + 8 * h));
    dof[kk] = as_bf16x8(*(const u32x4*)(dobase + (int64_t)qi_ld * p.dout.ss + 16 * kk + 8 * h));
  }
  f32x16 acc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[dt][r] = 0.f;

  TileOffsets<D> off;
  off.init(lane);
  float sl2 = 0.f;
  if (ALIBI) sl2 = p.slopes[hd] * kLog2e;
  float nlse_q = 0.f, d_q = 0.f;  // softmax: this lane's query statistics
  if (SOFTMAX) {
    nlse_q = -p.lse[(int64_t)bh * N + qi_ld] * kLog2e;
    d_q = p.dvec[(int64_t)bh * N + qi_ld];
  }

  const int q_hi = (qb * BR + BR < N ? qb * BR + BR : N) - 1;
  const int kv_len = CAUSAL ? (q_hi + 1) : N;
  const int n_tiles = (kv_len + BC - 1) / BC;

  PairStager<D, BC, NT> st;
  st.load(kbase, vbase, p.k.ss, p.v.ss, 0, N, tid);
  st.store(lds0, lds0 + TILE, tid);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): stationary fragments are in registers before the loop
  __syncthreads();

  for (int jt = 0; jt < n_tiles; ++jt) {
    const int j0 = jt * BC;
    const uint32_t ks = lds0 + (jt & 1) * (2 * TILE), vs = ks + TILE;
    const bool more = jt + 1 < n_tiles;
    if (more) st.load(kbase, vbase, p.k.ss, p.v.ss, j0 + BC, N, tid);
#pragma unroll
    for (int ck = 0; ck < NCK; ++ck) {
      const int jc = j0 + 32 * ck;
      if (jc >= N) break;
      if (CAUSAL && jc > q_wave0 + 31) break;
      const uint32_t cko = ck * 32 * (D * 2);
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < KD; ++kk) {
        s = mfma32(as_bf16x8(lds_read_b128(ks + cko + off.row[kk])), qf[kk], s);
        dp = mfma32(as_bf16x8(lds_read_b128(vs + cko + off.row[kk])), dof[kk], dp);
      }
      const int jl = jc + 8 * h;
      float pr[16];
      float ds[16];
      if (SOFTMAX) {
        softmax16<ALIBI, false>(s, pr, -p.nscale_log2, sl2, (float)(qi - jl), -1.0f, &nlse_q);
#pragma unroll
        for (int r = 0; r < 16; ++r) ds[r] = pr[r] * (dp[r] - d_q);
      } else {
        sigmoid16<ALIBI>(s, pr, p.nscale_log2, p.nbias_log2, sl2, (float)(qi - jl), -1.0f);
#pragma unroll
        for (int r = 0; r < 16; ++r) ds[r] = pr[r] * (1.0f - pr[r]) * dp[r];
      }
      if ((jc + 31 >= N) || (CAUSAL && jc + 31 > q_wave0)) {
        int lim = N - 1 - jl;
        if (CAUSAL) lim = lim < qi - jl ? lim : qi - jl;
#pragma unroll
        for (int r = 0; r < 16; ++r) ds[r] = key_of_reg(r) <= lim ? ds[r] : 0.f;
      }
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2) {
        bf16x8 dsb = pack8(ds + 8 * ks2);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          uint32_t a0 = ks + cko + ks2 * 16 * (D * 2);
          bf16x8 a = join_tr(lds_read_tr16(a0 + off.tr[dt][0]), lds_read_tr16(a0 + off.tr[dt][1]));
          acc[dt] = mfma32(a, dsb, acc[dt]);
        }
      }
    }
    if (more) st.store(lds0 + ((jt + 1) & 1) * (2 * TILE), lds0 + ((jt + 1) & 1) * (2 * TILE) + TILE, tid);
    __syncthreads();
  }
  if (qi < N) {
    __bf16* row = dqbase + (int64_t)qi * p.dq.ss;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w;
        w[0] = pack_bf16(acc[dt][4 * g] * p.inv_sqrt_d, acc[dt][4 * g + 1] * p.inv_sqrt_d);
        w[1] = pack_bf16(acc[dt][4 * g + 2] * p.inv_sqrt_d, acc[dt][4 * g + 3] * p.inv_sqrt_d);
        *(u32x2*)(row + 32 * dt + 8 * g + 4 * h) = w;
      }
  }
}

// ------------------------------------------------------------------ dK/dV kernel
template <int D, int BQ, int NW, bool CAUSAL, bool ALIBI, bool SOFTMAX>
__global__ void __launch_bounds__(64 * NW, 1)
attn_bwd_dkdv_kernel(const BwdParams p) {
  constexpr int NT = 64 * NW, BK = 32 * NW, KD = D / 16, DT = D / 32, NCK = BQ / 32;
  constexpr int TILE = BQ * D * 2;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(SATTN_LDS(char)*)smem;
  // softmax: per-query statistics of the staged tile, [stage][0: -lse*log2e | 1: D][BQ]
  SATTN_LDS(float)* stat = (SATTN_LDS(float)*)(smem + 4 * TILE);
  static_assert(NT >= 2 * BQ, "statistics are staged by the first 2*BQ threads");

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int total = p.n_blocks * p.B * p.H;
  const int logical = xcd_remap(blockIdx.x, total);
  const int bh = logical / p.n_blocks;
  const int kb = logical % p.n_blocks;  // causal: early key blocks are the heavy ones and come first
  const int b = bh / p.H, hd = bh % p.H, N = p.N;

  const __bf16* qbase = (const __bf16*)p.q.ptr + b * p.q.sb + hd * p.q.sh;
  const __bf16* kbase = (const __bf16*)p.k.ptr + b * p.k.sb + hd * p.k.sh;
  const __bf16* vbase = (const __bf16*)p.v.ptr + b * p.v.sb + hd * p.v.sh;
  const __bf16* dobase = (const __bf16*)p.dout.ptr + b * p.dout.sb + hd * p.dout.sh;
  __bf16* dkbase = (__bf16*)p.dk.ptr + b * p.dk.sb + hd * p.dk.sh;
  __bf16* dvbase = (__bf16*)p.dv.ptr + b * p.dv.sb + hd * p.dv.sh;

  const int k_wave0 = kb * BK + wave * 32, kj = k_wave0 + l32, kj_ld = kj < N ? kj : N - 1;
  // K and V fragments: B operands (column = key, k = d)
  bf16x8 kf[KD], vf[KD];
#pragma unroll
  for (int kk = 0; kk < KD; ++kk) {
    kf[kk] = as_bf16x8(*(const u32x4*)(kbase + (int64_t)kj_ld * p.k.ss + 16 * kk + 8 * h));
    vf[kk] = as_bf16x8(*(const u32x4*)(vbase + (int64_t)kj_ld * p.v.ss + 16 * kk + 8 * h));
  }
  f32x16 dkacc[DT], dvacc[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dkacc[dt][r] = 0.f; dvacc[dt][r] = 0.f; }

  TileOffsets<D> off;
  off.init(lane);
  float sl2 = 0.f;
  if (ALIBI) sl2 = p.slopes[hd] * kLog2e;

  const int it0 = CAUSAL ? (kb * BK) / BQ : 0;  // first query tile that can see this key block
  const int n_tiles = (N + BQ - 1) / BQ;

  PairStager<D, BQ, NT> st;
  float statreg = 0.f;
  auto load_stat = [&](int i0) {
    if (SOFTMAX && tid < 2 * BQ) {
      int row = i0 + (tid & (BQ - 1));
      row = row < N ? row : N - 1;
      statreg = tid < BQ ? -p.lse[(int64_t)bh * N + row] * kLog2e : p.dvec[(int64_t)bh * N + row];
    }
  };
  auto store_stat = [&](int stage) {
    if (SOFTMAX && tid < 2 * BQ) stat[stage * 2 * BQ + tid] = statreg;
  };
  if (it0 < n_tiles) {
    st.load(qbase, dobase, p.q.ss, p.dout.ss, it0 * BQ, N, tid);
    load_stat(it0 * BQ);
    st.store(lds0 + (it0 & 1) * (2 * TILE), lds0 + (it0 & 1) * (2 * TILE) + TILE, tid);
    store_stat(it0 & 1);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): stationary fragments are in registers before the loop
  __syncthreads();

  for (int it = it0; it < n_tiles; ++it) {
    const int i0 = it * BQ;
    const uint32_t qs = lds0 + (it & 1) * (2 * TILE), dos = qs + TILE;
    const bool more = it + 1 < n_tiles;
    if (more) {
      st.load(qbase, dobase, p.q.ss, p.dout.ss, i0 + BQ, N, tid);
      load_stat(i0 + BQ);
    }
#pragma unroll
    for (int ck = 0; ck < NCK; ++ck) {
      const int ic = i0 + 32 * ck;  // first query row of the chunk
      if (ic >= N) break;
      if (CAUSAL && ic + 31 < k_wave0) continue;  // every query of the chunk precedes every key of the wave
      const uint32_t cko = ck * 32 * (D * 2);
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < KD; ++kk) {
        s = mfma32(as_bf16x8(lds_read_b128(qs + cko + off.row[kk])), kf[kk], s);
        dp = mfma32(as_bf16x8(lds_read_b128(dos + cko + off.row[kk])), vf[kk], dp);
      }
      const int il = ic + 8 * h;  // query row of register 0 for this lane half
      float pr[16];
      float dq_r[16];  // softmax: D of the query held by register r
      if (SOFTMAX) {
        float nl[16];
        const SATTN_LDS(float)* sl = stat + (it & 1) * 2 * BQ + 32 * ck + 8 * h;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          nl[r] = sl[key_of_reg(r)];
          dq_r[r] = sl[BQ + key_of_reg(r)];
        }
        softmax16<ALIBI, true>(s, pr, -p.nscale_log2, sl2, (float)(il - kj), 1.0f, nl);
      } else {
        sigmoid16<ALIBI>(s, pr, p.nscale_log2, p.nbias_log2, sl2, (float)(il - kj), 1.0f);
      }
      if ((ic + 31 >= N) || (CAUSAL && ic < k_wave0 + 31)) {
        // keep rows il + key_of_reg(r) in [max(kj, .), N-1]
        const int hi = N - 1 - il;
        const int lo = CAUSAL ? kj - il : -1000000;
#pragma unroll
        for (int r = 0; r < 16; ++r) pr[r] = (key_of_reg(r) <= hi && key_of_reg(r) >= lo) ? pr[r] : 0.f;
      }
      float ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) ds[r] = SOFTMAX ? pr[r] * (dp[r] - dq_r[r]) : pr[r] * (1.0f - pr[r]) * dp[r];
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2) {
        bf16x8 pb = pack8(pr + 8 * ks2), dsb = pack8(ds + 8 * ks2);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          uint32_t a0 = cko + ks2 * 16 * (D * 2);
          bf16x8 ado = join_tr(lds_read_tr16(dos + a0 + off.tr[dt][0]), lds_read_tr16(dos + a0 + off.tr[dt][1]));
          dvacc[dt] = mfma32(ado, pb, dvacc[dt]);
          bf16x8 aq = join_tr(lds_read_tr16(qs + a0 + off.tr[dt][0]), lds_read_tr16(qs + a0 + off.tr[dt][1]));
          dkacc[dt] = mfma32(aq, dsb, dkacc[dt]);
        }
      }
    }
    if (more) {
      st.store(lds0 + ((it + 1) & 1) * (2 * TILE), lds0 + ((it + 1) & 1) * (2 * TILE) + TILE, tid);
      store_stat((it + 1) & 1);
    }
    __syncthreads();
  }
  if (kj < N) {
    __bf16* krow = dkbase + (int64_t)kj * p.dk.ss;
    __bf16* vrow = dvbase + (int64_t)kj * p.dv.ss;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w;
        w[0] = pack_bf16(dkacc[dt][4 * g] * p.inv_sqrt_d, dkacc[dt][4 * g + 1] * p.inv_sqrt_d);
        w[1] = pack_bf16(dkacc[dt][4 * g + 2] * p.inv_sqrt_d, dkacc[dt][4 * g + 3] * p.inv_sqrt_d);
        *(u32x2*)(krow + 32 * dt + 8 * g + 4 * h) = w;
        w[0] = pack_bf16(dvacc[dt][4 * g], dvacc[dt][4 * g + 1]);
        w[1] = pack_bf16(dvacc[dt][4 * g + 2], dvacc[dt][4 * g + 3]);
        *(u32x2*)(vrow + 32 * dt + 8 * g + 4 * h) = w;
      }
  }
}

// D_i = sum_t dO[i][t] * O[i][t] (fp32), the row term of the softmax backward.  16 lanes per
// row, 8 elements per lane and pass.
template <int D>
__global__ void __launch_bounds__(256)
rowsum_do_o_kernel(TensorRef o, TensorRef dout, float* dvec, int B, int H, int N) {
  const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int sub = threadIdx.x & 15;
  const int64_t rows = (int64_t)B * H * N;
  float acc = 0.f;
  if (row < rows) {
    const int64_t bh = row / N;
    const int i = (int)(row % N);
    const int b = (int)(bh / H), hd = (int)(bh % H);
    const __bf16* op = (const __bf16*)o.ptr + b * o.sb + hd * o.sh + (int64_t)i * o.ss;
    const __bf16* dp = (const __bf16*)dout.ptr + b * dout.sb + hd * dout.sh + (int64_t)i * dout.ss;
#pragma unroll
    for (int c = sub * 8; c < D; c += 128) {
      bf16x8 a = as_bf16x8(*(const u32x4*)(op + c));
      bf16x8 g = as_bf16x8(*(const u32x4*)(dp + c));
#pragma unroll
      for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)g[e];
    }
  }
#pragma unroll
  for (int m = 8; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 16);
  if (row < rows && sub == 0) dvec[row] = acc;
}

}  // namespace sattn
