// Fused sigmoid-attention forward for gfx950 (Algorithm 1 of the paper's Appendix F.1),
// bf16 operands, fp32 logits / sigmoid / accumulation.
//
// Work split: one workgroup = NW waves, each wave owns 32 query rows (B_r = 32*NW); the
// workgroup streams K/V tiles of 64 keys through LDS (three K slots, three V slots) with
// direct-to-LDS loads issued two tiles ahead.
// Per 32-key chunk c a wave computes
//     S^T (32 keys x 32 queries) = K_c Q_i^T               8 (d=128) MFMA 32x32x16
//     P^T = sigmoid(S^T / sqrt(d) + b [+ ALiBi])            fp32 VALU, no row max / row sum
//     O_i^T (d x 32 queries)    += V_c^T P^T                8 MFMA, V read with the
//                                                           transposing LDS load
// Computing the transposed products lets the S^T accumulator registers be used, after the
// bf16 round, as the B operand of the second product with no cross-lane traffic.
//
// The three stages are software-pipelined inside each wave: step c issues the MFMAs of
// S^T(c+1) and of the O^T update with P^T(c-1) while the VALU evaluates sigmoid(c), and
// refills each operand fragment from LDS (K(c+2), V(c)) right after the MFMA that consumed
// it, a full step before its next use.  Matrix and vector pipes are fed from one
// instruction stream whose order is pinned with scheduling barriers.
#pragma once
#include "sattn_common.hpp"

namespace sattn {

struct FwdParams {
  TensorRef q, k, v, o;
  const float* slopes;  // [H] or nullptr
  float* lse;           // softmax only: [B,H,N]
  int B, H, N;
  int n_qblocks;
  int head_group;     // causal: heads walked abreast in the dispatch order (head_and_rank); 1 otherwise
  float nscale_log2;  // -log2(e)/sqrt(d)   (softmax: +log2(e)/sqrt(d))
  float nbias_log2;   // -b*log2(e)
  // variable-length batches (nullptr otherwise): sequence b owns tokens cu_seqlens[b] ..
  // cu_seqlens[b+1]-1 of the packed [tokens, H, d] tensors (batch stride 0); N is then the
  // longest length the grid covers; bias_vec, if given, holds one bias per sequence
  const int* cu_seqlens;
  const float* bias_vec;
  // shared key/value heads: query head h reads K/V head h / kv_group (1 = one per query head)
  int kv_group;
  // number of keys when it differs from the number of queries N (0: same)
  int Nk;
  // position of query 0 on the key axis (Nk - N when the queries are the last N positions of the
  // key sequence, else 0): the causal mask keeps key j for query i iff j <= i + qoff, and ALiBi
  // measures |i + qoff - j|.  A multiple of 32 in these kernels (a wave's query rows and a key
  // chunk then still meet in one diagonal chunk).
  int qoff;
  // 64-row causal kernel: every workgroup handles two query blocks of its head, the r-th longest
  // and the r-th shortest (n_qblocks even), so that all workgroups of a launch do the same work
  int pair;
  ClockProbe clock;  // measurement aid, {nullptr, 0} otherwise
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

// Stage one tile (BC x D bf16) global -> LDS with the direct-to-LDS load: no staging
// registers, no LDS write instructions.  One wave-level instruction moves 64 x 16 bytes to
// 1 KB of LDS at M0 + 16*lane, so the XOR swizzle is applied on the global side: the lane
// that fills physical chunk pc of row r fetches logical chunk pc ^ swz(r).  Completion is
// tracked by hand (vmcnt), the compiler never sees these loads.
template <int D, int BC, int NW, bool IS_V>
struct DmaStager {
  static constexpr int CPR = D / 8;               // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;            // rows filled by one instruction
  static constexpr int NI = (BC * CPR) / (64 * NW);  // instructions per wave per tile
  static_assert((BC * CPR) % (64 * NW) == 0, "tile must split evenly over the waves");
  const char* base;       // first row of the next tile to stage (wave-uniform, advances per tile)
  const char* base_last;  // row N-1 (wave-uniform)
  // This lane's byte offset inside a tile for instruction n is
  //   row_of(n) * row_bytes + col_bytes(n) = (rowoff0 + n * RPI * row_bytes) + (col0 ^ XCOL * n'):
  // successive instructions of a wave move RPI rows down, which flips swizzle bits that no
  // lane-dependent term touches, so two registers describe all NI offsets; the row step goes
  // into the scalar base.
  uint32_t rowoff0, col0;
  uint32_t tile_bytes, row_bytes;
  int j0;                 // first key of the next tile to stage
  __device__ __forceinline__ static int row_of(int n, int wave, int lane) { return (wave * NI + n) * RPI + lane / CPR; }
  __device__ __forceinline__ static uint32_t col_bytes(int n, int wave, int lane) {
    const int r = row_of(n, wave, lane);
    return (uint32_t)(((lane % CPR) ^ (IS_V ? Swz<D>::v(r) : Swz<D>::k(r))) * 16);
  }
  // col_bytes(n) ^ col_bytes(0): the K swizzle takes row bits 0..3 (D = 128) or 1..3 (D = 64),
  // instruction n adds n * RPI = 4n (8n) to the row; the V swizzle only takes bits the lane sets.
  __host__ __device__ static constexpr uint32_t xcol(int n) {
    return IS_V ? 0u : (uint32_t)((D == 128 ? (4 * n) & 15 : (4 * n) & 7) << 4);
  }
  static_assert(IS_V || (D == 128 ? 4 * (NI - 1) < 16 && (NI * RPI) % 8 == 0 : NI <= 2), "row step must stay inside the swizzle field");
  // The host side guarantees that one (batch, head) slice spans < 4 GiB.
  __device__ __forceinline__ void init(const __bf16* b, int64_t ss, int N, int wave, int lane) {
    base = (const char*)b;
    base_last = (const char*)(b + (int64_t)(N - 1) * ss);
    row_bytes = (uint32_t)(ss * 2);
    tile_bytes = BC * row_bytes;
    j0 = 0;
    rowoff0 = row_of(0, wave, lane) * row_bytes;
    col0 = col_bytes(0, wave, lane);
  }
  __device__ __forceinline__ static void load(uint32_t o, const char* sbase, uint32_t m0v) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(o), "s"(sbase), "s"(m0v) : "memory");
  }
  // Same with the lane offset (c ^ X) + r formed in place, so that it never occupies a register
  // between tiles.  The instruction offset moves the LDS target and the global address alike:
  // the NI loads of a wave (consecutive 1 KB pieces) share the M0 value set by the first one
  // and carry 1024 * n in their offset field, which the scalar base takes out again.  M0 is
  // not otherwise used in these kernels (checked on the generated assembly by isa_check.py).
  template <uint32_t X, int n>
  __device__ __forceinline__ static void load_xad(uint32_t c, uint32_t r, const char* sbase, uint32_t m0v) {
    uint32_t t;
    if constexpr (n == 0)
      asm volatile("v_xad_u32 %0, %1, %2, %3\n\ts_mov_b32 m0, %5\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %4"
                   : "=&v"(t) : "v"(c), "s"(X), "v"(r), "s"(sbase), "s"(m0v) : "memory");
    else
      asm volatile("v_xad_u32 %0, %1, %2, %3\n\tglobal_load_lds_dwordx4 %0, %4 offset:%5"
                   : "=&v"(t) : "v"(c), "s"(X), "v"(r), "s"(sbase), "n"(1024 * n) : "memory");
  }
  static_assert(NI * 1024 <= 4096 && RPI * D * 2 >= 1024, "offset field of the load: 0 .. 4095, never below the row step");
  template <int n>
  __device__ __forceinline__ void issue_full(uint32_t lds, int wave) const {
    if constexpr (n < NI) {
      load_xad<xcol(n), n>(col0, rowoff0, base + (uint32_t)n * (RPI * row_bytes - 1024), lds + wave * NI * 1024);
      issue_full<n + 1>(lds, wave);
    }
  }
  // The same staging one instruction at a time, for a tile that lies wholly inside the tensor
  // (for interleaving with a pinned step).  lane_off(n) is this lane's complete byte offset for
  // instruction n relative to `base` (the instruction's own offset field, which moves the
  // global address along with the LDS target, already taken out), so that all NI loads share
  // one scalar base; the caller keeps the NI values in registers and calls issue_off<n> for
  // n = 0 .. NI-1 in this order with no other staging in between (n = 0 sets M0 for all of
  // them: lds_wave = the wave's first 1 KB piece of the LDS tile), then advance().
  __device__ __forceinline__ uint32_t lane_off(int n) const {
    return (col0 ^ xcol(n)) + rowoff0 + (uint32_t)n * (RPI * row_bytes - 1024);
  }
  template <int n>
  __device__ __forceinline__ static void issue_off(uint32_t off, const char* sbase, uint32_t lds_wave) {
    if constexpr (n == 0)
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(off), "s"(sbase), "s"(lds_wave) : "memory");
    else
      asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" : : "v"(off), "s"(sbase), "n"(1024 * n) : "memory");
  }
  __device__ __forceinline__ void advance() { base += tile_bytes; j0 += BC; }
  // Issue the loads of the next tile into the LDS tile at byte address `lds` (wave-uniform)
  // and advance.  Rows past the end re-read row N-1.
  __device__ __forceinline__ void issue(uint32_t lds, int N, int wave, int lane) {
    if (j0 + BC <= N) {
      issue_full<0>(lds, wave);
    } else if (j0 < N) {
      const uint32_t to_last = (uint32_t)(N - 1 - j0) * row_bytes;
#pragma unroll
      for (int n = 0; n < NI; ++n) {
        const int r = row_of(n, wave, lane);
        const uint32_t o = (j0 + r < N ? r * row_bytes : to_last) + col_bytes(n, wave, lane);
        load(o, base, lds + (wave * NI + n) * 1024);
      }
    } else {
#pragma unroll
      for (int n = 0; n < NI; ++n) load(col_bytes(n, wave, lane), base_last, lds + (wave * NI + n) * 1024);
    }
    base += tile_bytes;
    j0 += BC;
  }
};

// Running row statistics of the softmax comparison kernel (log2 units), one query per lane.
struct SoftmaxState {
  float m;  // running maximum of the scaled logits
  float l;  // this lane half's partial sum of 2^(x - m)
};

// Per-wave state of the forward pipeline.
template <int D>
struct FwdWave {
  static constexpr int KD = D / 16, DT = D / 32;
  uint32_t koff[KD];   // LDS byte address of this lane's K fragment kk in (slot 0, chunk 0)
  uint32_t voff[DT];   // LDS byte address of this lane's V fragment dt in (slot 0, chunk 0, ks 0, rd 0)
  bf16x8 qf[KD];       // Q fragment (B operand of S^T)
  bf16x8 kf[KD];       // K fragments of the chunk whose S^T is computed next
  bf16x8 vf[2 * DT];   // V fragments of the chunk whose P^T is consumed next
  f32x16 oacc[DT];     // O^T accumulator
  f32x16 s[2];         // S^T of chunk c in s[c&1]
  f32x16 cinit;        // FOLD: initial value of every S^T accumulator (the key term of causal ALiBi)
  bf16x8 p[2][2];      // bf16 P^T of chunk c in p[c&1][ks]
  SoftmaxState sm;
  int qi, h;
  float nscale, nbias, sl2;
};

enum StepKind { STEP_FULL = 0, STEP_LAST = 1, STEP_TAIL = 2 };

// One pipeline step for chunk c (PAR = c & 1).
//   FULL: S^T(c+1) MFMAs + refill kf with K(c+2); sigmoid(c); O^T += V(c-1)^T P^T(c-1) + refill vf with V(c)
//   LAST: the wave's last chunk (diagonal / ragged end): no S^T; masked sigmoid(c); O^T update; refill vf
//   TAIL: only the O^T update with P^T(c-1)
// kaddr: byte offset (compile-time) of K chunk c+2 inside LDS; vaddr: of V chunk c.
//
// FOLD (sigmoid, causal, ALiBi): every unmasked key lies at or before its query, so the
// ALiBi term slope*(i - j) splits into a per-lane, per-step part slope*(i - jc - 8h), added
// to the bias with one fma per step, and a per-register part -slope*key_of_reg(r), which is
// a constant of the kernel and goes into the accumulators as the initial value of S^T
// (divided by the logit scale).  The sigmoid then costs what it costs without ALiBi.
template <int D, bool ALIBI, bool SOFTMAX, int KIND, int PAR, bool FOLD = false>
__device__ __forceinline__ void fwd_step(FwdWave<D>& W, uint32_t kaddr, uint32_t vaddr, int jc, int N, bool causal) {
  constexpr int KD = D / 16, DT = D / 32;
  constexpr int NM = KD;  // == 2*DT
  static_assert(KD == 2 * DT, "one S^T MFMA pairs with one O^T MFMA");
  constexpr int EPS = 16 / NM;  // sigmoid elements evaluated per MFMA pair
  constexpr bool QK = KIND == STEP_FULL, SIG = KIND != STEP_TAIL;
  f32x16& s_cur = W.s[PAR];
  f32x16& s_nxt = W.s[PAR ^ 1];
  bf16x8* p_cur = W.p[PAR];
  const bf16x8* p_prv = W.p[PAR ^ 1];

  float pr[16];
  float alpha = 1.0f;
  const int jl = jc + 8 * W.h;  // key held by register 0 of this lane half
  if (SIG && SOFTMAX) {
    // x = (s/sqrt(d) - slope|i-j|) log2(e); masked keys -> -inf.  Under the causal mask every
    // kept key has i - j >= 0: the term splits into one constant of the lane and step and a
    // multiple of the register's key offset (a masked key gets -inf below whatever this gives).
    const bool split = ALIBI && causal;
    const float wstep = split ? -W.sl2 * (float)(W.qi - jl) : 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float x = __builtin_fmaf(s_cur[r], W.nscale, wstep);
      if (split) x = __builtin_fmaf(W.sl2, (float)key_of_reg(r), x);
      else if (ALIBI) x = __builtin_fmaf(-W.sl2, __builtin_fabsf((float)(W.qi - jl) - (float)key_of_reg(r)), x);
      pr[r] = x;
    }
    if (KIND == STEP_LAST) {
      int lim2 = N - 1 - jl;
      if (causal) lim2 = lim2 < W.qi - jl ? lim2 : W.qi - jl;
#pragma unroll
      for (int r = 0; r < 16; ++r) pr[r] = key_of_reg(r) <= lim2 ? pr[r] : -__builtin_inff();
    }
    float mx = pr[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = __builtin_fmaxf(mx, pr[r]);
    mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));  // the other half of this query's keys
    const float m_new = __builtin_fmaxf(W.sm.m, mx);
    alpha = __builtin_amdgcn_exp2f(W.sm.m - m_new);
    W.sm.m = m_new;
#pragma unroll
    for (int r = 0; r < 16; ++r) pr[r] -= m_new;
  }
  float dist0 = 0.f;
  if (SIG && !SOFTMAX && ALIBI) dist0 = (float)(W.qi - jl);
  const float wfold = FOLD ? __builtin_fmaf(W.sl2, dist0, W.nbias) : W.nbias;
  int lim = N - 1 - jl;  // STEP_LAST: registers whose key offset exceeds lim are masked
  if (causal) lim = lim < W.qi - jl ? lim : W.qi - jl;
  u32x4 pw = {0, 0, 0, 0};

  if (QK) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s_nxt[r] = FOLD ? W.cinit[r] : 0.f;
  }
#pragma unroll
  for (int m = 0; m < NM; ++m) {
    // ---- sub-slot A: S^T MFMA, refill its K fragment, first half of two sigmoids
    if (QK) {
      s_nxt = mfma32(W.kf[m], W.qf[m], s_nxt);
      W.kf[m] = as_bf16x8(lds_read_b128(W.koff[m] + kaddr));
    }
    if (SIG && !SOFTMAX) {
      // p = 1 / (1 + 2^u), u = -(s/sqrt(d) + b - slope|i-j|) log2(e)
#pragma unroll
      for (int r = EPS * m; r < EPS * m + EPS; ++r) {
        float w = wfold;
        if (ALIBI && !FOLD) w = __builtin_fmaf(W.sl2, __builtin_fabsf(dist0 - (float)key_of_reg(r)), W.nbias);
        pr[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[r], W.nscale, w));
      }
    }
    if (SIG && SOFTMAX) {
#pragma unroll
      for (int r = EPS * m; r < EPS * m + EPS; ++r) pr[r] = __builtin_amdgcn_exp2f(pr[r]);
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- sub-slot B: O^T MFMA, refill its V fragment, second half of the two sigmoids
    W.oacc[m % DT] = mfma32(W.vf[m], p_prv[m / DT], W.oacc[m % DT]);
    if (SIG) {
      const uint32_t a0 = W.voff[m % DT] + vaddr + (m / DT) * 16 * (D * 2);
      W.vf[m] = join_tr(lds_read_tr16(a0), lds_read_tr16(a0 + 4 * (D * 2)));
    }
    if (SIG && !SOFTMAX) {
#pragma unroll
      for (int r = EPS * m; r < EPS * m + EPS; ++r) {
        pr[r] = __builtin_amdgcn_rcpf(1.0f + pr[r]);
        if (KIND == STEP_LAST) pr[r] = key_of_reg(r) <= lim ? pr[r] : 0.f;
      }
      // registers 8ks..8ks+7 form the P^T operand of contraction step ks
#pragma unroll
      for (int r = EPS * m; r < EPS * m + EPS; r += 2) {
        pw[(r & 7) >> 1] = pack_bf16(pr[r], pr[r + 1]);
        if ((r & 7) == 6) p_cur[r >> 3] = as_bf16x8(pw);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  if (SIG && SOFTMAX) {
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += pr[r];
    W.sm.l = __builtin_fmaf(W.sm.l, alpha, sum);
    // O^T holds sums relative to the previous maximum: rescale only when some maximum moved
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) W.oacc[dt][r] *= alpha;
    }
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
#pragma unroll
      for (int w = 0; w < 4; ++w) pw[w] = pack_bf16(pr[8 * ks2 + 2 * w], pr[8 * ks2 + 2 * w + 1]);
      p_cur[ks2] = as_bf16x8(pw);
    }
  }
}

// ---- The steady-state step with a hand-pinned instruction order.
// Every instruction below is a volatile asm statement, which the compiler neither reorders
// nor drops, so the stream that reaches the SIMD is exactly: one MFMA, one fragment refill
// from LDS, then a slice of the sigmoid whose dependent operations sit a full slice apart.
// (The compiler still allocates registers and inserts the LDS wait counts: the refills are
// ordinary loads.)  The MFMA asm carries a memory clobber to keep those loads in place.
__device__ __forceinline__ void a_mfma(f32x16& c, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b) : "memory");
}
__device__ __forceinline__ void a_mfma_zero(f32x16& c, const bf16x8& a, const bf16x8& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(c) : "v"(a), "v"(b) : "memory");
}

__device__ __forceinline__ void a_mfma_init(f32x16& c, const bf16x8& a, const bf16x8& b, const f32x16& init) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(c) : "v"(a), "v"(b), "v"(init) : "memory");
}

// Sigmoid of the 16 accumulator registers as 4 groups x 18 operations.  Inside a group of
// four elements the order is F F F F  X X X X  A A A A  R R R R  C C (scale+bias fma, exp2,
// 1+e, reciprocal, bf16 pack), so a result is consumed four instructions after it was issued.
template <int D, bool ALIBI, int I>
__device__ __forceinline__ void sig_op(const FwdWave<D>& W, const f32x16& s, float (&u)[16], uint32_t (&wp)[8],
                                       float nbias_v, float sl2_v, float dist0) {
  constexpr int G = I / 18, i = I % 18, e = 4 * G + (i & 3);
  if constexpr (i < 4) {
    if constexpr (ALIBI) {
      float t, w;
      const float keyf = (float)key_of_reg(e);
      asm volatile("v_sub_f32 %0, %1, %2" : "=v"(t) : "v"(dist0), "v"(keyf));
      asm volatile("v_fma_f32 %0, %1, |%2|, %3" : "=v"(w) : "v"(sl2_v), "v"(t), "v"(nbias_v));
      asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(u[e]) : "v"(s[e]), "s"(W.nscale), "v"(w));
    } else {
      asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(u[e]) : "v"(s[e]), "s"(W.nscale), "v"(nbias_v));
    }
  } else if constexpr (i < 8) {
    asm volatile("v_exp_f32 %0, %0" : "+v"(u[e]));
  } else if constexpr (i < 12) {
    asm volatile("v_add_f32 %0, 1.0, %0" : "+v"(u[e]));
  } else if constexpr (i < 16) {
    asm volatile("v_rcp_f32 %0, %0" : "+v"(u[e]));
  } else {
    constexpr int j = 2 * G + (i - 16);  // word j packs elements 2j, 2j+1
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(wp[j]) : "v"(u[2 * j]), "v"(u[2 * j + 1]));
  }
}
template <int D, bool ALIBI, int LO, int HI>
__device__ __forceinline__ void sig_ops(const FwdWave<D>& W, const f32x16& s, float (&u)[16], uint32_t (&wp)[8],
                                        float nbias_v, float sl2_v, float dist0) {
  if constexpr (LO < HI) {
    sig_op<D, ALIBI, LO>(W, s, u, wp, nbias_v, sl2_v, dist0);
    sig_ops<D, ALIBI, LO + 1, HI>(W, s, u, wp, nbias_v, sl2_v, dist0);
  }
}

// First sigmoid operation of sub-slot K.  The 72 operations are cut so that every group of
// transcendental instructions (X x4, R x4) ends a slice, i.e. is followed by the next
// sub-slot's MFMA: a plain VALU instruction right behind a transcendental one costs a wait
// state (an s_nop from the compiler, one more issue slot).  Per group of 18 operations the
// cuts are  [C2 of the previous group, F4] [X4] [A4] [R4]  with 4 sub-slots per group, or
// [C2, F4, X4] [A4, R4] with 2; the last C2 joins the last slice.
template <int NSUB>
__device__ constexpr int sig_lo(int K) {
  if (K <= 0) return 0;
  if (K >= NSUB) return 72;
  constexpr int PER = NSUB / 4;  // sub-slots per group
  const int g = K / PER, ph = K % PER;
  if (PER == 4) return ph == 0 ? 18 * g - 2 : 18 * g + 4 * ph;
  if (PER == 2) return ph == 0 ? 18 * g - 2 : 18 * g + 8;
  return (K * 72) / NSUB;
}

template <int D, bool ALIBI, int PAR, bool FOLD, int K>
__device__ __forceinline__ void full_subslots(FwdWave<D>& W, uint32_t kaddr, uint32_t vaddr, float (&u)[16],
                                              uint32_t (&wp)[8], float nbias_v, float sl2_v, float dist0) {
  constexpr int KD = D / 16, DT = D / 32, NSUB = 2 * KD, NOPS = 72;
  if constexpr (K < NSUB) {
    constexpr int m = K / 2;
    if constexpr ((K & 1) == 0) {
      if constexpr (m == 0 && FOLD) a_mfma_init(W.s[PAR ^ 1], W.kf[m], W.qf[m], W.cinit);
      else if constexpr (m == 0) a_mfma_zero(W.s[PAR ^ 1], W.kf[m], W.qf[m]);
      else a_mfma(W.s[PAR ^ 1], W.kf[m], W.qf[m]);
      W.kf[m] = as_bf16x8(lds_read_b128(W.koff[m] + kaddr));
    } else {
      a_mfma(W.oacc[m % DT], W.vf[m], W.p[PAR ^ 1][m / DT]);
      const uint32_t a0 = W.voff[m % DT] + vaddr + (m / DT) * 16 * (D * 2);
      W.vf[m] = join_tr(lds_read_tr16(a0), lds_read_tr16(a0 + 4 * (D * 2)));
    }
    sig_ops<D, ALIBI, sig_lo<NSUB>(K), sig_lo<NSUB>(K + 1)>(W, W.s[PAR], u, wp, nbias_v, sl2_v, dist0);
    full_subslots<D, ALIBI, PAR, FOLD, K + 1>(W, kaddr, vaddr, u, wp, nbias_v, sl2_v, dist0);
  }
}

template <int D, bool ALIBI, int PAR, bool FOLD>
__device__ __forceinline__ void fwd_step_full_pinned(FwdWave<D>& W, uint32_t kaddr, uint32_t vaddr, int jc) {
  float u[16];
  uint32_t wp[8];
  const float dist0 = (float)(W.qi - (jc + 8 * W.h));
  if constexpr (FOLD)  // the per-element arithmetic is the one without ALiBi, on a per-step bias
    full_subslots<D, false, PAR, true, 0>(W, kaddr, vaddr, u, wp, __builtin_fmaf(W.sl2, dist0, W.nbias), W.sl2, dist0);
  else
    full_subslots<D, ALIBI, PAR, false, 0>(W, kaddr, vaddr, u, wp, W.nbias, W.sl2, dist0);
  W.p[PAR][0] = as_bf16x8(u32x4{wp[0], wp[1], wp[2], wp[3]});
  W.p[PAR][1] = as_bf16x8(u32x4{wp[4], wp[5], wp[6], wp[7]});
}

// ---- The same hand-pinned stream for the softmax comparison kernel: what the sigmoid slices
// are replaced with is the online softmax of the chunk (Appendix F.1 table, left half).  With
// the logits transposed a lane holds 16 of its query's 32 keys of the chunk, the other lane half
// the other 16, so the row maximum is a register tree plus one exchange between the halves.
//   Y  x16 (ALiBi only)  y = s - (slope/scale)|i-j|: two operations per element; one under the
//        causal mask, where i-j >= 0 splits into a constant of the lane and step (added where the
//        maximum is scaled) and a multiple of the register's key offset (a literal)
//   M  x8   tree of three-input maxima over y (raw logits: the scale is positive)
//   X       exchange with the other half; m_new = max(m, scale*max), alpha = 2^(m - m_new)
//   per group of four elements:  F x4 (u = y*scale - m_new)  E x4 (2^u)  A x4 (partial sums)  C x2 (pack)
// The row sum (l = l*alpha + sum) and the rescaling of O^T by alpha follow the stream; O^T is
// only touched when some lane's maximum moved, which stops early in a long key loop.
template <int D, int AL>
struct SmxLayout {
  static constexpr int nY = AL == 1 ? 32 : AL == 2 ? 16 : 0, oM = nY, oX = oM + 8, oG = oX + 1, OPG = 14, NOPS = oG + 4 * OPG;
};
template <int D, int AL, int I>
__device__ __forceinline__ void smx_op(FwdWave<D>& W, const f32x16& s, float (&y)[16], float (&u)[16],
                                       float (&acc)[4], uint32_t (&wp)[8], float& nm, float& alpha, float cal, float dist0,
                                       float wstep) {
  using L = SmxLayout<D, AL>;
  constexpr bool ALIBI = AL != 0;
  if constexpr (I < L::oM && AL == 2) {
    constexpr int e = I;
    // y = cal * key_of_reg(e) + s  (cal = slope*log2(e) / scale here)
    asm volatile("v_fmamk_f32 %0, %1, %2, %3" : "=v"(y[e]) : "v"(cal), "n"(__builtin_bit_cast(int, (float)key_of_reg(e))), "v"(s[e]));
  } else if constexpr (I < L::oM) {
    constexpr int e = I / 2;
    if constexpr ((I & 1) == 0) {
      const float keyf = (float)key_of_reg(e);
      asm volatile("v_sub_f32 %0, %1, %2" : "=v"(u[e]) : "v"(dist0), "v"(keyf));
    } else {
      asm volatile("v_fma_f32 %0, %1, |%2|, %3" : "=v"(y[e]) : "v"(cal), "v"(u[e]), "v"(s[e]));
    }
  } else if constexpr (I < L::oX) {
    constexpr int j = I - L::oM;
    // without ALiBi the tree reads the accumulator registers themselves
#define SATTN_SMX_Y(e) (ALIBI ? y[e] : s[e])
    // (the temporaries are the first five entries of u, which the F stage overwrites later)
    if constexpr (j < 5)
      asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(u[j]) : "v"(SATTN_SMX_Y(3 * j)), "v"(SATTN_SMX_Y(3 * j + 1)), "v"(SATTN_SMX_Y(3 * j + 2)));
    else if constexpr (j == 5)
      asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(u[0]) : "v"(u[1]), "v"(u[2]));
    else if constexpr (j == 6)
      asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(u[3]) : "v"(u[4]), "v"(SATTN_SMX_Y(15)));
    else
      asm volatile("v_max_f32 %0, %0, %1" : "+v"(u[0]) : "v"(u[3]));
  } else if constexpr (I < L::oG) {
    // compiler-scheduled island between the pinned halves (its inputs and outputs pin it there)
    float mx = __builtin_fmaf(u[0], W.nscale, wstep);
    mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = __builtin_fmaxf(W.sm.m, mx);
    alpha = __builtin_amdgcn_exp2f(W.sm.m - m_new);
    W.sm.m = m_new;
    nm = wstep - m_new;
  } else {
    constexpr int G = (I - L::oG) / L::OPG, i = (I - L::oG) % L::OPG, e = 4 * G + (i & 3);
    if constexpr (i < 4) {
      asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(u[e]) : "v"(SATTN_SMX_Y(e)), "s"(W.nscale), "v"(nm));
    } else if constexpr (i < 8) {
      asm volatile("v_exp_f32 %0, %0" : "+v"(u[e]));
    } else if constexpr (i < 12) {
      if constexpr (G == 0) asm volatile("v_mov_b32 %0, %1" : "=v"(acc[i & 3]) : "v"(u[e]));
      else asm volatile("v_add_f32 %0, %0, %1" : "+v"(acc[i & 3]) : "v"(u[e]));
    } else {
      constexpr int j = 2 * G + (i - 12);
      asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(wp[j]) : "v"(u[2 * j]), "v"(u[2 * j + 1]));
    }
#undef SATTN_SMX_Y
  }
}
template <int D, int AL, int LO, int HI>
__device__ __forceinline__ void smx_ops(FwdWave<D>& W, const f32x16& s, float (&y)[16], float (&u)[16],
                                        float (&acc)[4], uint32_t (&wp)[8], float& nm, float& alpha, float cal, float dist0,
                                       float wstep) {
  if constexpr (LO < HI) {
    smx_op<D, AL, LO>(W, s, y, u, acc, wp, nm, alpha, cal, dist0, wstep);
    smx_ops<D, AL, LO + 1, HI>(W, s, y, u, acc, wp, nm, alpha, cal, dist0, wstep);
  }
}

template <int D, int AL, int PAR, int K>
__device__ __forceinline__ void smx_subslots(FwdWave<D>& W, uint32_t kaddr, uint32_t vaddr, float (&y)[16], float (&u)[16],
                                             float (&acc)[4], uint32_t (&wp)[8], float& nm, float& alpha,
                                             float cal, float dist0, float wstep) {
  constexpr int KD = D / 16, DT = D / 32, NSUB = 2 * KD, NOPS = SmxLayout<D, AL>::NOPS;
  if constexpr (K < NSUB) {
    constexpr int m = K / 2;
    if constexpr ((K & 1) == 0) {
      if constexpr (m == 0) a_mfma_zero(W.s[PAR ^ 1], W.kf[m], W.qf[m]);
      else a_mfma(W.s[PAR ^ 1], W.kf[m], W.qf[m]);
      W.kf[m] = as_bf16x8(lds_read_b128(W.koff[m] + kaddr));
    } else {
      a_mfma(W.oacc[m % DT], W.vf[m], W.p[PAR ^ 1][m / DT]);
      const uint32_t a0 = W.voff[m % DT] + vaddr + (m / DT) * 16 * (D * 2);
      W.vf[m] = join_tr(lds_read_tr16(a0), lds_read_tr16(a0 + 4 * (D * 2)));
    }
    smx_ops<D, AL, (K * NOPS) / NSUB, ((K + 1) * NOPS) / NSUB>(W, W.s[PAR], y, u, acc, wp, nm, alpha, cal, dist0, wstep);
    smx_subslots<D, AL, PAR, K + 1>(W, kaddr, vaddr, y, u, acc, wp, nm, alpha, cal, dist0, wstep);
  }
}

// (The sigmoid step keeps the register term of causal ALiBi in the S^T accumulators' initial
// value, sixteen registers that this step, with its running statistics, does not have to spare.)
template <int D, bool ALIBI, int PAR, bool CAUSAL>
__device__ __forceinline__ void fwd_step_full_pinned_softmax(FwdWave<D>& W, uint32_t kaddr, uint32_t vaddr, int jc) {
  constexpr int DT = D / 32;
  float y[16], u[16], acc[4];
  uint32_t wp[8];
  float nm = 0.f, alpha = 1.f;
  const float dist0 = (float)(W.qi - (jc + 8 * W.h));
  constexpr int AL = !ALIBI ? 0 : CAUSAL ? 2 : 1;
  // y*scale = s*scale - slope*log2(e)*|i-j|
  const float cal = !ALIBI ? 0.f : CAUSAL ? W.sl2 / W.nscale : -W.sl2 / W.nscale;
  const float wstep = AL == 2 ? -W.sl2 * dist0 : 0.f;
  smx_subslots<D, AL, PAR, 0>(W, kaddr, vaddr, y, u, acc, wp, nm, alpha, cal, dist0, wstep);
  W.p[PAR][0] = as_bf16x8(u32x4{wp[0], wp[1], wp[2], wp[3]});
  W.p[PAR][1] = as_bf16x8(u32x4{wp[4], wp[5], wp[6], wp[7]});
  W.sm.l = __builtin_fmaf(W.sm.l, alpha, (acc[0] + acc[1]) + (acc[2] + acc[3]));
  // O^T holds sums relative to the previous maximum: rescale only when some maximum moved
  if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
    // the stream's last MFMAs must have written O^T before the vector ALU reads it, and the
    // products must be that old before the next step's MFMA reads them (the compiler knows of neither)
    asm volatile("s_nop 15\n\ts_nop 3" ::: "memory");
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) W.oacc[dt][r] *= alpha;
      asm volatile("" : "+v"(W.oacc[dt]) : : "memory");
    }
    asm volatile("s_nop 1" ::: "memory");
  }
}

// Dispatch one step of chunk c for a wave that owns chunks 0..cw-1.
template <int D, bool ALIBI, bool SOFTMAX, int PAR, bool FOLD, bool PIN, bool CAUSAL>
__device__ __forceinline__ void fwd_step_any(FwdWave<D>& W, int c, int cw, uint32_t kaddr, uint32_t vaddr, int N,
                                             bool causal) {
  if (c + 1 < cw) {
    if constexpr (!PIN) fwd_step<D, ALIBI, SOFTMAX, STEP_FULL, PAR, FOLD>(W, kaddr, vaddr, 32 * c, N, causal);
    else if constexpr (SOFTMAX) fwd_step_full_pinned_softmax<D, ALIBI, PAR, CAUSAL>(W, kaddr, vaddr, 32 * c);
    else fwd_step_full_pinned<D, ALIBI, PAR, FOLD>(W, kaddr, vaddr, 32 * c);
  }
  else if (c + 1 == cw) fwd_step<D, ALIBI, SOFTMAX, STEP_LAST, PAR, FOLD>(W, kaddr, vaddr, 32 * c, N, causal);
  else if (c == cw) fwd_step<D, ALIBI, SOFTMAX, STEP_TAIL, PAR, FOLD>(W, kaddr, vaddr, 32 * c, N, causal);
}

// PIN = false runs the steady-state step in its compiler-scheduled form as well (measurement
// aid: what the hand-pinned order is worth, for either method).
// VS = V ring slots (3, or 2: the V tile is then staged one tile ahead instead of two, which
// brings the ring of D = 128 down to 80 KB so that two 4-wave workgroups share a compute unit).
template <int D, int NW, bool CAUSAL, bool ALIBI, bool SOFTMAX, bool PIN = true, int VS = 3>
__global__ void __launch_bounds__(64 * NW, 8 / NW)
attn_fwd_kernel(const FwdParams p) {
  static_assert(VS == 2 || VS == 3, "V ring of two or three slots");
  constexpr int BR = 32 * NW, BC = 64;
  constexpr int KD = D / 16, DT = D / 32;
  constexpr bool FOLD = !SOFTMAX && CAUSAL && ALIBI;  // see fwd_step
  constexpr int TILE = BC * D * 2;    // bytes of one K or V tile
  constexpr int CHUNK = 32 * D * 2;   // bytes of a 32-key chunk

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(SATTN_LDS(char)*)smem;
  const uint32_t kring = lds0, vring = lds0 + 3 * TILE;  // 3 K slots, then VS V slots

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, h = lane >> 5;
  ClockStart clk = clock_probe_begin(p.clock);

  const int total = p.n_qblocks * p.B * p.H;
  const int logical = xcd_remap(blockIdx.x, total);
  int bh, rank;
  head_and_rank(logical, p.n_qblocks, p.B * p.H, CAUSAL ? p.head_group : 1, bh, rank);
  // causal: heavy (late) query blocks first
  const int qb = CAUSAL ? (p.n_qblocks - 1 - rank) : rank;
  const int b = bh / p.H, hd = bh % p.H;
  int N = p.N;
  int64_t tok0 = 0;
  float nbias_log2 = p.nbias_log2;
  if (p.cu_seqlens) {
    tok0 = p.cu_seqlens[b];
    N = min(p.cu_seqlens[b + 1] - (int)tok0, p.N);  // never beyond the span the host checked
    if (p.bias_vec) nbias_log2 = -p.bias_vec[b] * kLog2e;
    if (qb * BR >= N) return;  // this sequence has no such query block (whole workgroup)
  }

  const __bf16* qbase = (const __bf16*)p.q.ptr + b * p.q.sb + hd * p.q.sh + tok0 * p.q.ss;
  const int hkv = hd / p.kv_group;
  const __bf16* kbase = (const __bf16*)p.k.ptr + b * p.k.sb + hkv * p.k.sh + tok0 * p.k.ss;
  const __bf16* vbase = (const __bf16*)p.v.ptr + b * p.v.sb + hkv * p.v.sh + tok0 * p.v.ss;
  __bf16* obase = (__bf16*)p.o.ptr + b * p.o.sb + hd * p.o.sh + tok0 * p.o.ss;

  const int q_wave0 = qb * BR + wave * 32;  // first query row of this wave
  const int qi = q_wave0 + l32;             // this lane's query row
  const int qi_ld = qi < N ? qi : N - 1;

  FwdWave<D> W;
  // Q fragment: B operand of S^T = K Q^T, column = query, k = d
#pragma unroll
  for (int kk = 0; kk < KD; ++kk)
    W.qf[kk] = as_bf16x8(*(const u32x4*)(qbase + (int64_t)qi_ld * p.q.ss + 16 * kk + 8 * h));
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) W.oacc[dt][r] = 0.f;
  {
    const int kap = kappa(l32);
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) W.koff[kk] = kring + kap * (D * 2) + (((2 * kk + h) ^ Swz<D>::k(kap)) << 4);
    const int i16 = lane & 15, blk1 = (lane >> 4) & 1;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      int row = 8 * h + (i16 >> 2);
      int c = 4 * dt + 2 * blk1 + ((i16 & 3) >> 1);
      W.voff[dt] = vring + row * (D * 2) + ((c ^ Swz<D>::v(row)) << 4) + ((i16 & 1) << 3);
    }
    W.qi = qi + p.qoff; W.h = h;  // (W.qi is only ever used as a position)
    W.nscale = p.nscale_log2; W.nbias = nbias_log2;
    W.sl2 = ALIBI ? p.slopes[hd] * kLog2e : 0.f;
    W.sm = SoftmaxState{-__builtin_inff(), 0.f};
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      W.cinit[r] = FOLD ? -W.sl2 * (float)key_of_reg(r) / W.nscale : 0.f;
      W.s[0][r] = W.cinit[r];  // step -1 accumulates S^T(0) on top of it
      W.s[1][r] = 0.f;
    }
    const bf16x8 z = as_bf16x8(u32x4{0, 0, 0, 0});
    W.p[0][0] = W.p[0][1] = W.p[1][0] = W.p[1][1] = z;
#pragma unroll
    for (int m = 0; m < 2 * DT; ++m) W.vf[m] = z;  // step 0 multiplies these by P^T(-1) = 0
  }

  // keys this workgroup must visit, and chunks this wave must visit
  const int q_hi = (qb * BR + BR < N ? qb * BR + BR : N) - 1;  // last valid query row of the block
  const int Nk = p.Nk > 0 ? p.Nk : N;  // keys (N counts the queries)
  auto visible = [&](int rows) {  // keys visible to the first `rows` queries: positions < rows + qoff
    const int kv = rows + p.qoff;
    return kv < 0 ? 0 : (kv < Nk ? kv : Nk);
  };
  const int kv_len = CAUSAL ? visible(q_hi + 1) : Nk;
  const int n_tiles = (kv_len + BC - 1) / BC;
  int kv_wave = Nk;
  if (CAUSAL) kv_wave = visible(q_wave0 + 32 < N ? q_wave0 + 32 : N);
  const int cw = q_wave0 < N ? (kv_wave + 31) / 32 : 0;  // chunks 0..cw-1; waves past the end idle

  // LDS rings: K tile t in K slot t%3, V tile t in V slot t%VS.  At the start of tile t the
  // loads of K(t+3) and V(t+2) are issued; they must have landed by the end of tile t+1.
  // K(t+3) overwrites K(t), whose last reads happened during tile t-1; V(t+2) overwrites
  // V(t-1), ditto: the barrier that ends tile t-1 orders both.  With VS = 2 it is V(t+1) that
  // is issued at the start of tile t (first, so that the wait at the end of the tile can leave
  // K(t+3) in flight), again into the slot of V(t-1).
  DmaStager<D, BC, NW, false> kst;
  DmaStager<D, BC, NW, true> vst;
  constexpr int NIK = DmaStager<D, BC, NW, false>::NI, NIV = DmaStager<D, BC, NW, true>::NI;
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  kst.init(kbase, p.k.ss, Nk, uwave, lane);
  vst.init(vbase, p.v.ss, Nk, uwave, lane);
  kst.issue(kring, Nk, uwave, lane);
  vst.issue(vring, Nk, uwave, lane);
  if (n_tiles > 1) {
    kst.issue(kring + TILE, Nk, uwave, lane);
    if (VS == 3) vst.issue(vring + TILE, Nk, uwave, lane);
  }
  if (n_tiles > 2) kst.issue(kring + 2 * TILE, Nk, uwave, lane);
  SATTN_WAIT_VMCNT(0);  // prologue tiles landed; the Q fragment is in registers
  __syncthreads();

  clock_probe_mark(p.clock, clk, kMarkFirstProduct);
  // step -1: S^T(0) into s[0], then fetch K(1)
  if (cw > 0) {
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) W.kf[kk] = as_bf16x8(lds_read_b128(W.koff[kk]));
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) W.s[0] = mfma32(W.kf[kk], W.qf[kk], W.s[0]);
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) W.kf[kk] = as_bf16x8(lds_read_b128(W.koff[kk] + CHUNK));
  }
  __syncthreads();  // every wave has read K tile 0 before tile 0 lets K(3) overwrite it

  // Tile t: steps 2t, 2t+1.  Step c refills kf from K chunk c+2 (tile t+1, slot (t+1)%3) and
  // vf from V chunk c (tile t, slot t%3).  The per-lane LDS addresses rotate with the rings.
#pragma unroll
  for (int kk = 0; kk < KD; ++kk) W.koff[kk] += TILE;  // K reads now point at tile 1
  int kslot = 0;  // ring slot of K tile t == slot that K(t+3) will overwrite; with VS = 3 V tile t is in the same slot index
  // (this kernel picks the form of every step on the fly: its whole tile loop counts as steady)
  clock_probe_mark(p.clock, clk, kMarkSteadyBegin);
  clk.steady_tiles = clk.tiles = n_tiles;
  for (int t = 0; t < n_tiles; ++t) {
    const bool k_more = t + 3 < n_tiles, v_more = t + (VS == 3 ? 2 : 1) < n_tiles;
    if (VS == 3) {
      const int vslot2 = kslot == 0 ? 2 : kslot - 1;  // (t+2)%3
      if (k_more) kst.issue(kring + kslot * TILE, Nk, uwave, lane);
      if (v_more) vst.issue(vring + vslot2 * TILE, Nk, uwave, lane);
    } else {
      if (v_more) vst.issue(vring + ((t + 1) & 1) * TILE, Nk, uwave, lane);
      if (k_more) kst.issue(kring + kslot * TILE, Nk, uwave, lane);
    }
    fwd_step_any<D, ALIBI, SOFTMAX, 0, FOLD, PIN, CAUSAL>(W, 2 * t, cw, 0, 0, Nk, CAUSAL);
    fwd_step_any<D, ALIBI, SOFTMAX, 1, FOLD, PIN, CAUSAL>(W, 2 * t + 1, cw, CHUNK, CHUNK, Nk, CAUSAL);
    // advance the read addresses by one ring slot: K reads are at slot (t+1)%3, V reads at t%3
    const int kadv = kslot == 1 ? -2 * TILE : TILE;  // slot (t+1)%3 == 2 wraps to 0
    const int vadv = VS == 3 ? (kslot == 2 ? -2 * TILE : TILE) : ((t & 1) ? -TILE : TILE);
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) W.koff[kk] += kadv;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) W.voff[dt] += vadv;
    kslot = kslot == 2 ? 0 : kslot + 1;
    // everything issued before this tile must have landed; this tile's own loads may fly on
    if (VS == 3) {
      if (k_more) SATTN_WAIT_VMCNT(NIK + NIV);
      else if (v_more) SATTN_WAIT_VMCNT(NIV);
      else SATTN_WAIT_VMCNT(0);
    } else {
      if (k_more) SATTN_WAIT_VMCNT(NIK);  // V(t+1) was issued first and has landed
      else SATTN_WAIT_VMCNT(0);
    }
    __syncthreads();
  }
  clock_probe_mark(p.clock, clk, kMarkSteadyEnd);
  // flush: O^T update of the last chunk when it fell on the last step of the loop
  if (cw == 2 * n_tiles && cw > 0) fwd_step<D, ALIBI, SOFTMAX, STEP_TAIL, 0, FOLD>(W, 0, 0, 0, Nk, CAUSAL);
  clock_probe_mark(p.clock, clk, kMarkStore);

  if (SOFTMAX) {
    // normalise by the row sum (both lane halves) and write the natural-log row log-sum-exp
    const float l_tot = W.sm.l + __shfl_xor(W.sm.l, 32);
    const float inv = 1.0f / l_tot;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) W.oacc[dt][r] *= inv;
    if (qi < N && h == 0) p.lse[(int64_t)bh * N + qi] = (W.sm.m + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }
  // ---- store O (bf16): register 4g+t of tile dt is O[qi][32dt + 8g + 4h + t]
  if (qi < N) {
    __bf16* orow = obase + (int64_t)qi * p.o.ss;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w;
        w[0] = pack_bf16(W.oacc[dt][4 * g], W.oacc[dt][4 * g + 1]);
        w[1] = pack_bf16(W.oacc[dt][4 * g + 2], W.oacc[dt][4 * g + 3]);
        *(u32x2*)(orow + 32 * dt + 8 * g + 4 * h) = w;
      }
  }
  clock_probe_end(p.clock, clk);
}

}  // namespace sattn
