// Fused sigmoid-attention forward for gfx950 (Algorithm 1 of the paper's Appendix F.1), the
// shape for long key loops: 64 query rows per wave, one wave per SIMD.
//
// The 32-rows-per-wave kernel (sattn_fwd.hpp) reads 1 KB of K or V fragment from LDS for
// every MFMA it issues; with eight waves per compute unit that keeps the LDS pipe as busy as
// the matrix pipe.  Here a wave owns two blocks of 32 query rows (rb = 0, 1), so that every
// K fragment feeds two S^T MFMAs and every V fragment two O^T MFMAs: half the LDS traffic per
// MFMA.  The price is the register budget: O^T (128 registers at d = 128) and the Q fragments
// (64) live in AGPRs, the wave takes up to 512 registers, and a SIMD holds one wave.
//
// Same data flow as the 32-row kernel, per 32-key chunk c and row block rb:
//     S^T[rb] (32 keys x 32 queries) = K_c Q[rb]^T          MFMA 32x32x16 bf16
//     P^T[rb] = sigmoid(S^T[rb] / sqrt(d) + b [+ ALiBi])    fp32 VALU, no row max / row sum
//     O^T[rb] (d x 32 queries)      += V_c^T P^T[rb]        MFMA, V through the transposing read
// software-pipelined over three chunks inside the wave (S^T of c+1 and the O^T update with
// P^T of c-1 are issued while the VALU evaluates the sigmoid of c).
//
// PRESCALE (no ALiBi): Q is multiplied by -log2(e)/sqrt(d) and rounded to bf16 once, when its
// fragments are loaded, so the accumulators hold u' = -s*log2(e)/sqrt(d) directly, and the bias
// enters as the factor E = 2^(-b*log2(e)) = exp(-b) of  p = 1/(1 + E * 2^u'):  the "1 +" becomes
// an fma and the per-element arithmetic is exp2, fma, rcp and half a pack, with no
// scale-and-bias fma in front of the exp2.  This costs one more bf16 rounding on an operand (the
// same kind the inputs already carry); the other variant keeps the scale-and-bias fma and is
// bit-identical to the 32-row kernels.
#pragma once
#include <type_traits>

#include "sattn_fwd.hpp"

namespace sattn {

// ---- MFMA statements with fixed register files.  S-type: C/D in VGPRs (the VALU reads them),
// A = K fragment (VGPR, from LDS), B = Q fragment (AGPR).  O-type: C/D in AGPRs, A = V^T
// fragment (VGPR, from LDS), B = P^T (VGPR).  GUARD puts two wait states in front: a vector-ALU
// result must be that old before an MFMA reads it; the compiler-scheduled step needs it
// (register copies may sit right in front of the statement), the pinned step orders its own
// instructions and is verified on the generated assembly (isa_check.py).
template <bool GUARD>
__device__ __forceinline__ void f64_mfma_s(f32x16& c, const bf16x8& a, const bf16x8& bq) {
  if constexpr (GUARD) asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "a"(bq) : "memory");
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "a"(bq) : "memory");
}
template <bool GUARD>
__device__ __forceinline__ void f64_mfma_s_init(f32x16& c, const bf16x8& a, const bf16x8& bq, const f32x16& init) {
  if constexpr (GUARD) asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(c) : "v"(a), "a"(bq), "v"(init) : "memory");
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(c) : "v"(a), "a"(bq), "v"(init) : "memory");
}
template <bool GUARD>
__device__ __forceinline__ void f64_mfma_s_zero(f32x16& c, const bf16x8& a, const bf16x8& bq) {
  if constexpr (GUARD) asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(c) : "v"(a), "a"(bq) : "memory");
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(c) : "v"(a), "a"(bq) : "memory");
}
template <bool GUARD>
__device__ __forceinline__ void f64_mfma_o(f32x16& c_agpr, const bf16x8& a, const bf16x8& b) {
  if constexpr (GUARD) asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c_agpr) : "v"(a), "v"(b) : "memory");
  else asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c_agpr) : "v"(a), "v"(b) : "memory");
}
// Wait until the MFMAs issued so far have written their results, and keep the named S^T
// accumulators in their registers up to this point.
__device__ __forceinline__ void f64_settle(f32x16& a, f32x16& b) {
  asm volatile("s_nop 15\n\ts_nop 3" : "+v"(a), "+v"(b) : : "memory");
}
__device__ __forceinline__ void f64_settle() { asm volatile("s_nop 15\n\ts_nop 3" ::: "memory"); }

template <int D>
struct F64Wave {
  static constexpr int KD = D / 16, DT = D / 32;
  uint32_t koff[KD];    // LDS byte address of this lane's K fragment kk in the K tile read next
  uint32_t voff[DT];    // LDS byte address of this lane's V fragment dt (ks 0, first row group) in the V tile read next
  bf16x8 qf[2][KD];     // Q fragments of the two row blocks (AGPR operands)
  bf16x8 kf[KD];        // K fragments of the chunk whose S^T is computed next
  bf16x8 vf[2 * DT];    // V fragments of the chunk whose P^T is consumed next
  f32x16 oacc[2][DT];   // O^T accumulators (AGPR operands)
  f32x16 s[2][2];       // S^T of chunk c, row block rb, in s[c & 1][rb]
  f32x16 cinit;         // FOLD: initial value of every S^T accumulator (the key term of causal ALiBi)
  bf16x8 p[2][2][2];    // bf16 P^T of chunk c in p[c & 1][rb][ks]
  int qi0, h;           // this lane's query row in row block 0 (row block 1: +32), lane half
  float nscale, nbias, sl2;
  float ebias;          // PRESCALE: exp(-b), the factor of 2^u' in 1 + exp(-b) 2^u'
};

// ---- One pipeline step for chunk c (PAR = c & 1) with a hand-pinned instruction order.  For
// both row blocks it issues S^T(c+1) and refills the K fragments with chunk c+2, evaluates the
// sigmoid of chunk c, issues O^T += V(c-1)^T P^T(c-1) and refills the V fragments with chunk c.
// Sub-slot K = 4m + ph, m = fragment index 0..KD-1:
//   ph 0: S^T[0] MFMA with K fragment m          ph 1: O^T[0] MFMA with V fragment m
//   ph 2: S^T[1] MFMA, refill K fragment m       ph 3: O^T[1] MFMA, refill V fragment m
// and after each MFMA a slice of the sigmoid of chunk c.  The 32 elements of a lane (16 per row
// block) form 4 groups of eight; a group takes eight sub-slots (two values of m), two per kind of
// operation, four elements each:
//   [scale+bias fma x4,] exp2 x4 | same | 1+e (PRESCALE: 1+E*e) x4 | same | rcp x4 | same | pack x2 | pack x2
// so a result is consumed two MFMAs later (closer than that the compiler separates dependent
// asm statements with an s_nop of its own), and every run of transcendental instructions is
// followed by an MFMA rather than by a plain vector instruction.
//
// MASK: the steps at the end of a row block's key range (its diagonal / ragged last chunk, the
// two steps that drain the pipeline, and steps a wave only sits through because another wave of
// the workgroup still has keys to visit) run the same stream with a select per element after the
// reciprocal: element r is kept if key_of_reg(r) <= thr, with thr a per-lane threshold -- the
// distance to the lane's last visible key in the last chunk, "keep everything" before it, "keep
// nothing" after it.  A select, not a product: S^T of a chunk past the range is computed from
// whatever the ring holds, P^T must be exactly zero whatever that is.  The S^T MFMAs of a finished
// row block are wasted work on a handful of steps per wave.
template <int D, bool PRESCALE, bool MASK, int G, int Q>
__device__ __forceinline__ void f64_sig_slice(const F64Wave<D>& W, const f32x16& s, float (&u)[8], uint32_t (&wp)[8],
                                              float wv, int thr) {
  constexpr int e0 = 8 * (G & 1);      // first element of the group inside its row block
  constexpr int i0 = 4 * (Q & 1);      // this slice's half of the group
  if constexpr (Q < 2) {
    if constexpr (!PRESCALE) {
#pragma unroll
      for (int i = i0; i < i0 + 4; ++i) asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(u[i]) : "v"(s[e0 + i]), "s"(W.nscale), "v"(wv));
#pragma unroll
      for (int i = i0; i < i0 + 4; ++i) asm volatile("v_exp_f32 %0, %0" : "+v"(u[i]));
    } else {
#pragma unroll
      for (int i = i0; i < i0 + 4; ++i) asm volatile("v_exp_f32 %0, %1" : "=v"(u[i]) : "v"(s[e0 + i]));
    }
  } else if constexpr (Q < 4) {
    if constexpr (PRESCALE) {
#pragma unroll
      for (int i = i0; i < i0 + 4; ++i) asm volatile("v_fma_f32 %0, %0, %1, 1.0" : "+v"(u[i]) : "s"(W.ebias));
    } else {
#pragma unroll
      for (int i = i0; i < i0 + 4; ++i) asm volatile("v_add_f32 %0, 1.0, %0" : "+v"(u[i]));
    }
  } else if constexpr (Q < 6) {
#pragma unroll
    for (int i = i0; i < i0 + 4; ++i) asm volatile("v_rcp_f32 %0, %0" : "+v"(u[i]));
  } else {
    constexpr int j = (e0 + i0) / 2;  // word j packs elements 2j, 2j+1 of the row block
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(wp[j]) : "v"(u[i0]), "v"(u[i0 + 1]));
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(wp[j + 1]) : "v"(u[i0 + 2]), "v"(u[i0 + 3]));
  }
  if constexpr (MASK && (Q == 5 || Q == 6)) {
    // selects of the half whose reciprocals were issued one sub-slot earlier (Q 5: first half,
    // Q 6: second half; the pack of a half follows its selects by one sub-slot)
    constexpr int m0 = 4 * (Q - 5);
#pragma unroll
    for (int i = m0; i < m0 + 4; ++i) {
      uint64_t keep;
      asm volatile("v_cmp_le_i32_e64 %0, %2, %3\n\tv_cndmask_b32_e64 %1, 0, %1, %0"
                   : "=&s"(keep), "+v"(u[i]) : "n"(key_of_reg(e0 + i)), "v"(thr));
    }
  }
}

// DMA: one staging instruction (of the K tile three ahead or the V tile two ahead, see the
// kernel) every DSTEP sub-slots: doff = this lane's offsets, dbase = the tile's first row,
// dma_lds = this wave's first piece of the LDS tile.
template <int D, bool FOLD, bool PRESCALE, int PAR, bool DMA, bool MASK, int K>
__device__ __forceinline__ void f64_subslots(F64Wave<D>& W, uint32_t kaddr, uint32_t vaddr, float (&u)[8],
                                             uint32_t (&wp0)[8], uint32_t (&wp1)[8], float wv0, float wv1,
                                             int thr0, int thr1,
                                             const uint32_t (&doff)[4], const char* dbase, uint32_t dma_lds) {
  constexpr int KD = D / 16, DT = D / 32, NSUB = 4 * KD;
  if constexpr (K < NSUB) {
    constexpr int m = K / 4, ph = K % 4;
    if constexpr (ph == 0 || ph == 2) {
      constexpr int rb = ph / 2;
      if constexpr (m == 0 && FOLD) f64_mfma_s_init<false>(W.s[PAR ^ 1][rb], W.kf[0], W.qf[rb][0], W.cinit);
      else if constexpr (m == 0) f64_mfma_s_zero<false>(W.s[PAR ^ 1][rb], W.kf[0], W.qf[rb][0]);
      else f64_mfma_s<false>(W.s[PAR ^ 1][rb], W.kf[m], W.qf[rb][m]);
      if constexpr (ph == 2) W.kf[m] = as_bf16x8(lds_read_b128(W.koff[m] + kaddr));
    } else if constexpr (ph == 1) {
      f64_mfma_o<false>(W.oacc[0][m % DT], W.vf[m], W.p[PAR ^ 1][0][m / DT]);
    } else {
      f64_mfma_o<false>(W.oacc[1][m % DT], W.vf[m], W.p[PAR ^ 1][1][m / DT]);
      const uint32_t a0 = W.voff[m % DT] + vaddr + (m / DT) * 16 * (D * 2);
      W.vf[m] = join_tr(lds_read_tr16(a0), lds_read_tr16(a0 + 4 * (D * 2)));
    }
    // sigmoid of chunk c: group g = K / 8 (two per row block)
    static_assert(NSUB == 32, "four groups of eight sub-slots");
    if constexpr (K < 16) f64_sig_slice<D, PRESCALE, MASK, K / 8, K % 8>(W, W.s[PAR][0], u, wp0, wv0, thr0);
    else f64_sig_slice<D, PRESCALE, MASK, K / 8, K % 8>(W, W.s[PAR][1], u, wp1, wv1, thr1);
    if constexpr (DMA) {
      constexpr int NI = 4, DSTEP = NSUB / NI;
      if constexpr (K % DSTEP == 2) DmaStager<D, 64, 4, false>::template issue_off<K / DSTEP>(doff[K / DSTEP], dbase, dma_lds);
    }
    f64_subslots<D, FOLD, PRESCALE, PAR, DMA, MASK, K + 1>(W, kaddr, vaddr, u, wp0, wp1, wv0, wv1, thr0, thr1, doff, dbase,
                                                            dma_lds);
  }
}

// kaddr / vaddr: compile-time-constant byte offsets of the K chunk c+2 / V chunk c relative to
// W.koff / W.voff.  thr0 / thr1 (MASK only): per-lane thresholds of the two row blocks.
template <int D, bool FOLD, bool PRESCALE, int PAR, bool DMA, bool MASK = false>
__device__ __forceinline__ void f64_step_pinned(F64Wave<D>& W, uint32_t kaddr, uint32_t vaddr, int jc,
                                                const uint32_t (&doff)[4], const char* dbase, uint32_t dma_lds,
                                                int thr0 = 0, int thr1 = 0) {
  static_assert(D == 128, "the pinned 64-row step is written for head dimension 128");
  float u[8];
  uint32_t wp0[8], wp1[8];
  const float dist0 = (float)(W.qi0 - (jc + 8 * W.h));
  const float wv0 = FOLD ? __builtin_fmaf(W.sl2, dist0, W.nbias) : W.nbias;
  const float wv1 = FOLD ? __builtin_fmaf(W.sl2, dist0 + 32.0f, W.nbias) : W.nbias;
  f64_subslots<D, FOLD, PRESCALE, PAR, DMA, MASK, 0>(W, kaddr, vaddr, u, wp0, wp1, wv0, wv1, thr0, thr1, doff, dbase, dma_lds);
  W.p[PAR][0][0] = as_bf16x8(u32x4{wp0[0], wp0[1], wp0[2], wp0[3]});
  W.p[PAR][0][1] = as_bf16x8(u32x4{wp0[4], wp0[5], wp0[6], wp0[7]});
  W.p[PAR][1][0] = as_bf16x8(u32x4{wp1[0], wp1[1], wp1[2], wp1[3]});
  W.p[PAR][1][1] = as_bf16x8(u32x4{wp1[4], wp1[5], wp1[6], wp1[7]});
}

// One steady-state tile t with U = t % 3 known at compile time, so that every ring address is
// an immediate: K chunks c+2 are read from slot (U+1)%3, V chunks c from slot U (W.koff / W.voff
// point at slot 0), K(t+3) is staged into slot U and V(t+2) into slot (U+2)%3.
template <int D, bool FOLD, bool PRESCALE, int U>
__device__ __forceinline__ void f64_tile_pinned(F64Wave<D>& W, int t, DmaStager<D, 64, 4, false>& kst,
                                                DmaStager<D, 64, 4, true>& vst, const uint32_t (&kdoff)[4],
                                                const uint32_t (&vdoff)[4], uint32_t kring_wave, uint32_t vring_wave) {
  constexpr int TILE = 64 * D * 2, CHUNK = 32 * D * 2;
  constexpr uint32_t kimm = ((U + 1) % 3) * TILE, vimm = U * TILE;
  f64_step_pinned<D, FOLD, PRESCALE, 0, true>(W, kimm, vimm, 64 * t, kdoff, kst.base, kring_wave + U * TILE);
  kst.advance();
  f64_step_pinned<D, FOLD, PRESCALE, 1, true>(W, kimm + CHUNK, vimm + CHUNK, 64 * t + 32, vdoff, vst.base,
                                              vring_wave + ((U + 2) % 3) * TILE);
  vst.advance();
  SATTN_WAIT_VMCNT(8);  // everything issued before this tile has landed; its own eight loads may fly on
  __builtin_amdgcn_s_barrier();
}

// One query block (256 rows of head bh) from the first load to the last store; `record` is its
// slot in the clock probe's buffer.
template <int D, bool CAUSAL, bool ALIBI, bool PRESCALE>
__device__ __forceinline__ void attn_fwd64_block(const FwdParams& p, const int bh, const int qb, const int record) {
  static_assert(!ALIBI || CAUSAL, "ALiBi only in the causal form whose per-element cost folds away");
  static_assert(!(ALIBI && PRESCALE), "the pre-scaled form has no per-step bias");
  constexpr int NW = 4, BR = 64 * NW, BC = 64;
  constexpr int KD = D / 16, DT = D / 32;
  constexpr bool FOLD = CAUSAL && ALIBI;
  constexpr int TILE = BC * D * 2;    // bytes of one K or V tile
  constexpr int CHUNK = 32 * D * 2;   // bytes of a 32-key chunk

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(SATTN_LDS(char)*)smem;
  const uint32_t kring = lds0, vring = lds0 + 3 * TILE;  // 3 K slots, then 3 V slots

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, h = lane >> 5;
  ClockStart clk = clock_probe_begin(p.clock);

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

  const int q_wave0 = qb * BR + wave * 64;  // first query row of this wave
  const int qi0 = q_wave0 + l32;            // this lane's query row in row block 0

  // keys this workgroup must visit, and chunks each row block of this wave must visit
  const int q_hi = (qb * BR + BR < N ? qb * BR + BR : N) - 1;  // last valid query row of the block
  const int Nk = p.Nk > 0 ? p.Nk : N;  // keys (N counts the queries)
  auto visible = [&](int rows) {  // keys visible to the first `rows` queries: positions < rows + qoff
    const int kv = rows + p.qoff;
    return kv < 0 ? 0 : (kv < Nk ? kv : Nk);
  };
  const int kv_len = CAUSAL ? visible(q_hi + 1) : Nk;
  const int n_tiles = (kv_len + BC - 1) / BC;
  int cw[2];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
    const int q0 = q_wave0 + 32 * rb;
    int kv = Nk;
    if (CAUSAL) kv = visible(q0 + 32 < N ? q0 + 32 : N);
    cw[rb] = __builtin_amdgcn_readfirstlane(q0 < N ? (kv + 31) / 32 : 0);  // chunks 0..cw-1; row blocks past the end idle
  }

  // (staged first of all: the ring loads do not depend on Q and their latency overlaps the Q loads)
  // LDS rings as in the 32-row kernel: K tile t in K slot t%3, V tile t in V slot t%3.  During
  // tile t the loads of K(t+3) (into the slot of K(t), last read during tile t-1) and V(t+2)
  // (into the slot of V(t-1)) are issued; they must have landed by the end of tile t+1.
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
    vst.issue(vring + TILE, Nk, uwave, lane);
  }
  if (n_tiles > 2) kst.issue(kring + 2 * TILE, Nk, uwave, lane);
  F64Wave<D> W;
  // Q fragments: B operand of S^T = K Q^T, column = query, k = d.  All sixteen loads are issued
  // before the first one is consumed (the fragments then move into their AGPRs one by one).
  {
    u32x4 raw[2][KD];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const int qi = qi0 + 32 * rb, qi_ld = qi < N ? qi : N - 1;
#pragma unroll
      for (int kk = 0; kk < KD; ++kk) raw[rb][kk] = *(const u32x4*)(qbase + (int64_t)qi_ld * p.q.ss + 16 * kk + 8 * h);
    }
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int kk = 0; kk < KD; ++kk) {
        bf16x8 f = as_bf16x8(raw[rb][kk]);
        if constexpr (PRESCALE) {
          u32x4 w;
#pragma unroll
          for (int j = 0; j < 4; ++j)
            w[j] = pack_bf16((float)f[2 * j] * p.nscale_log2, (float)f[2 * j + 1] * p.nscale_log2);
          f = as_bf16x8(w);
        }
        W.qf[rb][kk] = f;
        // into its AGPRs now: sixteen converted fragments at once would not fit the VGPR file
        asm volatile("" : "+a"(W.qf[rb][kk]) : : "memory");
      }
  }
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) W.oacc[rb][dt][r] = 0.f;
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
    W.qi0 = qi0 + p.qoff; W.h = h;  // (a position: the row's place on the key axis)
    W.nscale = p.nscale_log2; W.nbias = nbias_log2;
    W.sl2 = ALIBI ? p.slopes[hd] * kLog2e : 0.f;
    // wave-uniform: into a scalar register, so that the fma reads it as its one scalar operand
    W.ebias = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, __builtin_amdgcn_exp2f(nbias_log2))));
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      // FOLD: the per-register key term of causal ALiBi over the logit scale
      W.cinit[r] = FOLD ? -W.sl2 * (float)key_of_reg(r) / W.nscale : 0.f;
      W.s[0][0][r] = W.s[0][1][r] = W.cinit[r];  // step -1 accumulates S^T(0) on top of it
      W.s[1][0][r] = W.s[1][1][r] = 0.f;
    }
    const bf16x8 z = as_bf16x8(u32x4{0, 0, 0, 0});
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) W.p[0][rb][0] = W.p[0][rb][1] = W.p[1][rb][0] = W.p[1][rb][1] = z;
#pragma unroll
    for (int m = 0; m < 2 * DT; ++m) W.vf[m] = z;  // step 0 multiplies these by P^T(-1) = 0
  }

  SATTN_WAIT_VMCNT(0);  // prologue tiles landed; the Q fragments are in registers
  __syncthreads();

  clock_probe_mark(p.clock, clk, kMarkFirstProduct);
  // step -1: S^T(0) into s[0], then fetch K(1).  (cw[1] is either 0, row block 1 lying past
  // the end, or >= cw[0]; cw[0] alone is 0 when only row block 0 lies before the first key.)
  if (cw[0] > 0 || cw[1] > 0) {
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) W.kf[kk] = as_bf16x8(lds_read_b128(W.koff[kk]));
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int kk = 0; kk < KD; ++kk) f64_mfma_s<true>(W.s[0][rb], W.kf[kk], W.qf[rb][kk]);
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) W.kf[kk] = as_bf16x8(lds_read_b128(W.koff[kk] + CHUNK));
    f64_settle(W.s[0][0], W.s[0][1]);
  }
  __syncthreads();  // every wave has read K tile 0 before tile 0 lets K(3) overwrite it

  // Tile t: steps 2t, 2t+1.  Step c refills the K fragments from chunk c+2 (tile t+1, slot
  // (t+1)%3) and the V fragments from chunk c (tile t, slot t%3).
  //
  // Steady state: both steps of the tile are full for both row blocks of this wave (step c is
  // full for a row block while c + 1 < cw[rb]) and the staged tiles K(t+3), V(t+2) lie wholly
  // inside the tensor, so their loads need no clamping and are interleaved with the pinned
  // stream.  The loop is unrolled over the three ring positions, which turns every ring address
  // into an immediate: a wave issues about one instruction every six cycles whatever the
  // instruction, so address rotation and slot selection would sit on the critical path.  Every
  // variant of a tile has its one barrier at the same place, so the waves of a workgroup may be
  // in different loops.
  int t = 0;
  clock_probe_mark(p.clock, clk, kMarkSteadyBegin);
  if constexpr (D == 128) {
    static_assert(NIK == 4 && NIV == 4, "four staging instructions per wave and tile");
    const int t_full = (cw[0] - 1) / 2;       // tiles t < t_full: 2t + 2 < cw[0]
    const int t_dma = Nk / BC - 3;            // tiles t < t_dma: (t + 3) * 64 + 64 <= Nk
    const int t_steady = t_full < t_dma ? t_full : t_dma;
    if (t_steady > 0) {
      uint32_t kdoff[4], vdoff[4];
#pragma unroll
      for (int n = 0; n < 4; ++n) { kdoff[n] = kst.lane_off(n); vdoff[n] = vst.lane_off(n); }
      const uint32_t kring_wave = kring + uwave * (NIK * 1024), vring_wave = vring + uwave * (NIV * 1024);
      for (; t + 3 <= t_steady; t += 3) {
        f64_tile_pinned<D, FOLD, PRESCALE, 0>(W, t, kst, vst, kdoff, vdoff, kring_wave, vring_wave);
        f64_tile_pinned<D, FOLD, PRESCALE, 1>(W, t + 1, kst, vst, kdoff, vdoff, kring_wave, vring_wave);
        f64_tile_pinned<D, FOLD, PRESCALE, 2>(W, t + 2, kst, vst, kdoff, vdoff, kring_wave, vring_wave);
      }
      // the one or two steady tiles left over by the unrolling (t is a multiple of 3 here)
      if (t + 1 <= t_steady) {
        f64_tile_pinned<D, FOLD, PRESCALE, 0>(W, t, kst, vst, kdoff, vdoff, kring_wave, vring_wave);
        ++t;
      }
      if (t + 1 <= t_steady) {
        f64_tile_pinned<D, FOLD, PRESCALE, 1>(W, t, kst, vst, kdoff, vdoff, kring_wave, vring_wave);
        ++t;
      }
      f64_settle();  // the compiler does not know the statements above are MFMAs
    }
  }
  clock_probe_mark(p.clock, clk, kMarkSteadyEnd);
  clk.steady_tiles = t;
  clk.tiles = n_tiles;
  // The remaining tiles take the ring position from t: K reads at slot (t+1)%3, V reads at t%3.
  int kslot = t % 3;  // ring slot of K tile t == slot that K(t+3) will overwrite; V tile t is in the same slot index
  {
    const int kadv = (kslot == 2 ? 0 : kslot + 1) * TILE, vadv = kslot * TILE;
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) W.koff[kk] += kadv;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) W.voff[dt] += vadv;
  }
  auto rotate = [&]() {
    const int kadv = kslot == 1 ? -2 * TILE : TILE;  // slot (t+1)%3 == 2 wraps to 0
    const int vadv = kslot == 2 ? -2 * TILE : TILE;
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) W.koff[kk] += kadv;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) W.voff[dt] += vadv;
    kslot = kslot == 2 ? 0 : kslot + 1;
  };
  // The remaining steps of this wave: the last chunk of a row block (mask), the drain of its
  // pipeline, steps it only sits through, and full steps whose staged tiles reach past the
  // tensor's last full tile.  Per row block: FULL while c + 1 < cw, LAST (masked) at c + 1 == cw,
  // TAIL at c == cw (only the O^T update counts), nothing afterwards.
  const uint32_t nodma[4] = {0, 0, 0, 0};
  auto run_step = [&](auto par_tag, int c) {
    constexpr int PAR = decltype(par_tag)::value;
    int thr[2];
    bool live = false;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const int n = cw[rb];
      const bool full = c + 1 < n, last = c + 1 == n, tail = c == n && n > 0;
      live = live || full || last || tail;
      const int jl = 32 * c + 8 * h;           // key held by register 0 of this lane half
      int lim = Nk - 1 - jl;                    // LAST: registers whose key offset exceeds lim are masked
      if (CAUSAL) lim = lim < W.qi0 + 32 * rb - jl ? lim : W.qi0 + 32 * rb - jl;
      thr[rb] = full ? 1000 : last ? lim : -1000;
    }
    if (!live) return;
    f64_step_pinned<D, FOLD, PRESCALE, PAR, false, true>(W, PAR * CHUNK, PAR * CHUNK, 32 * c, nodma, nullptr, 0, thr[0], thr[1]);
    f64_settle();  // compiler-generated code follows: let the last MFMAs retire first
  };
  for (; t < n_tiles; ++t) {
    const bool k_more = t + 3 < n_tiles, v_more = t + 2 < n_tiles;
    const int vslot2 = kslot == 0 ? 2 : kslot - 1;  // (t+2)%3
    if (k_more) kst.issue(kring + kslot * TILE, Nk, uwave, lane);
    if (v_more) vst.issue(vring + vslot2 * TILE, Nk, uwave, lane);
    run_step(std::integral_constant<int, 0>{}, 2 * t);
    run_step(std::integral_constant<int, 1>{}, 2 * t + 1);
    rotate();
    if (k_more) SATTN_WAIT_VMCNT(NIK + NIV);
    else if (v_more) SATTN_WAIT_VMCNT(NIV);
    else SATTN_WAIT_VMCNT(0);
    __syncthreads();
  }
  // flush: O^T update of the last chunk when it fell on the last step of the loop
  run_step(std::integral_constant<int, 0>{}, 2 * n_tiles);

  clock_probe_mark(p.clock, clk, kMarkStore);
  // ---- store O (bf16).  Register 4g+t of tile dt is O[qi][32dt + 8g + 4h + t]: a lane holds 4
  // consecutive features of ITS row, so storing from the registers would scatter 8-byte pieces
  // over 64 rows per instruction.  The wave instead transposes through its own 17 KB of the (now
  // free) ring -- rows padded to 272 bytes, which spreads the 32 rows of a write over the banks --
  // and stores whole 256-byte rows, 16 bytes per lane, four rows per instruction.
  {
    constexpr int ROWB = D * 2 + 16;  // padded row
    // every wave is past its last fragment read of the ring, but other waves may not be
    __syncthreads();
    const uint32_t obuf = lds0 + wave * (64 * ROWB);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 w;
          w[0] = pack_bf16(W.oacc[rb][dt][4 * g], W.oacc[rb][dt][4 * g + 1]);
          w[1] = pack_bf16(W.oacc[rb][dt][4 * g + 2], W.oacc[rb][dt][4 * g + 3]);
          *(SATTN_LDS(u32x2)*)(uintptr_t)(obuf + (32 * rb + l32) * ROWB + (32 * dt + 8 * g + 4 * h) * 2) = w;
        }
    // the wave reads back what its own lanes wrote: only the LDS counter has to drain
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    const int r4 = lane >> 4, c16 = lane & 15;  // row within a group of four, 16-byte chunk of the row
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = 4 * i + r4, qi = q_wave0 + row;
      const u32x4 v4 = lds_read_b128(obuf + row * ROWB + c16 * 16);
      if (qi < N) *(u32x4*)(obase + (int64_t)qi * p.o.ss + c16 * 8) = v4;
    }
  }
  clock_probe_end(p.clock, clk, record);
}

template <int D, bool CAUSAL, bool ALIBI, bool PRESCALE>
__global__ void __launch_bounds__(256, 1)
attn_fwd64_kernel(const FwdParams p) {
  // blocks of a head this launch deals out: pairs (longest with shortest, ...) or single blocks
  const int places = (CAUSAL && p.pair) ? p.n_qblocks / 2 : p.n_qblocks;
  const int logical = xcd_remap(blockIdx.x, places * p.B * p.H);
  int bh, rank;
  head_and_rank(logical, places, p.B * p.H, CAUSAL ? p.head_group : 1, bh, rank);
  // Under the causal mask block q of a head visits q + 1 key tiles (in units of the block):
  // blocks n-1-r and r together visit n + 1 whatever r is.  Equal workgroups leave no ragged
  // end of the launch, and a compute unit pays the gap between two workgroups half as often.
  const int n_parts = (CAUSAL && p.pair) ? 2 : 1;
#pragma nounroll
  for (int part = 0; part < n_parts; ++part) {
    // causal: heavy first, within a pair and (single blocks) within the launch
    const int qb = (CAUSAL && part == 0) ? p.n_qblocks - 1 - rank : rank;
    attn_fwd64_block<D, CAUSAL, ALIBI, PRESCALE>(p, bh, qb, (int)(blockIdx.x + part * gridDim.x));
    // the block's epilogue reads the ring that the next block's first loads refill
    if (part + 1 < n_parts) __syncthreads();
  }
}

}  // namespace sattn
