// Sigmoid-attention backward for gfx950 (Algorithm 2 of the paper's Appendix F.1), bf16
// operands, fp32 logits / sigmoid / accumulation.  P is recomputed from Q and K; nothing
// but Q, K, V, dO is read.
//
// Algorithm 2 keeps dK_j, dV_j on chip and read-modify-writes dQ_i in HBM.  Here the pass
// is split in two launches of one kernel template so that every output tile has exactly
// one owner and no atomics or fp32 dQ workspace are needed (results are bit-reproducible):
//   DQ   : query block stationary (Q, dO fragments in registers), streams K/V tiles
//          S^T = K Q^T, dP^T = V dO^T, dS^T = P^T(1-P^T)dP^T, dQ^T += K^T dS^T
//   DKDV : key block stationary (K, V fragments in registers), streams Q/dO tiles
//          S = Q K^T, dP = dO V^T, dS = P(1-P)dP, dV^T += dO^T P, dK^T += Q^T dS
// In both, the streamed rows land on the rows of the first products' accumulators, so after
// the bf16 round those registers are the B operand of the second products; the A operand
// of the second products is a transposing LDS read of the same row-major tiles.
//
// One workgroup = 4 waves (one per SIMD, up to 512 registers each), 32 stationary rows per
// wave, 64-row streamed tiles in a 4-slot LDS ring filled by direct-to-LDS loads two tiles
// ahead (issued one instruction at a time inside the second step of a tile).  Work is
// software pipelined over 32-row chunks: step s issues the first products of chunk s,
// evaluates the sigmoid / dS of chunk s-1 and issues the second products of chunk s-2.
// The steady-state step is a fixed instruction stream of asm statements (MFMA, LDS refill,
// a slice of the sigmoid arithmetic); tiles at the ends of a wave's range, masked tiles and
// the softmax variant run a compiler-scheduled step with the same data flow.
#pragma once
#include "sattn_common.hpp"

namespace sattn {

// BWD_DQ_DB is the dQ pass that also sums dS along every query row (the gradient of a bias
// added to that row's logits); everything that is not BWD_DKDV is a dQ pass.
enum BwdMode { BWD_DQ = 0, BWD_DKDV = 1, BWD_DQ_DB = 2 };

struct BwdParams {
  TensorRef q, k, v, dout, dq, dk, dv;
  const float* slopes;
  // softmax only, written by the pre-pass: per query row -lse*log2(e) and rowsum(dO o O), each
  // [B*H, npad] with rows padded to a multiple of 64 (pad entries are zero)
  const float* nlse2;
  const float* dvec;
  int npad;
  int B, H, N;
  int n_blocks;        // blocks of 128 stationary rows
  int head_group;      // causal: heads walked abreast in the dispatch order (head_and_rank); 1 otherwise
  float nscale_log2;   // -log2(e)/sqrt(d)
  float nbias_log2;    // -b*log2(e)
  float inv_sqrt_d;
  // variable-length batches (nullptr otherwise), as in the forward parameters
  const int* cu_seqlens;
  const float* bias_vec;
  // BWD_DQ_DB: row sums of dS, element (b, h, i) at b*db_sb + h*db_sh + i
  float* db_rows;
  int64_t db_sb, db_sh;
  // shared key/value heads: query head h reads K/V head h / kv_group (1 = one per query head);
  // k, v, dk, dv then have H / kv_group heads
  int kv_group;
  // grouped dK/dV pass only: a group's query heads are split over n_split workgroups (a divisor
  // of kv_group; 0 or 1: no split), each of which writes its fp32 partial dK, dV (unscaled) to
  // part[(which * n_split + split) * B * (H / kv_group) + b * (H / kv_group) + head][key][d],
  // which = 0 for dK, 1 for dV; a second kernel adds the partials up
  int n_split;
  float* part;
  // number of keys when it differs from the number of queries N (0: same)
  int Nk;
  // position of query 0 on the key axis (see FwdParams::qoff); a multiple of 32
  int qoff;
  // causal passes: every workgroup handles two blocks of its head, the r-th longest and the r-th
  // shortest (n_blocks even), so that all workgroups of a launch do the same work
  int pair;
  ClockProbe clock;  // measurement aid, {nullptr, 0} otherwise
};

// One swizzle for tiles that are read both row-wise (ds_read_b128, 32 rows at one logical
// chunk) and transposed (4 consecutive rows x 64 contiguous bytes).
template <int D>
struct SwzX {
  __device__ static __forceinline__ int f(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
  }
};

// Direct-to-LDS staging of one 64-row tile: one wave-level global_load_lds_dwordx4 moves
// 64 x 16 bytes to 1 KB of LDS at M0 + offset + 16*lane; the XOR swizzle is applied on the
// global side.  Completion is tracked by hand (vmcnt), the compiler never sees these loads.
// The instruction offset moves the LDS target and the global address alike, so the NI loads
// of a wave (consecutive 1 KB pieces of the tile) share one M0 value and differ in their
// offset field; the per-lane global offsets are stored with that offset taken out.  M0 is
// not otherwise used in these kernels (checked on the generated assembly by isa_check.py).
template <int D, int NW>
struct DmaStagerX {
  static constexpr int BC = 64, CPR = D / 8, RPI = 64 / CPR, NI = (BC * CPR) / (64 * NW);
  const char* base;       // first row of the next tile to stage (wave-uniform, advances per tile)
  const char* base_last;  // row N-1 (wave-uniform)
  uint32_t off[NI];       // this lane's byte offset inside a tile, minus 1024 * n (constant)
  uint32_t tile_bytes, row_bytes;
  int j0;                 // first row of the next tile to stage
  static_assert(RPI * D * 2 >= 1024 && NI * 1024 <= 4096, "offset field of the load: 0 .. 4095, never below the row step");
  __device__ __forceinline__ static int row_of(int n, int wave, int lane) { return (wave * NI + n) * RPI + lane / CPR; }
  __device__ __forceinline__ static uint32_t col_bytes(int n, int wave, int lane) {
    return (uint32_t)(((lane % CPR) ^ SwzX<D>::f(row_of(n, wave, lane))) * 16);
  }
  __device__ __forceinline__ void init(const __bf16* b, int64_t ss, int N, int first_row, int wave, int lane) {
    base = (const char*)(b + (int64_t)first_row * ss);
    base_last = (const char*)(b + (int64_t)(N - 1) * ss);
    row_bytes = (uint32_t)(ss * 2);
    tile_bytes = BC * row_bytes;
    j0 = first_row;
#pragma unroll
    for (int n = 0; n < NI; ++n) off[n] = row_of(n, wave, lane) * row_bytes + col_bytes(n, wave, lane) - 1024 * n;
  }
  __device__ __forceinline__ static void load(uint32_t o, const char* sbase, uint32_t m0v) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(o), "s"(sbase), "s"(m0v) : "memory");
  }
  // Load n of a wave's NI: the first one sets M0 to the wave's first piece, the others reuse it.
  template <int n>
  __device__ __forceinline__ static void load_nth(uint32_t o, const char* sbase, uint32_t m0v) {
    if constexpr (n == 0)
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(o), "s"(sbase), "s"(m0v) : "memory");
    else
      asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" : : "v"(o), "s"(sbase), "n"(1024 * n) : "memory");
  }
  template <int n>
  __device__ __forceinline__ void issue_rest(uint32_t lds_wave) const {
    if constexpr (n < NI) {
      load_nth<n>(off[n], base, lds_wave);
      issue_rest<n + 1>(lds_wave);
    }
  }
  __device__ __forceinline__ void advance() { base += tile_bytes; j0 += BC; }
  // Advance unless the tile after the next one does not lie wholly inside the tensor: the
  // stager then stays where it is and a further issue_one() stages the same tile again.
  __device__ __forceinline__ void advance_inside(int N) {
    if (j0 + 2 * BC <= N) advance();
  }
  // Before a run of issue_one() calls on a tensor that ends on a tile boundary: a stager that
  // has already staged the last tile steps back onto it.
  __device__ __forceinline__ void step_back_inside(int N) {
    if (j0 + BC > N) {
      const int back = (j0 + BC - N) / BC;
      base -= (int64_t)back * tile_bytes;
      j0 -= back * BC;
    }
  }
  // Stage the whole next tile.  Rows past the end re-read row N-1.
  __device__ __forceinline__ void issue(uint32_t lds, int N, int wave, int lane) {
    if (j0 + BC <= N) {
      issue_rest<0>(lds + wave * NI * 1024);
    } else if (j0 < N) {
      const uint32_t to_last = (uint32_t)(N - 1 - j0) * row_bytes;
#pragma unroll
      for (int n = 0; n < NI; ++n) {
        const uint32_t o = (j0 + row_of(n, wave, lane) < N) ? off[n] + 1024 * n : to_last + col_bytes(n, wave, lane);
        load(o, base, lds + (wave * NI + n) * 1024);
      }
    } else {
#pragma unroll
      for (int n = 0; n < NI; ++n) load(col_bytes(n, wave, lane), base_last, lds + (wave * NI + n) * 1024);
    }
    advance();
  }
  // One instruction of the same staging for a tile that lies inside the tensor (for
  // interleaving with a pinned step; the caller calls advance() after the last one).
  template <int n>
  __device__ __forceinline__ void issue_one(uint32_t lds, int wave) const {
    load_nth<n>(off[n], base, lds + wave * NI * 1024);
  }
};

// Softmax dK/dV pass: the row statistics of a streamed tile of 64 queries (-lse*log2e and D, two
// fp32 per query, from the [B*H, npad] vectors of the pre-pass) travel with the tile: 256 + 256
// bytes into a side ring of four slots behind the tile ring, by the same asynchronous loads
// (one dword per lane; every wave issues them, all writing the same values).
struct StatStager {
  static constexpr int SLOT = 512;
  const float* l;  // -lse*log2e of this (batch, head), wave-uniform
  const float* d;  // D of this (batch, head)
  int last_tile;   // npad / 64 - 1
  __device__ __forceinline__ static const float* scalar_ptr(const float* ptr) {
    const uint64_t u = (uint64_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
    return (const float*)(((uint64_t)hi << 32) | lo);
  }
  __device__ __forceinline__ void init(const float* l_, const float* d_, int npad) {
    l = scalar_ptr(l_); d = scalar_ptr(d_); last_tile = npad / 64 - 1;
  }
  // stage the statistics of tile `tile` (clamped to the last one) into the side-ring slot at `lds`
  __device__ __forceinline__ void issue(uint32_t lds, int tile, int lane) const {
    const int t = tile < last_tile ? tile : last_tile;
    const uint32_t o = (uint32_t)lane * 4;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" : : "v"(o), "s"(l + 64 * t), "s"(lds) : "memory");
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" : : "v"(o), "s"(d + 64 * t), "s"(lds + 256) : "memory");
  }
};

// A wave-uniform flag as a per-lane value the compiler cannot prove uniform.
__device__ __forceinline__ bool lane_flag(bool uniform) {
  int x;
  asm("v_mov_b32 %0, %1" : "=v"(x) : "s"((int)uniform));
  return x != 0;
}

__device__ __forceinline__ bf16x8 pack8(const float* x) {
  u32x4 w;
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = pack_bf16(x[2 * i], x[2 * i + 1]);
  return as_bf16x8(w);
}

// Per-wave pipeline state.
template <int D, int MODE>
struct BwdWave {
  static constexpr int KD = D / 16, DT = D / 32;
  uint32_t row0[KD];    // LDS address (streamed tensor 1) of row fragment kk in tile t (t = current tile)
  uint32_t row1[KD];    // same in tile t+1
  uint32_t tr[DT][2];   // LDS address of the transposed-read pair for d-tile dt in tile t-1 (tensor 1)
  bf16x8 x1[KD], x2[KD];  // stationary B operands of the first products
  bf16x8 F[2 * KD];       // streamed row fragments: F[2kk] from tensor 1, F[2kk+1] from tensor 2
  f32x16 acc0[DT];        // DQ: dQ^T ; DKDV: dK^T
  f32x16 acc1[MODE == BWD_DKDV ? DT : 1];  // DKDV: dV^T
  f32x16 s[2], dp[2];     // first products of chunk c in [c&1]
  f32x16 cinit;           // FOLD: initial value of the S accumulators (register term of causal ALiBi)
  bf16x8 pb[2][2];        // bf16 P of chunk c in [c&1][ks]   (DKDV only)
  bf16x8 dsb[2][2];       // bf16 dS of chunk c in [c&1][ks]
  int ai, h;              // this lane's stationary row, lane half
  float nscale, nbias, sl2;
  float nlse, dstat;      // softmax DQ: this lane's -lse*log2e and D
  float dbs[4];           // BWD_DQ_DB: partial sums of this lane's dS elements (element e in [e & 3])
};

// Every MFMA of the backward kernel is a volatile asm statement with fixed register classes:
// stationary fragments and output accumulators are AGPR operands, streamed fragments and the
// first products VGPR operands.  The compiler does not see these as MFMAs, so the code below
// covers the read-after-MFMA hazards itself (mfma_settle).
// GUARD puts two wait states in front of the MFMA: a vector-ALU result has to be that old
// before an MFMA may read it.  The compiler-scheduled step needs it (register copies and
// packs may sit right in front of the statement); the pinned step orders its own
// instructions and is verified on the generated assembly instead (isa_check.py).
#define SATTN_BWD_MFMA(PRE, ACC) PRE "v_mfma_f32_32x32x16_bf16 %0, %1, %2, " ACC
template <bool GUARD>
__device__ __forceinline__ void b_mfma_v(f32x16& c, const bf16x8& a, const bf16x8& b_agpr) {
  if constexpr (GUARD) asm volatile(SATTN_BWD_MFMA("s_nop 1\n\t", "%0") : "+v"(c) : "v"(a), "a"(b_agpr) : "memory");
  else asm volatile(SATTN_BWD_MFMA("", "%0") : "+v"(c) : "v"(a), "a"(b_agpr) : "memory");
}
template <bool GUARD>
__device__ __forceinline__ void b_mfma_v0(f32x16& c, const bf16x8& a, const bf16x8& b_agpr) {
  if constexpr (GUARD) asm volatile(SATTN_BWD_MFMA("s_nop 1\n\t", "0") : "=&v"(c) : "v"(a), "a"(b_agpr) : "memory");
  else asm volatile(SATTN_BWD_MFMA("", "0") : "=&v"(c) : "v"(a), "a"(b_agpr) : "memory");
}
// First MFMA of an S product whose accumulator starts from `init` instead of zero.  C and D
// of an MFMA share one register file, so `init` is a VGPR tuple like the result; under
// register pressure the compiler parks it in AGPRs and copies it back right here, hence the
// two wait states in front of the MFMA in every variant.
__device__ __forceinline__ void b_mfma_vinit(f32x16& c, const bf16x8& a, const bf16x8& b_agpr, const f32x16& init) {
  asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(c) : "v"(a), "a"(b_agpr), "v"(init) : "memory");
}
template <bool GUARD>
__device__ __forceinline__ void b_mfma_a(f32x16& c_agpr, const bf16x8& a, const bf16x8& b) {
  if constexpr (GUARD) asm volatile(SATTN_BWD_MFMA("s_nop 1\n\t", "%0") : "+a"(c_agpr) : "v"(a), "v"(b) : "memory");
  else asm volatile(SATTN_BWD_MFMA("", "%0") : "+a"(c_agpr) : "v"(a), "v"(b) : "memory");
}
// Wait until the MFMAs issued so far have written their results, and keep the named first
// products in their registers up to this point (a register copy placed earlier would read
// them before the matrix pipeline has written them).
__device__ __forceinline__ void mfma_settle(f32x16& a, f32x16& b) {
  asm volatile("s_nop 15\n\ts_nop 3" : "+v"(a), "+v"(b) : : "memory");
}
__device__ __forceinline__ void mfma_settle() { asm volatile("s_nop 15\n\ts_nop 3" ::: "memory"); }
// Same pin without the wait, for places where enough independent MFMAs have issued since.
__device__ __forceinline__ void mfma_pin(f32x16& a, f32x16& b) { asm volatile("" : "+v"(a), "+v"(b) : : "memory"); }

// One pipeline step s (PAR = s & 1), compiler-scheduled:
//   A : first products of chunk s (fragments F, loaded by the previous step)
//   SG: p / dS of chunk s-1 (first row cs), masked when `mask`
//   B : second products of chunk s-2 (transposed reads at tr + trimm)
// then F is refilled with the rows of chunk s+1 (nextrow + nextimm).
template <int D, int MODE, bool CAUSAL, bool ALIBI, bool SOFTMAX, int PAR>
__device__ __forceinline__ void bwd_step(BwdWave<D, MODE>& W, bool doA, bool doS, bool doB, bool mask, uint32_t trimm,
                                         const uint32_t* nextrow, uint32_t nextimm, int cs, int N,
                                         const float* stat_l, const float* stat_d) {
  constexpr int KD = D / 16, DT = D / 32;
  constexpr uint32_t T2OFF = 64 * D * 2;  // tensor 2's tile follows tensor 1's inside a ring slot
  // FOLD (sigmoid, causal, ALiBi): every unmasked pair has its key at or before its query, so
  // slope*(i - j) splits into a per-lane, per-step part added to the bias and a per-register
  // part that is a constant of the kernel and sits in the S accumulators from the start
  // (W.cinit, already divided by the logit scale): no ALiBi arithmetic per element.
  constexpr bool FOLD = !SOFTMAX && CAUSAL && ALIBI;
  if (doA) {
    if constexpr (FOLD) b_mfma_vinit(W.s[PAR], W.F[0], W.x1[0], W.cinit);
    else b_mfma_v0<true>(W.s[PAR], W.F[0], W.x1[0]);
    b_mfma_v0<true>(W.dp[PAR], W.F[1], W.x2[0]);
#pragma unroll
    for (int kk = 1; kk < KD; ++kk) {
      b_mfma_v<true>(W.s[PAR], W.F[2 * kk], W.x1[kk]);
      b_mfma_v<true>(W.dp[PAR], W.F[2 * kk + 1], W.x2[kk]);
    }
    mfma_settle(W.s[PAR], W.dp[PAR]);
  }
  if (doS) {
    // chunk s-1 lives in buffers [PAR^1]; streamed index of register r: b = cs + 8h + key_of_reg(r)
    const int bl = cs + 8 * W.h;
    float pr[16], ds[16];
    // softmax dK/dV: the statistics of the 16 streamed queries this lane's registers belong to
    // (queries bl .. bl+7 and bl+16 .. bl+23), straight from global memory: every lane of a wave
    // half reads the same 2 x 32 bytes, which the vector cache serves as one request
    f32x4 sl[4], sd[4];
    if (SOFTMAX && MODE == BWD_DKDV) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        sl[g] = *(const f32x4*)(stat_l + bl + 16 * (g >> 1) + 4 * (g & 1));
        sd[g] = *(const f32x4*)(stat_d + bl + 16 * (g >> 1) + 4 * (g & 1));
      }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int b = bl + key_of_reg(r);
      const int qrow = MODE == BWD_DKDV ? b : W.ai, krow = MODE == BWD_DKDV ? W.ai : b;
      if (SOFTMAX) {
        // p = 2^(s*log2e/sqrt(d) - slope|i-j|log2e - lse*log2e), dS = p (dP - D)
        float w = MODE == BWD_DKDV ? sl[r >> 2][r & 3] : W.nlse;
        if (ALIBI) w = __builtin_fmaf(-W.sl2, __builtin_fabsf((float)(qrow - krow)), w);
        pr[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(W.s[PAR ^ 1][r], -W.nscale, w));
        const float dd = MODE == BWD_DKDV ? sd[r >> 2][r & 3] : W.dstat;
        ds[r] = pr[r] * (W.dp[PAR ^ 1][r] - dd);
      } else {
        // p = 1/(1 + 2^u), dS = (p - p^2) dP
        float w = W.nbias;
        if (FOLD) w = __builtin_fmaf(W.sl2, MODE == BWD_DKDV ? (float)(bl - W.ai) : (float)(W.ai - bl), w);
        else if (ALIBI) w = __builtin_fmaf(W.sl2, __builtin_fabsf((float)(qrow - krow)), w);
        const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(W.s[PAR ^ 1][r], W.nscale, w));
        pr[r] = __builtin_amdgcn_rcpf(1.0f + e);
        ds[r] = __builtin_fmaf(-pr[r], pr[r], pr[r]) * W.dp[PAR ^ 1][r];
      }
      if (mask) {
        const bool keep = b < N && (!CAUSAL || krow <= qrow);
        pr[r] = keep ? pr[r] : 0.f;
        ds[r] = keep ? ds[r] : 0.f;
      }
      if (MODE == BWD_DQ_DB) W.dbs[r & 3] += ds[r];
    }
    if (MODE == BWD_DKDV) { W.pb[PAR ^ 1][0] = pack8(pr); W.pb[PAR ^ 1][1] = pack8(pr + 8); }
    W.dsb[PAR ^ 1][0] = pack8(ds);
    W.dsb[PAR ^ 1][1] = pack8(ds + 8);
  }
  if (doB) {
    // chunk s-2 lives in buffers [PAR]
#pragma unroll
    for (int j = 0; j < 2 * DT; ++j) {
      const uint32_t a0 = W.tr[j % DT][0] + trimm + (j / DT) * 16 * (D * 2);
      const uint32_t a1 = W.tr[j % DT][1] + trimm + (j / DT) * 16 * (D * 2);
      if (MODE == BWD_DKDV) {
        bf16x8 ado = join_tr(lds_read_tr16(a0 + T2OFF), lds_read_tr16(a1 + T2OFF));
        b_mfma_a<true>(W.acc1[j % DT], ado, W.pb[PAR][j / DT]);
      }
      bf16x8 a1t = join_tr(lds_read_tr16(a0), lds_read_tr16(a1));
      b_mfma_a<true>(W.acc0[j % DT], a1t, W.dsb[PAR][j / DT]);
    }
    mfma_settle();
  }
#pragma unroll
  for (int kk = 0; kk < KD; ++kk) {
    W.F[2 * kk] = as_bf16x8(lds_read_b128(nextrow[kk] + nextimm));
    W.F[2 * kk + 1] = as_bf16x8(lds_read_b128(nextrow[kk] + nextimm + T2OFF));
  }
}

// ---- The steady-state step (all three stages active, no mask) with a hand-pinned
// instruction order: every instruction is a volatile asm statement, so the stream is exactly
// one MFMA, the LDS refill of the fragment it consumed, then a slice of the sigmoid / dS
// arithmetic whose dependent operations sit four instructions apart.  Stationary fragments
// and output accumulators are AGPR operands, which keeps the VALU-visible registers < 256.
// One fragment buffer serves both kinds of LDS operand: a slot is refilled with the
// transposed fragment right after the first-product MFMA that used it, and with the next
// chunk's row fragment right after the second-product MFMA that used that.

// Arithmetic of one chunk as 4 groups of four elements.  Per group:
//   F x4 (u = s*scale + bias[+alibi])  X x4 (2^u)  A x4 (1+e)  R x4 (p = 1/.)  [C x4]
//   Q x4 (p - p^2)  M x4 (dS = . * dP)  [D x4]  [B x4 row sum]  [CP x2 pack P]  CD x2 pack dS
// MASK adds C (keep = key_of_reg(e) >= thr for DKDV, <= thr for DQ; p = keep ? p : 0) and
// D (dS = keep ? dS : 0): selects, so that a masked element is exactly zero whatever the
// logit and dP registers hold (they are not even finite in a dead pipeline stage).
// SMX: the softmax comparison kernel's arithmetic in the same stream (dQ pass, where the row
// statistics are per lane): per group F x4 (x = s*scale - lse[- alibi], in log2 units) X x4
// (p = 2^x) [C x4] Q x4 (dP - D) M x4 (dS = . * p) [D x4] CD x2: no 1+e, no reciprocal.
template <int MODE, bool MASK, bool SMX = false>
struct BsigLayout {
  static constexpr int nC = MASK ? 4 : 0, nP = MODE == BWD_DKDV ? 2 : 0, nB = MODE == BWD_DQ_DB ? 4 : 0;
  static constexpr int nAR = SMX ? 0 : 4;
  static constexpr int oX = 4, oA = 8, oR = oA + nAR, oC = oR + nAR, oQ = oC + nC, oM = oQ + 4, oD = oM + 4, oB = oD + nC,
                       oP = oB + nB, oS = oP + nP, OPG = oS + 2, NOPS = 4 * OPG;
};
// nbias_v: the bias term of the exponent (SMX: -lse of the lane's row, log2 units); sl2_v: the
// ALiBi slope (SMX: negated, the exponent has the other sign); dstat_v (SMX): D of the lane's row.
// SMX in the dK/dV pass: the statistics belong to the streamed queries, one pair per element.
// The lane's sixteen queries are rows bl..bl+7 and bl+16..bl+23 of the chunk (bl = 8h), group G
// of four elements rows 4(G&1) + 16(G>>1) + 0..3: two 16-byte LDS reads per group from the side
// ring (stat = address of row bl's -lse; D is 256 bytes further), issued one group ahead.
struct BsigStats {
  f32x4 l[4], d[4];
  uint32_t stat;
};
template <int G>
__device__ __forceinline__ void bsig_load_stats(BsigStats& st) {
  constexpr uint32_t off = (4 * (G & 1) + 16 * (G >> 1)) * 4;
  st.l[G] = *(SATTN_LDS(f32x4)*)(uintptr_t)(st.stat + off);
  st.d[G] = *(SATTN_LDS(f32x4)*)(uintptr_t)(st.stat + off + 256);
}
template <int D, int MODE, bool ALIBI, bool MASK, bool SMX, int I>
__device__ __forceinline__ void bsig_op(BwdWave<D, MODE>& W, const f32x16& s, const f32x16& dp, float (&u)[16],
                                        float (&v)[16], uint32_t (&wp)[8], uint32_t (&wd)[8], uint64_t (&km)[16],
                                        float nbias_v, float sl2_v, float dist0, float dstep, int thr, float dstat_v,
                                        BsigStats& st) {
  using L = BsigLayout<MODE, MASK, SMX>;
  constexpr int G = I / L::OPG, i = I % L::OPG, e = 4 * G + (i & 3);
  if constexpr (SMX && MODE == BWD_DKDV) {
    if constexpr (I == 0) { bsig_load_stats<0>(st); bsig_load_stats<1>(st); }
    else if constexpr (i == 0 && G + 1 < 4) bsig_load_stats<G + 1>(st);
    if constexpr (i < L::oX) nbias_v = st.l[G][i & 3];
    if constexpr (i >= L::oQ && i < L::oM) dstat_v = st.d[G][i & 3];
  }
  if constexpr (i < L::oX) {
    if constexpr (ALIBI) {
      float t, w;
      const float keyf = (float)key_of_reg(e);
      asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(t) : "v"(dstep), "v"(keyf), "v"(dist0));
      asm volatile("v_fma_f32 %0, %1, |%2|, %3" : "=v"(w) : "v"(sl2_v), "v"(t), "v"(nbias_v));
      if constexpr (SMX) asm volatile("v_fma_f32 %0, %1, -%2, %3" : "=v"(u[e]) : "v"(s[e]), "s"(W.nscale), "v"(w));
      else asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(u[e]) : "v"(s[e]), "s"(W.nscale), "v"(w));
    } else {
      if constexpr (SMX) asm volatile("v_fma_f32 %0, %1, -%2, %3" : "=v"(u[e]) : "v"(s[e]), "s"(W.nscale), "v"(nbias_v));
      else asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(u[e]) : "v"(s[e]), "s"(W.nscale), "v"(nbias_v));
    }
  } else if constexpr (i < L::oA) {
    asm volatile("v_exp_f32 %0, %0" : "+v"(u[e]));
  } else if constexpr (i < L::oR) {
    asm volatile("v_add_f32 %0, 1.0, %0" : "+v"(u[e]));
  } else if constexpr (i < L::oC) {
    asm volatile("v_rcp_f32 %0, %0" : "+v"(u[e]));
  } else if constexpr (i < L::oQ) {
    constexpr int kor = key_of_reg(e);
    if constexpr (MODE == BWD_DKDV)
      asm volatile("v_cmp_ge_i32_e64 %0, %2, %3\n\tv_cndmask_b32_e64 %1, 0, %1, %0" : "=&s"(km[e]), "+v"(u[e]) : "n"(kor), "v"(thr));
    else
      asm volatile("v_cmp_le_i32_e64 %0, %2, %3\n\tv_cndmask_b32_e64 %1, 0, %1, %0" : "=&s"(km[e]), "+v"(u[e]) : "n"(kor), "v"(thr));
  } else if constexpr (i < L::oM) {
    if constexpr (SMX) asm volatile("v_sub_f32 %0, %1, %2" : "=v"(v[e]) : "v"(dp[e]), "v"(dstat_v));
    else asm volatile("v_fma_f32 %0, -%1, %1, %1" : "=v"(v[e]) : "v"(u[e]));
  } else if constexpr (i < L::oD) {
    if constexpr (SMX) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(v[e]) : "v"(u[e]));
    else asm volatile("v_mul_f32 %0, %0, %1" : "+v"(v[e]) : "v"(dp[e]));
  } else if constexpr (i < L::oB) {
    asm volatile("v_cndmask_b32_e64 %0, 0, %0, %1" : "+v"(v[e]) : "s"(km[e]));
  } else if constexpr (i < L::oP) {
    asm volatile("v_add_f32 %0, %0, %1" : "+v"(W.dbs[i - L::oB]) : "v"(v[e]));
  } else if constexpr (i < L::oS) {
    constexpr int j = 2 * G + (i - L::oP);
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(wp[j]) : "v"(u[2 * j]), "v"(u[2 * j + 1]));
  } else {
    constexpr int j = 2 * G + (i - L::oS);
    asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(wd[j]) : "v"(v[2 * j]), "v"(v[2 * j + 1]));
  }
}
template <int D, int MODE, bool ALIBI, bool MASK, bool SMX, int LO, int HI>
__device__ __forceinline__ void bsig_ops(BwdWave<D, MODE>& W, const f32x16& s, const f32x16& dp, float (&u)[16],
                                         float (&v)[16], uint32_t (&wp)[8], uint32_t (&wd)[8], uint64_t (&km)[16],
                                         float nbias_v, float sl2_v, float dist0, float dstep, int thr, float dstat_v,
                                         BsigStats& st) {
  if constexpr (LO < HI) {
    bsig_op<D, MODE, ALIBI, MASK, SMX, LO>(W, s, dp, u, v, wp, wd, km, nbias_v, sl2_v, dist0, dstep, thr, dstat_v, st);
    bsig_ops<D, MODE, ALIBI, MASK, SMX, LO + 1, HI>(W, s, dp, u, v, wp, wd, km, nbias_v, sl2_v, dist0, dstep, thr, dstat_v, st);
  }
}

template <int D, int MODE, bool ALIBI, int PAR, bool DMA, bool MASK, bool FOLD, bool GUARD, bool SMX, int K>
__device__ __forceinline__ void bwd_full_subslots(BwdWave<D, MODE>& W, uint32_t trimm, const uint32_t* nextrow,
                                                  uint32_t nextimm, float (&u)[16], float (&v)[16], uint32_t (&wp)[8],
                                                  uint32_t (&wd)[8], uint64_t (&km)[16], float nbias_v, float sl2_v,
                                                  float dist0, float dstep, int thr, float dstat_v, BsigStats& stats,
                                                  const DmaStagerX<D, 4>& st1,
                                                  const DmaStagerX<D, 4>& st2, uint32_t dma_lds, int uwave) {
  constexpr int KD = D / 16, DT = D / 32;
  constexpr uint32_t T2OFF = 64 * D * 2;
  constexpr int NA = 2 * KD;                               // first-product MFMAs
  constexpr int NB = MODE == BWD_DKDV ? 2 * KD : KD;       // second-product MFMAs
  constexpr int NSUB = NA + NB;
  constexpr int NOPS = BsigLayout<MODE, MASK, SMX>::NOPS;
  if constexpr (K < NSUB) {
    if constexpr (K < NA) {
      constexpr int kk = K / 2;
      if constexpr ((K & 1) == 0) {
        // S-type product from tensor 1, then fetch the transposed tensor-1 fragment kk
        if constexpr (kk == 0 && FOLD) b_mfma_vinit(W.s[PAR], W.F[K], W.x1[kk], W.cinit);
        else if constexpr (kk == 0) b_mfma_v0<GUARD>(W.s[PAR], W.F[K], W.x1[kk]);
        else b_mfma_v<GUARD>(W.s[PAR], W.F[K], W.x1[kk]);
        const uint32_t off = trimm + (kk / DT) * 16 * (D * 2);
        W.F[K] = join_tr(lds_read_tr16(W.tr[kk % DT][0] + off), lds_read_tr16(W.tr[kk % DT][1] + off));
      } else {
        // dP-type product from tensor 2
        if constexpr (kk == 0) b_mfma_v0<GUARD>(W.dp[PAR], W.F[K], W.x2[kk]);
        else b_mfma_v<GUARD>(W.dp[PAR], W.F[K], W.x2[kk]);
        if constexpr (MODE == BWD_DKDV) {
          const uint32_t off = trimm + (kk / DT) * 16 * (D * 2) + T2OFF;
          W.F[K] = join_tr(lds_read_tr16(W.tr[kk % DT][0] + off), lds_read_tr16(W.tr[kk % DT][1] + off));
        } else {
          W.F[K] = as_bf16x8(lds_read_b128(nextrow[kk] + nextimm + T2OFF));  // DQ: V is only read row-wise
        }
      }
    } else {
      constexpr int KB = K - NA;
      if constexpr (KB == 2) mfma_pin(W.s[PAR], W.dp[PAR]);
      if constexpr (MODE == BWD_DKDV) {
        constexpr int j = KB / 2;
        if constexpr ((KB & 1) == 0) {
          b_mfma_a<GUARD>(W.acc0[j % DT], W.F[2 * j], W.dsb[PAR][j / DT]);      // dK^T += Q^T dS
          W.F[2 * j] = as_bf16x8(lds_read_b128(nextrow[j] + nextimm));
        } else {
          b_mfma_a<GUARD>(W.acc1[j % DT], W.F[2 * j + 1], W.pb[PAR][j / DT]);   // dV^T += dO^T P
          W.F[2 * j + 1] = as_bf16x8(lds_read_b128(nextrow[j] + nextimm + T2OFF));
        }
      } else {
        constexpr int j = KB;
        b_mfma_a<GUARD>(W.acc0[j % DT], W.F[2 * j], W.dsb[PAR][j / DT]);        // dQ^T += K^T dS^T
        W.F[2 * j] = as_bf16x8(lds_read_b128(nextrow[j] + nextimm));
      }
    }
    bsig_ops<D, MODE, ALIBI, MASK, SMX, (K * NOPS) / NSUB, ((K + 1) * NOPS) / NSUB>(W, W.s[PAR ^ 1], W.dp[PAR ^ 1], u, v, wp,
                                                                                    wd, km, nbias_v, sl2_v, dist0, dstep,
                                                                                    thr, dstat_v, stats);
    if constexpr (DMA) {
      // one staging instruction of the tile two ahead every DSTEP sub-slots
      constexpr int NI = DmaStagerX<D, 4>::NI, DSTEP = NSUB / (2 * NI);
      if constexpr (K % DSTEP == 1 && K / DSTEP < 2 * NI) {
        constexpr int n = K / DSTEP;
        if constexpr (n < NI) st1.template issue_one<n>(dma_lds, uwave);
        else st2.template issue_one<n - NI>(dma_lds + 64 * D * 2, uwave);
      }
    }
    bwd_full_subslots<D, MODE, ALIBI, PAR, DMA, MASK, FOLD, GUARD, SMX, K + 1>(W, trimm, nextrow, nextimm, u, v, wp, wd, km,
                                                                               nbias_v, sl2_v, dist0, dstep, thr, dstat_v,
                                                                               stats, st1, st2, dma_lds, uwave);
  }
}

// thr (MASK only): elements with key_of_reg(e) >= thr (DKDV) / <= thr (DQ) are kept.
// GUARD puts the two wait states in front of every MFMA (for kernels whose register pressure
// makes the compiler park streamed fragments in AGPRs and copy them back right before use).
// SETTLE = false leaves the wait for the last MFMAs to the caller (a loop of pinned steps only,
// which waits once after the loop).
// SMX: the softmax arithmetic (dQ pass: W.nlse and W.dstat hold the lane's row statistics; dK/dV
// pass: `stat` = LDS address of the statistics of the lane's first query in the chunk).
template <int D, int MODE, bool ALIBI, bool FOLD, int PAR, bool DMA, bool MASK = false, bool SETTLE = true, bool GUARD = false,
          bool SMX = false>
__device__ __forceinline__ void bwd_step_full_pinned(BwdWave<D, MODE>& W, uint32_t trimm, const uint32_t* nextrow,
                                                     uint32_t nextimm, int cs, const DmaStagerX<D, 4>& st1,
                                                     const DmaStagerX<D, 4>& st2, uint32_t dma_lds, int uwave,
                                                     int thr = 0, uint32_t stat = 0) {
  float u[16], v[16];
  uint32_t wp[8], wd[8];
  uint64_t km[16];
  BsigStats stats;
  stats.stat = stat;
  // |i-j| of register r: DKDV streams queries (b - a), DQ streams keys (a - b)
  const int bl = cs + 8 * W.h;
  const float dist0 = MODE == BWD_DKDV ? (float)(bl - W.ai) : (float)(W.ai - bl);
  const float dstep = MODE == BWD_DKDV ? 1.0f : -1.0f;
  static_assert(!SMX || !FOLD, "softmax: ALiBi in its |i-j| form");
  if constexpr (FOLD)  // the per-element arithmetic is the one without ALiBi, on a per-step bias
    bwd_full_subslots<D, MODE, false, PAR, DMA, MASK, true, GUARD, false, 0>(W, trimm, nextrow, nextimm, u, v, wp, wd, km,
                                                                      __builtin_fmaf(W.sl2, dist0, W.nbias), W.sl2, dist0,
                                                                      dstep, thr, 0.f, stats, st1, st2, dma_lds, uwave);
  else
    bwd_full_subslots<D, MODE, ALIBI, PAR, DMA, MASK, false, GUARD, SMX, 0>(W, trimm, nextrow, nextimm, u, v, wp, wd, km,
                                                                     SMX ? W.nlse : W.nbias, SMX ? -W.sl2 : W.sl2, dist0,
                                                                     dstep, thr, W.dstat, stats, st1, st2, dma_lds, uwave);
  // The compiler does not know that the asm statements above are MFMAs: let the last ones
  // retire before it may touch their accumulators (copies at the join with the other path).
  if constexpr (SETTLE) mfma_settle();
  if (MODE == BWD_DKDV) {
    W.pb[PAR ^ 1][0] = as_bf16x8(u32x4{wp[0], wp[1], wp[2], wp[3]});
    W.pb[PAR ^ 1][1] = as_bf16x8(u32x4{wp[4], wp[5], wp[6], wp[7]});
  }
  W.dsb[PAR ^ 1][0] = as_bf16x8(u32x4{wd[0], wd[1], wd[2], wd[3]});
  W.dsb[PAR ^ 1][1] = as_bf16x8(u32x4{wd[4], wd[5], wd[6], wd[7]});
}

// PIN = false runs every step in its compiler-scheduled form (the form the softmax variant
// always uses): the like-for-like counterpart for comparisons.
// GROUPS (dK/dV pass only) compiles the loop over the query heads that share a K/V head; without
// it the pass handles exactly one query head per K/V head and p.kv_group must be 1.
// One block (128 rows of the stationary side) of head bh -- a K/V head in the dK/dV pass, a
// query head in the dQ pass -- from the first load to the last store; `record` is its slot in
// the clock probe's buffer.
template <int D, int MODE, bool CAUSAL, bool ALIBI, bool SOFTMAX, bool PIN = true, bool GROUPS = false>
__device__ __forceinline__ void attn_bwd_body(const BwdParams& p, const int bh, const int blk, const int record,
                                              const int tid) {
  static_assert(!GROUPS || MODE == BWD_DKDV, "only the dK/dV pass iterates over query heads");
  constexpr int NW = 4, BS = 32 * NW, BC = 64, KD = D / 16, DT = D / 32;
  constexpr bool FOLD = !SOFTMAX && CAUSAL && ALIBI;  // see bwd_step
  // kernels that carry the pinned steps; kStats: the softmax dK/dV pass, whose pinned steps read
  // the row statistics of the streamed queries from a side ring in LDS
  constexpr bool kPinned = PIN;
  constexpr bool kStats = SOFTMAX && MODE == BWD_DKDV && kPinned;
  constexpr int TILE = BC * D * 2, SLOT = 2 * TILE, CHUNK = 32 * D * 2, NSLOT = 4;
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(SATTN_LDS(char)*)smem;

  const int wave = tid >> 6, lane = tid & 63, l32 = lane & 31, h = lane >> 5;
  const int uwave = __builtin_amdgcn_readfirstlane(wave);
  ClockStart clk = clock_probe_begin(p.clock);
  // the dK/dV pass runs one workgroup per K/V head and key block and streams the query heads
  // of that head's group one after the other; the dQ pass runs per query head
  const int kv_group = (MODE == BWD_DKDV && !GROUPS) ? 1 : p.kv_group;
  const int heads = MODE == BWD_DKDV ? p.H / kv_group : p.H;
  // (a split group: bh counts (batch, K/V head, split) triples, the split running fastest)
  const int n_split = (GROUPS && p.n_split > 1) ? p.n_split : 1;
  const int split = GROUPS ? bh % n_split : 0, bh_g = GROUPS ? bh / n_split : bh;
  const int b = bh_g / heads, hd = bh_g % heads;  // hd: K/V head (dK/dV pass) or query head (dQ pass)
  const int hkv = MODE == BWD_DKDV ? hd : hd / kv_group;
  const int n_hq = MODE == BWD_DKDV ? kv_group / n_split : 1;
  const int hq0 = MODE == BWD_DKDV ? hd * kv_group + split * n_hq : hd;
  int N = p.N;
  int64_t tok0 = 0;
  float nbias_log2 = p.nbias_log2;
  if (p.cu_seqlens) {
    tok0 = p.cu_seqlens[b];
    N = min(p.cu_seqlens[b + 1] - (int)tok0, p.N);  // never beyond the span the host checked
    if (p.bias_vec) nbias_log2 = -p.bias_vec[b] * kLog2e;
    if (blk * BS >= N) return;  // this sequence has no such block (whole workgroup)
  }
  // keys may differ in number from queries (cross attention): N counts the
  // queries, Nk the keys; Ns / Nt are the row counts of this pass's stationary / streamed side
  const int Nk = p.Nk > 0 ? p.Nk : N;
  const int Ns = MODE == BWD_DKDV ? Nk : N, Nt = MODE == BWD_DKDV ? N : Nk;

  const __bf16* kbase = (const __bf16*)p.k.ptr + b * p.k.sb + hkv * p.k.sh + tok0 * p.k.ss;
  const __bf16* vbase = (const __bf16*)p.v.ptr + b * p.v.sb + hkv * p.v.sh + tok0 * p.v.ss;
  // query-side tensors of query head hq
  auto qhead = [&](int hq) { return (const __bf16*)p.q.ptr + b * p.q.sb + hq * p.q.sh + tok0 * p.q.ss; };
  auto dohead = [&](int hq) { return (const __bf16*)p.dout.ptr + b * p.dout.sb + hq * p.dout.sh + tok0 * p.dout.ss; };
  // stationary tensors x1, x2 and streamed tensors y1, y2 (per query head in the dK/dV pass)
  const __bf16* x1b = MODE == BWD_DKDV ? kbase : qhead(hq0);
  const __bf16* x2b = MODE == BWD_DKDV ? vbase : dohead(hq0);
  const int64_t x1s = MODE == BWD_DKDV ? p.k.ss : p.q.ss, x2s = MODE == BWD_DKDV ? p.v.ss : p.dout.ss;
  const int64_t y1s = MODE == BWD_DKDV ? p.q.ss : p.k.ss, y2s = MODE == BWD_DKDV ? p.dout.ss : p.v.ss;

  const int a_wave0 = blk * BS + wave * 32, ai = a_wave0 + l32, ai_ld = ai < Ns ? ai : Ns - 1;

  BwdWave<D, MODE> W;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      W.acc0[dt][r] = 0.f;
      if (MODE == BWD_DKDV) W.acc1[dt][r] = 0.f;
    }
  // W.ai is only ever used as a position, compared with or subtracted from the streamed side's
  // row index: a key's place on the query axis in the dK/dV pass, a query's place on the key
  // axis in the dQ pass
  W.ai = MODE == BWD_DKDV ? ai - p.qoff : ai + p.qoff; W.h = h;
  W.nscale = p.nscale_log2; W.nbias = nbias_log2;
  W.nlse = 0.f; W.dstat = 0.f;
  W.dbs[0] = W.dbs[1] = W.dbs[2] = W.dbs[3] = 0.f;
  if (SOFTMAX && MODE != BWD_DKDV) {
    W.nlse = p.nlse2[((int64_t)b * p.H + hq0) * p.npad + ai_ld];
    W.dstat = p.dvec[((int64_t)b * p.H + hq0) * p.npad + ai_ld];
  }

  // chunk range of the streamed side: workgroup [wg_lo, wg_hi], this wave [c_lo, c_hi]
  const int n_chunks = (Nt + 31) / 32;
  int wg_lo = 0, wg_hi = n_chunks - 1, c_lo = 0, c_hi = n_chunks - 1;
  if (CAUSAL) {
    if (MODE == BWD_DKDV) {
      // queries before the block's first key (at place key - qoff on the query axis) see none of its keys
      const int first = blk * BS - p.qoff, first_w = a_wave0 - p.qoff;
      wg_lo = (first > 0 ? first : 0) / 32;
      c_lo = (first_w > 0 ? first_w : 0) / 32;
    } else {
      // keys after the block's last query (at place query + qoff on the key axis) are masked
      const int a_hi = (blk * BS + BS < Ns ? blk * BS + BS : Ns) - 1 + p.qoff;
      const int last_w = (a_wave0 + 31 < Ns ? a_wave0 + 31 : Ns - 1) + p.qoff;
      wg_hi = (a_hi < 0 ? 0 : (a_hi < Nt ? a_hi : Nt - 1)) / 32;
      c_hi = (last_w < Nt ? last_w : Nt - 1) / 32;
      if (last_w < 0) { c_lo = 1; c_hi = 0; }  // every key lies after this wave's queries
    }
  }
  if (a_wave0 >= Ns) { c_lo = 1; c_hi = 0; }  // wave past the end: no chunks
  // The per-step flags are wave-uniform: evaluate them on the scalar unit.  The branch itself
  // stays an exec-mask branch on an opaque VGPR copy of the flag (lane_flag), which keeps the
  // two step variants in one linear region for the register allocator.
  const int c_lo_s = __builtin_amdgcn_readfirstlane(c_lo), c_hi_s = __builtin_amdgcn_readfirstlane(c_hi);
  // step s handles chunks s, s-1, s-2; tile t holds chunks 2t, 2t+1 and runs steps 2t, 2t+1
  const int t_lo = wg_lo / 2, t_hi = (wg_hi + 2) / 2;  // the last step is wg_hi + 2
  const int t_data_hi = wg_hi / 2;                      // last tile that has to be staged

  auto load_stationary = [&]() {
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) {
      W.x1[kk] = as_bf16x8(*(const u32x4*)(x1b + (int64_t)ai_ld * x1s + 16 * kk + 8 * h));
      W.x2[kk] = as_bf16x8(*(const u32x4*)(x2b + (int64_t)ai_ld * x2s + 16 * kk + 8 * h));
    }
  };
  // (with a loop over query heads the fragments are loaded once, ahead of the loop)
  if constexpr (GROUPS) load_stationary();
  for (int hq = hq0; hq < hq0 + n_hq; ++hq) {  // one pass of the pipeline per query head
  const __bf16* y1b = MODE == BWD_DKDV ? qhead(hq) : kbase;
  const __bf16* y2b = MODE == BWD_DKDV ? dohead(hq) : vbase;
  // softmax statistics of query head hq
  const float* stat_l = SOFTMAX ? p.nlse2 + ((int64_t)b * p.H + hq) * p.npad : nullptr;
  const float* stat_d = SOFTMAX ? p.dvec + ((int64_t)b * p.H + hq) * p.npad : nullptr;
  W.sl2 = ALIBI ? p.slopes[hq] * kLog2e : 0.f;
  // the pipeline starts empty: the second-product stage of the first steps must add zeros
  {
    const bf16x8 z = as_bf16x8(u32x4{0, 0, 0, 0});
    W.pb[0][0] = W.pb[0][1] = W.pb[1][0] = W.pb[1][1] = z;
    W.dsb[0][0] = W.dsb[0][1] = W.dsb[1][0] = W.dsb[1][1] = z;
#pragma unroll
    for (int r = 0; r < 16; ++r) { W.s[0][r] = W.s[1][r] = W.dp[0][r] = W.dp[1][r] = 0.f; }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r)  // DKDV: |i-j| = (bl - ai) + key_of_reg(r); DQ: (ai - bl) - key_of_reg(r)
    W.cinit[r] = FOLD ? (MODE == BWD_DKDV ? W.sl2 : -W.sl2) * (float)key_of_reg(r) / p.nscale_log2 : 0.f;
  // (With a loop over query heads the set-up below goes through an opaque copy of the thread
  // index made inside the loop: otherwise everything that depends on the lane alone -- these
  // addresses, the stagers' offsets -- is hoisted out of the loop and held in registers across
  // the whole pipeline, which these kernels cannot afford.)
  int tid_s = tid;
  if constexpr (GROUPS) asm volatile("" : "+v"(tid_s));
  const int lane_s = tid_s & 63, l32_s = lane_s & 31, h_s = lane_s >> 5;
  // per-lane LDS addresses (the ring slot of tile t is t % 4)
  {
    const int kap = kappa(l32_s), i16 = lane_s & 15, blk1 = (lane_s >> 4) & 1;
    const int h = h_s;
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) {
      const uint32_t o = lds0 + kap * (D * 2) + (((2 * kk + h) ^ SwzX<D>::f(kap)) << 4);
      W.row0[kk] = o + (t_lo % NSLOT) * SLOT;
      W.row1[kk] = o + ((t_lo + 1) % NSLOT) * SLOT;
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int rd = 0; rd < 2; ++rd) {
        const int r = 8 * h + 4 * rd + (i16 >> 2);
        const int c = 4 * dt + 2 * blk1 + ((i16 & 3) >> 1);
        W.tr[dt][rd] = lds0 + ((t_lo + NSLOT - 1) % NSLOT) * SLOT + r * (D * 2) + ((c ^ SwzX<D>::f(r)) << 4) +
                       ((i16 & 1) << 3);
      }
  }

  DmaStagerX<D, NW> st1, st2;
  constexpr int NI_TILE = DmaStagerX<D, NW>::NI;  // staging instructions per wave, tensor and tile
  st1.init(y1b, y1s, Nt, t_lo * BC, uwave, lane_s);
  st2.init(y2b, y2s, Nt, t_lo * BC, uwave, lane_s);
  // side ring of the streamed queries' statistics (softmax dK/dV): slot of tile t = t % 4, behind the tile ring
  const uint32_t stat_base = lds0 + NSLOT * SLOT;
  StatStager sst;
  if constexpr (kStats) sst.init(stat_l, stat_d, p.npad);
  auto stage_stats = [&](int tile, int slot_of) {  // the statistics of `tile` into the side-ring slot of tile `slot_of`
    if constexpr (kStats) sst.issue(stat_base + (slot_of % NSLOT) * StatStager::SLOT, tile, lane);
  };
  // address of the statistics of this lane's first query in chunk c
  // (c = -1, the empty stage of the very first step, maps to a slot like any other: its elements are masked)
  auto stat_of_chunk = [&](int c) { return stat_base + ((c >> 1) & (NSLOT - 1)) * StatStager::SLOT + ((c & 1) * 32 + 8 * h) * 4; };
  // Prologue.  The workgroup's first loads share the compute unit's one path from memory, so
  // they are kept few and ordered by need: tile t_lo, the stationary fragments, then tile
  // t_lo+1, which may land while the first tile is computed (every tile waits for the next
  // one before its barrier anyway).  The pinned steps run their second-product stage from the
  // first step on, with zero P / dS until the pipeline has filled, so the slot of tile t_lo-1
  // must hold finite data: zeros, written here.
  {
    const uint32_t zslot = lds0 + ((t_lo + NSLOT - 1) % NSLOT) * SLOT + tid_s * 16;
#pragma unroll
    for (int i = 0; i < SLOT / (256 * 16); ++i) lds_write_b128(zslot + i * (256 * 16), u32x4{0, 0, 0, 0});
  }
  st1.issue(lds0 + (t_lo % NSLOT) * SLOT, Nt, uwave, lane);
  st2.issue(lds0 + (t_lo % NSLOT) * SLOT + TILE, Nt, uwave, lane);
  stage_stats(t_lo, t_lo);
  if constexpr (!GROUPS) load_stationary();
  if (t_lo + 1 <= t_data_hi) {
    st1.issue(lds0 + ((t_lo + 1) % NSLOT) * SLOT, Nt, uwave, lane);
    st2.issue(lds0 + ((t_lo + 1) % NSLOT) * SLOT + TILE, Nt, uwave, lane);
    stage_stats(t_lo + 1, t_lo + 1);
    // all but the newest 2 NI loads (+ 2 for the statistics): tile t_lo has landed, the
    // stationary fragments are in registers
    if constexpr (kStats) SATTN_WAIT_VMCNT(2 * NI_TILE + 2);
    else SATTN_WAIT_VMCNT(2 * NI_TILE);
  } else {
    SATTN_WAIT_VMCNT(0);
  }
  __syncthreads();
  clock_probe_mark(p.clock, clk, kMarkFirstProduct);
  // rows of chunk 2*t_lo for the first step
#pragma unroll
  for (int kk = 0; kk < KD; ++kk) {
    W.F[2 * kk] = as_bf16x8(lds_read_b128(W.row0[kk]));
    W.F[2 * kk + 1] = as_bf16x8(lds_read_b128(W.row0[kk] + TILE));
  }

  // Iteration t runs steps 2t and 2t+1 with one barrier between them.  Tile t+2 is staged
  // during step 2t+1 (into the slot of tile t-2, whose last reads were in step 2t-1, before
  // this iteration's barrier) and has landed before the next iteration's barrier, after which
  // step 2t+3 reads its first rows.
  auto flags = [&](int s, bool& doA, bool& doS, bool& doB, bool& mask) {
    doA = s >= c_lo_s && s <= c_hi_s;
    doS = s - 1 >= c_lo_s && s - 1 <= c_hi_s;
    doB = s - 2 >= c_lo_s && s - 2 <= c_hi_s;
    mask = (s - 1 == c_hi_s) || (CAUSAL && MODE == BWD_DKDV && s - 1 == c_lo_s);
  };
  // Outside the steady state the sigmoid passes still run the pinned step, in its masked
  // form: a stage whose chunk lies outside this wave's range works on whatever finite data
  // the ring and the registers hold and its P / dS are forced to zero (thr = keep nothing);
  // the diagonal / ragged chunk gets its per-lane threshold.  Only the ragged last query
  // chunk of the dK/dV pass (upper and lower bound at once) and the softmax variant take
  // the compiler-scheduled step.
  auto step_kind = [&](int s, bool& pin, int& thr) {
    constexpr int NONE = MODE == BWD_DKDV ? 1000 : -1000, ALL = -NONE;
    const bool doA = s >= c_lo_s && s <= c_hi_s;
    const bool doS = s - 1 >= c_lo_s && s - 1 <= c_hi_s;
    const bool doB = s - 2 >= c_lo_s && s - 2 <= c_hi_s;
    const int cs = 32 * (s - 1), bl = cs + 8 * h;
    const bool ragged = doS && s - 1 == c_hi_s && cs + 32 > Nt;
    // a step with at most one live stage (first and last step of the wave's range, steps
    // outside it) is cheaper in the flag-driven form, which skips the dead stages
    pin = kPinned && !(MODE == BWD_DKDV && ragged) && (int)doA + (int)doS + (int)doB >= 2;
    if (!doS) thr = NONE;
    else if (MODE == BWD_DKDV) thr = (CAUSAL && s - 1 == c_lo_s) ? W.ai - bl : ALL;
    else thr = (s - 1 == c_hi_s) ? ((CAUSAL && W.ai < Nt - 1 ? W.ai : Nt - 1) - bl) : ALL;
  };
  // A wave issues about one instruction every six cycles whatever the instruction, so the
  // per-tile control flow is kept out of the steady state: tiles whose two steps are both
  // full (chunks s, s-1, s-2 inside this wave's range, no mask: c_lo+2 <= s <= c_hi) run a
  // loop of pinned steps only; the tiles before and after run the flag-driven general body.
  // Every variant has its one barrier per tile at the same place, so waves of a workgroup
  // may be in different loops.
  const int t_s0 = !kPinned ? t_hi + 1 : (c_lo_s + 3) / 2;          // first tile with 2t >= c_lo+2
  // last tile with 2t+1 <= c_hi / last tile whose staging needs no clamping.  The steady loop
  // stages tile t+2 during tile t without looking at the tensor's end: when the tensor ends on
  // a tile boundary the stager stops at the last tile and tiles t+2 past it are that tile
  // again, written to a ring slot nobody reads; a ragged last tile needs the clamped form,
  // so the loop ends before it.
  const int t_s1a = (c_hi_s + 1) / 2 - 1, t_s1b = Nt % BC == 0 ? t_s1a : Nt / BC - 3;
  const int t_s1 = !kPinned ? t_lo - 1 : (t_s1a < t_s1b ? t_s1a : t_s1b);
  auto rotate = [&](int t) {
    // rotate the per-lane addresses by one ring slot
    const int s0 = t % NSLOT;  // row0 points at slot s0, row1 at s0+1, tr at s0-1 (mod 4)
    const int adv0 = s0 == NSLOT - 1 ? -(NSLOT - 1) * SLOT : SLOT;
    const int adv1 = s0 == NSLOT - 2 ? -(NSLOT - 1) * SLOT : SLOT;
    const int advt = s0 == 0 ? -(NSLOT - 1) * SLOT : SLOT;
#pragma unroll
    for (int kk = 0; kk < KD; ++kk) { W.row0[kk] += adv0; W.row1[kk] += adv1; }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) { W.tr[dt][0] += advt; W.tr[dt][1] += advt; }
  };
  int t = t_lo;
  int general_end = t_s0 < t_hi + 1 ? t_s0 : t_hi + 1;
  for (int phase = 0; phase < 2; ++phase) {
    for (; t < general_end; ++t) {
      {
        const int s = 2 * t;
        bool doA_s, doS_s, doB_s, mask_s;
        flags(s, doA_s, doS_s, doB_s, mask_s);
        // rows of chunk s+1 come from tile t (second half); transposed reads of chunk s-2 from tile t-1 (first half)
        bool pin_s;
        int thr;
        step_kind(s, pin_s, thr);
        // (the other kernels do not carry the pinned code at all)
        if (kPinned && lane_flag(pin_s)) {
          if constexpr (kPinned)
            bwd_step_full_pinned<D, MODE, ALIBI, FOLD, 0, false, true, true, GROUPS, SOFTMAX>(W, 0, W.row0, CHUNK, 32 * (s - 1), st1, st2, 0, uwave, thr, stat_of_chunk(s - 1));
        } else
          bwd_step<D, MODE, CAUSAL, ALIBI, SOFTMAX, 0>(W, lane_flag(doA_s), lane_flag(doS_s), lane_flag(doB_s),
                                                       lane_flag(mask_s), 0, W.row0, CHUNK, 32 * (s - 1), Nt, stat_l, stat_d);
      }
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): tile t+1 has landed
      // A bare barrier: fragment reads of the tiles that stay in the ring may remain in flight
      // across it.
      __builtin_amdgcn_s_barrier();
      {
        const int s = 2 * t + 1;
        bool doA_s, doS_s, doB_s, mask_s;
        flags(s, doA_s, doS_s, doB_s, mask_s);
        bool pin_s;
        int thr;
        step_kind(s, pin_s, thr);
        const bool more = t + 2 <= t_data_hi;
        if (more) {  // stage tile t+2 up front (the steady-state loop interleaves it instead)
          const uint32_t dma_lds = lds0 + ((t + 2) % NSLOT) * SLOT;
          st1.issue(dma_lds, Nt, uwave, lane);
          st2.issue(dma_lds + TILE, Nt, uwave, lane);
          stage_stats(t + 2, t + 2);
        }
        // rows of chunk s+1 come from tile t+1 (first half); transposed reads of chunk s-2 from tile t-1 (second half)
        // (the other kernels do not carry the pinned code at all)
        if (kPinned && lane_flag(pin_s)) {
          if constexpr (kPinned)
            bwd_step_full_pinned<D, MODE, ALIBI, FOLD, 1, false, true, true, GROUPS, SOFTMAX>(W, CHUNK, W.row1, 0, 32 * (s - 1), st1, st2, 0, uwave, thr, stat_of_chunk(s - 1));
        } else
          bwd_step<D, MODE, CAUSAL, ALIBI, SOFTMAX, 1>(W, lane_flag(doA_s), lane_flag(doS_s), lane_flag(doB_s),
                                                       lane_flag(mask_s), CHUNK, W.row1, 0, 32 * (s - 1), Nt, stat_l, stat_d);
      }
      rotate(t);
    }
    if constexpr (kPinned) if (phase == 0) {
      const bool any_steady = t <= t_s1;
      clock_probe_mark(p.clock, clk, kMarkSteadyBegin);
      const int t_steady_begin = t;
      // (a ragged tensor's steady loop ends early enough that its stagers never reach the end)
      const int n_sat = Nt % BC == 0 ? Nt : 0x7fffff00;
      if (any_steady) {
        st1.step_back_inside(n_sat);
        st2.step_back_inside(n_sat);
      }
      for (; t <= t_s1; ++t) {
        bwd_step_full_pinned<D, MODE, ALIBI, FOLD, 0, false, false, false, false, SOFTMAX>(W, 0, W.row0, CHUNK, 32 * (2 * t - 1), st1, st2, 0, uwave, 0, stat_of_chunk(2 * t - 1));
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): tile t+1 has landed
        __builtin_amdgcn_s_barrier();
        stage_stats(st1.j0 / BC, t + 2);  // (the tile the stager is at: t + 2, or the last one again, see above)
        bwd_step_full_pinned<D, MODE, ALIBI, FOLD, 1, true, false, false, false, SOFTMAX>(W, CHUNK, W.row1, 0, 32 * (2 * t), st1, st2,
                                                                    lds0 + ((t + 2) % NSLOT) * SLOT, uwave, 0,
                                                                    stat_of_chunk(2 * t));
        st1.advance_inside(n_sat);
        st2.advance_inside(n_sat);
        rotate(t);
      }
      if (any_steady) mfma_settle();  // once for the whole loop of pinned steps
      clock_probe_mark(p.clock, clk, kMarkSteadyEnd);
      clk.steady_tiles = t - t_steady_begin;
      clk.tiles = t_hi + 1 - t_lo;
    }
    general_end = t_hi + 1;
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // no staging may be in flight when the workgroup's LDS is released
  // the next query head refills the ring: every wave must have finished reading it
  if (hq + 1 < hq0 + n_hq) __syncthreads();
  }  // query heads

  if (MODE == BWD_DQ_DB) {
    // the two halves of the wave hold the sums over different keys of the same query row
    float rs = (W.dbs[0] + W.dbs[1]) + (W.dbs[2] + W.dbs[3]);
    rs += __shfl_xor(rs, 32);
    if (h == 0 && ai < Ns) p.db_rows[b * p.db_sb + hq0 * p.db_sh + tok0 + ai] = rs;
  }
  clock_probe_mark(p.clock, clk, kMarkStore);
  // Outputs as whole rows, transposed through the ring (free once every wave has left the loop).
  __syncthreads();
  if (GROUPS && n_split > 1) {
    // fp32 partial sums of this workgroup's share of the group, straight from the accumulators:
    // register 4g+t of tile dt is element [row ai][32dt + 8g + 4h + t]
    if (ai < Ns) {
      const int64_t slab = (int64_t)p.B * heads * Ns * D;  // one [B, Hkv, keys, d] tensor
      float* pk = p.part + (int64_t)split * slab + (((int64_t)b * heads + hd) * Ns + ai) * D;
      float* pv = pk + (int64_t)n_split * slab;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          *(f32x4*)(pk + 32 * dt + 8 * g + 4 * h) =
              f32x4{W.acc0[dt][4 * g], W.acc0[dt][4 * g + 1], W.acc0[dt][4 * g + 2], W.acc0[dt][4 * g + 3]};
          if constexpr (MODE == BWD_DKDV)
            *(f32x4*)(pv + 32 * dt + 8 * g + 4 * h) =
                f32x4{W.acc1[dt][4 * g], W.acc1[dt][4 * g + 1], W.acc1[dt][4 * g + 2], W.acc1[dt][4 * g + 3]};
        }
    }
  } else {
    const int rows_valid = Ns - a_wave0;  // <= 0 for a wave past the end
    const uint32_t obuf = lds0 + wave * (2 * RowStore<D>::BYTES);
    __bf16* o0 = (MODE == BWD_DKDV ? (__bf16*)p.dk.ptr + b * p.dk.sb + hkv * p.dk.sh + (tok0 + a_wave0) * p.dk.ss
                                   : (__bf16*)p.dq.ptr + b * p.dq.sb + hq0 * p.dq.sh + (tok0 + a_wave0) * p.dq.ss);
    // dQ and dK carry the 1/sqrt(d) of the logits
    RowStore<D>::run(W.acc0, p.inv_sqrt_d, obuf, lane, o0, MODE == BWD_DKDV ? p.dk.ss : p.dq.ss, rows_valid);
    if constexpr (MODE == BWD_DKDV) {
      __bf16* o1 = (__bf16*)p.dv.ptr + b * p.dv.sb + hkv * p.dv.sh + (tok0 + a_wave0) * p.dv.ss;
      RowStore<D>::run(W.acc1, 1.0f, obuf + RowStore<D>::BYTES, lane, o1, p.dv.ss, rows_valid);
    }
  }
  clock_probe_end(p.clock, clk, record);
}

// Place `logical` of a pass (consecutive places share a head) -> head and block, a head's blocks
// in heavy-first order under the causal mask (late query blocks for the dQ pass, early key
// blocks for the dK/dV pass); `places` = blocks dealt out per head.
template <int MODE, bool CAUSAL, bool GROUPS>
__device__ __forceinline__ void bwd_place(const BwdParams& p, int logical, int places, int& bh, int& rank) {
  const int kv_group = (MODE == BWD_DKDV && !GROUPS) ? 1 : p.kv_group;
  const int heads = MODE == BWD_DKDV ? p.H / kv_group : p.H;
  const int n_split = (GROUPS && p.n_split > 1) ? p.n_split : 1;
  head_and_rank(logical, places, p.B * heads * n_split, CAUSAL ? p.head_group : 1, bh, rank);
}
template <int MODE, bool CAUSAL>
__device__ __forceinline__ int bwd_block_of_rank(const BwdParams& p, int rank) {
  return (CAUSAL && MODE != BWD_DKDV) ? (p.n_blocks - 1 - rank) : rank;
}

// At d = 64 the ring takes 64 KB, so two workgroups fit a compute unit if the kernel stays within
// 256 registers.  The compiler-scheduled forms (softmax, PIN = false) need that second wave per
// SIMD to hide their schedule and sit right at the limit, so they are held to it; the pinned
// forms use more VGPRs than a two-wave split of the register file leaves (128 + 128).
template <int D, int MODE, bool CAUSAL, bool ALIBI, bool SOFTMAX, bool PIN = true, bool GROUPS = false>
__global__ void __launch_bounds__(256, ((D == 64 && !PIN) ? 2 : 1))
attn_bwd_kernel(const BwdParams p) {
  const int kv_group = (MODE == BWD_DKDV && !GROUPS) ? 1 : p.kv_group;
  // Under the causal mask the r-th longest and the r-th shortest block of a head together stream
  // the same number of tiles whatever r is: a workgroup that runs such a pair makes all
  // workgroups of the launch equal (no ragged end) and halves the gaps between workgroups.
  // (only the pinned passes carry the loop: it costs a few registers, which the kernels held to
  // 256 of them do not have)
  constexpr bool kCanPair = CAUSAL && PIN && MODE != BWD_DQ_DB;
  const bool pair = kCanPair && p.pair;
  const int places = pair ? p.n_blocks / 2 : p.n_blocks;
  const int total = places * p.B * (MODE == BWD_DKDV ? p.H / kv_group : p.H) * ((GROUPS && p.n_split > 1) ? p.n_split : 1);
  int bh, rank;
  bwd_place<MODE, CAUSAL, GROUPS>(p, xcd_remap(blockIdx.x, total), places, bh, rank);
  if constexpr (!kCanPair) {
    attn_bwd_body<D, MODE, CAUSAL, ALIBI, SOFTMAX, PIN, GROUPS>(p, bh, bwd_block_of_rank<MODE, CAUSAL>(p, rank),
                                                                (int)blockIdx.x, (int)threadIdx.x);
    return;
  }
  const int n_parts = pair ? 2 : 1;
#pragma nounroll
  for (int part = 0; part < n_parts; ++part) {
    const int blk = bwd_block_of_rank<MODE, CAUSAL>(p, part == 0 ? rank : p.n_blocks - 1 - rank);
    // The thread index goes in through an opaque copy made inside the loop: nothing derived from
    // it (lane addresses, swizzles, folded constants) can then be hoisted out of the loop and
    // held in registers across the whole block, which cost 60-90 registers and spills.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    attn_bwd_body<D, MODE, CAUSAL, ALIBI, SOFTMAX, PIN, GROUPS>(p, bh, blk, (int)(blockIdx.x + part * gridDim.x), tid);
    // the block's epilogue transposes through the ring that the next block's first loads refill
    if (part + 1 < n_parts) __syncthreads();
  }
}

// Both passes of the pinned backward in one grid (self-attention, one K/V head per query
// head): even places run the dK/dV workgroup, odd places the dQ workgroup of the same
// (head, block) place, each pass in its own heavy-first order.  The grid is one launch, so a
// pass's last, ragged round of workgroups is filled by the other pass, and a head's two
// passes run on the same XCD next to each other and share its L2.  (SOFTMAX: the comparison
// kernel's two passes; its pre-pass stays a launch of its own.)
template <int D, bool CAUSAL, bool ALIBI, bool SOFTMAX = false>
__global__ void __launch_bounds__(256, 1)
attn_bwd_merged_kernel(const BwdParams p) {
  const int total = p.n_blocks * p.B * p.H;
  const int logical = xcd_remap(blockIdx.x, 2 * total);
  int bh, rank;
  if (logical & 1) {
    bwd_place<BWD_DQ, CAUSAL, false>(p, logical >> 1, p.n_blocks, bh, rank);
    attn_bwd_body<D, BWD_DQ, CAUSAL, ALIBI, SOFTMAX, true, false>(p, bh, bwd_block_of_rank<BWD_DQ, CAUSAL>(p, rank), (int)blockIdx.x, (int)threadIdx.x);
  } else {
    bwd_place<BWD_DKDV, CAUSAL, false>(p, logical >> 1, p.n_blocks, bh, rank);
    attn_bwd_body<D, BWD_DKDV, CAUSAL, ALIBI, SOFTMAX, true, false>(p, bh, bwd_block_of_rank<BWD_DKDV, CAUSAL>(p, rank), (int)blockIdx.x, (int)threadIdx.x);
  }
}

// Second kernel of a split grouped dK/dV pass: dK = inv_sqrt_d * sum of the dK partials, dV =
// sum of the dV partials, rounded to bf16 once.  One thread per eight consecutive features;
// blockIdx.y = 0 for dK, 1 for dV.
template <int D>
__global__ void __launch_bounds__(256)
group_partials_reduce_kernel(const float* part, TensorRef dk, TensorRef dv, int n_split, int B, int Hkv, int Nk,
                             float inv_sqrt_d) {
  const int which = blockIdx.y;
  const int64_t slab = (int64_t)B * Hkv * Nk * D;
  const int64_t e0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (e0 >= slab) return;
  const float* src = part + (int64_t)which * n_split * slab + e0;
  f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < n_split; ++s) {
    const f32x4 a = *(const f32x4*)(src + (int64_t)s * slab), c = *(const f32x4*)(src + (int64_t)s * slab + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) { lo[i] += a[i]; hi[i] += c[i]; }
  }
  const float scale = which == 0 ? inv_sqrt_d : 1.0f;
  const int col = (int)(e0 % D);
  const int64_t row_all = e0 / D;
  const int row = (int)(row_all % Nk);
  const int bh = (int)(row_all / Nk), b = bh / Hkv, hd = bh % Hkv;
  const TensorRef& o = which == 0 ? dk : dv;
  u32x4 w;
  w[0] = pack_bf16(lo[0] * scale, lo[1] * scale);
  w[1] = pack_bf16(lo[2] * scale, lo[3] * scale);
  w[2] = pack_bf16(hi[0] * scale, hi[1] * scale);
  w[3] = pack_bf16(hi[2] * scale, hi[3] * scale);
  *(u32x4*)((__bf16*)o.ptr + b * o.sb + hd * o.sh + (int64_t)row * o.ss + col) = w;
}

// Pre-pass of the softmax backward: per query row D_i = sum_t dO[i][t] * O[i][t] (fp32) and
// -lse_i * log2(e), written to [B*H, npad] vectors (npad = N rounded up to 64; pad entries 0 so
// that the kernels may read whole chunks).  16 lanes per row, 8 elements per lane and pass.
template <int D>
__global__ void __launch_bounds__(256)
softmax_bwd_prepass_kernel(TensorRef o, TensorRef dout, const float* lse, float* nlse2, float* dvec, int B, int H,
                           int N, int npad) {
  const int64_t prow = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);  // padded row index
  const int sub = threadIdx.x & 15;
  const int64_t prows = (int64_t)B * H * npad;
  if (prow >= prows) return;  // whole 16-lane group
  const int64_t bh = prow / npad;
  const int i = (int)(prow % npad);
  float acc = 0.f;
  if (i < N) {
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
  if (sub == 0) {
    dvec[prow] = acc;
    nlse2[prow] = i < N ? -lse[bh * N + i] * kLog2e : 0.f;
  }
}

}  // namespace sattn
