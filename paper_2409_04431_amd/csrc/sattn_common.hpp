// Device-side building blocks shared by the gfx950 attention kernels: vector types, MFMA
// wrappers, fragment/LDS index maps.  HIP for CDNA4 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sattn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define SATTN_LDS(T) __attribute__((address_space(3))) T

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// One tensor as the kernels see it: base pointer plus element strides (d contiguous).
struct TensorRef {
  void* ptr;
  int64_t sb, sh, ss;
};

// ---- MFMA 32x32x16 bf16 (D = A*B + C).  Fragment maps for lane l (l32 = l%32, h = l/32):
//   A (32 x 16): row l32, k = 8h + slot            (8 bf16 per lane)
//   B (16 x 32): col l32, k = 8h + slot
//   C (32 x 32): col l32, row = 8*(r/4) + 4h + r%4 (16 fp32 per lane, r = register)
// The contraction index may be permuted freely as long as A and B use the same map.
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// fp32 pair -> packed bf16 (round to nearest even), low half = a.
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  bf16x2 v = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(uint32_t, v);
}

// Row permutation that makes the accumulator of S^T = K Q^T directly usable as the B
// operand of the next product.  A-row m of the S^T MFMA is fed with key kappa(m) (bits 2
// and 3 of m swapped); then register r = 4g + t of lane half h holds key
// 16*(g/2) + 8h + 4*(g%2) + t, i.e. registers 8ks..8ks+7 are eight consecutive keys
// 16ks + 8h + (0..7): exactly the k-slots of B for contraction step ks.
__device__ __forceinline__ int kappa(int m) { return (m & 0x13) | ((m & 4) << 1) | ((m & 8) >> 1); }
// key offset (inside a 32-key chunk, without the 8h lane-half term) held by register r
__host__ __device__ constexpr int key_of_reg(int r) { return 16 * (r >> 3) + (r & 7); }

// Transposing LDS read (ds_read_b64_tr_b16).  Within each block of 16 lanes, lane i
// receives 16-bit element (i % 4) of the 8 bytes addressed by lane 4j + i/4, for j = 0..3.
// Pointing lanes 4j..4j+3 at 16 contiguous elements of row j therefore hands lane i the
// four rows' element i: a 4 (k) x 16 (m) block read in "k-major per lane" order.
__device__ __forceinline__ s16x4 lds_read_tr16(uint32_t lds_byte_addr) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((SATTN_LDS(s16x4)*)(uintptr_t)lds_byte_addr);
}

__device__ __forceinline__ bf16x8 join_tr(s16x4 lo, s16x4 hi) {
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ u32x4 lds_read_b128(uint32_t lds_byte_addr) {
  return *(SATTN_LDS(u32x4)*)(uintptr_t)lds_byte_addr;
}
__device__ __forceinline__ void lds_write_b128(uint32_t lds_byte_addr, u32x4 v) {
  *(SATTN_LDS(u32x4)*)(uintptr_t)lds_byte_addr = v;
}

// s_waitcnt vmcnt(n), other counters untouched (gfx9 encoding, n < 16).
#define SATTN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | (n))

// Store a wave's 32 x D accumulator tile (DT transposed 32x32 MFMA results: register 4g+t of
// tile dt, lane (l32, h) = element [row l32][32dt + 8g + 4h + t]) as bf16 rows of a global
// tensor.  A lane holds four consecutive features of ITS row, so a store from the registers
// scatters 8-byte pieces over 32 rows per instruction; the wave instead transposes through a
// private LDS region -- rows padded by 16 bytes, which spreads the 32 rows of a write over the
// banks -- and stores whole rows, 16 bytes per lane.  `buf` must not be in use by any wave
// (the caller synchronises); only this wave touches it here, so the LDS counter is the only wait.
template <int D>
struct RowStore {
  static constexpr int DT = D / 32, ROWB = D * 2 + 16, BYTES = 32 * ROWB;
  static constexpr int LPR = D / 8, RPI = 64 / LPR;  // lanes per row, rows per store instruction
  __device__ __forceinline__ static void run(const f32x16 (&acc)[DT], float scale, uint32_t buf, int lane,
                                             __bf16* row0, int64_t stride, int rows_valid) {
    const int l32 = lane & 31, h = lane >> 5;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w;
        w[0] = pack_bf16(acc[dt][4 * g] * scale, acc[dt][4 * g + 1] * scale);
        w[1] = pack_bf16(acc[dt][4 * g + 2] * scale, acc[dt][4 * g + 3] * scale);
        *(SATTN_LDS(u32x2)*)(uintptr_t)(buf + l32 * ROWB + (32 * dt + 8 * g + 4 * h) * 2) = w;
      }
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    const int rr = lane / LPR, cc = lane % LPR;
    u32x4 v4[32 / RPI];
#pragma unroll
    for (int i = 0; i < 32 / RPI; ++i) v4[i] = lds_read_b128(buf + (RPI * i + rr) * ROWB + cc * 16);
#pragma unroll
    for (int i = 0; i < 32 / RPI; ++i) {
      const int row = RPI * i + rr;
      if (row < rows_valid) *(u32x4*)(row0 + (int64_t)row * stride + cc * 8) = v4[i];
    }
  }
};

// Measurement aid: when `out` is set, workgroup w < cap writes eight values to out[8w ..]:
// [0] the core cycles and [1] the ticks of the constant-rate counter it spent in the kernel
// (their ratio is the engine clock the kernel actually ran at: the clock drops under matrix
// load), then the ticks since the kernel's start at which wave 0 [2] issued its first tile
// product, [3] entered and [4] left the steady-state loop of pinned steps, [5] began to store
// its outputs, and [6] the tiles it ran in that loop, [7] the tiles of the workgroup.
struct ClockProbe {
  long long* out;
  int cap;
};
struct ClockStart {
  long long cycles, ticks;
  int mark[4];   // phase stamps, ticks since `ticks`
  int steady_tiles, tiles;
};
enum ClockMark { kMarkFirstProduct = 0, kMarkSteadyBegin = 1, kMarkSteadyEnd = 2, kMarkStore = 3 };
__device__ __forceinline__ ClockStart clock_probe_begin(const ClockProbe& c) {
  ClockStart s{0, 0, {0, 0, 0, 0}, 0, 0};
  if (c.out) { s.cycles = clock64(); s.ticks = wall_clock64(); }
  return s;
}
__device__ __forceinline__ void clock_probe_mark(const ClockProbe& c, ClockStart& s, int which) {
  if (c.out) s.mark[which] = (int)(wall_clock64() - s.ticks);
}
// `record`: the slot written (one per workgroup, or one per block of a workgroup that handles several)
__device__ __forceinline__ void clock_probe_end(const ClockProbe& c, const ClockStart& s, int record) {
  if (c.out && threadIdx.x == 0 && record < c.cap) {
    long long* o = c.out + 8 * (int64_t)record;
    o[0] = clock64() - s.cycles;
    o[1] = wall_clock64() - s.ticks;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[2 + i] = s.mark[i];
    o[6] = s.steady_tiles;
    o[7] = s.tiles;
  }
}
__device__ __forceinline__ void clock_probe_end(const ClockProbe& c, const ClockStart& s) {
  clock_probe_end(c, s, (int)blockIdx.x);
}

// Workgroup id -> logical tile id so that consecutive logical ids (which share a head's
// K/V) land on the same XCD and hence the same L2: hardware deals workgroup ids round-robin
// over the 8 XCDs.
__device__ __forceinline__ int xcd_remap(int bid, int total) {
  constexpr int kXcd = 8;
  int xcd = bid % kXcd, slot = bid / kXcd;
  int c = total / kXcd, r = total % kXcd;
  return xcd * c + (xcd < r ? xcd : r) + slot;
}

// Place of a workgroup in its launch -> (head, rank of the block in that head's dispatch
// order).  With group > 1 consecutive places walk one rank over `group` heads before moving on
// to the next rank.  A causal head's blocks differ widely in length and are dispatched longest
// first; when a head has fewer blocks than an XCD has compute units, the units would otherwise
// hold the short tail of one head next to the long start of the next all the time, and the
// launch ends with long blocks still running on a few units.  Walking a few heads abreast keeps
// blocks of similar length together and the short ones for the end.
__device__ __forceinline__ void head_and_rank(int place, int n_blocks, int n_heads, int group, int& head, int& rank) {
  const int per_group = group * n_blocks;
  const int G = place / per_group, r = place - G * per_group;
  const int left = n_heads - G * group, g_this = left < group ? left : group;
  rank = r / g_this;
  head = G * group + (r - rank * g_this);
}

}  // namespace sattn
