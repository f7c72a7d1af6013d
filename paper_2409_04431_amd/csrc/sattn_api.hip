// C ABI of the sigmoid-attention library: argument validation and kernel dispatch.
// See include/sattn.h (product contract) and include/sattn_bench.h (measurement aids).
#include "../../include/sattn.h"
#include "../../include/sattn_bench.h"

#include <hip/hip_runtime.h>
#include <math.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <map>
#include <utility>

#include "sattn_f32.hpp"
#include "sattn_launch.hpp"
#include "sattn_norm.hpp"

using namespace sattn;

namespace sattn {

bool ensure_dynamic_lds(const void* kernel, int dev, size_t lds) {
  static std::mutex mu;
  static std::map<std::pair<const void*, int>, size_t> granted;  // (kernel, device) -> largest size set so far
  const std::pair<const void*, int> key(kernel, dev);
  std::lock_guard<std::mutex> lock(mu);
  auto it = granted.find(key);
  if (it != granted.end() && it->second >= lds) return true;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return false;
  granted[key] = lds;
  return true;
}

}  // namespace sattn

// Scratch of softmax_attn_bwd_noalloc: what softmax_attn_bwd takes as its workspace (two fp32
// per padded query row), held in the library's own device image so that the call allocates
// nothing.  Every GPU the library runs on holds its own copy until the process ends.
constexpr size_t kNoAllocRows = (size_t)1 << 20;  // padded query rows B*H*roundup(N, 64)
static __device__ __align__(256) float scratch[2 * kNoAllocRows];  // 8 MiB

namespace {

// Device address of `scratch` on the current device.  In host code the array's name is only
// a handle; the address kernels can use comes from the runtime, once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
float* g_scratch_ptr[kMaxDevices] = {};

int scratch_on_current_device(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return SATTN_ERR_LAUNCH;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return SATTN_ERR_LAUNCH;
    }
    g_scratch_ptr[dev] = (float*)ptr;
  }
  *out = g_scratch_ptr[dev];
  return SATTN_OK;
}

int elem_size(sattn_dtype t) { return t == SATTN_BF16 ? 2 : 4; }

// Register-resident MFMA loop of the matrix-rate probe: 4 accumulators, 8 MFMAs per iteration.
__global__ void __launch_bounds__(256) mfma_bf16_probe_kernel(float* sink, int iters) {
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(0.01f * (float)((threadIdx.x % 7) + e));
    b[e] = (__bf16)(0.02f * (float)((threadIdx.x % 5) + e));
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u & 3] = mfma32(a, b, acc[u & 3]);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// out[bh] = sum over i < N of rows[b*sb + h*sh + i], in a fixed order (deterministic).
__global__ void __launch_bounds__(256)
rowsum_reduce_kernel(const float* rows, float* out, int H, int N, int64_t sb, int64_t sh) {
  __shared__ float part[256];
  const int bh = blockIdx.x, tid = threadIdx.x;
  const float* r = rows + (bh / H) * sb + (bh % H) * sh;
  float acc = 0.f;
  for (int i = tid; i < N; i += 256) acc += r[i];
  part[tid] = acc;
  __syncthreads();
#pragma unroll
  for (int m = 128; m >= 1; m >>= 1) {
    if (tid < m) part[tid] += part[tid + m];
    __syncthreads();
  }
  if (tid == 0) out[bh] = part[0];
}

// Packed sequences: out[b*H + h] = sum of rows[h*total + t] over the tokens t of sequence b that the
// backward pass covered (its first min(length, max_seqlen) tokens), in a fixed order.
__global__ void __launch_bounds__(256)
rowsum_reduce_varlen_kernel(const float* rows, float* out, const int* cu_seqlens, int H, int64_t total, int max_seqlen) {
  __shared__ float part[256];
  const int bh = blockIdx.x, tid = threadIdx.x, b = bh / H, h = bh % H;
  const int t0 = cu_seqlens[b], n = min(cu_seqlens[b + 1] - t0, max_seqlen);
  const float* r = rows + (int64_t)h * total + t0;
  float acc = 0.f;
  for (int i = tid; i < n; i += 256) acc += r[i];
  part[tid] = acc;
  __syncthreads();
#pragma unroll
  for (int m = 128; m >= 1; m >>= 1) {
    if (tid < m) part[tid] += part[tid + m];
    __syncthreads();
  }
  if (tid == 0) out[bh] = part[0];
}

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
  // the kernels address the rows of one (batch, head) slice with 32-bit byte offsets
  if (((int64_t)N + 256) * ss * elem_size(dt) > 0xffffffffLL) return SATTN_ERR_SHAPE;
  out->ptr = const_cast<void*>(ptr);
  out->sb = sb; out->sh = sh; out->ss = ss;
  return SATTN_OK;
}

// Shape of a forward workgroup: waves (32 query rows each) and depth of the V ring.
// Head dimension 64: two 4-wave workgroups share a compute unit (their LDS rings both fit) and
// overlap each other's barriers, which measured faster than one 8-wave workgroup at every size.
// Head dimension 128: the 96 KB ring of the three-slot V ring admits one workgroup per compute
// unit, so 4 waves halve the occupancy; that only pays while the problem is too small to give
// every compute unit an 8-wave workgroup (causal problems a little longer: their workgroups run
// heavy-first, so a second, light round costs less than idle compute units in the first).  With a
// two-slot V ring (80 KB) two 4-wave workgroups fit again; they win while a workgroup's key loop
// is short (per-workgroup prologue, diagonal and barrier waits overlap with the neighbour) and
// lose a few percent on long loops, where V is staged only one tile ahead.
std::atomic<int> g_fwd_waves{0};   // 0: choose per problem; 4, 8, 64, 65, 66: forced; 32: choose among the 32-row shapes
std::atomic<int> g_fwd_vslots{0};  // 0: choose per problem; 2 or 3: forced (sattn_set_fwd_v_slots)
std::atomic<int> g_bwd_merged{0};  // 0: choose per problem; 1: one grid wherever that form exists; 2: never; 3: never, and single blocks (sattn_set_bwd_merged)
std::atomic<long long*> g_clock_out{nullptr};  // sattn_set_clock_probe
std::atomic<int> g_clock_cap{0};
ClockProbe clock_probe() { return ClockProbe{g_clock_out.load(std::memory_order_relaxed), g_clock_cap.load(std::memory_order_relaxed)}; }

int compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
    (void)hipGetLastError();
    return 256;
  }
  return n;
}

struct FwdShape { int waves, v_slots; };

// allow64 = false: the choice among the 32-row shapes only (the kernels that have no 64-row form)
FwdShape pick_fwd_shape(int B, int H, int N, int d, int causal, bool allow64 = true) {
  int forced_waves = g_fwd_waves.load(std::memory_order_relaxed);
  if (forced_waves == 32) { allow64 = false; forced_waves = 0; }
  FwdShape s{8, 3};
  if (d == 64) {
    s.waves = 4;
  } else {
    const int64_t wg4 = (int64_t)B * H * ((N + 127) / 128);
    const int64_t cus = compute_units();
    const int64_t avg_tiles = (causal ? (N + 1) / 2 : N) / 64;  // 64-key tiles a workgroup visits on average
    if (wg4 <= (causal ? cus + cus / 2 : cus)) s = FwdShape{4, 3};
    else if (avg_tiles < (causal ? 16 : 48)) s = FwdShape{4, 2};
    // Long key loops with at least one 256-row workgroup per compute unit: four waves of 64 query
    // rows, which read half as much K/V from LDS per MFMA (waves = 64).  From a sweep over B, N
    // and the mask (with the causal launches walking several heads abreast, head_and_rank): 3-12 %
    // faster than the best 32-row shape from 16 tiles per workgroup on average with the causal
    // mask (N >= 2048) and from 24 without (N >= 1536); slower below.
    const int64_t wg64 = (int64_t)B * H * ((N + 255) / 256);
    if (allow64 && wg64 >= cus && avg_tiles >= (causal ? 16 : 24)) s = FwdShape{64, 3};
  }
  const int forced_vslots = g_fwd_vslots.load(std::memory_order_relaxed);
  if (forced_waves) {
    if (forced_waves != s.waves) s.v_slots = 3;
    s.waves = forced_waves;
  }
  if (forced_vslots) s.v_slots = forced_vslots;
  if (s.waves >= 64 && (d != 128 || !allow64)) s = FwdShape{4, 3};  // (a forced 64 where no such kernel exists)
  if (s.waves != 4 || d != 128) s.v_slots = 3;  // the only shape with a two-slot V ring
  return s;
}

// The two passes of the sigmoid backward as one grid (where the launcher has that form: both
// passes asked for, self-attention, one K/V head per query head).  It pays while a pass alone
// cannot fill the chip: measured 10-28 % faster below two workgroups per pass and compute unit
// (three without the causal mask), equal within 1.5 % from there to 16, and 9 % slower on very
// large grids (48 per unit, d = 64), where the two passes compete for the L2.
bool pick_bwd_merged(int B, int H, int N, int causal) {
  const int mode = g_bwd_merged.load(std::memory_order_relaxed);
  if (mode) return mode == 1;
  const int64_t wgs = (int64_t)B * H * ((N + 127) / 128), cus = compute_units();
  return wgs < (causal ? 2 : 3) * cus;
}

// Workgroups over which the dK/dV pass splits the query heads of one K/V head (a power of two
// that divides the group): one per K/V head and key block leaves compute units idle when there
// are few K/V heads -- with one K/V head, 8 sequences of 4096 tokens make 256 workgroups of
// unequal causal work -- so the group is split until the pass has two workgroups per compute
// unit under the causal mask (enough to deal the blocks out in pairs of equal work), one without.
int pick_group_split(int B, int Hkv, int group, int N, int causal) {
  const int64_t wgs = (int64_t)B * Hkv * ((N + 127) / 128), want = (int64_t)(causal ? 2 : 1) * compute_units();
  int s = 1;
  while (wgs * s < want && group % (2 * s) == 0) s *= 2;
  return s;
}

int check_shape(int B, int H, int N, int d, sattn_dtype dt) {
  if (dt != SATTN_BF16 && dt != SATTN_F32) return SATTN_ERR_UNSUPPORTED;
  if (d != 64 && d != 128) return SATTN_ERR_UNSUPPORTED;
  if (B <= 0 || H <= 0 || N <= 0) return SATTN_ERR_SHAPE;
  if ((int64_t)N > (1 << 24)) return SATTN_ERR_SHAPE;               // key distances are formed in fp32
  if ((int64_t)B * H * ((N + 31) / 32) > 0x7fffffffLL) return SATTN_ERR_SHAPE;  // 1-D grid of workgroups
  return SATTN_OK;
}

// ---------------------------------------------------------------- forward
template <int D>
int launch_fwd_f32(F32Params p, int causal, bool alibi, hipStream_t st) {
  p.n_blocks = (p.N + 127) / 128;
  dim3 grid(p.n_blocks * p.B * p.H), block(256);
  int rc = SATTN_OK;
  SATTN_DISPATCH2(causal, alibi, rc = launch(sigmoid_f32_kernel<D, F32_FWD, A, B2>, grid, block, 0, st, p));
  return rc;
}

struct FwdArgs {
  const void *q, *k, *v; void* o; float* lse;
  int B, H, N, d; sattn_dtype dtype; float bias; int causal; const float* slopes;
  const sattn_strides *sq, *sk, *sv, *so; void* stream;
  const int* cu_seqlens = nullptr; const float* bias_vec = nullptr;  // variable-length batches
  int Hkv = 0;                                                       // K/V heads (0: one per query head)
  int Nk = 0;                                                        // keys (0: as many as queries)
  bool end_aligned = false;                                          // queries = the last N positions of the key sequence
};

// A key count that differs from the query count: sigmoid attention with one K/V head per query
// head.  Without `end_aligned` plain attention only (no mask, no ALiBi: positions undefined);
// with it the queries sit at the end of the key sequence, which defines both; the bf16 kernels
// then need the offset Nk - N to be a multiple of 32 under the causal mask (a wave's query rows
// and a key chunk must meet in one diagonal chunk), the fp32 kernel takes any.
template <typename Args>
int check_cross(const Args& a, bool softmax, bool pin, int Hkv, int* Nk) {
  *Nk = a.Nk > 0 ? a.Nk : a.N;
  if (*Nk == a.N) return SATTN_OK;
  if (softmax || !pin || a.cu_seqlens || Hkv != a.H) return SATTN_ERR_UNSUPPORTED;
  if (!a.end_aligned && (a.causal || a.slopes)) return SATTN_ERR_UNSUPPORTED;
  if (a.end_aligned && a.causal && a.dtype == SATTN_BF16 && (*Nk - a.N) % 32 != 0) return SATTN_ERR_UNSUPPORTED;
  return check_shape(a.B, a.H, *Nk, a.d, a.dtype);
}

template <bool SOFTMAX, bool PIN = true>
int fwd_impl(const FwdArgs& a) {
  int rc = check_shape(a.B, a.H, a.N, a.d, a.dtype);
  if (rc) return rc;
  const int Hkv = a.Hkv ? a.Hkv : a.H;
  if (Hkv <= 0 || a.H % Hkv) return SATTN_ERR_SHAPE;
  if (Hkv != a.H && (SOFTMAX || !PIN)) return SATTN_ERR_UNSUPPORTED;
  int Nk;
  if ((rc = check_cross(a, SOFTMAX, PIN, Hkv, &Nk))) return rc;
  TensorRef q, k, v, o;
  if ((rc = make_ref(a.q, a.sq, a.H, a.N, a.d, a.dtype, &q))) return rc;
  if ((rc = make_ref(a.k, a.sk, Hkv, Nk, a.d, a.dtype, &k))) return rc;
  if ((rc = make_ref(a.v, a.sv, Hkv, Nk, a.d, a.dtype, &v))) return rc;
  if ((rc = make_ref(a.o, a.so, a.H, a.N, a.d, a.dtype, &o))) return rc;
  if (SOFTMAX && !a.lse) return SATTN_ERR_NULL;
  hipStream_t st = (hipStream_t)a.stream;
  const bool alibi = a.slopes != nullptr;
  const float inv_sqrt_d = 1.0f / sqrtf((float)a.d);
  if (a.dtype == SATTN_F32) {
    if (SOFTMAX || !PIN) return SATTN_ERR_UNSUPPORTED;  // comparison kernels and twins: bf16 only
    F32Params p{};
    p.q = q; p.k = k; p.v = v; p.out0 = o;
    p.slopes = a.slopes; p.B = a.B; p.H = a.H; p.N = a.N;
    p.scale = inv_sqrt_d; p.bias = a.bias;
    p.cu_seqlens = a.cu_seqlens; p.bias_vec = a.bias_vec;
    p.kv_group = a.H / Hkv;
    p.Nk = Nk == a.N ? 0 : Nk;
    p.qoff = a.end_aligned ? Nk - a.N : 0;
    if (a.d == 128) return launch_fwd_f32<128>(p, a.causal, alibi, st);
    return launch_fwd_f32<64>(p, a.causal, alibi, st);
  }
  FwdParams p{};
  p.q = q; p.k = k; p.v = v; p.o = o;
  p.slopes = a.slopes; p.lse = a.lse;
  p.B = a.B; p.H = a.H; p.N = a.N;
  p.nscale_log2 = (SOFTMAX ? kLog2e : -kLog2e) * inv_sqrt_d;
  p.nbias_log2 = -a.bias * kLog2e;
  p.cu_seqlens = a.cu_seqlens; p.bias_vec = a.bias_vec;
  p.kv_group = a.H / Hkv;
  p.Nk = Nk == a.N ? 0 : Nk;
  p.qoff = a.end_aligned ? Nk - a.N : 0;
  p.clock = clock_probe();
  // the 64-row waves exist for the pinned sigmoid kernel at d = 128, ALiBi only in its causal form
  const bool has64 = !SOFTMAX && PIN && a.d == 128 && !(alibi && !a.causal);
  const FwdShape shape = pick_fwd_shape(a.B, a.H, a.N, a.d, a.causal, has64);
  // The 64-row causal kernel deals a head's blocks out in pairs of equal work (longest with
  // shortest) where that still leaves a workgroup per compute unit.  Measured against single
  // blocks: 2-3.5 % faster from 16 blocks per head (N >= 4096), 3 % slower at 8 (B16 H16 N2048).
  // (66: single blocks, for that comparison.)
  const int nb64 = (a.N + 255) / 256;
  p.pair = shape.waves != 66 && a.causal && nb64 >= 16 && (int64_t)a.B * a.H * (nb64 / 2) >= compute_units();
  if (a.d == 128) return launch_fwd_bf16<128>(p, shape.waves, shape.v_slots, SOFTMAX, PIN, a.causal, alibi, st);
  return launch_fwd_bf16<64>(p, shape.waves, shape.v_slots, SOFTMAX, PIN, a.causal, alibi, st);
}

// ---------------------------------------------------------------- backward
template <int D>
int launch_bwd_f32(F32Params p, int causal, bool alibi, int parts, TensorRef dq, TensorRef dk, TensorRef dv,
                   hipStream_t st) {
  // the dQ pass runs one workgroup per query head and 128 queries, the dK/dV pass one per K/V
  // head and 128 keys
  const int nb_q = (p.N + 127) / 128, nb_k = ((p.Nk > 0 ? p.Nk : p.N) + 127) / 128;
  dim3 grid_q(nb_q * p.B * p.H), grid_kv(nb_k * p.B * (p.H / p.kv_group)), block(256);
  int rc = SATTN_OK;
  if (parts & kBwdDkDv) {
    p.n_blocks = nb_k;
    p.out0 = dk; p.out1 = dv;
    SATTN_DISPATCH2(causal, alibi, rc = launch(sigmoid_f32_kernel<D, F32_DKDV, A, B2>, grid_kv, block, 0, st, p));
  }
  if (rc == SATTN_OK && (parts & kBwdDq)) {
    p.n_blocks = nb_q;
    p.out0 = dq; p.out1 = TensorRef{};
    SATTN_DISPATCH2(causal, alibi, rc = launch(sigmoid_f32_kernel<D, F32_DQ, A, B2>, grid_q, block, 0, st, p));
  }
  return rc;
}

struct BwdArgs {
  const void *q, *k, *v, *o; const float* lse; const void* dout; void *dq, *dk, *dv;
  int B, H, N, d; sattn_dtype dtype; float bias; int causal; const float* slopes;
  const sattn_strides *sq, *sk, *sv, *so, *sdout, *sdq, *sdk, *sdv;
  void* workspace; size_t workspace_bytes; int parts; void* stream;
  const int* cu_seqlens = nullptr; const float* bias_vec = nullptr;  // variable-length batches
  float* db_rows = nullptr; float* db = nullptr;                     // bias gradient (sigmoid only)
  int64_t db_tokens = 0;                                             // packed sequences: tokens in db_rows' [H, tokens]
  int Hkv = 0;                                                       // K/V heads (0: one per query head)
  int Nk = 0;                                                        // keys (0: as many as queries)
  bool end_aligned = false;                                          // queries = the last N positions of the key sequence
  bool group_split = false;                                          // shared K/V heads: split a group over workgroups (workspace)
};

template <bool SOFTMAX, bool PIN = true>
int bwd_impl(const BwdArgs& a) {
  int rc = check_shape(a.B, a.H, a.N, a.d, a.dtype);
  if (rc) return rc;
  const int Hkv = a.Hkv ? a.Hkv : a.H;
  if (Hkv <= 0 || a.H % Hkv) return SATTN_ERR_SHAPE;
  if (Hkv != a.H && (SOFTMAX || !PIN)) return SATTN_ERR_UNSUPPORTED;
  int Nk;
  if ((rc = check_cross(a, SOFTMAX, PIN, Hkv, &Nk))) return rc;
  if (Nk != a.N && a.db_rows) return SATTN_ERR_UNSUPPORTED;
  TensorRef q, k, v, dout, dq{}, dk{}, dv{}, o{};
  if ((rc = make_ref(a.q, a.sq, a.H, a.N, a.d, a.dtype, &q))) return rc;
  if ((rc = make_ref(a.k, a.sk, Hkv, Nk, a.d, a.dtype, &k))) return rc;
  if ((rc = make_ref(a.v, a.sv, Hkv, Nk, a.d, a.dtype, &v))) return rc;
  if ((rc = make_ref(a.dout, a.sdout, a.H, a.N, a.d, a.dtype, &dout))) return rc;
  if ((a.parts & kBwdDq) && (rc = make_ref(a.dq, a.sdq, a.H, a.N, a.d, a.dtype, &dq))) return rc;
  if ((a.parts & kBwdDkDv) && (rc = make_ref(a.dk, a.sdk, Hkv, Nk, a.d, a.dtype, &dk))) return rc;
  if ((a.parts & kBwdDkDv) && (rc = make_ref(a.dv, a.sdv, Hkv, Nk, a.d, a.dtype, &dv))) return rc;
  hipStream_t st = (hipStream_t)a.stream;
  const bool alibi = a.slopes != nullptr;
  const float inv_sqrt_d = 1.0f / sqrtf((float)a.d);
  if (a.dtype == SATTN_F32) {
    if (SOFTMAX || !PIN) return SATTN_ERR_UNSUPPORTED;  // comparison kernels and twins: bf16 only
    F32Params p{};
    p.q = q; p.k = k; p.v = v; p.dout = dout;
    p.slopes = a.slopes; p.B = a.B; p.H = a.H; p.N = a.N;
    p.scale = inv_sqrt_d; p.bias = a.bias;
    p.cu_seqlens = a.cu_seqlens; p.bias_vec = a.bias_vec;
    p.kv_group = a.H / Hkv;
    p.Nk = Nk == a.N ? 0 : Nk;
    p.qoff = a.end_aligned ? Nk - a.N : 0;
    p.db_rows = a.db_rows; p.db_sb = (int64_t)a.H * a.N; p.db_sh = a.N;
    if (a.cu_seqlens && a.db_rows) { p.db_sb = 0; p.db_sh = a.db_tokens; }  // [H, tokens], as in the bf16 path
    if (a.d == 128) rc = launch_bwd_f32<128>(p, a.causal, alibi, a.parts, dq, dk, dv, st);
    else rc = launch_bwd_f32<64>(p, a.causal, alibi, a.parts, dq, dk, dv, st);
    if (rc == SATTN_OK && a.db) {
      if (a.cu_seqlens)
        rc = launch(rowsum_reduce_varlen_kernel, dim3(a.B * a.H), dim3(256), 0, st, (const float*)a.db_rows, a.db,
                    a.cu_seqlens, a.H, a.db_tokens, a.N);
      else
        rc = launch(rowsum_reduce_kernel, dim3(a.B * a.H), dim3(256), 0, st, (const float*)a.db_rows, a.db, a.H, a.N,
                    p.db_sb, p.db_sh);
    }
    return rc;
  }
  BwdParams p{};
  p.q = q; p.k = k; p.v = v; p.dout = dout; p.dq = dq; p.dk = dk; p.dv = dv;
  p.slopes = a.slopes;
  p.B = a.B; p.H = a.H; p.N = a.N;
  p.inv_sqrt_d = inv_sqrt_d;
  p.nscale_log2 = -kLog2e * inv_sqrt_d;
  p.nbias_log2 = -a.bias * kLog2e;
  p.cu_seqlens = a.cu_seqlens; p.bias_vec = a.bias_vec;
  p.db_rows = a.db_rows; p.db_sb = (int64_t)a.H * a.N; p.db_sh = a.N;
  if (a.cu_seqlens && a.db_rows) { p.db_sb = 0; p.db_sh = a.db_tokens; }  // [H, tokens]: the kernel adds the sequence's first token
  p.kv_group = a.H / Hkv;
  p.Nk = Nk == a.N ? 0 : Nk;
  p.qoff = a.end_aligned ? Nk - a.N : 0;
  p.clock = clock_probe();
  if (SOFTMAX) {
    if (!a.lse) return SATTN_ERR_NULL;
    if ((rc = make_ref(a.o, a.so, a.H, a.N, a.d, a.dtype, &o))) return rc;
    const int npad = (a.N + 63) / 64 * 64;
    const int64_t prows = (int64_t)a.B * a.H * npad;
    const size_t need = 2 * (size_t)prows * sizeof(float);
    if (!a.workspace || a.workspace_bytes < need) return SATTN_ERR_WORKSPACE;
    if (((uintptr_t)a.workspace & 15) != 0) return SATTN_ERR_ALIGN;
    if ((prows + 15) / 16 > 0x7fffffffLL) return SATTN_ERR_SHAPE;
    float* nlse2 = (float*)a.workspace;
    float* dvec = nlse2 + prows;
    dim3 grid((unsigned)((prows + 15) / 16)), block(256);
    if (a.d == 128)
      rc = launch(softmax_bwd_prepass_kernel<128>, grid, block, 0, st, o, dout, a.lse, nlse2, dvec, a.B, a.H, a.N, npad);
    else
      rc = launch(softmax_bwd_prepass_kernel<64>, grid, block, 0, st, o, dout, a.lse, nlse2, dvec, a.B, a.H, a.N, npad);
    if (rc) return rc;
    p.nlse2 = nlse2; p.dvec = dvec; p.npad = npad;
  }
  const bool merged = pick_bwd_merged(a.B, a.H, a.N, a.causal);
  int n_split = 1;
  if (a.group_split && !SOFTMAX && PIN && Hkv != a.H && !a.cu_seqlens && Nk == a.N && (a.parts & kBwdDkDv)) {
    n_split = pick_group_split(a.B, Hkv, a.H / Hkv, a.N, a.causal);
    if (n_split > 1) {
      const size_t need = 2 * (size_t)n_split * a.B * Hkv * a.N * a.d * sizeof(float);
      if (!a.workspace || a.workspace_bytes < need) return SATTN_ERR_WORKSPACE;
      if (((uintptr_t)a.workspace & 15) != 0) return SATTN_ERR_ALIGN;
      p.n_split = n_split;
      p.part = (float*)a.workspace;
    }
  }
  // causal passes deal a head's blocks out in pairs of equal work (longest with shortest) where
  // a pair per compute unit remains (see the 64-row forward)
  p.pair = a.causal && PIN && g_bwd_merged.load(std::memory_order_relaxed) != 3 &&
           (int64_t)a.B * Hkv * n_split * ((std::min(a.N, Nk) + 127) / 128 / 2) >= compute_units();
  if (a.d == 128) rc = launch_bwd_bf16<128>(p, SOFTMAX, PIN, a.causal, alibi, a.parts, merged, st);
  else rc = launch_bwd_bf16<64>(p, SOFTMAX, PIN, a.causal, alibi, a.parts, merged, st);
  if (rc == SATTN_OK && a.db) {
    if (a.cu_seqlens)
      rc = launch(rowsum_reduce_varlen_kernel, dim3(a.B * a.H), dim3(256), 0, st, (const float*)a.db_rows, a.db,
                  a.cu_seqlens, a.H, a.db_tokens, a.N);
    else
      rc = launch(rowsum_reduce_kernel, dim3(a.B * a.H), dim3(256), 0, st, (const float*)a.db_rows, a.db, a.H, a.N,
                  p.db_sb, p.db_sh);
  }
  return rc;
}

template <bool RMS, bool BACKWARD>
int launch_norm(const NormParams& p, hipStream_t st) {
  const int nchunks = p.H * (p.d / 8);
  const int64_t tokens = (int64_t)p.B * p.N;
  dim3 grid((unsigned)((tokens + 3) / 4)), block(256);
  if (nchunks <= 64) return launch(headconcat_norm_kernel<1, RMS, BACKWARD>, grid, block, 0, st, p);
  if (nchunks <= 128) return launch(headconcat_norm_kernel<2, RMS, BACKWARD>, grid, block, 0, st, p);
  if (nchunks <= 256) return launch(headconcat_norm_kernel<4, RMS, BACKWARD>, grid, block, 0, st, p);
  if (nchunks <= 512) return launch(headconcat_norm_kernel<8, RMS, BACKWARD>, grid, block, 0, st, p);
  return launch(headconcat_norm_kernel<16, RMS, BACKWARD>, grid, block, 0, st, p);
}

int norm_impl(bool backward, const void* x, const void* dy, void* out, float* stats, int B, int H, int N, int d,
              sattn_dtype dtype, int kind, float eps, const sattn_strides* sx, const sattn_strides* sdy,
              const sattn_strides* sout, void* stream) {
  int rc = check_shape(B, H, N, d, dtype);
  if (rc) return rc;
  if (dtype != SATTN_BF16 || (kind != SATTN_NORM_LAYER && kind != SATTN_NORM_RMS)) return SATTN_ERR_UNSUPPORTED;
  if ((int64_t)H * d > 8192) return SATTN_ERR_SHAPE;  // a wave keeps one token's features in registers
  if (((int64_t)B * N + 3) / 4 > 0x7fffffffLL) return SATTN_ERR_SHAPE;  // 1-D grid, four tokens per workgroup
  if (!(eps >= 0.f)) return SATTN_ERR_SHAPE;
  if (!stats) return SATTN_ERR_NULL;
  if (((uintptr_t)stats & 7) != 0) return SATTN_ERR_ALIGN;
  NormParams p{};
  if ((rc = make_ref(x, sx, H, N, d, dtype, &p.x))) return rc;
  if ((rc = make_ref(out, sout, H, N, d, dtype, &p.y))) return rc;
  if (backward && (rc = make_ref(dy, sdy, H, N, d, dtype, &p.dy))) return rc;
  p.stats = stats; p.B = B; p.H = H; p.N = N; p.d = d; p.eps = eps;
  hipStream_t st = (hipStream_t)stream;
  if (kind == SATTN_NORM_RMS) return backward ? launch_norm<true, true>(p, st) : launch_norm<true, false>(p, st);
  return backward ? launch_norm<false, true>(p, st) : launch_norm<false, false>(p, st);
}

}  // namespace

extern "C" {

int sigmoid_attn_fwd(const void* q, const void* k, const void* v, void* o, int B, int H, int N, int d,
                     sattn_dtype dtype, float bias, int causal, const float* alibi_slopes, const sattn_strides* sq,
                     const sattn_strides* sk, const sattn_strides* sv, const sattn_strides* so, void* stream) {
  FwdArgs a{q, k, v, o, nullptr, B, H, N, d, dtype, bias, causal, alibi_slopes, sq, sk, sv, so, stream};
  return fwd_impl<false>(a);
}

int sigmoid_attn_bwd(const void* q, const void* k, const void* v, const void* dout, void* dq, void* dk, void* dv,
                     int B, int H, int N, int d, sattn_dtype dtype, float bias, int causal,
                     const float* alibi_slopes, const sattn_strides* sq, const sattn_strides* sk,
                     const sattn_strides* sv, const sattn_strides* sdout, const sattn_strides* sdq,
                     const sattn_strides* sdk, const sattn_strides* sdv, void* workspace, size_t workspace_bytes,
                     void* stream) {
  // the split by output owner needs no workspace
  BwdArgs a{q, k, v, nullptr, nullptr, dout, dq, dk, dv, B, H, N, d, dtype, bias, causal, alibi_slopes,
            sq, sk, sv, nullptr, sdout, sdq, sdk, sdv, workspace, workspace_bytes, kBwdDkDv | kBwdDq, stream};
  return bwd_impl<false>(a);
}

int sigmoid_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* dout, void* dk, void* dv,
                          int B, int H, int N, int d, sattn_dtype dtype, float bias, int causal,
                          const float* alibi_slopes, const sattn_strides* sq, const sattn_strides* sk,
                          const sattn_strides* sv, const sattn_strides* sdout, const sattn_strides* sdk,
                          const sattn_strides* sdv, void* stream) {
  BwdArgs a{q, k, v, nullptr, nullptr, dout, nullptr, dk, dv, B, H, N, d, dtype, bias, causal, alibi_slopes,
            sq, sk, sv, nullptr, sdout, nullptr, sdk, sdv, nullptr, 0, kBwdDkDv, stream};
  return bwd_impl<false>(a);
}

int sigmoid_attn_bwd_dq(const void* q, const void* k, const void* v, const void* dout, void* dq, int B, int H,
                        int N, int d, sattn_dtype dtype, float bias, int causal, const float* alibi_slopes,
                        const sattn_strides* sq, const sattn_strides* sk, const sattn_strides* sv,
                        const sattn_strides* sdout, const sattn_strides* sdq, void* stream) {
  BwdArgs a{q, k, v, nullptr, nullptr, dout, dq, nullptr, nullptr, B, H, N, d, dtype, bias, causal, alibi_slopes,
            sq, sk, sv, nullptr, sdout, sdq, nullptr, nullptr, nullptr, 0, kBwdDq, stream};
  return bwd_impl<false>(a);
}

int sigmoid_attn_bwd_bias_grad(const void* q, const void* k, const void* v, const void* dout, void* dq, void* dk,
                               void* dv, float* db_rows, float* db, int B, int H, int N, int d, sattn_dtype dtype,
                               float bias, int causal, const float* alibi_slopes, const sattn_strides* sq,
                               const sattn_strides* sk, const sattn_strides* sv, const sattn_strides* sdout,
                               const sattn_strides* sdq, const sattn_strides* sdk, const sattn_strides* sdv,
                               void* stream) {
  if (!db_rows) return SATTN_ERR_NULL;
  if (((uintptr_t)db_rows & 3) != 0 || ((uintptr_t)db & 3) != 0) return SATTN_ERR_ALIGN;
  BwdArgs a{q, k, v, nullptr, nullptr, dout, dq, dk, dv, B, H, N, d, dtype, bias, causal, alibi_slopes,
            sq, sk, sv, nullptr, sdout, sdq, sdk, sdv, nullptr, 0, kBwdDkDv | kBwdDq, stream};
  a.db_rows = db_rows; a.db = db;
  return bwd_impl<false>(a);
}

size_t sigmoid_attn_bwd_workspace_bytes(int, int, int, int, sattn_dtype) { return 0; }

int sigmoid_attn_fwd_compiler_scheduled(const void* q, const void* k, const void* v, void* o, int B, int H, int N,
                                        int d, sattn_dtype dtype, float bias, int causal, const float* alibi_slopes,
                                        const sattn_strides* sq, const sattn_strides* sk, const sattn_strides* sv,
                                        const sattn_strides* so, void* stream) {
  FwdArgs a{q, k, v, o, nullptr, B, H, N, d, dtype, bias, causal, alibi_slopes, sq, sk, sv, so, stream};
  return fwd_impl<false, false>(a);
}

int sigmoid_attn_bwd_compiler_scheduled(const void* q, const void* k, const void* v, const void* dout, void* dq,
                                        void* dk, void* dv, int B, int H, int N, int d, sattn_dtype dtype, float bias,
                                        int causal, const float* alibi_slopes, const sattn_strides* sq,
                                        const sattn_strides* sk, const sattn_strides* sv, const sattn_strides* sdout,
                                        const sattn_strides* sdq, const sattn_strides* sdk, const sattn_strides* sdv,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  BwdArgs a{q, k, v, nullptr, nullptr, dout, dq, dk, dv, B, H, N, d, dtype, bias, causal, alibi_slopes,
            sq, sk, sv, nullptr, sdout, sdq, sdk, sdv, workspace, workspace_bytes, kBwdDkDv | kBwdDq, stream};
  return bwd_impl<false, false>(a);
}

int softmax_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int N, int d,
                     sattn_dtype dtype, int causal, const float* alibi_slopes, const sattn_strides* sq,
                     const sattn_strides* sk, const sattn_strides* sv, const sattn_strides* so, void* stream) {
  FwdArgs a{q, k, v, o, lse, B, H, N, d, dtype, 0.0f, causal, alibi_slopes, sq, sk, sv, so, stream};
  return fwd_impl<true>(a);
}

int softmax_attn_fwd_compiler_scheduled(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H,
                                        int N, int d, sattn_dtype dtype, int causal, const float* alibi_slopes,
                                        const sattn_strides* sq, const sattn_strides* sk, const sattn_strides* sv,
                                        const sattn_strides* so, void* stream) {
  FwdArgs a{q, k, v, o, lse, B, H, N, d, dtype, 0.0f, causal, alibi_slopes, sq, sk, sv, so, stream};
  return fwd_impl<true, false>(a);
}

int softmax_attn_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dout,
                     void* dq, void* dk, void* dv, int B, int H, int N, int d, sattn_dtype dtype, int causal,
                     const float* alibi_slopes, const sattn_strides* sq, const sattn_strides* sk,
                     const sattn_strides* sv, const sattn_strides* so, const sattn_strides* sdout,
                     const sattn_strides* sdq, const sattn_strides* sdk, const sattn_strides* sdv, void* workspace,
                     size_t workspace_bytes, void* stream) {
  BwdArgs a{q, k, v, o, lse, dout, dq, dk, dv, B, H, N, d, dtype, 0.0f, causal, alibi_slopes,
            sq, sk, sv, so, sdout, sdq, sdk, sdv, workspace, workspace_bytes, kBwdDkDv | kBwdDq, stream};
  return bwd_impl<true>(a);
}

int softmax_attn_bwd_compiler_scheduled(const void* q, const void* k, const void* v, const void* o, const float* lse,
                                        const void* dout, void* dq, void* dk, void* dv, int B, int H, int N, int d,
                                        sattn_dtype dtype, int causal, const float* alibi_slopes,
                                        const sattn_strides* sq, const sattn_strides* sk, const sattn_strides* sv,
                                        const sattn_strides* so, const sattn_strides* sdout, const sattn_strides* sdq,
                                        const sattn_strides* sdk, const sattn_strides* sdv, void* workspace,
                                        size_t workspace_bytes, void* stream) {
  BwdArgs a{q, k, v, o, lse, dout, dq, dk, dv, B, H, N, d, dtype, 0.0f, causal, alibi_slopes,
            sq, sk, sv, so, sdout, sdq, sdk, sdv, workspace, workspace_bytes, kBwdDkDv | kBwdDq, stream};
  return bwd_impl<true, false>(a);
}

size_t softmax_attn_bwd_workspace_bytes(int B, int H, int N, int d, sattn_dtype dtype) {
  if (check_shape(B, H, N, d, dtype) != SATTN_OK) return 0;
  // rowsum(dO o O) and the rescaled log-sum-exp: two fp32 per query row, rows padded to 64
  return 2 * (size_t)B * H * ((N + 63) / 64 * 64) * sizeof(float);
}

size_t softmax_attn_bwd_noalloc_max_rows(void) { return kNoAllocRows; }

int softmax_attn_bwd_noalloc(const void* q, const void* k, const void* v, const void* o, const float* lse,
                             const void* dout, void* dq, void* dk, void* dv, int B, int H, int N, int d,
                             sattn_dtype dtype, int causal, const float* alibi_slopes, const sattn_strides* sq,
                             const sattn_strides* sk, const sattn_strides* sv, const sattn_strides* so,
                             const sattn_strides* sdout, const sattn_strides* sdq, const sattn_strides* sdk,
                             const sattn_strides* sdv, void* stream) {
  int rc = check_shape(B, H, N, d, dtype);
  if (rc) return rc;
  // the pre-pass writes every padded row it later reads, so the last call's contents need no clearing
  const size_t rows = (size_t)B * H * ((size_t)(N + 63) / 64 * 64);
  if (rows > kNoAllocRows) return SATTN_ERR_TOO_LARGE;
  float* ws = nullptr;
  if ((rc = scratch_on_current_device(&ws))) return rc;
  BwdArgs a{q, k, v, o, lse, dout, dq, dk, dv, B, H, N, d, dtype, 0.0f, causal, alibi_slopes,
            sq, sk, sv, so, sdout, sdq, sdk, sdv, ws, 2 * kNoAllocRows * sizeof(float), kBwdDkDv | kBwdDq, stream};
  return bwd_impl<true>(a);
}

const char* sattn_strerror(int code) {
  switch (code) {
    case SATTN_OK: return "success";
    case SATTN_ERR_NULL: return "a required pointer is NULL";
    case SATTN_ERR_SHAPE: return "B, H and N must be positive and within the supported range";
    case SATTN_ERR_UNSUPPORTED: return "unsupported head dimension or dtype (d must be 64 or 128; softmax is bf16 only)";
    case SATTN_ERR_ALIGN: return "pointers and strides must keep rows 16-byte aligned";
    case SATTN_ERR_WORKSPACE: return "workspace missing or too small";
    case SATTN_ERR_LAUNCH: return "the HIP runtime rejected the kernel launch";
    case SATTN_ERR_TOO_LARGE: return "problem exceeds the fixed scratch of the allocation-free entry point";
    default: return "unknown error code";
  }
}

// Packed [tokens, H, d] strides for a variable-length call: batch stride 0; head and token
// strides from the caller, or contiguous.
static sattn_strides varlen_strides(const sattn_strides* s, int H, int d) {
  sattn_strides r;
  r.batch = 0;
  r.head = s ? s->head : d;
  r.seq = s ? s->seq : (int64_t)H * d;
  return r;
}

int sigmoid_attn_varlen_fwd(const void* q, const void* k, const void* v, void* o, const int32_t* cu_seqlens,
                            const float* bias_per_seq, int B, int H, int max_seqlen, int d, sattn_dtype dtype,
                            float bias, int causal, const float* alibi_slopes, const sattn_strides* sq,
                            const sattn_strides* sk, const sattn_strides* sv, const sattn_strides* so,
                            void* stream) {
  if (!cu_seqlens) return SATTN_ERR_NULL;
  const sattn_strides tq = varlen_strides(sq, H, d), tk = varlen_strides(sk, H, d), tv = varlen_strides(sv, H, d),
                      to = varlen_strides(so, H, d);
  FwdArgs a{q, k, v, o, nullptr, B, H, max_seqlen, d, dtype, bias, causal, alibi_slopes, &tq, &tk, &tv, &to, stream};
  a.cu_seqlens = cu_seqlens; a.bias_vec = bias_per_seq;
  return fwd_impl<false>(a);
}

int sigmoid_attn_varlen_bwd(const void* q, const void* k, const void* v, const void* dout, void* dq, void* dk,
                            void* dv, const int32_t* cu_seqlens, const float* bias_per_seq, int B, int H,
                            int max_seqlen, int d, sattn_dtype dtype, float bias, int causal,
                            const float* alibi_slopes, const sattn_strides* sq, const sattn_strides* sk,
                            const sattn_strides* sv, const sattn_strides* sdout, const sattn_strides* sdq,
                            const sattn_strides* sdk, const sattn_strides* sdv, void* stream) {
  if (!cu_seqlens) return SATTN_ERR_NULL;
  const sattn_strides tq = varlen_strides(sq, H, d), tk = varlen_strides(sk, H, d), tv = varlen_strides(sv, H, d),
                      tdo = varlen_strides(sdout, H, d), tdq = varlen_strides(sdq, H, d),
                      tdk = varlen_strides(sdk, H, d), tdv = varlen_strides(sdv, H, d);
  BwdArgs a{q, k, v, nullptr, nullptr, dout, dq, dk, dv, B, H, max_seqlen, d, dtype, bias, causal, alibi_slopes,
            &tq, &tk, &tv, nullptr, &tdo, &tdq, &tdk, &tdv, nullptr, 0, kBwdDkDv | kBwdDq, stream};
  a.cu_seqlens = cu_seqlens; a.bias_vec = bias_per_seq;
  return bwd_impl<false>(a);
}

int sigmoid_attn_varlen_bwd_bias_grad(const void* q, const void* k, const void* v, const void* dout, void* dq,
                                      void* dk, void* dv, float* db_rows, float* db, const int32_t* cu_seqlens,
                                      const float* bias_per_seq, int B, int H, int max_seqlen, int64_t total_tokens,
                                      int d, sattn_dtype dtype, float bias, int causal, const float* alibi_slopes,
                                      const sattn_strides* sq, const sattn_strides* sk, const sattn_strides* sv,
                                      const sattn_strides* sdout, const sattn_strides* sdq, const sattn_strides* sdk,
                                      const sattn_strides* sdv, void* stream) {
  if (!cu_seqlens || !db_rows) return SATTN_ERR_NULL;
  if (((uintptr_t)db_rows & 3) != 0 || ((uintptr_t)db & 3) != 0) return SATTN_ERR_ALIGN;
  if (total_tokens <= 0) return SATTN_ERR_SHAPE;
  const sattn_strides tq = varlen_strides(sq, H, d), tk = varlen_strides(sk, H, d), tv = varlen_strides(sv, H, d),
                      tdo = varlen_strides(sdout, H, d), tdq = varlen_strides(sdq, H, d),
                      tdk = varlen_strides(sdk, H, d), tdv = varlen_strides(sdv, H, d);
  BwdArgs a{q, k, v, nullptr, nullptr, dout, dq, dk, dv, B, H, max_seqlen, d, dtype, bias, causal, alibi_slopes,
            &tq, &tk, &tv, nullptr, &tdo, &tdq, &tdk, &tdv, nullptr, 0, kBwdDkDv | kBwdDq, stream};
  a.cu_seqlens = cu_seqlens; a.bias_vec = bias_per_seq;
  a.db_rows = db_rows; a.db = db; a.db_tokens = total_tokens;
  return bwd_impl<false>(a);
}

int sigmoid_attn_mqa_fwd(const void* q, const void* k, const void* v, void* o, int B, int H, int Hkv, int N, int d,
                         sattn_dtype dtype, float bias, int causal, const float* alibi_slopes,
                         const sattn_strides* sq, const sattn_strides* sk, const sattn_strides* sv,
                         const sattn_strides* so, void* stream) {
  if (Hkv <= 0) return SATTN_ERR_SHAPE;
  FwdArgs a{q, k, v, o, nullptr, B, H, N, d, dtype, bias, causal, alibi_slopes, sq, sk, sv, so, stream};
  a.Hkv = Hkv;
  return fwd_impl<false>(a);
}

int sigmoid_attn_mqa_bwd(const void* q, const void* k, const void* v, const void* dout, void* dq, void* dk,
                         void* dv, int B, int H, int Hkv, int N, int d, sattn_dtype dtype, float bias, int causal,
                         const float* alibi_slopes, const sattn_strides* sq, const sattn_strides* sk,
                         const sattn_strides* sv, const sattn_strides* sdout, const sattn_strides* sdq,
                         const sattn_strides* sdk, const sattn_strides* sdv, void* stream) {
  if (Hkv <= 0) return SATTN_ERR_SHAPE;
  BwdArgs a{q, k, v, nullptr, nullptr, dout, dq, dk, dv, B, H, N, d, dtype, bias, causal, alibi_slopes,
            sq, sk, sv, nullptr, sdout, sdq, sdk, sdv, nullptr, 0, kBwdDkDv | kBwdDq, stream};
  a.Hkv = Hkv;
  return bwd_impl<false>(a);
}

size_t sigmoid_attn_mqa_bwd_workspace_bytes(int B, int H, int Hkv, int N, int d, sattn_dtype dtype, int causal) {
  if (check_shape(B, H, N, d, dtype) != SATTN_OK || Hkv <= 0 || H % Hkv || Hkv == H || dtype != SATTN_BF16) return 0;
  const int s = pick_group_split(B, Hkv, H / Hkv, N, causal);
  return s > 1 ? 2 * (size_t)s * B * Hkv * N * d * sizeof(float) : 0;
}

int sigmoid_attn_mqa_bwd_split(const void* q, const void* k, const void* v, const void* dout, void* dq, void* dk,
                               void* dv, int B, int H, int Hkv, int N, int d, sattn_dtype dtype, float bias,
                               int causal, const float* alibi_slopes, const sattn_strides* sq,
                               const sattn_strides* sk, const sattn_strides* sv, const sattn_strides* sdout,
                               const sattn_strides* sdq, const sattn_strides* sdk, const sattn_strides* sdv,
                               void* workspace, size_t workspace_bytes, void* stream) {
  if (Hkv <= 0) return SATTN_ERR_SHAPE;
  BwdArgs a{q, k, v, nullptr, nullptr, dout, dq, dk, dv, B, H, N, d, dtype, bias, causal, alibi_slopes,
            sq, sk, sv, nullptr, sdout, sdq, sdk, sdv, workspace, workspace_bytes, kBwdDkDv | kBwdDq, stream};
  a.Hkv = Hkv;
  a.group_split = true;
  return bwd_impl<false>(a);
}

int sigmoid_attn_cross_fwd(const void* q, const void* k, const void* v, void* o, int B, int H, int Nq, int Nk, int d,
                           sattn_dtype dtype, float bias, const sattn_strides* sq, const sattn_strides* sk,
                           const sattn_strides* sv, const sattn_strides* so, void* stream) {
  if (Nk <= 0) return SATTN_ERR_SHAPE;
  FwdArgs a{q, k, v, o, nullptr, B, H, Nq, d, dtype, bias, 0, nullptr, sq, sk, sv, so, stream};
  a.Nk = Nk;
  return fwd_impl<false>(a);
}

int sigmoid_attn_cross_bwd(const void* q, const void* k, const void* v, const void* dout, void* dq, void* dk,
                           void* dv, int B, int H, int Nq, int Nk, int d, sattn_dtype dtype, float bias,
                           const sattn_strides* sq, const sattn_strides* sk, const sattn_strides* sv,
                           const sattn_strides* sdout, const sattn_strides* sdq, const sattn_strides* sdk,
                           const sattn_strides* sdv, void* stream) {
  if (Nk <= 0) return SATTN_ERR_SHAPE;
  BwdArgs a{q, k, v, nullptr, nullptr, dout, dq, dk, dv, B, H, Nq, d, dtype, bias, 0, nullptr,
            sq, sk, sv, nullptr, sdout, sdq, sdk, sdv, nullptr, 0, kBwdDkDv | kBwdDq, stream};
  a.Nk = Nk;
  return bwd_impl<false>(a);
}

int sigmoid_attn_cross_aligned_fwd(const void* q, const void* k, const void* v, void* o, int B, int H, int Nq, int Nk,
                                   int d, sattn_dtype dtype, float bias, int causal, const float* alibi_slopes,
                                   const sattn_strides* sq, const sattn_strides* sk, const sattn_strides* sv,
                                   const sattn_strides* so, void* stream) {
  if (Nk <= 0) return SATTN_ERR_SHAPE;
  FwdArgs a{q, k, v, o, nullptr, B, H, Nq, d, dtype, bias, causal, alibi_slopes, sq, sk, sv, so, stream};
  a.Nk = Nk;
  a.end_aligned = true;
  return fwd_impl<false>(a);
}

int sigmoid_attn_cross_aligned_bwd(const void* q, const void* k, const void* v, const void* dout, void* dq, void* dk,
                                   void* dv, int B, int H, int Nq, int Nk, int d, sattn_dtype dtype, float bias,
                                   int causal, const float* alibi_slopes, const sattn_strides* sq,
                                   const sattn_strides* sk, const sattn_strides* sv, const sattn_strides* sdout,
                                   const sattn_strides* sdq, const sattn_strides* sdk, const sattn_strides* sdv,
                                   void* stream) {
  if (Nk <= 0) return SATTN_ERR_SHAPE;
  BwdArgs a{q, k, v, nullptr, nullptr, dout, dq, dk, dv, B, H, Nq, d, dtype, bias, causal, alibi_slopes,
            sq, sk, sv, nullptr, sdout, sdq, sdk, sdv, nullptr, 0, kBwdDkDv | kBwdDq, stream};
  a.Nk = Nk;
  a.end_aligned = true;
  return bwd_impl<false>(a);
}

int sattn_mfma_bf16_probe(int blocks, int iters, float* sink, void* stream) {
  if (!sink) return SATTN_ERR_NULL;
  if (blocks <= 0 || iters <= 0) return SATTN_ERR_SHAPE;
  return launch(mfma_bf16_probe_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, sink, iters);
}

int sattn_headconcat_norm_fwd(const void* x, void* y, float* stats, int B, int H, int N, int d, sattn_dtype dtype,
                              int kind, float eps, const sattn_strides* sx, const sattn_strides* sy, void* stream) {
  return norm_impl(false, x, nullptr, y, stats, B, H, N, d, dtype, kind, eps, sx, nullptr, sy, stream);
}

int sattn_headconcat_norm_bwd(const void* x, const void* dy, const float* stats, void* dx, int B, int H, int N, int d,
                              sattn_dtype dtype, int kind, const sattn_strides* sx, const sattn_strides* sdy,
                              const sattn_strides* sdx, void* stream) {
  return norm_impl(true, x, dy, dx, const_cast<float*>(stats), B, H, N, d, dtype, kind, 0.f, sx, sdy, sdx, stream);
}

int sattn_set_fwd_waves(int waves) {
  if (waves != 0 && waves != 4 && waves != 8 && waves != 32 && (waves < 64 || waves > 66)) return SATTN_ERR_UNSUPPORTED;
  g_fwd_waves.store(waves, std::memory_order_relaxed);
  return SATTN_OK;
}

int sattn_bwd_merged(int B, int H, int N, int causal) {
  if (B <= 0 || H <= 0 || N <= 0) return SATTN_ERR_SHAPE;
  return pick_bwd_merged(B, H, N, causal) ? 1 : 0;
}

int sattn_set_bwd_merged(int mode) {
  if (mode < 0 || mode > 3) return SATTN_ERR_UNSUPPORTED;
  g_bwd_merged.store(mode, std::memory_order_relaxed);
  return SATTN_OK;
}

int sattn_set_fwd_v_slots(int v_slots) {
  if (v_slots != 0 && v_slots != 2 && v_slots != 3) return SATTN_ERR_UNSUPPORTED;
  g_fwd_vslots.store(v_slots, std::memory_order_relaxed);
  return SATTN_OK;
}

int sattn_set_clock_probe(void* device_buffer, int capacity) {
  if (capacity < 0 || (device_buffer && ((uintptr_t)device_buffer & 7) != 0)) return SATTN_ERR_ALIGN;
  g_clock_cap.store(device_buffer ? capacity : 0, std::memory_order_relaxed);
  g_clock_out.store((long long*)device_buffer, std::memory_order_relaxed);
  return SATTN_OK;
}

int sattn_fwd_waves(int B, int H, int N, int d, int causal) {
  if (B <= 0 || H <= 0 || N <= 0) return SATTN_ERR_SHAPE;
  if (d != 64 && d != 128) return SATTN_ERR_UNSUPPORTED;
  return pick_fwd_shape(B, H, N, d, causal).waves;
}

int sattn_fwd_v_slots(int B, int H, int N, int d, int causal) {
  if (B <= 0 || H <= 0 || N <= 0) return SATTN_ERR_SHAPE;
  if (d != 64 && d != 128) return SATTN_ERR_UNSUPPORTED;
  return pick_fwd_shape(B, H, N, d, causal).v_slots;
}

int sattn_device_info(int* compute_units, int* clock_khz) {
  if (!compute_units || !clock_khz) return SATTN_ERR_NULL;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(compute_units, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipDeviceGetAttribute(clock_khz, hipDeviceAttributeClockRate, dev) != hipSuccess) {
    (void)hipGetLastError();
    return SATTN_ERR_LAUNCH;
  }
  return SATTN_OK;
}

int sattn_wall_clock_khz(void) {
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) {
    (void)hipGetLastError();
    return SATTN_ERR_LAUNCH;
  }
  return khz;
}

int sattn_version(void) { return 102; }

}  // extern "C"
