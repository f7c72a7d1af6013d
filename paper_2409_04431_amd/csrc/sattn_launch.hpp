// Host-side launch helpers, and the launchers of the bf16 kernels.  The launchers are
// templates on the head dimension whose definitions (sattn_fwd_launch.hpp,
// sattn_bwd_launch.hpp) are instantiated in one translation unit per head dimension, so the
// kernel instantiations compile in parallel; the API file only sees these declarations.
#pragma once
#include "../../include/sattn.h"

#include <hip/hip_runtime.h>

#include "sattn_bwd.hpp"
#include "sattn_fwd.hpp"

namespace sattn {

// Raises the dynamic-LDS limit of `kernel` on device `dev` to `lds` bytes unless an earlier
// launch already did (the attribute is a property of the loaded function per device, and the
// small problems are launch-latency bound, so the runtime call is made once, not per launch).
bool ensure_dynamic_lds(const void* kernel, int dev, size_t lds);

template <typename K, typename... Args>
int launch(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
  if (lds > 0) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || !ensure_dynamic_lds((const void*)kernel, dev, lds)) {
      (void)hipGetLastError();
      return SATTN_ERR_LAUNCH;
    }
  }
  // the launch's own status, not whatever error an earlier, unrelated call left behind
  void* argv[] = {(void*)&args...};
  if (hipLaunchKernel((const void*)kernel, grid, block, argv, lds, st) != hipSuccess) {
    (void)hipGetLastError();
    return SATTN_ERR_LAUNCH;
  }
  return SATTN_OK;
}

// Expand two runtime flags into the constexpr bools A and B2 visible to CALL.
#define SATTN_DISPATCH2(F1, F2, CALL)                          \
  do {                                                         \
    if (F1) {                                                  \
      if (F2) { constexpr bool A = true, B2 = true; CALL; }    \
      else { constexpr bool A = true, B2 = false; CALL; }      \
    } else {                                                   \
      if (F2) { constexpr bool A = false, B2 = true; CALL; }   \
      else { constexpr bool A = false, B2 = false; CALL; }     \
    }                                                          \
  } while (0)

enum BwdPart { kBwdDkDv = 1, kBwdDq = 2 };

// Heads walked abreast in the dispatch order of a causal launch (head_and_rank): enough of them
// that one rank of blocks covers the 32 compute units of an XCD, at most 8 (their K/V should
// stay in the XCD's L2 together).
inline int heads_abreast(int n_blocks) {
  const int g = n_blocks > 0 ? 32 / n_blocks : 1;
  return g < 1 ? 1 : (g > 8 ? 8 : g);
}

// Forward: `waves` (4 or 8) is the number of 32-query-row waves per workgroup (sets
// p.n_qblocks accordingly), `v_slots` (2 or 3) the depth of the V ring of 4-wave workgroups
// at D = 128.  softmax selects the comparison kernel, pin the hand-ordered step.
// waves = 64 / 65 selects the kernel with four waves of 64 query rows (D = 128, sigmoid,
// pinned; 65: Q fragments pre-scaled, no ALiBi).
template <int D>
int launch_fwd_bf16(FwdParams p, int waves, int v_slots, bool softmax, bool pin, int causal, bool alibi,
                    hipStream_t st);

// Backward: `parts` is a mask of BwdPart; p.db_rows selects the dQ pass with row sums; `merged`
// lets the two passes of the pinned sigmoid backward share one grid where that form exists.
template <int D>
int launch_bwd_bf16(BwdParams p, bool softmax, bool pin, int causal, bool alibi, int parts, bool merged,
                    hipStream_t st);

}  // namespace sattn
