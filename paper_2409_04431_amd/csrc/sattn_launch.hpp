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

template <typename K, typename... Args>
int launch(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t st, Args... args) {
  if (lds > 0 &&
      hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return SATTN_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
  return hipGetLastError() == hipSuccess ? SATTN_OK : SATTN_ERR_LAUNCH;
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

// Forward: `waves` (4 or 8) is the number of 32-query-row waves per workgroup (sets
// p.n_qblocks accordingly), `v_slots` (2 or 3) the depth of the V ring of 4-wave workgroups
// at D = 128.  softmax selects the comparison kernel, pin the hand-ordered step.
template <int D>
int launch_fwd_bf16(FwdParams p, int waves, int v_slots, bool softmax, bool pin, int causal, bool alibi,
                    hipStream_t st);

// Backward: `parts` is a mask of BwdPart; p.db_rows selects the dQ pass with row sums.
template <int D>
int launch_bwd_bf16(BwdParams p, bool softmax, bool pin, int causal, bool alibi, int parts, hipStream_t st);

}  // namespace sattn
