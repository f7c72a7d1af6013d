// Definition of launch_fwd_bf16<D>; included by the one translation unit that instantiates it.
#pragma once
#include "sattn_fwd64.hpp"
#include "sattn_launch.hpp"

namespace sattn {

template <int D, int NW, int VS, bool SOFTMAX, bool PIN>
int launch_fwd_variant(FwdParams p, int causal, bool alibi, hipStream_t st) {
  constexpr size_t lds = (3 + VS) * 64 * D * 2;  // 3 K slots + VS V slots of 64 keys
  p.n_qblocks = (p.N + 32 * NW - 1) / (32 * NW);
  p.head_group = heads_abreast(p.n_qblocks);
  dim3 grid(p.n_qblocks * p.B * p.H), block(64 * NW);
  int rc = SATTN_OK;
  SATTN_DISPATCH2(causal, alibi, rc = launch(attn_fwd_kernel<D, NW, A, B2, SOFTMAX, PIN, VS>, grid, block, lds, st, p));
  return rc;
}

template <int D, int NW, int VS>
int launch_fwd_shape(const FwdParams& p, bool softmax, bool pin, int causal, bool alibi, hipStream_t st) {
  if (softmax && pin) return launch_fwd_variant<D, NW, VS, true, true>(p, causal, alibi, st);
  if (softmax) return launch_fwd_variant<D, NW, VS, true, false>(p, causal, alibi, st);
  if (pin) return launch_fwd_variant<D, NW, VS, false, true>(p, causal, alibi, st);
  return launch_fwd_variant<D, NW, VS, false, false>(p, causal, alibi, st);
}

// The 64-rows-per-wave sigmoid kernel (head dimension 128; ALiBi only in its causal form).
template <int D>
int launch_fwd64(FwdParams p, int causal, bool alibi, bool prescale, bool pair, hipStream_t st) {
  if constexpr (D != 128) {
    return SATTN_ERR_UNSUPPORTED;
  } else {
    constexpr size_t lds = 6 * 64 * D * 2;  // 3 K slots + 3 V slots of 64 keys
    p.n_qblocks = (p.N + 255) / 256;
    p.head_group = heads_abreast(p.n_qblocks);
    // pairs of blocks: causal launches of equal-length sequences with an even number of blocks
    p.pair = causal && !p.cu_seqlens && p.n_qblocks % 2 == 0 && pair;
    if (p.pair) p.head_group = 1;
    dim3 grid((p.pair ? p.n_qblocks / 2 : p.n_qblocks) * p.B * p.H), block(256);
    if (alibi && !causal) return SATTN_ERR_UNSUPPORTED;
    if (alibi) return launch(attn_fwd64_kernel<D, true, true, false>, grid, block, lds, st, p);
    if (causal) {
      if (prescale) return launch(attn_fwd64_kernel<D, true, false, true>, grid, block, lds, st, p);
      return launch(attn_fwd64_kernel<D, true, false, false>, grid, block, lds, st, p);
    }
    if (prescale) return launch(attn_fwd64_kernel<D, false, false, true>, grid, block, lds, st, p);
    return launch(attn_fwd64_kernel<D, false, false, false>, grid, block, lds, st, p);
  }
}

template <int D>
int launch_fwd_bf16(FwdParams p, int waves, int v_slots, bool softmax, bool pin, int causal, bool alibi,
                    hipStream_t st) {
  if (p.kv_group < 1 || p.H % p.kv_group) return SATTN_ERR_SHAPE;
  if (waves >= 64 && waves <= 66) {  // 64-row waves: 65 = with the pre-scaled Q fragments, 66 = one block per workgroup
    if (softmax || !pin) return SATTN_ERR_UNSUPPORTED;
    return launch_fwd64<D>(p, causal, alibi, waves == 65 && !alibi, p.pair != 0, st);
  }
  if (waves == 4) {
    // the two-slot V ring only matters at D = 128, where it lets two workgroups share a compute unit
    if constexpr (D == 128) {
      if (v_slots == 2) return launch_fwd_shape<D, 4, 2>(p, softmax, pin, causal, alibi, st);
    }
    return launch_fwd_shape<D, 4, 3>(p, softmax, pin, causal, alibi, st);
  }
  return launch_fwd_shape<D, 8, 3>(p, softmax, pin, causal, alibi, st);
}

}  // namespace sattn
