// Definition of launch_bwd_bf16<D>; included by the one translation unit that instantiates it.
#pragma once
#include "sattn_launch.hpp"

namespace sattn {

template <int D, bool SOFTMAX, bool PIN>
int launch_bwd_variant(BwdParams p, int causal, bool alibi, int parts, bool merged, hipStream_t st) {
  // the dQ pass runs one workgroup per 128 queries, the dK/dV pass one per 128 keys
  const int nb_q = (p.N + 127) / 128, nb_k = ((p.Nk > 0 ? p.Nk : p.N) + 127) / 128;
  // pairs of blocks per workgroup: causal pinned sigmoid passes over equal-length sequences with
  // an even number of blocks per head (measured from 4 blocks up: 0-3 % faster than single
  // blocks, never slower)
  const bool may_pair = p.pair && causal && PIN && !p.cu_seqlens;
  const bool pair_q = may_pair && !p.db_rows && nb_q % 2 == 0 && nb_q >= 4, pair_k = may_pair && nb_k % 2 == 0 && nb_k >= 4;
  dim3 grid((pair_q ? nb_q / 2 : nb_q) * p.B * p.H), grid_k((pair_k ? nb_k / 2 : nb_k) * p.B * p.H),
      grid_kv((pair_k ? nb_k / 2 : nb_k) * p.B * (p.H / p.kv_group) * (p.n_split > 1 ? p.n_split : 1));
  int rc = SATTN_OK;
  constexpr size_t lds = 4 * 2 * 64 * D * 2;                    // 4 ring slots of two 64-row tiles
  dim3 block(256);
  if (p.kv_group < 1 || p.H % p.kv_group) return SATTN_ERR_SHAPE;
  if (p.kv_group > 1 && (SOFTMAX || !PIN)) return SATTN_ERR_UNSUPPORTED;  // only the product kernels share K/V heads
  if constexpr (PIN) {
    // self-attention with one K/V head per query head and both passes wanted: one grid
    if (parts == (kBwdDkDv | kBwdDq) && p.kv_group == 1 && nb_q == nb_k && p.Nk == 0 && !p.db_rows && merged) {
      p.n_blocks = nb_q;
      p.head_group = heads_abreast(nb_q);
      p.pair = 0;
      dim3 grid2(2 * nb_q * p.B * p.H);
      SATTN_DISPATCH2(causal, alibi, rc = launch(attn_bwd_merged_kernel<D, A, B2, SOFTMAX>, grid2, block,
                                                 lds + (SOFTMAX ? 4 * StatStager::SLOT : 0), st, p));
      return rc;
    }
  }
  if (parts & kBwdDkDv) {
    p.n_blocks = nb_k;
    p.head_group = heads_abreast(nb_k);
    p.pair = pair_k;
    if constexpr (!SOFTMAX && PIN) {
      if (p.kv_group > 1) {  // one workgroup per K/V head (and split) streams the query heads of its group
        SATTN_DISPATCH2(causal, alibi,
                        rc = launch(attn_bwd_kernel<D, BWD_DKDV, A, B2, false, true, true>, grid_kv, block, lds, st, p));
        if (rc == SATTN_OK && p.n_split > 1) {
          const int Hkv = p.H / p.kv_group, Nk = p.Nk > 0 ? p.Nk : p.N;
          const int64_t threads = ((int64_t)p.B * Hkv * Nk * D + 7) / 8;
          rc = launch(group_partials_reduce_kernel<D>, dim3((unsigned)((threads + 255) / 256), 2), dim3(256), 0, st,
                      (const float*)p.part, p.dk, p.dv, p.n_split, p.B, Hkv, Nk, p.inv_sqrt_d);
        }
      }
    }
    // (the pinned softmax dK/dV pass keeps the streamed queries' statistics in a side ring behind the tiles)
    if (p.kv_group == 1)
      SATTN_DISPATCH2(causal, alibi, rc = launch(attn_bwd_kernel<D, BWD_DKDV, A, B2, SOFTMAX, PIN>, grid_k, block,
                                                 lds + ((SOFTMAX && PIN) ? 4 * StatStager::SLOT : 0), st, p));
  }
  p.n_blocks = nb_q;
  p.head_group = heads_abreast(nb_q);
  p.pair = pair_q;
  if (rc == SATTN_OK && (parts & kBwdDq)) {
    if constexpr (!SOFTMAX && PIN) {
      if (p.db_rows) {  // the dQ pass that also writes the row sums of dS
        SATTN_DISPATCH2(causal, alibi,
                        rc = launch(attn_bwd_kernel<D, BWD_DQ_DB, A, B2, false, true>, grid, block, lds, st, p));
        return rc;
      }
    }
    SATTN_DISPATCH2(causal, alibi, rc = launch(attn_bwd_kernel<D, BWD_DQ, A, B2, SOFTMAX, PIN>, grid, block, lds, st, p));
  }
  return rc;
}

template <int D>
int launch_bwd_bf16(BwdParams p, bool softmax, bool pin, int causal, bool alibi, int parts, bool merged,
                    hipStream_t st) {
  if (softmax && pin) return launch_bwd_variant<D, true, true>(p, causal, alibi, parts, merged, st);
  if (softmax) return launch_bwd_variant<D, true, false>(p, causal, alibi, parts, false, st);
  if (pin) return launch_bwd_variant<D, false, true>(p, causal, alibi, parts, merged, st);
  return launch_bwd_variant<D, false, false>(p, causal, alibi, parts, false, st);
}

}  // namespace sattn
