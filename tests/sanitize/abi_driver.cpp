// Drives the host side of the C ABI (argument validation, dispatch, the per-kernel launch
// cache) without a GPU, for a build whose host code carries -fsanitize=address,undefined.
// Every call either fails validation or, with a well-formed problem on fake device pointers,
// reaches the runtime and is refused there (no device): both paths are host code only.  If a
// device is visible after all, the well-formed calls are skipped (they would launch kernels on
// the fake pointers) and reported as refused.
#include <cstdint>
#include <cstdio>

#include "../../include/sattn.h"
#include "../../include/sattn_bench.h"

int main() {
  void *q = (void*)0x10000, *k = (void*)0x20000, *v = (void*)0x30000, *o = (void*)0x40000, *g = (void*)0x50000;
  void *dq = (void*)0x60000, *dk = (void*)0x70000, *dv = (void*)0x80000;
  float* f = (float*)0x90000;
  int32_t* cu = (int32_t*)0xa0000;
  int rc[64], n = 0;
  int cus = 0, khz = 0;
  const bool gpu = sattn_device_info(&cus, &khz) == SATTN_OK;
#define WELL_FORMED(call) (gpu ? (int)SATTN_ERR_LAUNCH : (call))
  sattn_strides bad{1027, 1024, 64}, ok{1 << 20, 1 << 16, 128};
  rc[n++] = sigmoid_attn_fwd(nullptr, k, v, o, 1, 1, 16, 64, SATTN_BF16, 0.f, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  rc[n++] = sigmoid_attn_fwd(q, k, v, o, 1, 1, 16, 96, SATTN_BF16, 0.f, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  rc[n++] = sigmoid_attn_fwd(q, k, v, o, 1, 1, 16, 64, SATTN_BF16, 0.f, 0, nullptr, &bad, nullptr, nullptr, nullptr, nullptr);
  rc[n++] = WELL_FORMED(sigmoid_attn_fwd(q, k, v, o, 2, 3, 300, 128, SATTN_BF16, -5.f, 1, f, &ok, &ok, &ok, &ok, nullptr));
  rc[n++] = WELL_FORMED(sigmoid_attn_fwd(q, k, v, o, 2, 3, 300, 64, SATTN_F32, -5.f, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr));
  rc[n++] = sigmoid_attn_bwd(q, k, v, g, dq, dk, nullptr, 1, 1, 16, 64, SATTN_BF16, 0.f, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr);
  rc[n++] = WELL_FORMED(sigmoid_attn_bwd(q, k, v, g, dq, dk, dv, 2, 2, 500, 128, SATTN_BF16, -6.f, 1, f, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr));
  rc[n++] = sigmoid_attn_bwd_bias_grad(q, k, v, g, dq, dk, dv, nullptr, nullptr, 1, 1, 16, 64, SATTN_BF16, 0.f, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  rc[n++] = softmax_attn_fwd(q, k, v, o, nullptr, 1, 1, 16, 64, SATTN_BF16, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  rc[n++] = WELL_FORMED(softmax_attn_bwd(q, k, v, o, f, g, dq, dk, dv, 1, 2, 100, 64, SATTN_BF16, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr));
  rc[n++] = softmax_attn_bwd_noalloc(q, k, v, o, f, g, dq, dk, dv, 64, 64, 4096, 64, SATTN_BF16, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  rc[n++] = WELL_FORMED(sigmoid_attn_varlen_fwd(q, k, v, o, cu, f, 3, 4, 700, 128, SATTN_BF16, 0.f, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr));
  rc[n++] = sigmoid_attn_varlen_bwd_bias_grad(q, k, v, g, dq, dk, dv, f, f, cu, nullptr, 3, 4, 700, 0, 128, SATTN_BF16, 0.f, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  rc[n++] = sigmoid_attn_mqa_fwd(q, k, v, o, 1, 6, 4, 64, 64, SATTN_BF16, 0.f, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr);
  rc[n++] = WELL_FORMED(sigmoid_attn_mqa_bwd(q, k, v, g, dq, dk, dv, 1, 8, 2, 640, 128, SATTN_BF16, 0.f, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr));
  rc[n++] = sigmoid_attn_cross_fwd(q, k, v, o, 1, 2, 64, 0, 64, SATTN_BF16, 0.f, nullptr, nullptr, nullptr, nullptr, nullptr);
  rc[n++] = WELL_FORMED(sigmoid_attn_cross_bwd(q, k, v, g, dq, dk, dv, 1, 2, 64, 96, 64, SATTN_BF16, 0.f, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr));
  rc[n++] = sattn_headconcat_norm_fwd(q, o, f, 1, 128, 32, 128, SATTN_BF16, 0, 1e-5f, nullptr, nullptr, nullptr);
  rc[n++] = WELL_FORMED(sattn_headconcat_norm_fwd(q, o, f, 2, 16, 32, 128, SATTN_BF16, 1, 1e-5f, nullptr, nullptr, nullptr));
  rc[n++] = sattn_set_fwd_waves(3);
  rc[n++] = sattn_set_fwd_waves(64);
  rc[n++] = sattn_fwd_waves(1, 2, 512, 128, 0);
  rc[n++] = sattn_set_fwd_waves(0);
  rc[n++] = sattn_fwd_waves(1, 32, 16384, 128, 1);
  rc[n++] = sattn_fwd_v_slots(8, 16, 4096, 128, 1);
  rc[n++] = (int)softmax_attn_bwd_workspace_bytes(8, 16, 4096, 128, SATTN_BF16);
  rc[n++] = sattn_mfma_bf16_probe(0, 1, f, nullptr);
  for (int i = 0; i < n; ++i) printf("%d%c", rc[i], i + 1 < n ? ' ' : '\n');
  for (int c = 0; c >= -8; --c) printf("%s\n", sattn_strerror(c));
  printf("ok\n");
  return 0;
}
