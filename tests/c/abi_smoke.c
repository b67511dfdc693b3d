/* The C boundary used from plain C: no Python, no torch.  Builds a two-layer stack (a standard layer and a
   sliding-window layer, arXiv 2409.15012 Section 3), appends tokens whose keys are all equal, and checks the
   closed form: equal keys give equal scores, so the output is the mean of the attended values, over all tokens for
   the standard layer and over the last `window` tokens for the sliding one.  Prints "abi smoke ok" and returns 0. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "mixattn.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define CHECK_MX(x) do { int s_ = (x); if (s_ != MIXATTN_OK) { printf("mixattn: %s (%d) at line %d\n", mixattn_strerror(s_), s_, __LINE__); return 3; } } while (0)

enum { B = 2, HQ = 4, HKV = 2, D = 64, W = 5, N = 12 };

int main(void) {
  const mixattn_layer_desc layers[2] = {{MIXATTN_FULL, 0, 0}, {MIXATTN_SLIDING, W, 1}};
  const int32_t capacity[B] = {N, N};
  mixattn_config cfg;
  cfg.n_layers = 2; cfg.layers = layers; cfg.batch = B; cfg.n_q_heads = HQ; cfg.n_kv_heads = HKV; cfg.head_dim = D;
  cfg.capacity = capacity; cfg.kv_dtype = MIXATTN_F32; cfg.out_dtype = MIXATTN_F32; cfg.softmax_scale = 0.f;
  mixattn_layout* L = NULL;
  CHECK_MX(mixattn_create_layout(&cfg, &L));

  const size_t kv_elems = (size_t)B * HKV * D, q_elems = (size_t)B * HQ * D;
  float *hk = malloc(kv_elems * sizeof(float)), *hv = malloc(kv_elems * sizeof(float));
  float *hq = malloc(q_elems * sizeof(float)), *ho = malloc(q_elems * sizeof(float));
  float *dk, *dv, *dq, *dout;
  CHECK_HIP(hipMalloc((void**)&dk, kv_elems * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&dv, kv_elems * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&dq, q_elems * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&dout, q_elems * sizeof(float)));
  for (size_t i = 0; i < kv_elems; ++i) hk[i] = 0.25f;  /* the same key for every token */
  for (size_t i = 0; i < q_elems; ++i) hq[i] = (float)(i % 7) - 3.f;
  CHECK_HIP(hipMemcpy(dk, hk, kv_elems * sizeof(float), hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dq, hq, q_elems * sizeof(float), hipMemcpyHostToDevice));

  double worst = 0.0;
  for (int t = 0; t < N; ++t) {
    /* value of token t: t + 1 in sequence 0, 10 (t + 1) in sequence 1, plus the dim index / 1000 */
    for (int b = 0; b < B; ++b)
      for (int h = 0; h < HKV; ++h)
        for (int d = 0; d < D; ++d) hv[((size_t)b * HKV + h) * D + d] = (b ? 10.f : 1.f) * (float)(t + 1) + d * 0.001f;
    CHECK_HIP(hipMemcpy(dv, hv, kv_elems * sizeof(float), hipMemcpyHostToDevice));
    for (int layer = 0; layer < 2; ++layer) {
      if (t % 2 == 0) {
        CHECK_MX(mixattn_append_kv(L, layer, dk, dv, NULL));
        CHECK_MX(mixattn_decode(L, layer, dq, dout, NULL));
      } else {
        CHECK_MX(mixattn_append_decode(L, layer, dk, dv, dq, dout, NULL));
      }
      CHECK_HIP(hipDeviceSynchronize());
      CHECK_HIP(hipMemcpy(ho, dout, q_elems * sizeof(float), hipMemcpyDeviceToHost));
      const int first = layer == 0 ? 0 : (t + 1 > W ? t + 1 - W : 0);  /* tokens first .. t are attended */
      const double mean_t = 0.5 * ((first + 1) + (t + 1));
      for (int b = 0; b < B; ++b)
        for (int j = 0; j < HQ; ++j)
          for (int d = 0; d < D; ++d) {
            const double expect = (b ? 10.0 : 1.0) * mean_t + d * 0.001;
            const double err = fabs((double)ho[((size_t)b * HQ + j) * D + d] - expect);
            if (err > worst) worst = err;
          }
    }
  }
  int64_t n = -1, slot = -1;
  CHECK_MX(mixattn_seq_len(L, 1, 1, &n));
  CHECK_MX(mixattn_slot_of(L, 1, N - 1, &slot));
  CHECK_MX(mixattn_destroy_layout(L));
  if (n != N || slot != (N - 1) % W) { printf("bookkeeping: n %lld slot %lld\n", (long long)n, (long long)slot); return 4; }
  if (!(worst < 2e-4)) { printf("worst error %g\n", worst); return 5; }
  printf("abi smoke ok (worst error %.3g)\n", worst);
  return 0;
}
