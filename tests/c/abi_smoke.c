/* The C boundary used from plain C: no Python, no torch.  Builds a two-layer stack (a standard layer and a
   sliding-window layer, arXiv 2409.15012 Section 3), appends tokens whose keys are all equal, and checks the
   closed form: equal keys give equal scores, so the output is the mean of the attended values, over all tokens for
   the standard layer and over the last `window` tokens for the sliding one.  Once on the scalar path (fp32,
   head_dim 64) and once on the MFMA path (bf16, head_dim 128, 4 query heads per KV head: a prompt through
   mixattn_prefill, then decode steps through mixattn_append_decode and mixattn_decode, with a reader layer on each
   cache).  Prints "abi smoke ok" and returns 0. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "mixattn.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define CHECK_MX(x) do { int s_ = (x); if (s_ != MIXATTN_OK) { printf("mixattn: %s (%d) at line %d\n", mixattn_strerror(s_), s_, __LINE__); return 3; } } while (0)

enum { B = 2, HQ = 4, HKV = 2, D = 64, W = 5, N = 12 };

/* ---- MFMA path: bf16, head_dim 128, group size 4 ---- */
enum { MB = 2, MHQ = 8, MHKV = 2, MD = 128, MW = 40, MS = 70, MSTEPS = 30 };

static uint16_t to_bf16(float f) { /* exact for the values used here (few significant bits) */
  union { float f; uint32_t u; } c;
  c.f = f;
  return (uint16_t)(c.u >> 16);
}
/* value of token t of sequence b in dim d: multiples of 1/4 below 4, exactly representable in bf16 */
static float mv(int b, int t, int d) { return (float)((t * 7 + b * 3) % 8) * 0.25f + (float)(d % 2) + (b ? 1.f : 0.f); }
/* mean of mv over tokens first .. last */
static double mean_mv(int b, int first, int last, int d) {
  double s = 0.0;
  for (int t = first; t <= last; ++t) s += mv(b, t, d);
  return s / (last - first + 1);
}

static int run_mfma_stack(double* worst_out) {
  /* standard layer (cache 0), sliding layer (cache 1), a reader of each */
  const mixattn_layer_desc layers[4] = {{MIXATTN_FULL, 0, 0}, {MIXATTN_SLIDING, MW, 1}, {MIXATTN_SLIDING, MW, 1}, {MIXATTN_FULL, 0, 0}};
  const int32_t capacity[MB] = {MS + MSTEPS, MS + MSTEPS};
  mixattn_config cfg;
  cfg.n_layers = 4; cfg.layers = layers; cfg.batch = MB; cfg.n_q_heads = MHQ; cfg.n_kv_heads = MHKV; cfg.head_dim = MD;
  cfg.capacity = capacity; cfg.kv_dtype = MIXATTN_BF16; cfg.out_dtype = MIXATTN_F32; cfg.softmax_scale = 0.f;
  mixattn_layout* L = NULL;
  CHECK_MX(mixattn_create_layout(&cfg, &L));
  CHECK_MX(mixattn_reserve_prefill(L, MS));

  const size_t pq = (size_t)MB * MS * MHQ * MD, pkv = (size_t)MB * MS * MHKV * MD;
  const size_t sq = (size_t)MB * MHQ * MD, skv = (size_t)MB * MHKV * MD;
  uint16_t *hq = malloc(pq * 2), *hk = malloc(pkv * 2), *hv = malloc(pkv * 2);
  float* ho = malloc(pq * sizeof(float));
  uint16_t *dq, *dk, *dv;
  float* dout;
  CHECK_HIP(hipMalloc((void**)&dq, pq * 2));
  CHECK_HIP(hipMalloc((void**)&dk, pkv * 2));
  CHECK_HIP(hipMalloc((void**)&dv, pkv * 2));
  CHECK_HIP(hipMalloc((void**)&dout, pq * sizeof(float)));
  for (size_t i = 0; i < pq; ++i) hq[i] = to_bf16((float)((int)(i % 13) - 6) * 0.125f);
  for (size_t i = 0; i < pkv; ++i) hk[i] = to_bf16(0.5f); /* the same key for every token */
  for (int b = 0; b < MB; ++b)
    for (int t = 0; t < MS; ++t)
      for (int h = 0; h < MHKV; ++h)
        for (int d = 0; d < MD; ++d) hv[(((size_t)b * MS + t) * MHKV + h) * MD + d] = to_bf16(mv(b, t, d));
  CHECK_HIP(hipMemcpy(dq, hq, pq * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dk, hk, pkv * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dv, hv, pkv * 2, hipMemcpyHostToDevice));

  double worst = 0.0;
  /* the prompt: writers get k, v; readers reuse the copy their writer staged (k = v = NULL) */
  for (int layer = 0; layer < 4; ++layer) {
    const int writer = layer < 2;
    CHECK_MX(mixattn_prefill(L, layer, dq, writer ? dk : NULL, writer ? dv : NULL, dout, MS, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(ho, dout, pq * sizeof(float), hipMemcpyDeviceToHost));
    const int sliding = layers[layer].kind == MIXATTN_SLIDING;
    for (int b = 0; b < MB; ++b)
      for (int i = 0; i < MS; ++i)
        for (int j = 0; j < MHQ; ++j)
          for (int d = 0; d < MD; ++d) {
            const int first = sliding && i + 1 > MW ? i + 1 - MW : 0;
            const double err = fabs((double)ho[(((size_t)b * MS + i) * MHQ + j) * MD + d] - mean_mv(b, first, i, d));
            if (err > worst) worst = err;
          }
  }
  /* decode steps: token MS + t */
  for (int t = 0; t < MSTEPS; ++t) {
    const int pos = MS + t;
    for (int b = 0; b < MB; ++b)
      for (int h = 0; h < MHKV; ++h)
        for (int d = 0; d < MD; ++d) hv[((size_t)b * MHKV + h) * MD + d] = to_bf16(mv(b, pos, d));
    CHECK_HIP(hipMemcpy(dv, hv, skv * 2, hipMemcpyHostToDevice));
    for (int layer = 0; layer < 4; ++layer) {
      if (layer < 2) CHECK_MX(mixattn_append_decode(L, layer, dk, dv, dq, dout, NULL));
      else CHECK_MX(mixattn_decode(L, layer, dq, dout, NULL));
      CHECK_HIP(hipDeviceSynchronize());
      CHECK_HIP(hipMemcpy(ho, dout, sq * sizeof(float), hipMemcpyDeviceToHost));
      const int sliding = layers[layer].kind == MIXATTN_SLIDING;
      const int first = sliding && pos + 1 > MW ? pos + 1 - MW : 0;
      for (int b = 0; b < MB; ++b)
        for (int j = 0; j < MHQ; ++j)
          for (int d = 0; d < MD; ++d) {
            const double err = fabs((double)ho[((size_t)b * MHQ + j) * MD + d] - mean_mv(b, first, pos, d));
            if (err > worst) worst = err;
          }
    }
  }
  int64_t n = -1, slot = -1;
  CHECK_MX(mixattn_seq_len(L, 1, 1, &n));
  CHECK_MX(mixattn_slot_of(L, 1, MS + MSTEPS - 1, &slot));
  /* the last token's V row, read back through the boundary, bit for bit */
  uint16_t row[MD];
  CHECK_MX(mixattn_read_cache(L, 1, 1, 1, slot, NULL, row));
  for (int d = 0; d < MD; ++d)
    if (row[d] != to_bf16(mv(1, MS + MSTEPS - 1, d))) { printf("cache row differs at dim %d\n", d); return 6; }
  CHECK_MX(mixattn_destroy_layout(L));
  if (n != MS + MSTEPS || slot != (MS + MSTEPS - 1) % MW) { printf("bookkeeping (MFMA stack): n %lld slot %lld\n", (long long)n, (long long)slot); return 4; }
  CHECK_HIP(hipFree(dq)); CHECK_HIP(hipFree(dk)); CHECK_HIP(hipFree(dv)); CHECK_HIP(hipFree(dout));
  free(hq); free(hk); free(hv); free(ho);
  *worst_out = worst;
  return 0;
}

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
  double worst_mfma = 0.0;
  const int rc = run_mfma_stack(&worst_mfma);
  if (rc != 0) return rc;
  /* bf16 inputs, fp32 accumulation: 2e-3 scaled by the largest value magnitude (4) */
  if (!(worst_mfma < 2e-3 * 4)) { printf("worst error on the MFMA path %g\n", worst_mfma); return 7; }
  printf("abi smoke ok (worst error %.3g scalar path, %.3g MFMA path)\n", worst, worst_mfma);
  return 0;
}
