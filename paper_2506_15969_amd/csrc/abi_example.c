/* The lazyev C ABI from plain C (C99): device memory from the HIP runtime's C API, no C++ and
 * no Python anywhere.  Decodes a tiny fp32 workload with deterministic inputs (one layer, one
 * sequence, two KV heads of two query heads each, head_dim 64, 5-row prompt, budget 8,
 * window 2, 12 steps) and prints the attention outputs' checksums per step and the surviving
 * token positions, which tests/test_gpu_c_abi.py compares with the CPU oracle on the same
 * inputs.  Exit code 0 on success. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "lazyev.h"

#define HQ 4
#define HKV 2
#define D 64
#define P 5
#define B 8
#define W 2
#define STEPS 12

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define LZ_OK(x) do { int c_ = (x); if (c_ != LAZYEV_OK) { \
  fprintf(stderr, "lazyev error %d (%s) at line %d\n", c_, lazyev_strerror(c_), __LINE__); return 3; } } while (0)

/* the inputs: small exact binary fractions, a function of (stream, token position, head, lane) */
static float value(int stream, int pos, int head, int lane) {
  const int x = (stream * 131 + pos * 31 + head * 17 + lane * 7) % 23 - 11;
  return (float)x / 8.0f;
}

int main(void) {
  lazyev_config cfg;
  memset(&cfg, 0, sizeof(cfg));
  cfg.n_layers = 1; cfg.batch = 1; cfg.n_q_heads = HQ; cfg.n_kv_heads = HKV; cfg.head_dim = D;
  cfg.budget = B; cfg.window = W; cfg.prompt_len = P;
  cfg.alpha = 0.125f; cfg.softmax_scale = 0.0f;
  cfg.dtype = LAZYEV_DTYPE_FP32; cfg.score_flags = LAZYEV_SCORE_H1 | LAZYEV_SCORE_H2;
  const int C = lazyev_capacity(&cfg);
  if (C != B + W) { fprintf(stderr, "unexpected capacity %d\n", C); return 1; }
  const size_t rows = (size_t)HKV * C;
  HIP_OK(hipMalloc(&cfg.k_cache, rows * D * sizeof(float)));
  HIP_OK(hipMalloc(&cfg.v_cache, rows * D * sizeof(float)));
  HIP_OK(hipMalloc((void **)&cfg.ts, rows * sizeof(int32_t)));
  HIP_OK(hipMalloc((void **)&cfg.mri, rows * sizeof(int32_t)));
  HIP_OK(hipMalloc((void **)&cfg.pos, rows * sizeof(int32_t)));
  cfg.workspace_bytes = lazyev_workspace_size(&cfg);
  HIP_OK(hipMalloc(&cfg.workspace, cfg.workspace_bytes));
  cfg.stream = NULL;

  /* prompt rows */
  float *host = (float *)malloc(rows * D * sizeof(float));
  for (int s = 0; s < 2; ++s) {
    memset(host, 0, rows * D * sizeof(float));
    for (int h = 0; h < HKV; ++h)
      for (int i = 0; i < P; ++i)
        for (int l = 0; l < D; ++l) host[((size_t)h * C + i) * D + l] = value(1 + s, i, h, l);
    HIP_OK(hipMemcpy(s == 0 ? cfg.k_cache : cfg.v_cache, host, rows * D * sizeof(float), hipMemcpyHostToDevice));
  }

  lazyev_ctx *ctx = NULL;
  LZ_OK(lazyev_init(&cfg, &ctx));

  float *q_d, *k_d, *v_d, *out_d;
  HIP_OK(hipMalloc((void **)&q_d, HQ * D * sizeof(float)));
  HIP_OK(hipMalloc((void **)&k_d, HKV * D * sizeof(float)));
  HIP_OK(hipMalloc((void **)&v_d, HKV * D * sizeof(float)));
  HIP_OK(hipMalloc((void **)&out_d, HQ * D * sizeof(float)));
  float q[HQ * D], kn[HKV * D], vn[HKV * D], out[HQ * D];

  for (int t = 1; t <= STEPS; ++t) {
    for (int h = 0; h < HQ; ++h)
      for (int l = 0; l < D; ++l) q[h * D + l] = value(3, t, h, l);
    for (int h = 0; h < HKV; ++h)
      for (int l = 0; l < D; ++l) {
        kn[h * D + l] = value(1, P + t - 1, h, l);
        vn[h * D + l] = value(2, P + t - 1, h, l);
      }
    HIP_OK(hipMemcpy(q_d, q, sizeof(q), hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(k_d, kn, sizeof(kn), hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(v_d, vn, sizeof(vn), hipMemcpyHostToDevice));
    LZ_OK(lazyev_decode_step(ctx, 0, t, q_d, k_d, v_d, out_d, NULL, NULL));
    int32_t n_evicted = -1;
    LZ_OK(lazyev_evict(ctx, 0, t, &n_evicted));
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(out, out_d, sizeof(out), hipMemcpyDeviceToHost));
    printf("step %d evicted %d out", t, (int)n_evicted);
    for (int i = 0; i < HQ * D; ++i) printf(" %.9e", (double)out[i]);   /* every element, [HQ][D] */
    printf("\n");
  }

  int32_t len = 0, last = 0;
  int64_t events = 0;
  lazyev_stats_t st;
  memset(&st, 0, sizeof(st));
  st.n_layers = 1; st.len = &len; st.last_step = &last; st.n_evict_events = &events;
  LZ_OK(lazyev_stats(ctx, &st));
  printf("len %d last_step %d evict_events %lld\n", (int)len, (int)last, (long long)events);
  int32_t *pos = (int32_t *)malloc(rows * sizeof(int32_t));
  HIP_OK(hipMemcpy(pos, cfg.pos, rows * sizeof(int32_t), hipMemcpyDeviceToHost));
  for (int h = 0; h < HKV; ++h) {
    printf("pos head %d", h);
    for (int i = 0; i < len; ++i) printf(" %d", (int)pos[(size_t)h * C + i]);
    printf("\n");
  }
  /* error paths answer with codes, not with aborts */
  if (lazyev_decode_step(ctx, 0, STEPS + 5, q_d, k_d, v_d, out_d, NULL, NULL) != LAZYEV_EINVAL) return 4;
  if (lazyev_evict(NULL, 0, 1, NULL) != LAZYEV_EINVAL) return 4;
  lazyev_destroy(ctx);
  free(pos); free(host);
  printf("ok\n");
  return 0;
}
