/* The C boundary used from plain C: no Python, no torch.  Device memory comes from hipMalloc, the
 * library gets raw pointers.  Every expected value is a closed form:
 *   - zero queries give a uniform softmax, so the output is the arithmetic mean of the live values
 *     (Notation and Preliminaries, attention equation);
 *   - after T steps with window W and chunk C the counters are len = T, base = C * ceil((T - W) / C)
 *     (lazy chunk eviction once the cache is full; Our Approach);
 *   - with the Frobenius Normalize the state has unit norm after the first eviction (the update rule).
 * Prints "abi_smoke ok" and returns 0, or says what failed and returns 1. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "ptenc.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); return 1; } } while (0)
#define CHECK_PT(x) do { ptenc_status s_ = (x); if (s_ != PTENC_OK) { printf("%s: %s (line %d)\n", #x, ptenc_status_string(s_), __LINE__); return 1; } } while (0)

enum { B = 3, HQ = 4, HKV = 2, D = 32, W = 16, C = 4, G = 4, R = 4, T = 27 };

static float value_of(int t, int b, int h, int i) { return (float)((t * 7 + b * 3 + h * 5 + i) % 11) - 5.0f; }

int main(void) {
  ptenc_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.batch = B; cfg.n_q_heads = HQ; cfg.n_kv_heads = HKV; cfg.head_dim = D; cfg.window = W; cfg.chunk = C;
  cfg.n_global = G; cfg.rank = R; cfg.dtype = PTENC_F32; cfg.norm_mode = PTENC_NORM_FROBENIUS;
  size_t cb, sb, xb;
  CHECK_PT(ptenc_query_sizes(&cfg, &cb, &sb, &xb));
  void *cache, *state, *scratch;
  CHECK_HIP(hipMalloc(&cache, cb)); CHECK_HIP(hipMalloc(&state, sb)); CHECK_HIP(hipMalloc(&scratch, xb));
  CHECK_HIP(hipMemset(cache, 0xff, cb));      /* every float reads as NaN: dead slots must never leak */
  CHECK_HIP(hipMemset(state, 0, sb));
  ptenc_ctx* ctx = NULL;
  CHECK_PT(ptenc_create(&cfg, cache, state, scratch, &ctx));

  /* encoder parameters: small deterministic numbers */
  const int dq = HQ * D, dkv = HKV * D;
  size_t n_enc = (size_t)G * dq + (size_t)dq * R + 2 * (size_t)dkv * R + 2 * (size_t)G * dkv;
  float* h_enc = (float*)malloc(n_enc * sizeof(float));
  for (size_t i = 0; i < n_enc; ++i) h_enc[i] = (float)((int)(i * 2654435761u % 17) - 8) / 64.0f;
  float* d_enc;
  CHECK_HIP(hipMalloc((void**)&d_enc, n_enc * sizeof(float)));
  CHECK_HIP(hipMemcpy(d_enc, h_enc, n_enc * sizeof(float), hipMemcpyHostToDevice));
  float *qg = d_enc, *WaQ = qg + (size_t)G * dq, *WaK = WaQ + (size_t)dq * R, *WaV = WaK + (size_t)dkv * R,
        *kg = WaV + (size_t)dkv * R, *vg = kg + (size_t)G * dkv;
  CHECK_PT(ptenc_set_encoder(ctx, qg, WaQ, WaK, WaV, kg, vg, NULL));
  CHECK_PT(ptenc_reset(ctx, NULL, NULL));

  /* T decode steps: q = 0, k arbitrary, v = value_of */
  const size_t nq = (size_t)B * HQ * D, nkv = (size_t)B * HKV * D;
  float *h_q = (float*)calloc(nq, sizeof(float)), *h_k = (float*)malloc(nkv * sizeof(float)),
        *h_v = (float*)malloc(nkv * sizeof(float)), *h_out = (float*)malloc(nq * sizeof(float));
  float *d_q, *d_k, *d_v, *d_out;
  CHECK_HIP(hipMalloc((void**)&d_q, nq * sizeof(float))); CHECK_HIP(hipMalloc((void**)&d_out, nq * sizeof(float)));
  CHECK_HIP(hipMalloc((void**)&d_k, nkv * sizeof(float))); CHECK_HIP(hipMalloc((void**)&d_v, nkv * sizeof(float)));
  CHECK_HIP(hipMemcpy(d_q, h_q, nq * sizeof(float), hipMemcpyHostToDevice));
  for (int t = 0; t < T; ++t) {
    for (int b = 0; b < B; ++b)
      for (int h = 0; h < HKV; ++h)
        for (int i = 0; i < D; ++i) {
          h_k[((size_t)b * HKV + h) * D + i] = 0.25f * value_of(t + 3, b, h, i);
          h_v[((size_t)b * HKV + h) * D + i] = value_of(t, b, h, i);
        }
    CHECK_HIP(hipMemcpy(d_k, h_k, nkv * sizeof(float), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_v, h_v, nkv * sizeof(float), hipMemcpyHostToDevice));
    CHECK_PT(ptenc_decode_step(ctx, d_q, d_k, d_v, d_out, NULL, NULL));
    CHECK_HIP(hipMemcpy(h_out, d_out, nq * sizeof(float), hipMemcpyDeviceToHost));
    /* live positions after this step: [base, t], base = C * ceil((t + 1 - W) / C) once t + 1 > W */
    const int n = t + 1, base = n > W ? C * ((n - W + C - 1) / C) : 0;
    for (int b = 0; b < B; ++b)
      for (int hq = 0; hq < HQ; ++hq)
        for (int i = 0; i < D; ++i) {
          double mean = 0.0;
          for (int p = base; p <= t; ++p) mean += value_of(p, b, hq / (HQ / HKV), i);
          mean /= (double)(t + 1 - base);
          const double got = h_out[((size_t)b * HQ + hq) * D + i];
          if (!(fabs(got - mean) <= 1e-5)) {
            printf("step %d rollout %d head %d column %d: got %g, mean of the live values is %g\n", t, b, hq, i, got, mean);
            return 1;
          }
        }
  }
  int64_t len[B], base[B];
  CHECK_PT(ptenc_get_counters(ctx, len, base, NULL));
  for (int b = 0; b < B; ++b)
    if (len[b] != T || base[b] != C * ((T - W + C - 1) / C)) { printf("counters of rollout %d: len %lld base %lld\n", b, (long long)len[b], (long long)base[b]); return 1; }
  float S[B * G * R];
  CHECK_PT(ptenc_get_state(ctx, S, NULL));
  for (int b = 0; b < B; ++b) {
    double ss = 0.0;
    for (int i = 0; i < G * R; ++i) ss += (double)S[b * G * R + i] * S[b * G * R + i];
    if (!(fabs(sqrt(ss) - 1.0) <= 1e-5)) { printf("state of rollout %d has norm %g, not 1\n", b, sqrt(ss)); return 1; }
  }
  int32_t flags = -1;
  CHECK_PT(ptenc_poll_error(ctx, &flags, NULL));
  if (flags != 0) { printf("device error word %d\n", flags); return 1; }
  /* misuse is an error code, never a crash */
  if (ptenc_decode_step(ctx, NULL, d_k, d_v, d_out, NULL, NULL) != PTENC_ERR_INVALID_ARG) { printf("NULL q was not rejected\n"); return 1; }
  CHECK_PT(ptenc_destroy(ctx));
  printf("abi_smoke ok\n");
  return 0;
}
