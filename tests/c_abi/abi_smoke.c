/* The C boundary used from plain C: no Python, no torch.  Device memory comes from hipMalloc, the
 * library gets raw pointers.  Every expected value is a closed form:
 *   - zero queries give a uniform softmax, so the output is the arithmetic mean of the live values
 *     (Notation and Preliminaries, attention equation);
 *   - after T steps with window W and chunk C the counters are len = T, base = C * ceil((T - W) / C)
 *     (lazy chunk eviction once the cache is full; Our Approach);
 *   - with the Frobenius Normalize the state has unit norm after the first eviction (the update rule).
 * A second part drives the bf16 MFMA step kernel the same way (run_bf16_mfma).
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

/* ---- the bf16 MFMA step kernel (head_dim 128, window a multiple of 32) from plain C ----
 * Inputs are small integers and one-hot vectors, all exact in bf16, so every expectation is a closed form:
 *   - step 1 attends over a single key: the weight is 1 and the output is the value itself, whatever the
 *     query is (Notation and Preliminaries, attention equation);
 *   - even query heads carry zero queries: uniform softmax, output = mean of the live values;
 *   - odd query heads carry 32 e_j against keys 8 e_(p mod 128): the key of position j scores 256 / sqrt(128)
 *     = 22.6 above every other, so it takes all but n e^-22.6 of the weight and the output is v_j to within
 *     the rounding of the output;
 *   - counters follow the lazy chunk eviction, and the state has unit Frobenius norm after an eviction. */
static uint16_t bf16_of(float f) {          /* exact for the values used here */
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}
static float f32_of(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

static int run_bf16_mfma(void) {
  enum { B2 = 2, HQ2 = 4, HKV2 = 2, D2 = 128, W2 = 64, C2 = 32, G2 = 4, R2 = 8, T2 = 64 + 32 + 7 };
  ptenc_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.batch = B2; cfg.n_q_heads = HQ2; cfg.n_kv_heads = HKV2; cfg.head_dim = D2; cfg.window = W2; cfg.chunk = C2;
  cfg.n_global = G2; cfg.rank = R2; cfg.dtype = PTENC_BF16; cfg.norm_mode = PTENC_NORM_FROBENIUS;
  size_t cb, sb, xb;
  CHECK_PT(ptenc_query_sizes(&cfg, &cb, &sb, &xb));
  void *cache, *state, *scratch;
  CHECK_HIP(hipMalloc(&cache, cb)); CHECK_HIP(hipMalloc(&state, sb)); CHECK_HIP(hipMalloc(&scratch, xb));
  CHECK_HIP(hipMemset(cache, 0xff, cb));      /* NaN everywhere: dead slots must never leak */
  CHECK_HIP(hipMemset(state, 0, sb));
  ptenc_ctx* ctx = NULL;
  CHECK_PT(ptenc_create(&cfg, cache, state, scratch, &ctx));
  int32_t attn_kernel = -1, n_splits = 0, enc_kernel = -1;
  CHECK_PT(ptenc_get_plan(ctx, &attn_kernel, &n_splits, &enc_kernel));
  if (attn_kernel != 1 || enc_kernel != 1) { printf("bf16 / head_dim 128 / window 64 did not select the MFMA kernels\n"); return 1; }

  const int dq = HQ2 * D2, dkv = HKV2 * D2;
  size_t n_enc = (size_t)G2 * dq + (size_t)dq * R2 + 2 * (size_t)dkv * R2 + 2 * (size_t)G2 * dkv;
  uint16_t* h_enc = (uint16_t*)malloc(n_enc * 2);
  for (size_t i = 0; i < n_enc; ++i) h_enc[i] = bf16_of((float)((int)(i * 2654435761u % 17) - 8) / 64.0f);
  uint16_t* d_enc;
  CHECK_HIP(hipMalloc((void**)&d_enc, n_enc * 2));
  CHECK_HIP(hipMemcpy(d_enc, h_enc, n_enc * 2, hipMemcpyHostToDevice));
  uint16_t *qg = d_enc, *WaQ = qg + (size_t)G2 * dq, *WaK = WaQ + (size_t)dq * R2, *WaV = WaK + (size_t)dkv * R2,
           *kg = WaV + (size_t)dkv * R2, *vg = kg + (size_t)G2 * dkv;
  CHECK_PT(ptenc_set_encoder(ctx, qg, WaQ, WaK, WaV, kg, vg, NULL));
  CHECK_PT(ptenc_reset(ctx, NULL, NULL));

  const size_t nq = (size_t)B2 * HQ2 * D2, nkv = (size_t)B2 * HKV2 * D2;
  uint16_t *h_q = (uint16_t*)malloc(nq * 2), *h_k = (uint16_t*)malloc(nkv * 2), *h_v = (uint16_t*)malloc(nkv * 2),
           *h_out = (uint16_t*)malloc(nq * 2);
  uint16_t *d_q, *d_k, *d_v, *d_out;
  CHECK_HIP(hipMalloc((void**)&d_q, nq * 2)); CHECK_HIP(hipMalloc((void**)&d_out, nq * 2));
  CHECK_HIP(hipMalloc((void**)&d_k, nkv * 2)); CHECK_HIP(hipMalloc((void**)&d_v, nkv * 2));
  for (int t = 0; t < T2; ++t) {
    const int n = t + 1, base = n > W2 ? C2 * ((n - W2 + C2 - 1) / C2) : 0;
    const int target = base + (t - base) / 2;                     /* a live position the odd heads look for */
    for (int b = 0; b < B2; ++b) {
      for (int h = 0; h < HKV2; ++h)
        for (int i = 0; i < D2; ++i) {
          h_k[((size_t)b * HKV2 + h) * D2 + i] = bf16_of(i == t % D2 ? 8.0f : 0.0f);
          h_v[((size_t)b * HKV2 + h) * D2 + i] = bf16_of(value_of(t, b, h, i));
        }
      for (int hq = 0; hq < HQ2; ++hq)
        for (int i = 0; i < D2; ++i)
          h_q[((size_t)b * HQ2 + hq) * D2 + i] = bf16_of((hq & 1) && i == target % D2 ? 32.0f : 0.0f);
    }
    CHECK_HIP(hipMemcpy(d_q, h_q, nq * 2, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_k, h_k, nkv * 2, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(d_v, h_v, nkv * 2, hipMemcpyHostToDevice));
    CHECK_PT(ptenc_decode_step(ctx, d_q, d_k, d_v, d_out, NULL, NULL));
    CHECK_HIP(hipMemcpy(h_out, d_out, nq * 2, hipMemcpyDeviceToHost));
    for (int b = 0; b < B2; ++b)
      for (int hq = 0; hq < HQ2; ++hq)
        for (int i = 0; i < D2; ++i) {
          const int h = hq / (HQ2 / HKV2);
          double want;
          if (hq & 1) {
            want = value_of(target, b, h, i);                     /* one key takes the weight */
          } else {
            want = 0.0;
            for (int p = base; p <= t; ++p) want += value_of(p, b, h, i);
            want /= (double)(t + 1 - base);
          }
          const double got = f32_of(h_out[((size_t)b * HQ2 + hq) * D2 + i]);
          /* the stated bar for bf16 outputs, against a value range of 5 */
          if (!(fabs(got - want) <= 1e-2 + 2e-2 * fabs(want))) {
            printf("bf16 step %d rollout %d head %d column %d: got %g, expected %g\n", t, b, hq, i, got, want);
            return 1;
          }
          if (t == 0 && got != value_of(0, b, h, i)) {            /* a single key: the value itself, exactly */
            printf("bf16 single key: rollout %d head %d column %d: got %g, the value is %g\n", b, hq, i, got, value_of(0, b, h, i));
            return 1;
          }
        }
  }
  int64_t len[B2], base[B2];
  CHECK_PT(ptenc_get_counters(ctx, len, base, NULL));
  for (int b = 0; b < B2; ++b)
    if (len[b] != T2 || base[b] != C2 * ((T2 - W2 + C2 - 1) / C2)) { printf("bf16 counters of rollout %d: len %lld base %lld\n", b, (long long)len[b], (long long)base[b]); return 1; }
  float S[B2 * G2 * R2];
  CHECK_PT(ptenc_get_state(ctx, S, NULL));
  for (int b = 0; b < B2; ++b) {
    double ss = 0.0;
    for (int i = 0; i < G2 * R2; ++i) ss += (double)S[b * G2 * R2 + i] * S[b * G2 * R2 + i];
    if (!(fabs(sqrt(ss) - 1.0) <= 1e-5)) { printf("bf16 state of rollout %d has norm %g, not 1\n", b, sqrt(ss)); return 1; }
  }
  int32_t flags = -1;
  CHECK_PT(ptenc_poll_error(ctx, &flags, NULL));
  if (flags != 0) { printf("bf16 device error word %d\n", flags); return 1; }
  /* the MFMA path wants 16-byte aligned rows: a misaligned pointer is an error code, and changes nothing */
  if (ptenc_decode_step(ctx, d_q + 1, d_k, d_v, d_out, NULL, NULL) != PTENC_ERR_INVALID_ARG) { printf("misaligned q was not rejected\n"); return 1; }
  CHECK_PT(ptenc_get_counters(ctx, len, base, NULL));
  if (len[0] != T2) { printf("a rejected call advanced the counters\n"); return 1; }
  CHECK_PT(ptenc_destroy(ctx));
  return 0;
}

int main(void) {
  if (run_bf16_mfma() != 0) return 1;
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
