// Shared tail of the thought encoder: given K_a and V_a of up to 32 tokens in LDS, accumulate
// S' += (Q_a K_a^T) V_a, and the state update S <- Normalize(S + S')
// (Our Approach, the Delta-W equation and the update rule).  THREADS = workgroup size (256 or 512).
#pragma once

#include "ptenc_internal.h"

constexpr int kEncThreads = 256;   // workgroup size of the plain-ALU encoder kernels
constexpr int kEncSub = 32;     // tokens per sub-chunk
constexpr int kEncMaxGR = 64;   // max G and r

struct EncTailSmem {
  float Ka[kEncSub][kEncMaxGR + 1];
  float Va[kEncSub][kEncMaxGR + 1];
  float P[kEncMaxGR][kEncSub + 1];
  float red[16];
};

// Thread t owns entries t, t+THREADS, ... of the row-major G x r accumulator sacc[16].
// Ka / Va rows at and beyond ntok must be zero or are ignored.  Ends with a barrier.
template <int THREADS>
__device__ inline void pt_encode_accumulate(EncTailSmem& sm, const float* __restrict__ Qa, int G, int r,
                                            int ntok, float sacc[16]) {
  const int t = threadIdx.x;
  for (int idx = t; idx < G * kEncSub; idx += THREADS) {   // P = Q_a K_a^T  (G x 32)
    const int g = idx / kEncSub, tk = idx - g * kEncSub;
    float p = 0.f;
    if (tk < ntok)
      for (int a = 0; a < r; ++a) p = fmaf(Qa[g * r + a], sm.Ka[tk][a], p);
    sm.P[g][tk] = p;
  }
  __syncthreads();
#pragma unroll
  for (int x = 0; x < 4096 / THREADS; ++x) {                               // S' += P V_a  (G x r)
    const int idx = t + THREADS * x;
    if (idx < G * r) {
      const int g = idx / r, col = idx - g * r;
      float s = sacc[x];
      for (int tk = 0; tk < ntok; ++tk) s = fmaf(sm.P[g][tk], sm.Va[tk][col], s);
      sacc[x] = s;
    }
  }
  __syncthreads();
}

template <int THREADS>
__device__ inline float pt_block_sum(float v, float* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float tot = 0.f;
  for (int i = 0; i < THREADS / 64; ++i) tot += red[i];
  return tot;
}

// S[b] <- Normalize(S[b] + S'), S' in sacc.  `stage` is G*r floats of LDS (row-norm mode only).
template <int THREADS>
__device__ inline void pt_state_update(const PtDev& c, int b, float sacc[16], float* stage, float* red) {
  const int t = threadIdx.x, n = c.G * c.r;
  float* S = c.S + (size_t)b * n;
  float ss = 0.f;
#pragma unroll
  for (int x = 0; x < 4096 / THREADS; ++x) {
    const int idx = t + THREADS * x;
    if (idx < n) {
      sacc[x] += S[idx];
      ss = fmaf(sacc[x], sacc[x], ss);
      if (c.norm_mode == PTENC_NORM_ROW_L2) stage[idx] = sacc[x];
    }
  }
  if (c.norm_mode == PTENC_NORM_FROBENIUS) {
    const float nrm = fmaxf(sqrtf(pt_block_sum<THREADS>(ss, red)), c.norm_eps);
#pragma unroll
    for (int x = 0; x < 4096 / THREADS; ++x) {
      const int idx = t + THREADS * x;
      if (idx < n) S[idx] = sacc[x] / nrm;
    }
  } else if (c.norm_mode == PTENC_NORM_ROW_L2) {
    __syncthreads();
#pragma unroll
    for (int x = 0; x < 4096 / THREADS; ++x) {
      const int idx = t + THREADS * x;
      if (idx < n) {
        const int g = idx / c.r;
        float rs = 0.f;
        for (int a = 0; a < c.r; ++a) rs = fmaf(stage[g * c.r + a], stage[g * c.r + a], rs);
        S[idx] = sacc[x] / fmaxf(sqrtf(rs), c.norm_eps);
      }
    }
  } else {
#pragma unroll
    for (int x = 0; x < 4096 / THREADS; ++x) {
      const int idx = t + THREADS * x;
      if (idx < n) S[idx] = sacc[x];
    }
  }
}
