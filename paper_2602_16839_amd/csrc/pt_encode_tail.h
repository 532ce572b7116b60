// Tail of the thought encoder: given K_a and V_a of up to 32 tokens in LDS, accumulate
// S' += (Q_a K_a^T) V_a (plain ALU: the encoder of the plain path; the MFMA kernel does this part on
// the matrix units), and the state update S <- Normalize(S + S') that both share
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

// S' += (Q_a K_a^T) V_a for the 32 tokens whose K_a and V_a rows are in LDS (rows that hold no token
// must be zero).  Qa: G rows of qa_stride floats, in LDS (staged) or in global memory.  Thread t owns
// entries t, t+THREADS, ... of the row-major G x r accumulator sacc[16].  Ends with a barrier.  All loops have fixed trip counts or independent accumulators, so the LDS reads
// of many terms are in flight together (the straightforward dot-product loops were latency-bound:
// ~12 us per 32 tokens).
template <int THREADS>
__device__ inline void pt_encode_accumulate(EncTailSmem& sm, const float* Qa, int qa_stride, int G, int r,
                                            float sacc[16]) {
  const int t = threadIdx.x;
  {
    // P = Q_a K_a^T (G x 32): entry t + THREADS x is (g = its index / 32, token = t % 32)
    constexpr int NX = kEncMaxGR * kEncSub / THREADS, DG = THREADS / kEncSub;
    const int tk = t & (kEncSub - 1), gq = t >> 5;
    float p[NX];
    int grow[NX];
#pragma unroll
    for (int x = 0; x < NX; ++x) { p[x] = 0.f; grow[x] = gq + DG * x < G ? gq + DG * x : 0; }   // clamped: computed, not stored
#pragma unroll 4
    for (int a = 0; a < r; ++a) {
      const float ka = sm.Ka[tk][a];
#pragma unroll
      for (int x = 0; x < NX; ++x) p[x] = fmaf(Qa[grow[x] * qa_stride + a], ka, p[x]);
    }
#pragma unroll
    for (int x = 0; x < NX; ++x)
      if (gq + DG * x < G) sm.P[gq + DG * x][tk] = p[x];
  }
  __syncthreads();
  {
    // S' += P V_a (G x r)
    int g = t / r, col = t - g * r;
    const int dg = THREADS / r, dc = THREADS - dg * r;
#pragma unroll
    for (int x = 0; x < 4096 / THREADS; ++x) {
      if (THREADS * x < G * r) {                       // uniform
        const bool mine = t + THREADS * x < G * r;
        const int gg = mine ? g : 0, cc = mine ? col : 0;
        // one chain over all tokens of the chunk, in order (rows of zeros leave it as it is), so S does
        // not depend on how the chunk falls into groups of 32
        float s = sacc[x];
#pragma unroll
        for (int tk = 0; tk < kEncSub; ++tk) s = fmaf(sm.P[gg][tk], sm.Va[tk][cc], s);
        if (mine) sacc[x] = s;
      }
      g += dg; col += dc;
      if (col >= r) { col -= r; ++g; }
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
// ADD_S = false: the caller has added S[b] to sacc already (it fetched S while it waited for something else).
template <int THREADS, bool ADD_S = true>
__device__ inline void pt_state_update(const PtDev& c, int b, float sacc[16], float* stage, float* red) {
  const int t = threadIdx.x, n = c.G * c.r;
  float* S = c.S + (size_t)b * n;
  float ss = 0.f;
#pragma unroll
  for (int x = 0; x < 4096 / THREADS; ++x) {
    const int idx = t + THREADS * x;
    if (idx < n) {
      if (ADD_S) sacc[x] += S[idx];
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
