// The plain-ALU thought encoder (any dtype, cache layout, G and r up to 64), shared by the kernels
// that evict: S' = (Q_a (K_e W^a_K)^T)(V_e W^a_V) (Our Approach, the Delta-W equation) in the
// paper's association, 32 tokens at a time, fp32 accumulation, one workgroup of kEncThreads threads.
#pragma once

#include "pt_encode_tail.h"

constexpr int kEncKB = 64;   // contraction block over d_kv

struct EncSmem {
  float Ks[kEncSub][kEncKB + 1];
  float Ws[kEncKB][kEncMaxGR];       // reused as the G x r staging area of the state update
  EncTailSmem tail;
};

// S' of a chunk of n_tok tokens; thread t ends up with entries t, t+256, ... of the row-major
// G x r result in sacc[].  dbg (may be null) receives the raw chunk [2][n_tok][d_kv].
template <typename T, typename Src>
__device__ void encode_chunk(EncSmem& sm, const Src& src, int n_tok, int dkv, int G, int r,
                             const float* __restrict__ Qa, const T* __restrict__ WaK,
                             const T* __restrict__ WaV, T* dbg, float sacc[16]) {
  const int t = threadIdx.x;
  const int tok = t & (kEncSub - 1), cg = t >> 5;   // 8 column groups
#pragma unroll
  for (int x = 0; x < 16; ++x) sacc[x] = 0.f;

  for (int sub0 = 0; sub0 < n_tok; sub0 += kEncSub) {
    const int ntok = min(kEncSub, n_tok - sub0);
    for (int which = 0; which < 2; ++which) {
      const T* Wsrc = which == 0 ? WaK : WaV;
      float acc[8];
#pragma unroll
      for (int x = 0; x < 8; ++x) acc[x] = 0.f;
      for (int kb = 0; kb < dkv; kb += kEncKB) {
        const int nk = min(kEncKB, dkv - kb);
        // all loads of the block first (nothing between them that could alias), then the stores
        constexpr int kPer = kEncSub * kEncKB / kEncThreads;
        float vals[kPer];
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
          const int idx = t + u * kEncThreads;
          const int tk = idx / kEncKB, kk = idx - tk * kEncKB;
          vals[u] = (tk < ntok && kk < nk) ? src.get(which, sub0 + tk, kb + kk) : 0.f;
        }
        for (int idx = t; idx < kEncKB * r; idx += kEncThreads) {
          const int kk = idx / r, col = idx - kk * r;
          sm.Ws[kk][col] = kk < nk ? pt_ld<T>(Wsrc + (size_t)(kb + kk) * r + col) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
          const int idx = t + u * kEncThreads;
          const int tk = idx / kEncKB, kk = idx - tk * kEncKB;
          sm.Ks[tk][kk] = vals[u];
          if (dbg && tk < ntok && kk < nk) pt_st<T>(dbg + ((size_t)which * n_tok + sub0 + tk) * dkv + kb + kk, vals[u]);
        }
        __syncthreads();
        for (int kk = 0; kk < kEncKB; ++kk) {
          const float kv = sm.Ks[tok][kk];
#pragma unroll
          for (int x = 0; x < 8; ++x) {
            const int col = cg + 8 * x;
            if (col < r) acc[x] = fmaf(kv, sm.Ws[kk][col], acc[x]);
          }
        }
        __syncthreads();
      }
#pragma unroll
      for (int x = 0; x < 8; ++x) {
        const int col = cg + 8 * x;
        if (col < r) (which == 0 ? sm.tail.Ka : sm.tail.Va)[tok][col] = acc[x];
      }
    }
    __syncthreads();
    pt_encode_accumulate<kEncThreads>(sm.tail, Qa, r, G, r, sacc);      // rows of tokens beyond ntok are zero
  }
}

