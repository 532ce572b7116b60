// Ring-buffer cache maintenance and the plain-ALU thought encoder.
//
//  * reset / gather / counters helpers
//  * step prologue: [evict the oldest chunk of a full window and fold it into S] then
//    [append the new k, v], one workgroup per rollout so the two never race on a slot
//  * encoder set-up: Q_a = q_g W^a_Q and S_0
//
// The encoder here is the general one (any dtype, layout, G and r up to 64).  It evaluates
// S' = (Q_a (K_e W^a_K)^T)(V_e W^a_V) (Our Approach, the Delta-W equation) in the paper's
// association, 32 tokens at a time, with fp32 accumulation.
#include "pt_prologue.h"

namespace {

constexpr int kThreads = kEncThreads;

template <typename T>
struct GlobalTokens { // k_g, v_g: row-major [G, d_kv]
  const T* kg; const T* vg; int dkv;
  __device__ float get(int which, int tok, int kk) const {
    return pt_ld<T>((which == 0 ? kg : vg) + (size_t)tok * dkv + kk);
  }
};

// ---- step prologue ----------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void step_prologue_kernel(PtDev c, int do_evict, int do_append,
                                                                const T* __restrict__ knew,
                                                                const T* __restrict__ vnew,
                                                                const uint8_t* __restrict__ active,
                                                                T* dbg_chunk, const int* __restrict__ ids,
                                                                int in_place) {
  __shared__ EncSmem sm;
  pt_step_prologue<T>(sm, c, blockIdx.x, do_evict, do_append, knew, vnew, active, dbg_chunk, ids, in_place);
}

// ---- reset / gather -----------------------------------------------------------------------------
__global__ void reset_kernel(PtDev c, const uint8_t* __restrict__ mask, int clear_err) {
  const int b = blockIdx.x;
  if (clear_err && b == 0 && threadIdx.x == 0) *c.err = 0;
  // arrival counters are zero between kernels anyway; a fresh context gets them zeroed here
  if (threadIdx.x == 0) { c.tick_rollout[b] = 0; c.tick_enc[b] = 0; }
  for (int h = threadIdx.x; h < c.Hkv; h += blockDim.x) c.tick_slab[b * c.Hkv + h] = 0;
  if (mask && !mask[b]) return;
  const int n = c.G * c.r;
  for (int i = threadIdx.x; i < n; i += blockDim.x) { c.S[(size_t)b * n + i] = c.S0[i]; c.pend[(size_t)b * n + i] = 0.f; }
  if (threadIdx.x == 0) c.enc_done[b] = 0;            // nothing of a next chunk is folded ahead of time
  // both counter buffers: a compact-list step merges into the other one by maximum
  if (threadIdx.x == 0) { c.len[b] = 0; c.base[b] = 0; c.len_nx[b] = 0; c.base_nx[b] = 0; c.n_prompt[b] = 0; }
  // importance scores: nothing waits to be folded, no eviction has happened
  for (int h = threadIdx.x; h < c.Hkv; h += blockDim.x) c.mtag[b * c.Hkv + h] = -1;
  for (int i = threadIdx.x; i < c.C; i += blockDim.x) c.victims[(size_t)b * c.C + i] = -1;
  if (threadIdx.x == 0) c.selected[b] = 0;
}

template <typename T>
__global__ void gather_kernel(PtDev c, T* __restrict__ Kout, T* __restrict__ Vout) {
  const int slab = blockIdx.x, b = slab / c.Hkv;
  const long long len = c.len[b], base = c.base[b];
  const int n_live = (int)(len - base), s0 = (int)(base % c.Wr), P = c.n_prompt[b];
  const T* src = (const T*)c.cache + (size_t)slab * pt_slab_elems(c.W, c.d);
  for (int j = blockIdx.y; j < c.W; j += gridDim.y) {
    int slot = j;                                  // question tokens first ...
    if (j >= P) { slot = s0 + (j - P); if (slot >= c.Wr) slot -= c.Wr; slot += c.n_sink; }   // ... then the ring
    for (int i = threadIdx.x; i < c.d; i += blockDim.x) {
      const size_t o = ((size_t)slab * c.W + j) * c.d + i;
      if (j < P + n_live) {
        Kout[o] = src[pt_k_off(c.tiled, c.W, c.d, slot, i)];
        Vout[o] = src[pt_v_off(c.tiled, c.W, c.d, slot, i)];
      } else {
        Kout[o] = (T)0; Vout[o] = (T)0;
      }
    }
  }
}

// Question tokens [B, p_max, H_kv, d] into the reserved slots: one workgroup per (slab, 32 tokens).
// The 32 x d tile is staged in LDS so that the tiled layout is written in whole 16-byte vectors.
// With a rollout list (ids, lens: row j of kin / vin belongs to rollout ids[j] and has lens[j] tokens)
// only the listed rollouts are touched, and their question-token counts are set here.
template <typename T>
__global__ __launch_bounds__(256) void prefill_kernel(PtDev c, const T* __restrict__ kin, const T* __restrict__ vin,
                                                      int p_max, const int* __restrict__ ids,
                                                      const int* __restrict__ lens) {
  __shared__ T tile[32][256 + 8];
  const int row = blockIdx.x / c.Hkv, h = blockIdx.x - row * c.Hkv, j0 = blockIdx.y * 32;
  int b = row;
  if (ids) {
    b = ids[row];
    if ((unsigned)b >= (unsigned)c.B) {            // never index with a bad id: flag it and leave
      if (threadIdx.x == 0 && h == 0 && j0 == 0) atomicOr(c.err, PTENC_DEVERR_BAD_ID);
      return;
    }
  }
  const int slab = b * c.Hkv + h;
  const int P = ids ? lens[row] : c.n_prompt[b];
  if (ids && h == 0 && j0 == 0 && threadIdx.x == 0) c.n_prompt[b] = P;   // read by later launches only
  if (j0 >= P) return;
  const int n = min(32, P - j0);
  T* dst = (T*)c.cache + (size_t)slab * pt_slab_elems(c.W, c.d);
  for (int which = 0; which < 2; ++which) {
    const T* in = which == 0 ? kin : vin;
    for (int idx = threadIdx.x; idx < 32 * c.d; idx += blockDim.x) {
      const int tk = idx / c.d, i = idx - tk * c.d;
      tile[tk][i] = tk < n ? in[(((size_t)row * p_max + j0 + tk) * c.Hkv + h) * c.d + i] : (T)0;
    }
    __syncthreads();
    if (c.tiled) {
      // d = 128: 512 vectors of 8 elements for the two K tiles, 512 for the token-minor V part
      typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
      union { u32x4 u; uint16_t s[8]; } vec;
      uint16_t* g = (uint16_t*)dst + (size_t)(j0 >> 5) * PT_GROUP_ELEMS + which * 4096;
      for (int vi = threadIdx.x; vi < 512; vi += blockDim.x) {
        if (which == 0) {
          const int t = vi >> 8, cc = (vi >> 6) & 3, kgrp = (vi >> 4) & 3, m = vi & 15;
#pragma unroll
          for (int e = 0; e < 8; ++e) vec.s[e] = (uint16_t)tile[16 * t + m][32 * cc + 8 * kgrp + e];
        } else {
          const int it = vi >> 6, kgrp = (vi >> 4) & 3, m = vi & 15;
#pragma unroll
          for (int e = 0; e < 8; ++e) vec.s[e] = (uint16_t)tile[(e >> 2) * 16 + 4 * kgrp + (e & 3)][16 * it + m];
        }
        *(u32x4*)(g + (size_t)vi * 8) = vec.u;
      }
    } else {
      for (int idx = threadIdx.x; idx < n * c.d; idx += blockDim.x) {
        const int tk = idx / c.d, i = idx - tk * c.d;
        const size_t off = which == 0 ? pt_k_off(0, c.W, c.d, j0 + tk, i) : pt_v_off(0, c.W, c.d, j0 + tk, i);
        dst[off] = tile[tk][i];
      }
    }
    __syncthreads();
  }
}

// ---- encoder set-up -----------------------------------------------------------------------------
template <typename T>
__global__ void qa_kernel(PtDev c, const T* __restrict__ qg, const T* __restrict__ WaQ) {
  const int g = blockIdx.x, a = threadIdx.x;
  if (a >= c.r) return;
  const int dq = c.Hq * c.d;
  float acc = 0.f;
  for (int x = 0; x < dq; ++x) acc = fmaf(pt_ld<T>(qg + (size_t)g * dq + x), pt_ld<T>(WaQ + (size_t)x * c.r + a), acc);
  c.Qa[g * c.r + a] = acc;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void s0_kernel(PtDev c, const T* __restrict__ kg, const T* __restrict__ vg) {
  __shared__ EncSmem sm;
  const int t = threadIdx.x;
  float sacc[16];
#pragma unroll
  for (int x = 0; x < 16; ++x) sacc[x] = 0.f;
  if (kg && vg) {
    GlobalTokens<T> src{kg, vg, c.Hkv * c.d};
    encode_chunk<T>(sm, src, c.G, c.Hkv * c.d, c.G, c.r, c.Qa, (const T*)c.WaK, (const T*)c.WaV, (T*)nullptr, sacc);
  }
#pragma unroll
  for (int x = 0; x < 16; ++x) {
    const int idx = t + kThreads * x;
    if (idx < c.G * c.r) c.S0[idx] = sacc[x];
  }
}

}  // namespace

hipError_t pt_launch_reset(const PtDev& c, const uint8_t* mask, bool clear_err, hipStream_t s) {
  hipLaunchKernelGGL(reset_kernel, dim3(c.B), dim3(256), 0, s, c, mask, clear_err ? 1 : 0);
  return hipGetLastError();
}

hipError_t pt_launch_step_prologue(const PtDev& c, bool do_evict, bool do_append,
                                   const void* k, const void* v, const uint8_t* active, void* dbg_chunk,
                                   const int* ids, int n_rows, bool in_place, hipStream_t s) {
  const dim3 grid(ids ? n_rows : c.B);
  const int ip = (ids != nullptr || in_place) ? 1 : 0;
  if (c.dtype == PTENC_F32)
    hipLaunchKernelGGL(step_prologue_kernel<float>, grid, dim3(kThreads), 0, s, c, do_evict ? 1 : 0,
                       do_append ? 1 : 0, (const float*)k, (const float*)v, active, (float*)dbg_chunk, ids, ip);
  else
    hipLaunchKernelGGL(step_prologue_kernel<uint16_t>, grid, dim3(kThreads), 0, s, c, do_evict ? 1 : 0,
                       do_append ? 1 : 0, (const uint16_t*)k, (const uint16_t*)v, active, (uint16_t*)dbg_chunk, ids, ip);
  return hipGetLastError();
}

hipError_t pt_launch_gather(const PtDev& c, void* K, void* V, hipStream_t s) {
  dim3 grid(c.B * c.Hkv, c.W < 64 ? c.W : 64);
  const int threads = c.d <= 64 ? 64 : (c.d <= 128 ? 128 : 256);
  if (c.dtype == PTENC_F32)
    hipLaunchKernelGGL(gather_kernel<float>, grid, dim3(threads), 0, s, c, (float*)K, (float*)V);
  else
    hipLaunchKernelGGL(gather_kernel<uint16_t>, grid, dim3(threads), 0, s, c, (uint16_t*)K, (uint16_t*)V);
  return hipGetLastError();
}

hipError_t pt_launch_prefill(const PtDev& c, const void* k, const void* v, int p_max, const int* ids, const int* lens,
                             int n_rows, hipStream_t s) {
  dim3 grid((ids ? n_rows : c.B) * c.Hkv, (c.n_sink + 31) / 32);
  if (c.dtype == PTENC_F32)
    hipLaunchKernelGGL(prefill_kernel<float>, grid, dim3(256), 0, s, c, (const float*)k, (const float*)v, p_max, ids, lens);
  else
    hipLaunchKernelGGL(prefill_kernel<uint16_t>, grid, dim3(256), 0, s, c, (const uint16_t*)k, (const uint16_t*)v, p_max, ids,
                       lens);
  return hipGetLastError();
}

hipError_t pt_launch_encoder_init(const PtDev& c, const void* qg, const void* WaQ, const void* kg,
                                  const void* vg, hipStream_t s) {
  if (c.dtype == PTENC_F32) {
    hipLaunchKernelGGL(qa_kernel<float>, dim3(c.G), dim3(64), 0, s, c, (const float*)qg, (const float*)WaQ);
    hipLaunchKernelGGL(s0_kernel<float>, dim3(1), dim3(kThreads), 0, s, c, (const float*)kg, (const float*)vg);
  } else {
    hipLaunchKernelGGL(qa_kernel<uint16_t>, dim3(c.G), dim3(64), 0, s, c, (const uint16_t*)qg, (const uint16_t*)WaQ);
    hipLaunchKernelGGL(s0_kernel<uint16_t>, dim3(1), dim3(kThreads), 0, s, c, (const uint16_t*)kg, (const uint16_t*)vg);
  }
  return hipGetLastError();
}
