// The context state applied as a per-rollout low-rank weight delta:  y[b] += ((x[b] A) S_b) B
// (Our Approach: Delta-W = A S B and theta' = theta + Delta-W; row convention, A is d_in x G and
// B is r x d_out).  A and B arrive transposed (A^T [G, d_in], B^T [d_out, r]) so that both long
// loops read contiguous memory.  One workgroup per rollout, fp32 accumulation:
//   u = x A      G dot products of length d_in, a wavefront per g, lanes strided over d_in
//   w = u S_b    G x r, one thread per column
//   y += w B     one thread per output column, r terms each
// 60 MFLOP and under 4 MB at the 7B shape: the launch, not the arithmetic, is what it costs; in a
// full model this belongs in the epilogue of the projection it adapts.
#include "ptenc_internal.h"

namespace {

constexpr int kThreads = 256;

// dot product of n elements, 8 at a time when T is bf16 and both rows are 16-byte aligned
template <typename T>
__device__ inline float lane_dot(const T* __restrict__ a, const T* __restrict__ b, int n, int lane) {
  float acc = 0.f;
  for (int i = lane; i < n; i += 64) acc = fmaf(pt_ld<T>(a + i), pt_ld<T>(b + i), acc);
  return acc;
}

template <>
__device__ inline float lane_dot<uint16_t>(const uint16_t* __restrict__ a, const uint16_t* __restrict__ b, int n,
                                           int lane) {
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  float acc = 0.f;
  int done = 0;
  if ((((uintptr_t)a | (uintptr_t)b) & 15) == 0) {
    const int nv = n >> 3;
    for (int v = lane; v < nv; v += 64) {
      union { u32x4 u; uint16_t s[8]; } va, vb;
      va.u = ((const u32x4*)a)[v];
      vb.u = ((const u32x4*)b)[v];
#pragma unroll
      for (int e = 0; e < 8; ++e) acc = fmaf(pt_bf16_to_f32(va.s[e]), pt_bf16_to_f32(vb.s[e]), acc);
    }
    done = nv << 3;
  }
  for (int i = done + lane; i < n; i += 64) acc = fmaf(pt_bf16_to_f32(a[i]), pt_bf16_to_f32(b[i]), acc);
  return acc;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void apply_delta_kernel(PtDev c, const T* __restrict__ x, const T* __restrict__ At,
                                                              const T* __restrict__ Bt, T* __restrict__ y, int d_in,
                                                              int d_out, const uint8_t* __restrict__ active,
                                                              const int* __restrict__ ids) {
  __shared__ float u[64], w[64];
  const int j_row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int b = j_row;
  if (ids) {
    b = ids[j_row];
    if ((unsigned)b >= (unsigned)c.B) {
      if (tid == 0) atomicOr(c.err, PTENC_DEVERR_BAD_ID);
      return;
    }
  }
  if (active && !active[b]) return;
  const T* xr = x + (size_t)j_row * d_in;
  for (int g = wave; g < c.G; g += kThreads / 64) {
    float acc = lane_dot<T>(xr, At + (size_t)g * d_in, d_in, lane);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) u[g] = acc;
  }
  __syncthreads();
  if (tid < c.r) {
    const float* S = c.S + (size_t)b * c.G * c.r;
    float acc = 0.f;
    for (int g = 0; g < c.G; ++g) acc = fmaf(u[g], S[g * c.r + tid], acc);
    w[tid] = acc;
  }
  __syncthreads();
  T* yr = y + (size_t)j_row * d_out;
  for (int j = tid; j < d_out; j += kThreads) {
    const T* br = Bt + (size_t)j * c.r;
    float acc = 0.f;
    for (int k = 0; k < c.r; ++k) acc = fmaf(w[k], pt_ld<T>(br + k), acc);
    pt_st<T>(yr + j, pt_ld<T>(yr + j) + acc);
  }
}

}  // namespace

hipError_t pt_launch_apply_delta(const PtDev& c, const void* x, const void* At, const void* Bt, void* y, int d_in,
                                 int d_out, const uint8_t* active, const int* ids, int n_rows, hipStream_t s) {
  const dim3 grid(ids ? n_rows : c.B);
  if (c.dtype == PTENC_F32)
    hipLaunchKernelGGL(apply_delta_kernel<float>, grid, dim3(kThreads), 0, s, c, (const float*)x, (const float*)At,
                       (const float*)Bt, (float*)y, d_in, d_out, active, ids);
  else
    hipLaunchKernelGGL(apply_delta_kernel<uint16_t>, grid, dim3(kThreads), 0, s, c, (const uint16_t*)x,
                       (const uint16_t*)At, (const uint16_t*)Bt, (uint16_t*)y, d_in, d_out, active, ids);
  return hipGetLastError();
}
