// The context state applied as a per-rollout low-rank weight delta:  y[b] += ((x[b] A) S_b) B
// (Our Approach: Delta-W = A S B and theta' = theta + Delta-W; row convention, A is d_in x G and
// B is r x d_out).  A and B arrive transposed (A^T [G, d_in], B^T [d_out, r]) so that both long
// loops read contiguous memory.  One workgroup per rollout, fp32 accumulation:
//   u = x A      every thread a slice of d_in for 32 columns at once, slices summed through LDS
//   w = u S_b    G x r, one thread per column
//   y += w B     one thread per output column, r terms each
// 60 MFLOP and under 4 MB at the 7B shape: the launch, not the arithmetic, is what it costs; in a
// full model this belongs in the epilogue of the projection it adapts.
#include "ptenc_internal.h"

namespace {

constexpr int kThreads = 512;
constexpr int kGBlock = 32;      // columns of A handled per pass over x
constexpr int kCols = 4;         // output columns per thread and batch

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
union Vec8 { u32x4 u; uint16_t s[8]; };

// Every phase of this kernel is one or two round trips to memory and little else, so the loads of a
// phase are issued together, and those that depend on nothing (the rollout's S, the first batch
// of B^T and y) before the first phase starts.
template <typename T>
__global__ __launch_bounds__(kThreads) void apply_delta_kernel(PtDev c, const T* __restrict__ x, const T* __restrict__ At,
                                                              const T* __restrict__ Bt, T* __restrict__ y, int d_in,
                                                              int d_out, const uint8_t* __restrict__ active,
                                                              const int* __restrict__ ids) {
  __shared__ float part[kThreads / 2][kGBlock + 1];   // per-thread partial sums, summed column-wise through LDS
  __shared__ float red[kThreads / 2 / kGBlock][kGBlock];
  __shared__ float u[64], w[64];
  constexpr bool kBf16 = sizeof(T) == 2;
  const int j_row = blockIdx.x, tid = threadIdx.x;
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
  T* yr = y + (size_t)j_row * d_out;
  const bool vec_a = kBf16 && ((((uintptr_t)xr | (uintptr_t)At) & 15) == 0) && (d_in & 7) == 0;
  const bool fast_b = kBf16 && c.r == 32 && (((uintptr_t)Bt) & 15) == 0;
  // All workgroups read the same A and B: each starts at its own offset, or they would all queue on
  // the same cache lines at the same moment.
  const int jblk = d_out >= kThreads ? d_out / kThreads : 1, jrot = (int)(blockIdx.x % jblk) * kThreads;

  // ---- early loads: this rollout's column of S, and the first batch of B^T and y ----
  const float* S = c.S + (size_t)b * c.G * c.r;
  float s_col[32];                       // rows 0..31 of the thread's column; further rows are read later
  if (tid < c.r) {
#pragma unroll
    for (int g = 0; g < 32; ++g) s_col[g] = g < c.G ? S[g * c.r + tid] : 0.f;
  }
  Vec8 bv[kCols][4];
  float yv[kCols];
  int jj[kCols];
  auto load_batch = [&](int j0) {
#pragma unroll
    for (int q = 0; q < kCols; ++q) {
      int j = j0 + q * kThreads;
      const bool ok = j < d_out;
      j += jrot;
      if (j >= d_out) j -= d_out;
      jj[q] = ok ? j : -1;
      const int jl = ok ? j : 0;
#pragma unroll
      for (int kv = 0; kv < 4; ++kv) bv[q][kv].u = ((const u32x4*)(Bt + (size_t)jl * 32))[kv];
      yv[q] = pt_ld<T>(yr + jl);
    }
  };
  if (fast_b) load_batch(tid);

  // ---- u = x A: every thread takes a slice of d_in for 32 columns at once, then the slices are added
  //      up column by column through LDS ----
  for (int g0 = 0; g0 < c.G; g0 += kGBlock) {
    float acc[kGBlock];
#pragma unroll
    for (int gi = 0; gi < kGBlock; ++gi) acc[gi] = 0.f;
    if (vec_a) {
      const int nv = d_in >> 3, nblk = nv >= 64 ? nv / 64 : 1, rot = (int)(blockIdx.x % nblk) * 64;
      for (int v0 = tid; v0 < nv; v0 += kThreads) {
        int v = v0 + rot;
        if (v >= nv) v -= nv;
        Vec8 xv, av[kGBlock];
        xv.u = ((const u32x4*)xr)[v];
#pragma unroll
        for (int gi = 0; gi < kGBlock; ++gi) {
          const int g = g0 + gi < c.G ? g0 + gi : c.G - 1;          // clamp: a valid row, result unused
          av[gi].u = ((const u32x4*)(At + (size_t)g * d_in))[v];
        }
        float xf[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) xf[e] = pt_bf16_to_f32(xv.s[e]);
#pragma unroll
        for (int gi = 0; gi < kGBlock; ++gi) {
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[gi] = fmaf(xf[e], pt_bf16_to_f32(av[gi].s[e]), acc[gi]);
        }
      }
    } else {
      for (int i = tid; i < d_in; i += kThreads) {
        const float xf = pt_ld<T>(xr + i);
#pragma unroll
        for (int gi = 0; gi < kGBlock; ++gi)
          if (g0 + gi < c.G) acc[gi] = fmaf(xf, pt_ld<T>(At + (size_t)(g0 + gi) * d_in + i), acc[gi]);
      }
    }
    // upper half of the workgroup hands its sums to the lower half, which then sums 256 rows by column
    constexpr int kHalf = kThreads / 2;
    if (tid >= kHalf) {
#pragma unroll
      for (int gi = 0; gi < kGBlock; ++gi) part[tid - kHalf][gi] = acc[gi];
    }
    __syncthreads();
    if (tid < kHalf) {
#pragma unroll
      for (int gi = 0; gi < kGBlock; ++gi) acc[gi] += part[tid][gi];
    }
    __syncthreads();
    if (tid < kHalf) {
#pragma unroll
      for (int gi = 0; gi < kGBlock; ++gi) part[tid][gi] = acc[gi];
    }
    __syncthreads();
    if (tid < kHalf) {
      const int gi = tid & (kGBlock - 1), seg = tid / kGBlock;      // 8 segments of 32 rows per column
      float a = 0.f;
#pragma unroll 8
      for (int t2 = 0; t2 < kGBlock; ++t2) a += part[seg * kGBlock + t2][gi];
      red[seg][gi] = a;
    }
    __syncthreads();
    if (tid < kGBlock && g0 + tid < c.G) {
      float a = 0.f;
#pragma unroll
      for (int seg = 0; seg < kHalf / kGBlock; ++seg) a += red[seg][tid];
      u[g0 + tid] = a;
    }
  }
  __syncthreads();

  // ---- w = u S_b ----
  if (tid < c.r) {
    float a = 0.f;
#pragma unroll
    for (int g = 0; g < 32; ++g) a = fmaf(g < c.G ? u[g] : 0.f, s_col[g], a);
    for (int g = 32; g < c.G; ++g) a = fmaf(u[g], S[g * c.r + tid], a);
    w[tid] = a;
  }
  __syncthreads();

  // ---- y += w B ----
  if (fast_b) {
    for (int j0 = tid; j0 < d_out; j0 += kCols * kThreads) {
      if (j0 != tid) load_batch(j0);
#pragma unroll
      for (int q = 0; q < kCols; ++q) {
        float a = 0.f;
#pragma unroll
        for (int kv = 0; kv < 4; ++kv)
#pragma unroll
          for (int e = 0; e < 8; ++e) a = fmaf(w[kv * 8 + e], pt_bf16_to_f32(bv[q][kv].s[e]), a);
        if (jj[q] >= 0) pt_st<T>(yr + jj[q], yv[q] + a);
      }
    }
  } else {
    for (int j0 = tid; j0 < d_out; j0 += kThreads) {
      int j = j0 + jrot;
      if (j >= d_out) j -= d_out;
      const T* br = Bt + (size_t)j * c.r;
      float a = 0.f;
      for (int k = 0; k < c.r; ++k) a = fmaf(w[k], pt_ld<T>(br + k), a);
      pt_st<T>(yr + j, pt_ld<T>(yr + j) + a);
    }
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
