// Calibration kernels: a plain streaming read and a plain copy of known size.  They give the
// achievable HBM ceiling next to the attention kernel and the scale factor of the profiler's
// FETCH_SIZE / WRITE_SIZE counters.
#include "ptenc_internal.h"

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// Every wavefront reads whole 16 KiB units (16 loads of 16 bytes per lane), units dealt round-robin
// to the wavefronts of the grid: the same access shape as the attention kernel's group walk.
template <bool NT>
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, size_t n_units,
                                                          uint32_t* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const size_t n_waves = (size_t)gridDim.x * 4;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (size_t u = wave; u < n_units; u += n_waves) {
    const u32x4* p = src + u * 1024 + lane;
    u32x4 r[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) r[i] = NT ? __builtin_nontemporal_load(p + i * 64) : p[i * 64];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc ^= r[i];
  }
  const uint32_t x = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if (x == 0x9e3779b9u) sink[0] = x;   // practically never: keeps the loads alive
}

__global__ __launch_bounds__(256) void copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                   size_t n_vec) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) dst[i] = src[i];
}

}  // namespace

extern "C" {

ptenc_status ptenc_util_stream_read(const void* d_src, size_t bytes, void* d_sink, int32_t n_blocks, void* stream) {
  if (!d_src || !d_sink || n_blocks < 1 || bytes < 16384 || ((uintptr_t)d_src & 15)) return PTENC_ERR_INVALID_ARG;
  hipLaunchKernelGGL(stream_read_kernel<false>, dim3(n_blocks), dim3(256), 0, (hipStream_t)stream, (const u32x4*)d_src,
                     bytes / 16384, (uint32_t*)d_sink);
  return hipGetLastError() == hipSuccess ? PTENC_OK : PTENC_ERR_HIP;
}

ptenc_status ptenc_util_stream_read_nt(const void* d_src, size_t bytes, void* d_sink, int32_t n_blocks, void* stream) {
  if (!d_src || !d_sink || n_blocks < 1 || bytes < 16384 || ((uintptr_t)d_src & 15)) return PTENC_ERR_INVALID_ARG;
  hipLaunchKernelGGL(stream_read_kernel<true>, dim3(n_blocks), dim3(256), 0, (hipStream_t)stream, (const u32x4*)d_src,
                     bytes / 16384, (uint32_t*)d_sink);
  return hipGetLastError() == hipSuccess ? PTENC_OK : PTENC_ERR_HIP;
}

ptenc_status ptenc_util_copy(void* d_dst, const void* d_src, size_t bytes, int32_t n_blocks, void* stream) {
  if (!d_dst || !d_src || n_blocks < 1 || bytes < 16 || (((uintptr_t)d_src | (uintptr_t)d_dst) & 15))
    return PTENC_ERR_INVALID_ARG;
  hipLaunchKernelGGL(copy_kernel, dim3(n_blocks), dim3(256), 0, (hipStream_t)stream, (u32x4*)d_dst,
                     (const u32x4*)d_src, bytes / 16);
  return hipGetLastError() == hipSuccess ? PTENC_OK : PTENC_ERR_HIP;
}

}  // extern "C"
