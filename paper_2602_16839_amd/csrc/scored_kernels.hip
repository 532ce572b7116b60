// Importance-based eviction: the stand-alone selection launch, and access to the scores.
//
// A decode step under the scored policy chooses the next victims itself, at its end, when its append
// fills the ring (decode_mfma.hip).  This launch covers what that misses: rings filled by a bare
// ptenc_cache_append, and selections invalidated by ptenc_set_scores.  It skips rollouts whose
// selection is still valid.
#include "pt_scored_select.h"

namespace {

__global__ __launch_bounds__(kSelThreads) void scored_select_kernel(PtDev c, const uint8_t* __restrict__ active,
                                                                   const int* __restrict__ ids) {
  __shared__ float work[PT_SCORED_MAX_ELIGIBLE + 2];
  __shared__ SelSmall sm;
  int b = blockIdx.x;
  if (ids) {
    b = ids[blockIdx.x];
    if ((unsigned)b >= (unsigned)c.B) {
      if (threadIdx.x == 0) atomicOr(c.err, PTENC_DEVERR_BAD_ID);
      return;
    }
  }
  if (active && !active[b]) return;
  const long long len = c.len[b], base = c.base[b];
  if (len - base != c.Wr || c.selected[b]) return;      // not full, or already chosen: nothing to do
  pt_scored_select<kSelThreads>(c, b, base, work, sm);
}

// Scores and position tags of the live ring entries in ring order (oldest ring entry first);
// entries past the live count read 0 and -1.
__global__ void scores_get_kernel(PtDev c, float* __restrict__ score, long long* __restrict__ pos) {
  const int b = blockIdx.x;
  const long long len = c.len[b], base = c.base[b];
  const int n_live = (int)(len - base), s0 = (int)(base % c.Wr);
  for (int i = threadIdx.x; i < c.W; i += blockDim.x) {
    float s = 0.f;
    long long p = -1;
    if (i < n_live) {
      int slot = s0 + i; if (slot >= c.Wr) slot -= c.Wr;
      slot += c.n_sink;
      for (int h = 0; h < c.Hkv; ++h) s += c.mass[(size_t)(b * c.Hkv + h) * c.W + slot];
      p = c.pos[(size_t)b * c.W + slot];
    }
    if (score) score[(size_t)b * c.W + i] = s;
    if (pos) pos[(size_t)b * c.W + i] = p;
  }
}

// Overwrites the scores of the live ring entries (ring order) and drops what waits to be folded.
__global__ void scores_set_kernel(PtDev c, const float* __restrict__ score) {
  const int b = blockIdx.x;
  const long long len = c.len[b], base = c.base[b];
  const int n_live = (int)(len - base), s0 = (int)(base % c.Wr);
  for (int i = threadIdx.x; i < n_live; i += blockDim.x) {
    int slot = s0 + i; if (slot >= c.Wr) slot -= c.Wr;
    slot += c.n_sink;
    for (int h = 0; h < c.Hkv; ++h)
      c.mass[(size_t)(b * c.Hkv + h) * c.W + slot] = h == 0 ? score[(size_t)b * c.W + i] : 0.f;
  }
  for (int h = threadIdx.x; h < c.Hkv; h += blockDim.x) c.mtag[b * c.Hkv + h] = -1;
  if (threadIdx.x == 0) c.selected[b] = 0;              // a choice made on the old scores no longer holds
}

}  // namespace

hipError_t pt_launch_scored_select(const PtDev& c, const uint8_t* active, const int* ids, int n_rows, hipStream_t s) {
  hipLaunchKernelGGL(scored_select_kernel, dim3(ids ? n_rows : c.B), dim3(kSelThreads), 0, s, c, active, ids);
  return hipGetLastError();
}

hipError_t pt_launch_scores_get(const PtDev& c, float* d_score, long long* d_pos, hipStream_t s) {
  hipLaunchKernelGGL(scores_get_kernel, dim3(c.B), dim3(256), 0, s, c, d_score, d_pos);
  return hipGetLastError();
}

hipError_t pt_launch_scores_set(const PtDev& c, const float* d_score, hipStream_t s) {
  hipLaunchKernelGGL(scores_set_kernel, dim3(c.B), dim3(256), 0, s, c, d_score);
  return hipGetLastError();
}
