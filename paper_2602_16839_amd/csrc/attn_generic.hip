// Plain-ALU windowed decode attention (any dtype / head_dim <= 256 / layout) and the split combine.
//
// out[b,h] = softmax(q[b,h] . K_live * scale) V_live over the live positions of rollout b
// (Notation and Preliminaries, attention equation, over the pruned context).  One workgroup per
// (rollout, query head, window split): a thread scores one token, the block reduces max and sum,
// then one thread per output column accumulates the values.  With several splits the partial
// results (m, l, unnormalised out; base-2 domain) are merged by combine_kernel.
//
// FUSED: the whole decode step of small problems in one launch.  The attention workgroups work out
// for themselves what the step's eviction and append leave (the same counter arithmetic), take the
// new token straight from the step's inputs instead of the cache, and one extra workgroup per rollout
// at the end of the grid runs the prologue (evict-and-encode, append, counters).  Nobody reads what
// that workgroup writes: the evicted slots are outside every attention range, the new token's slot
// is never read from the cache in this launch, and the counters go to the other buffer pair.
#include "pt_prologue.h"

namespace {

constexpr int kThreads = 256;

__device__ inline float block_reduce(float v, float* red, bool is_max) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float u = __shfl_xor(v, o, 64);
    v = is_max ? fmaxf(v, u) : v + u;
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
  for (int i = 1; i < kThreads / 64; ++i) r = is_max ? fmaxf(r, red[i]) : r + red[i];
  return r;
}

struct AttnSmem {
  float qs[256];
  float ps[kThreads];
  int slots[kThreads];
  float red[kThreads / 64];
};

template <bool FUSED> union StepSmem { AttnSmem a; };
template <> union StepSmem<true> { AttnSmem a; EncSmem e; };

template <typename T, bool FUSED>
__global__ __launch_bounds__(kThreads) void attn_generic_kernel(PtDev c, const T* __restrict__ q,
                                                               T* __restrict__ out,
                                                               const uint8_t* __restrict__ active,
                                                               const int* __restrict__ ids, int n_rows,
                                                               const T* __restrict__ knew,
                                                               const T* __restrict__ vnew) {
  // the two roles of a fused launch never meet in one workgroup: one block of LDS serves both
  __shared__ StepSmem<FUSED> smu;
  float* qs = smu.a.qs;
  float* ps = smu.a.ps;
  int* slots = smu.a.slots;
  float* red = smu.a.red;
  if constexpr (FUSED) {
    if ((int)blockIdx.x >= n_rows * c.Hq) {      // the prologue of rollout row blockIdx.x - n_rows * H_q
      if (blockIdx.y == 0)
        pt_step_prologue<T>(smu.e, c, blockIdx.x - n_rows * c.Hq, 1, 1, knew, vnew, active, (T*)nullptr, ids, 0);
      return;
    }
  }
  // bh = (row of q and out, query head); the row's rollout is b = row, or ids[row]
  const int bh = blockIdx.x, j_row = bh / c.Hq, h = bh - j_row * c.Hq, split = blockIdx.y, t = threadIdx.x;
  float* po = c.partial + ((size_t)bh * c.n_splits + split) * (c.d + 2);
  int b = j_row;
  bool bad = false;
  if (ids) { b = ids[j_row]; bad = (unsigned)b >= (unsigned)c.B; if (bad) b = 0; }
  const bool act = !bad && (!active || active[b]);
  long long len = c.len[b], base = c.base[b];
  bool newest = false;          // FUSED: the last live position is this step's token, still only in knew / vnew
  if constexpr (FUSED) {
    if (act) {
      if (len - base == c.Wr) base += c.C;                 // this step's eviction
      if (len - base < c.Wr) { newest = true; len += 1; }  // this step's append
    }
  }
  // logical order: the P question tokens (slots 0 .. P-1), then the live ring positions
  const int P = act ? c.n_prompt[b] : 0;
  const int n_live = act ? P + (int)(len - base) : 0;
  const int per = (n_live + c.n_splits - 1) / c.n_splits;
  const int j0 = split * per, j1 = min(n_live, j0 + per);
  const int s0 = (int)(base % c.Wr);
  const T* slab = (const T*)c.cache + (size_t)(b * c.Hkv + h / c.group) * pt_slab_elems(c.W, c.d);

  for (int i = t; i < c.d; i += kThreads) qs[i] = pt_ld<T>(q + (size_t)bh * c.d + i);
  __syncthreads();

  // values: all threads take part, thread t = (token part, column): part p adds tokens p, p + parts, ...
  const int parts = kThreads / c.d > 0 ? kThreads / c.d : 1;
  const int vcol = t % c.d, vpart = t / c.d;
  const bool vwork = vpart < parts && t < parts * c.d;
  const size_t new_off = FUSED ? ((size_t)j_row * c.Hkv + h / c.group) * c.d : 0;

  float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
  for (int jb = j0; jb < j1; jb += kThreads) {
    const int j = jb + t;
    float s = -INFINITY;
    int slot = 0;
    if (j < j1) {
      slot = j;
      if (j >= P) { slot = s0 + (j - P); if (slot >= c.Wr) slot -= c.Wr; slot += c.n_sink; }
      const bool from_input = FUSED && newest && j == n_live - 1;
      if (from_input) slot = -1;
      float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
      if (from_input || !c.tiled) {
        // a contiguous row: four independent chains, loads free to run ahead
        const T* kr = from_input ? knew + new_off : slab + (size_t)slot * c.d;
        int i = 0;
        for (; i + 4 <= c.d; i += 4) {
          d0 = fmaf(qs[i], pt_ld<T>(kr + i), d0);
          d1 = fmaf(qs[i + 1], pt_ld<T>(kr + i + 1), d1);
          d2 = fmaf(qs[i + 2], pt_ld<T>(kr + i + 2), d2);
          d3 = fmaf(qs[i + 3], pt_ld<T>(kr + i + 3), d3);
        }
        for (; i < c.d; ++i) d0 = fmaf(qs[i], pt_ld<T>(kr + i), d0);
      } else {
        // (the same four chains; d is a multiple of 8 in the tiled layout)
        for (int i = 0; i < c.d; i += 4) {
          d0 = fmaf(qs[i], pt_ld<T>(slab + pt_k_off(1, c.W, c.d, slot, i)), d0);
          d1 = fmaf(qs[i + 1], pt_ld<T>(slab + pt_k_off(1, c.W, c.d, slot, i + 1)), d1);
          d2 = fmaf(qs[i + 2], pt_ld<T>(slab + pt_k_off(1, c.W, c.d, slot, i + 2)), d2);
          d3 = fmaf(qs[i + 3], pt_ld<T>(slab + pt_k_off(1, c.W, c.d, slot, i + 3)), d3);
        }
      }
      s = ((d0 + d1) + (d2 + d3)) * c.scale_log2;
    }
    slots[t] = slot;
    const float mx = block_reduce(s, red, true);
    const float m_new = fmaxf(m_run, mx);
    const float p = j < j1 ? exp2f(s - m_new) : 0.f;
    ps[t] = p;
    const float sm = block_reduce(p, red, false);   // has barriers: ps/slots visible afterwards
    const float alpha = exp2f(m_run - m_new);
    l_run = l_run * alpha + sm;
    if (vwork) {
      acc *= alpha;
      const int n = min(kThreads, j1 - jb);
#pragma unroll 8
      for (int x = vpart; x < n; x += parts) {     // independent loads: eight in flight at a time (measured: -21 % per step at
                                                   // 4 rollouts x 4 heads x 256 tokens; sixteen are no better)
        const int sl = slots[x];
        const float vv = (FUSED && sl < 0) ? pt_ld<T>(vnew + new_off + vcol)
                                           : pt_ld<T>(slab + pt_v_off(c.tiled, c.W, c.d, sl, vcol));
        acc = fmaf(ps[x], vv, acc);
      }
    }
    m_run = m_new;
    __syncthreads();
  }
  // the token parts of a column, added in part order by the column's first thread
  ps[t] = vwork ? acc : 0.f;
  __syncthreads();
  if (t < c.d) {
    acc = 0.f;
    for (int pp = 0; pp < parts; ++pp) acc += ps[pp * c.d + t];
  }
  if (c.n_splits == 1) {
    // nothing to merge: normalise and write the output row here
    if (t < c.d) pt_st<T>(out + (size_t)bh * c.d + t, l_run > 0.f ? acc / l_run : 0.f);
    if (t == 0 && act && n_live == 0) atomicOr(c.err, PTENC_DEVERR_ATTEND_EMPTY);
    if (t == 0 && bad) atomicOr(c.err, PTENC_DEVERR_BAD_ID);
    return;
  }
  if (t == 0) { po[0] = m_run; po[1] = l_run; }
  if (t < c.d) po[2 + t] = acc;
}

// Merge the window splits of one (rollout, query head) and write the output row.
template <typename T>
__global__ void combine_kernel(PtDev c, T* __restrict__ out, const uint8_t* __restrict__ active,
                               const int* __restrict__ ids) {
  const int bh = blockIdx.x;
  int b = bh / c.Hq;
  bool bad = false;
  if (ids) { b = ids[b]; bad = (unsigned)b >= (unsigned)c.B; if (bad) b = 0; }
  const float* pp = c.partial + (size_t)bh * c.n_splits * (c.d + 2);
  const bool act = !bad && (!active || active[b]);
  float M = -INFINITY;
  if (act)
    for (int s = 0; s < c.n_splits; ++s) M = fmaxf(M, pp[(size_t)s * (c.d + 2)]);
  if (M == -INFINITY) {
    for (int i = threadIdx.x; i < c.d; i += blockDim.x) pt_st<T>(out + (size_t)bh * c.d + i, 0.f);
    if (act && threadIdx.x == 0) atomicOr(c.err, PTENC_DEVERR_ATTEND_EMPTY);
    if (bad && threadIdx.x == 0) atomicOr(c.err, PTENC_DEVERR_BAD_ID);
    return;
  }
  float L = 0.f;
  for (int s = 0; s < c.n_splits; ++s) {
    const float* p = pp + (size_t)s * (c.d + 2);
    L += exp2f(p[0] - M) * p[1];
  }
  for (int i = threadIdx.x; i < c.d; i += blockDim.x) {
    float o = 0.f;
    for (int s = 0; s < c.n_splits; ++s) {
      const float* p = pp + (size_t)s * (c.d + 2);
      const float f = exp2f(p[0] - M);
      if (f != 0.f) o = fmaf(f, p[2 + i], o);
    }
    pt_st<T>(out + (size_t)bh * c.d + i, o / L);
  }
}

}  // namespace

hipError_t pt_launch_attn_generic(const PtDev& c, const void* q, void* out, const uint8_t* active,
                                  const int* ids, int n_rows, hipStream_t s) {
  const int nr = ids ? n_rows : c.B, rows = nr * c.Hq;
  dim3 grid(rows, c.n_splits);
  const int cthreads = c.d <= 64 ? 64 : 128;
  if (c.dtype == PTENC_F32) {
    hipLaunchKernelGGL((attn_generic_kernel<float, false>), grid, dim3(kThreads), 0, s, c, (const float*)q, (float*)out, active,
                       ids, nr, (const float*)nullptr, (const float*)nullptr);
    if (c.n_splits > 1)
      hipLaunchKernelGGL(combine_kernel<float>, dim3(rows), dim3(cthreads), 0, s, c, (float*)out, active, ids);
  } else {
    hipLaunchKernelGGL((attn_generic_kernel<uint16_t, false>), grid, dim3(kThreads), 0, s, c, (const uint16_t*)q,
                       (uint16_t*)out, active, ids, nr, (const uint16_t*)nullptr, (const uint16_t*)nullptr);
    if (c.n_splits > 1)
      hipLaunchKernelGGL(combine_kernel<uint16_t>, dim3(rows), dim3(cthreads), 0, s, c, (uint16_t*)out, active, ids);
  }
  return hipGetLastError();
}

// The whole plain-ALU decode step (evict-and-encode, append, attention) in one launch; counters go to
// the other buffer pair (the caller rotates).  Full batch only.  With several splits the combine
// follows as a second launch (pt_launch_combine).
hipError_t pt_launch_step_generic(const PtDev& c, const void* q, const void* k, const void* v, void* out,
                                  const uint8_t* active, hipStream_t s) {
  const int rows = c.B * c.Hq;
  dim3 grid(rows + c.B, c.n_splits);
  if (c.dtype == PTENC_F32)
    hipLaunchKernelGGL((attn_generic_kernel<float, true>), grid, dim3(kThreads), 0, s, c, (const float*)q, (float*)out, active,
                       (const int*)nullptr, c.B, (const float*)k, (const float*)v);
  else
    hipLaunchKernelGGL((attn_generic_kernel<uint16_t, true>), grid, dim3(kThreads), 0, s, c, (const uint16_t*)q,
                       (uint16_t*)out, active, (const int*)nullptr, c.B, (const uint16_t*)k, (const uint16_t*)v);
  return hipGetLastError();
}

hipError_t pt_launch_combine(const PtDev& c, void* out, const uint8_t* active, hipStream_t s) {
  const int rows = c.B * c.Hq, cthreads = c.d <= 64 ? 64 : 128;
  if (c.dtype == PTENC_F32) hipLaunchKernelGGL(combine_kernel<float>, dim3(rows), dim3(cthreads), 0, s, c, (float*)out, active, (const int*)nullptr);
  else hipLaunchKernelGGL(combine_kernel<uint16_t>, dim3(rows), dim3(cthreads), 0, s, c, (uint16_t*)out, active, (const int*)nullptr);
  return hipGetLastError();
}
