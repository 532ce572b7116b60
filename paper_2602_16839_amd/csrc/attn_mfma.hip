// Windowed GQA decode attention for bf16, head_dim 128, on the MFMA-tiled cache layout.
//
// out[b,h] = softmax(q[b,h] . K_live * scale) V_live (Notation and Preliminaries, attention
// equation, over the pruned context of the cache policy).
//
// Work decomposition: one workgroup of 4 wavefronts per (rollout, KV head, window split).  A
// wavefront walks 32-slot groups of the ring (16 KiB each, contiguous in HBM).  Softmax does
// not care about the order of the keys, so the walk is in physical slot order starting at the
// group that holds the oldest live token; only the first and last group of the live range need
// a mask.  All H_q/H_kv query heads of the KV head ride in the N dimension of the MFMA
// (padded to 16), so every K/V byte is fetched from HBM exactly once per step and shared by
// the whole query group in registers.
//
// Per group and wavefront:
//   S^T[token, query]  = K_tile (16 x 32k) * Q^T (32k x 16), 4 k-chunks, two 16-token tiles
//   online softmax in the base-2 domain; lane (query = lane % 16) owns its query's statistics,
//       the max is exchanged between the 4 lane groups with two xor-shuffles per group
//   O^T[dcol, query]  += V^T_tile (16 dcols x 32 tokens) * P^T (32 tokens x 16 queries), 8 tiles
// The V part of a group is stored token-minor in exactly the order the first MFMA leaves the
// probabilities in each lane, so P goes from accumulator to operand with a bf16 pack only.
#include "ptenc_internal.h"

hipError_t pt_launch_combine(const PtDev& c, void* out, const uint8_t* active, hipStream_t s);

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

union Op {   // one MFMA operand = 16 bytes per lane
  u32x4 u;
  bf16x8 h;
};

struct Frag {   // one 32-token group in registers: 64 VGPRs
  Op k0[4], k1[4], v[8];
};

constexpr int kWaves = 4;
constexpr int kORow = 132;   // padded fp32 row of the cross-wave merge buffer

// NT = non-temporal loads: the stream is read once per step, so it should not displace anything
// in L2 / the memory-side cache; measured on MI355X a plain read-only stream gains ~15 % from it.
template <bool NT>
__device__ inline u32x4 ld16(const u32x4* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}

template <bool NT>
__device__ inline void load_group(Frag& f, const u32x4* __restrict__ grp, int lane) {
#pragma unroll
  for (int c = 0; c < 4; ++c) f.k0[c].u = ld16<NT>(grp + c * 64 + lane);
#pragma unroll
  for (int c = 0; c < 4; ++c) f.k1[c].u = ld16<NT>(grp + 256 + c * 64 + lane);
#pragma unroll
  for (int i = 0; i < 8; ++i) f.v[i].u = ld16<NT>(grp + 512 + i * 64 + lane);
}

struct Acc {
  f32x4 o[8];      // O^T: tile it, reg e -> dcol 16 it + 4 kgrp + e, query = lane % 16
  float m, l;      // running max (base-2 domain) and this lane's share of the running sum
};

__device__ inline void process_group(Frag& f, const Op q[4], Acc& a, int visit, int off0, int n_live,
                                     float scale_log2, int kgrp) {
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.k0[c].h, q[c].h, s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.k1[c].h, q[c].h, s1, 0, 0, 0);
  }
  // logical index of the group's first slot relative to the oldest live token
  const int jg = visit * PT_GROUP_TOKENS - off0;
  const bool interior = jg >= 0 && jg + PT_GROUP_TOKENS <= n_live;   // wave-uniform
  float s[8];
  if (interior) {
#pragma unroll
    for (int e = 0; e < 4; ++e) { s[e] = s0[e] * scale_log2; s[4 + e] = s1[e] * scale_log2; }
  } else {
    // edge group: dead slots may hold anything (stale tokens, never-written memory):
    // their scores become -inf and their value columns are zeroed before the second MFMA
    const int jl = jg + 4 * kgrp;
    uint32_t live = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool l0 = (unsigned)(jl + e) < (unsigned)n_live;
      const bool l1 = (unsigned)(jl + 16 + e) < (unsigned)n_live;
      s[e] = l0 ? s0[e] * scale_log2 : -INFINITY;
      s[4 + e] = l1 ? s1[e] * scale_log2 : -INFINITY;
      live |= (l0 ? 1u : 0u) << e | (l1 ? 1u : 0u) << (4 + e);
    }
    // V operand element e of this lane belongs to token (e/4)*16 + 4*kgrp + e%4: same bit order
    const uint32_t m01 = ((live & 1u) ? 0x0000ffffu : 0u) | ((live & 2u) ? 0xffff0000u : 0u);
    const uint32_t m23 = ((live & 4u) ? 0x0000ffffu : 0u) | ((live & 8u) ? 0xffff0000u : 0u);
    const uint32_t m45 = ((live & 16u) ? 0x0000ffffu : 0u) | ((live & 32u) ? 0xffff0000u : 0u);
    const uint32_t m67 = ((live & 64u) ? 0x0000ffffu : 0u) | ((live & 128u) ? 0xffff0000u : 0u);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      f.v[i].u[0] &= m01; f.v[i].u[1] &= m23; f.v[i].u[2] &= m45; f.v[i].u[3] &= m67;
    }
  }
  float mx = fmaxf(fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])), fmaxf(fmaxf(s[4], s[5]), fmaxf(s[6], s[7])));
  mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float m_new = fmaxf(a.m, mx);
  const float m_use = m_new == -INFINITY ? 0.f : m_new;   // nothing live yet: keep exp2 away from inf - inf
  const float alpha = __builtin_amdgcn_exp2f(a.m - m_use);
  float p[8], psum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) { p[e] = __builtin_amdgcn_exp2f(s[e] - m_use); psum += p[e]; }
  a.l = a.l * alpha + psum;
  a.m = m_new;
  if (__any(alpha != 1.f)) {
#pragma unroll
    for (int i = 0; i < 8; ++i) a.o[i] *= alpha;
  }
  Op pf;
#pragma unroll
  for (int e = 0; e < 8; ++e) pf.h[e] = (__bf16)p[e];
#pragma unroll
  for (int i = 0; i < 8; ++i) a.o[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.v[i].h, pf.h, a.o[i], 0, 0, 0);
}

template <bool NT>
__global__ __launch_bounds__(kWaves * 64, 2) void attn_mfma_kernel(PtDev c, const uint16_t* __restrict__ q,
                                                                   uint16_t* __restrict__ out,
                                                                   const uint8_t* __restrict__ active) {
  __shared__ float sm_o[kWaves][16][kORow];
  __shared__ float sm_m[kWaves][16], sm_l[kWaves][16];

  const int slab = blockIdx.x, split = blockIdx.y;
  const int b = slab / c.Hkv, hkv = slab - b * c.Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 15, kgrp = lane >> 4;
  const int g = c.group;
  const bool act = !active || active[b];

  const long long len = c.len[b], base = c.base[b];
  const int n_live = act ? (int)(len - base) : 0;
  const int s0 = (int)(base % c.W);
  const int g0 = s0 >> 5, off0 = s0 & 31;
  const int NG = c.W >> 5;
  const int n_visits = n_live > 0 ? (off0 + n_live + PT_GROUP_TOKENS - 1) >> 5 : 0;
  const int per = (n_visits + c.n_splits - 1) / c.n_splits;
  const int v0 = split * per, v1 = min(n_visits, v0 + per);

  Acc a;
#pragma unroll
  for (int i = 0; i < 8; ++i) a.o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  a.m = -INFINITY;
  a.l = 0.f;

  if (v0 < v1) {
    Op qf[4];
    if (n < g) {
      const u32x4* qp = (const u32x4*)(q + ((size_t)b * c.Hq + hkv * g + n) * 128);
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) qf[cc].u = qp[cc * 4 + kgrp];
    } else {
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) qf[cc].u = u32x4{0u, 0u, 0u, 0u};
    }
    const u32x4* slab_p = (const u32x4*)((const uint16_t*)c.cache + (size_t)slab * pt_slab_elems(c.W, 128));
    auto grp_ptr = [&](int visit) {
      int pg = g0 + visit;
      if (pg >= NG) pg -= NG;
      if (pg >= NG) pg -= NG;   // a full ring that starts mid-group visits its first group twice
      return slab_p + (size_t)pg * (PT_GROUP_ELEMS / 8);
    };
    int i = v0 + wave;
    Frag fa, fb;
    if (i < v1) load_group<NT>(fa, grp_ptr(i), lane);
    while (i < v1) {
      int nx = i + kWaves;
      if (nx < v1) load_group<NT>(fb, grp_ptr(nx), lane);
      process_group(fa, qf, a, i, off0, n_live, c.scale_log2, kgrp);
      i = nx;
      if (i >= v1) break;
      nx = i + kWaves;
      if (nx < v1) load_group<NT>(fa, grp_ptr(nx), lane);
      process_group(fb, qf, a, i, off0, n_live, c.scale_log2, kgrp);
      i = nx;
    }
  }

  // ---- merge the 4 wavefronts through LDS ----
  a.l += __shfl_xor(a.l, 16, 64);
  a.l += __shfl_xor(a.l, 32, 64);
  if (n < g) {
    if (kgrp == 0) { sm_m[wave][n] = a.m; sm_l[wave][n] = a.l; }
#pragma unroll
    for (int i = 0; i < 8; ++i) *(f32x4*)&sm_o[wave][n][16 * i + 4 * kgrp] = a.o[i];
  }
  __syncthreads();

  const int qn = tid >> 4, part = tid & 15;   // 16 threads per query, 8 columns each
  if (qn >= g) return;
  float M = -INFINITY;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sm_m[w][qn]);
  float L = 0.f, o[8];
#pragma unroll
  for (int x = 0; x < 8; ++x) o[x] = 0.f;
  if (M != -INFINITY) {
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float fw = exp2f(sm_m[w][qn] - M);
      L = fmaf(fw, sm_l[w][qn], L);
#pragma unroll
      for (int x = 0; x < 8; ++x) o[x] = fmaf(fw, sm_o[w][qn][part * 8 + x], o[x]);
    }
  }
  const size_t row = (size_t)b * c.Hq + hkv * g + qn;
  if (c.n_splits == 1) {
    const float inv = L > 0.f ? 1.f / L : 0.f;
    Op r;
#pragma unroll
    for (int x = 0; x < 8; ++x) r.h[x] = (__bf16)(o[x] * inv);
    *(u32x4*)(out + row * 128 + part * 8) = r.u;
    if (act && n_live == 0 && part == 0 && qn == 0 && hkv == 0) atomicOr(c.err, PTENC_DEVERR_ATTEND_EMPTY);
  } else {
    float* po = c.partial + (row * c.n_splits + split) * (128 + 2);
    if (part == 0) { po[0] = M; po[1] = L; }
#pragma unroll
    for (int x = 0; x < 8; ++x) po[2 + part * 8 + x] = o[x];
  }
}

}  // namespace

hipError_t pt_launch_attn_mfma(const PtDev& c, bool nontemporal, const void* q, void* out, const uint8_t* active,
                               hipStream_t s) {
  dim3 grid(c.B * c.Hkv, c.n_splits);
  if (nontemporal)
    hipLaunchKernelGGL(attn_mfma_kernel<true>, grid, dim3(kWaves * 64), 0, s, c, (const uint16_t*)q, (uint16_t*)out, active);
  else
    hipLaunchKernelGGL(attn_mfma_kernel<false>, grid, dim3(kWaves * 64), 0, s, c, (const uint16_t*)q, (uint16_t*)out, active);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || c.n_splits == 1) return e;
  return pt_launch_combine(c, out, active, s);
}
