// The bf16 / head_dim 128 decode step on the MFMA-tiled cache layout, as ONE kernel:
//   [evict the oldest chunk of a full window and fold it into S]  (Our Approach, Delta-W equation,
//                                                                  update rule)
//   [append the new k, v]                                         (Notation and Preliminaries,
//   [attend over the live window]                                  decode-stage / attention equations)
// Each part can be switched off, so the same kernel also serves the three separate entry points.
//
// Work decomposition: one workgroup of 4 or 8 wavefronts per (rollout, KV head, window split).
//
// Attention.  A wavefront walks 32-slot groups of the slab (16 KiB each, contiguous in HBM).
// Softmax does not care about the order of the keys, so the walk is in physical slot order and the
// groups are dealt to the wavefronts (and window splits) by their index alone: which groups a
// wavefront takes does not depend on the counters, only which of them are live does, so its first
// loads are on their way before the counters have arrived.  Only the groups at the two ends of the
// live range need a mask (one group when the ring's start lies inside it: its slots in front of the
// start are the newest).  All H_q/H_kv query heads of the KV head ride in the N dimension of
// the MFMA (padded to 16), so every K/V byte is fetched from HBM once per step and shared by
// the whole query group in registers.  Per group and wavefront:
//   S^T[token, query]  = K_tile (16 x 32k) * Q^T (32k x 16), 4 k-chunks, two 16-token tiles
//   online softmax in the base-2 domain; lane (query = lane % 16) owns its query's statistics,
//       the max is exchanged between the 4 lane groups with two xor-shuffles per group
//   O^T[dcol, query]  += V^T_tile (16 dcols x 32 tokens) * P^T (32 tokens x 16 queries), 8 tiles
// The V part of a group is stored token-minor in exactly the order the first MFMA leaves the
// probabilities in each lane, so P goes from accumulator to operand with a bf16 pack only.
// Window splits are merged by whichever workgroup of the (rollout, KV head) finishes last
// (a counter, no waiting), in split order, so the result does not depend on the arrival order.
//
// Eviction.  The encoder sums over the concatenated KV heads, so a rollout's chunk is folded into S by
// workgroups that read all heads (encode_groups: K_a = K_e W^a_K and V_a = V_e W^a_V with MFMA, then
// S' = (Q_a K_a^T) V_a; encode_rollout_finish: the update of S in fp32).  A chunk may be shared by c.enc_parts
// workgroups, each with a contiguous range of its 32-token groups; their shares of S' meet in memory and the
// last part to arrive adds them in part order, updates S and, the chunk's oldest slot being free now that
// every part has read its range, stores the new token there.  The rollout's attention never depends on any
// of this: it walks the window without the chunk and takes the new token from the step's inputs.  Who does
// the encoding depends on whether the launch fills the chip (see the launcher): encoding workgroups of their
// own behind the attention workgroups in the grid (encoder_role), which start at once where CUs are free; or
// the row's own workgroups before they walk (encode_part), where every CU is taken.
//
// Counters are double-buffered: a step reads (len, base) from one pair of arrays and writes the
// other, so no workgroup has to wait for the rest of its rollout before the step can end.  A compact
// list does the same for the rollouts it names, and one extra workgroup carries everybody's counters
// over to the other pair.  (With the in-place option, for steps a caller replays from a graph, the
// rollout's last workgroup to arrive writes them where they are, after every other one has read them.)
//
// Importance scores (template argument MASS, the scored eviction policy; the paper's ablation on
// token dropping strategies).  The attention probability every cached token received in the rollout's
// previous step is recomputed here, from that step's saved queries and softmax statistics riding in
// the idle columns 8..15 of the score MFMA, parked in LDS during the walk and added to the per-slot
// accumulators after it; the step whose append fills the ring also chooses the next victims
// (pt_scored_select.h) and leaves them in the ring's oldest chunk, so the eviction above needs no change.
#include "pt_encode_tail.h"
#include "pt_scored_select.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

union Op {   // one MFMA operand = 16 bytes per lane
  u32x4 u;
  bf16x8 h;
  uint16_t s[8];
};

struct Frag {   // one 32-token group in registers: 64 VGPRs
  Op k0[4], k1[4], v[8];
};

constexpr int kORow = 132;   // padded fp32 row of the cross-wave merge buffer

// NT = non-temporal loads: the stream is read once per step, so it should not displace anything
// in L2 / the memory-side cache; on MI355X a plain read-only stream gains ~15 % from it.
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

// Importance scores (the ablation on token dropping strategies; accumulated attention probability is
// the heavy-hitter score).  The probability every token received in the rollout's PREVIOUS step is
// recomputed while this step streams the same keys, at no extra matrix work: with at most 8 query heads
// per KV head, columns 8..15 of the score MFMA are free, and carry the previous step's queries (saved
// by that step, with its softmax maximum and 1 / sum).  Lane (kgrp, n >= 8) then holds, in p[], head
// n - 8's unnormalised probabilities of its 8 tokens; il = 1 / sum (0 in lanes that carry nothing).
// The sum over heads is taken among the eight lanes 8..15 of a row as a reduce-scatter: three
// exchanges (with the lane mirrored within the eight, then two apart, then one apart), each lane keeping
// the half of its values that its side of the exchange is responsible for, so that lane 8 + e ends with
// the total of the e-th of the lane's tokens, tl = (e / 4) * 16 + 4 kgrp + e % 4 (29 vector
// instructions per group instead of 56 for eight full sums; the walk pays for every one of them).
template <int CTRL>
__device__ inline float dpp_add(float keep, float send) {
  return keep + __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(send), CTRL, 0xf, 0xf, true));
}

__device__ inline void lagged_mass_park(const float p[8], float il, float* park_grp, int n, int kgrp) {
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = p[e] * il;       // 0 in the lanes of this step's own heads
  const bool lo4 = (n & 4) == 0, lo2 = (n & 2) == 0, lo1 = (n & 1) == 0;
  float r4[4], r2[2];
#pragma unroll
  for (int k = 0; k < 4; ++k) r4[k] = dpp_add<0x141>(lo4 ? v[k] : v[4 + k], lo4 ? v[4 + k] : v[k]);      // row_half_mirror
#pragma unroll
  for (int k = 0; k < 2; ++k) r2[k] = dpp_add<0x4E>(lo2 ? r4[k] : r4[2 + k], lo2 ? r4[2 + k] : r4[k]);   // quad_perm [2,3,0,1]
  const float mine = dpp_add<0xB1>(lo1 ? r2[0] : r2[1], lo1 ? r2[1] : r2[0]);                             // quad_perm [1,0,3,2]
  if (n >= 8) park_grp[((n - 8) >> 2) * 16 + 4 * kgrp + (n & 3)] = mine;
}

// jg = logical index of the group's first slot within its region (question tokens or ring walk),
// n_live = number of live logical indices of that region.
// MASS: lanes with `lag` set carry a query head of the rollout's PREVIOUS step in their column (see
// the kernel): their running maximum is frozen at that step's final one, so p[] comes out as that
// step's unnormalised probabilities, returned in p[], from which the importance scores are parked (park_grp: 32 floats of LDS, or null).
// wrap: 0, or the ring size for the one group that holds the ring's start (jg < 0 then: the slots in
// front of the start are the ring's newest, their logical indices are jg + i + wrap).
template <bool MASS = false>
__device__ inline void process_group(Frag& f, const Op q[4], Acc& a, int jg, int n_live, int wrap,
                                     float scale_log2, int kgrp, bool lag = false, float il = 0.f,
                                     float* park_grp = nullptr, int n = 0) {
  f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.k0[c].h, q[c].h, s0, 0, 0, 0);
    s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f.k1[c].h, q[c].h, s1, 0, 0, 0);
  }
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
      int j0 = jl + e, j1 = jl + 16 + e;
      j0 += j0 < 0 ? wrap : 0;
      j1 += j1 < 0 ? wrap : 0;
      const bool l0 = (unsigned)j0 < (unsigned)n_live;
      const bool l1 = (unsigned)j1 < (unsigned)n_live;
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
  float m_new = fmaxf(a.m, mx);
  if constexpr (MASS) m_new = lag ? a.m : m_new;
  const float m_use = m_new == -INFINITY ? 0.f : m_new;   // nothing live yet: keep exp2 away from inf - inf
  const float alpha = __builtin_amdgcn_exp2f(a.m - m_use);
  float p[8], psum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) { p[e] = __builtin_amdgcn_exp2f(s[e] - m_use); psum += p[e]; }
  if constexpr (MASS) {
    if (park_grp) lagged_mass_park(p, il, park_grp, n, kgrp);   // wave-uniform
  }
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

// kp[c] = this lane's 16 bytes of the new key (k-chunk c); new value column 16 i + (lane % 16) is the
// low (i even) or high (i odd) half of vp[i / 2]: four registers instead of eight.
__device__ inline void load_newest(Op kp[4], uint32_t vp[4], const uint16_t* __restrict__ knew,
                                   const uint16_t* __restrict__ vnew, size_t src, int n, int kgrp) {
#pragma unroll
  for (int cc = 0; cc < 4; ++cc) kp[cc].u = *(const u32x4*)(knew + src + (cc * 4 + kgrp) * 8);
#pragma unroll
  for (int i = 0; i < 4; ++i)
    vp[i] = (uint32_t)vnew[src + 32 * i + n] | ((uint32_t)vnew[src + 32 * i + 16 + n] << 16);
}

// One wavefront writes the new token into its ring slot: 16 key pieces of 16 bytes, 128 value elements.
__device__ inline void store_newest(uint16_t* __restrict__ dst, int W, int slot, const Op kp[4], const uint32_t vp[4],
                                    int n, int kgrp) {
  if (n == 0) {
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) *(u32x4*)(dst + pt_k_off(1, W, 128, slot, (cc * 4 + kgrp) * 8)) = kp[cc].u;
  }
  if (kgrp == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) dst[pt_v_off(1, W, 128, slot, 16 * i + n)] = (uint16_t)(vp[i >> 1] >> (16 * (i & 1)));
  }
}

// The newest token is stored to the cache and, for this step's attention, written straight into
// the registers of the wavefront that walks the last group: no wait for the store to land.
__device__ inline void patch_newest(Frag& f, const Op kp[4], const uint32_t vp[4], int tl, int n, int kgrp) {
  const int t = tl >> 4, m = tl & 15;
  if (n == m) {
    if (t == 0) {
#pragma unroll
      for (int c = 0; c < 4; ++c) f.k0[c].u = kp[c].u;
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) f.k1[c].u = kp[c].u;
    }
  }
  const int vkg = (tl & 15) >> 2, ve = ((tl >> 4) << 2) | (tl & 3);
  if (kgrp == vkg) {
    const int w = ve >> 1;
    const uint32_t sh = (uint32_t)(ve & 1) * 16u, keep = ~(0xffffu << sh);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const uint32_t val = ((vp[i >> 1] >> (16 * (i & 1))) & 0xffffu) << sh;
#pragma unroll
      for (int ww = 0; ww < 4; ++ww)
        if (ww == w) f.v[i].u[ww] = (f.v[i].u[ww] & keep) | val;
    }
  }
}

// Data handed from one workgroup to another inside this kernel (the window splits' partial results, the
// encoding workgroups' shares of S')
// is written and read with device-scope relaxed atomics: such stores write through and
// such loads bypass the per-CU and per-XCD caches, so the hand-over needs no cache write-back or
// invalidation.  Order is given by: stores, every wavefront waits until its own stores have been
// acknowledged (wait_own_stores), barrier, ticket.  A workgroup-scope fence is NOT that wait: with a
// workgroup's wavefronts on one CU the compiler turns it into a wait for LDS and scalar traffic only,
// and the ticket (another wavefront's atomic, to another memory channel) could overtake the stores.
__device__ inline void wait_own_stores() {
  // loads and stores share the vector-memory counter on this GPU
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}
// (two adjacent floats, 8-byte aligned, as one 64-bit access)
__device__ inline void st_agent2(float* p, float a, float b) {
  const unsigned long long u = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
  __hip_atomic_store((unsigned long long*)p, u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_agent1(float* p, float a) {
  __hip_atomic_store(p, a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float ld_agent1(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void ld_agent2(const float* p, float& a, float& b) {
  const unsigned long long u = __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  a = __uint_as_float((unsigned)u);
  b = __uint_as_float((unsigned)(u >> 32));
}

// A workgroup-uniform value that no workgroup of this launch writes (id lists and the like): read
// through the constant address space, i.e. with a scalar load, which comes back sooner than a vector
// load and costs no vector register.  (Loads only: nothing is ever written that way.)
template <typename T>
__device__ inline T ld_uniform(const T* p) {
  return *(const __attribute__((address_space(4))) T*)(uintptr_t)p;
}

// A workgroup-uniform value that a workgroup of this launch MAY overwrite once every reader has taken
// it (the tag of the saved queries; the counters below, when they are updated in place): a scalar load
// as well, but issued by hand, because memory behind the constant address space is taken never to
// change and a load from it may legally be repeated later.
__device__ inline long long ld_scalar(const long long* p) {
  long long v;
  asm volatile(
      "s_load_dwordx2 %0, %1, 0x0\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(v)
      : "s"(p)
      : "memory");
  return v;
}

// What a step must know before its first K/V load: the rollout's counters, its number of question
// tokens, its mask byte and how much of its next chunk is folded already.  All five are fetched together (scalar loads, one wait), so the step
// pays one round trip to memory for them instead of one per dependent load; the mask byte comes
// as the aligned dword that holds it (an aligned dword shares its page with every byte in it).
// Issued by hand like ld_scalar above: the counters may be rewritten in place later in the launch.
//
// The same wait also covers one dword of every 64-byte line of the kernel's argument block
// (TOUCH): the arguments the compiler fetches later, in several dependent batches, then come from
// the scalar cache instead of costing a round trip each.  The touched values are discarded.
struct StepHead { long long len, base; int n_prompt; uint32_t mask_word; int enc_done; };
typedef const void* KernargPtr;   // generic pointer to the argument block

// offset of the k-th touched dword inside an argument block of ARG_BYTES bytes
#define PT_TOUCH_OFF(k) ((k) * 64 < ARG_BYTES - 4 ? (k) * 64 : ARG_BYTES - 4)
#define PT_TOUCH_OFFSETS \
  "i"(PT_TOUCH_OFF(0)), "i"(PT_TOUCH_OFF(1)), "i"(PT_TOUCH_OFF(2)), "i"(PT_TOUCH_OFF(3)), "i"(PT_TOUCH_OFF(4)), \
  "i"(PT_TOUCH_OFF(5)), "i"(PT_TOUCH_OFF(6)), "i"(PT_TOUCH_OFF(7))

// TOUCH: with the argument-block lines (a launch over all rollouts); else the five values only
template <int ARG_BYTES, bool TOUCH>
__device__ inline StepHead load_step_head(const long long* len_p, const long long* base_p, const int* n_prompt_p,
                                          const uint32_t* mask_word_p, const int* enc_done_p, KernargPtr ka) {
  static_assert(ARG_BYTES >= 4 && ARG_BYTES <= 8 * 64, "argument block larger than the lines touched");
  StepHead h;
  if (TOUCH) {
    int t0, t1, t2, t3, t4, t5, t6, t7;
    asm volatile(
        "s_load_dwordx2 %0, %13, 0x0\n\t"
        "s_load_dwordx2 %1, %14, 0x0\n\t"
        "s_load_dword %2, %15, 0x0\n\t"
        "s_load_dword %3, %16, 0x0\n\t"
        "s_load_dword %4, %17, 0x0\n\t"
        "s_load_dword %5, %18, %19\n\t"
        "s_load_dword %6, %18, %20\n\t"
        "s_load_dword %7, %18, %21\n\t"
        "s_load_dword %8, %18, %22\n\t"
        "s_load_dword %9, %18, %23\n\t"
        "s_load_dword %10, %18, %24\n\t"
        "s_load_dword %11, %18, %25\n\t"
        "s_load_dword %12, %18, %26\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&s"(h.len), "=&s"(h.base), "=&s"(h.n_prompt), "=&s"(h.mask_word), "=&s"(h.enc_done), "=&s"(t0), "=&s"(t1),
          "=&s"(t2), "=&s"(t3), "=&s"(t4), "=&s"(t5), "=&s"(t6), "=&s"(t7)
        : "s"(len_p), "s"(base_p), "s"(n_prompt_p), "s"(mask_word_p), "s"(enc_done_p), "s"(ka), PT_TOUCH_OFFSETS
        : "memory");
  } else {
    asm volatile(
        "s_load_dwordx2 %0, %5, 0x0\n\t"
        "s_load_dwordx2 %1, %6, 0x0\n\t"
        "s_load_dword %2, %7, 0x0\n\t"
        "s_load_dword %3, %8, 0x0\n\t"
        "s_load_dword %4, %9, 0x0\n\t"
        "s_waitcnt lgkmcnt(0)"
        : "=&s"(h.len), "=&s"(h.base), "=&s"(h.n_prompt), "=&s"(h.mask_word), "=&s"(h.enc_done)
        : "s"(len_p), "s"(base_p), "s"(n_prompt_p), "s"(mask_word_p), "s"(enc_done_p)
        : "memory");
  }
  return h;
}

// a compact list's entry for this row, with the argument-block lines (the counters depend on it,
// so they follow in a second round trip)
template <int ARG_BYTES>
__device__ inline int load_row_id(const int* id_p, KernargPtr ka) {
  static_assert(ARG_BYTES >= 4 && ARG_BYTES <= 8 * 64, "argument block larger than the lines touched");
  int id, t0, t1, t2, t3, t4, t5, t6, t7;
  asm volatile(
      "s_load_dword %0, %9, 0x0\n\t"
      "s_load_dword %1, %10, %11\n\t"
      "s_load_dword %2, %10, %12\n\t"
      "s_load_dword %3, %10, %13\n\t"
      "s_load_dword %4, %10, %14\n\t"
      "s_load_dword %5, %10, %15\n\t"
      "s_load_dword %6, %10, %16\n\t"
      "s_load_dword %7, %10, %17\n\t"
      "s_load_dword %8, %10, %18\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&s"(id), "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&s"(t3), "=&s"(t4), "=&s"(t5), "=&s"(t6), "=&s"(t7)
      : "s"(id_p), "s"(ka), PT_TOUCH_OFFSETS
      : "memory");
  return id;
}

struct StepArgs {
  const uint16_t* q;       // [B, H_q, 128]
  uint16_t* out;           // [B, H_q, 128]
  const uint16_t* knew;    // [B, H_kv, 128]
  const uint16_t* vnew;
  const uint8_t* active;   // [B] or null
  uint16_t* dbg_chunk;     // [B, 2, C, H_kv*128] or null
  const int* ids;          // null, or the rollouts this launch works on: row j of q/k/v/out is rollout ids[j]
  int do_evict, do_append, do_attend;
  int in_place;            // counters written in place by the rollout's last workgroup (graph replay)
  int enc_inline;          // who folds an evicted chunk into S: 1 the row's own workgroups before their walk, 0 encoding
                           // workgroups of their own behind the attention workgroups in the grid (see the launcher)
  int carry;               // compact list with two counter buffers: one extra workgroup carries every
                           // rollout's counters over to the buffer this step writes (see the kernel)
};

// WAVES wavefronts per workgroup: 4 (up to 16 query heads per KV head) or 8 (up to 8), the same LDS.
template <int WAVES>
union StepSmem {
  struct {
    float o[WAVES][64 / WAVES][kORow];
    float m[WAVES][64 / WAVES], l[WAVES][64 / WAVES];
  } merge;
  struct {           // an encoding workgroup
    // one group's V part of one KV head, per V wavefront (operand transposition): the 16-byte piece of
    // (value-column tile it, lane group k, row m) sits at 16-byte index (4 it + k) * 18 + m + m / 8, a pitch
    // that spreads the pieces one gather touches over all banks (2-way conflicts instead of 16-way)
    uint16_t vstage[2][32 * 18 * 8];
    struct {                    // K_a and V_a of the group in hand; together (contiguous, >= G*r floats)
      float Ka[kEncSub][kEncMaxGR + 1];   //   they double as the staging area of S'
      float Va[kEncSub][kEncMaxGR + 1];
      float red[16];
    } tail;
  } enc;
  SelSmall sel;      // scored policy: the choice of the next victims, by the rollout's last workgroup
};

// The evicted chunk of one rollout (or this workgroup's part of it: see below), by a workgroup that
// does nothing else in this launch, so that a rollout's eviction is not on the path of its own or
// anybody's attention: K_a = K_e W^a_K and
// V_a = V_e W^a_V over the concatenated KV heads (MFMA, accumulated over the heads in head order),
// S' = (Q_a K_a^T) V_a, S <- Normalize(S + S')  (Our Approach, the Delta-W equation and the update rule).
// The chunk is the ring-relative slots [s0, s0 + C) (wrapping), walked as 32-slot groups; rows of a group
// outside the chunk count as zero.  Wavefronts 0..3 each own one 16-token tile of K_a or of V_a of the
// group in hand; wavefront w < ceil(G / 16) then adds the group to rows 16 w .. 16 w + 15 of S'.
//
// ROLE 0: a K_a tile, 1: a V_a tile, 2: neither (wavefronts 4..7 of an 8-wavefront workgroup only pass
// the barriers).  One instance per role, so that each keeps its own operand buffer in registers; every
// instance passes the same barriers.
//
// The caller names a contiguous range [v_lo, v_hi) of the chunk's groups (0 = the group that holds the chunk's
// oldest token; see pt_chunk_groups); their contribution to S' is left in LDS, row-major G x r.
__device__ inline int pt_chunk_groups(const PtDev& c, int s0) { return ((s0 & 31) + c.C + PT_GROUP_TOKENS - 1) >> 5; }

template <int WAVES, int ROLE>
__device__ inline void encode_groups(const PtDev& c, StepSmem<WAVES>& sm, int b, int s0, int v_lo, int v_hi) {
  constexpr int NP = ROLE == 0 ? 4 : 8;          // 16-byte pieces per lane, KV head and group
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, kgrp = lane >> 4;
  const int g0 = s0 >> 5, off0 = s0 & 31, NG = c.Wr >> 5, gs = c.n_sink >> 5;
  const int t = wave & 1;
  const size_t slab_u = pt_slab_elems(c.W, 128) / 8;                 // a slab in 16-byte units
  const u32x4* cache0 = (const u32x4*)c.cache + (size_t)b * c.Hkv * slab_u;
  const u32x4* Wp = (const u32x4*)(ROLE == 1 ? c.WVp : c.WKp);
  // this lane's token within the group as the A-operand row, and where the V part keeps it
  const int tl = t * 16 + n, vkg = (tl & 15) >> 2, ve = ((tl >> 4) << 2) | (tl & 3);
  // Operands of a batch of HB KV heads of one group, all loads in flight together; the next batch (of
  // this group or the next) is requested as soon as this one has been consumed, so its latency hides
  // behind the arithmetic and the tail.
  constexpr int HB = 2;      // (4 for the K tiles gained nothing and made the code larger)
  const int n_batches = (c.Hkv + HB - 1) / HB;
  u32x4 buf[HB][NP];
  auto load_batch = [&](int vis, int h0) {
    int pg = g0 + vis;
    if (pg >= NG) pg -= NG;
    if (pg >= NG) pg -= NG;
#pragma unroll
    for (int hh = 0; hh < HB; ++hh) {
      const int h = h0 + hh < c.Hkv ? h0 + hh : c.Hkv - 1;        // clamped: loaded, not used
      const u32x4* grp = cache0 + (size_t)h * slab_u + (size_t)(gs + pg) * (PT_GROUP_ELEMS / 8);
#pragma unroll
      for (int i = 0; i < NP; ++i) buf[hh][i] = ROLE == 0 ? grp[t * 256 + i * 64 + lane] : grp[512 + i * 64 + lane];
    }
  };
  if (ROLE != 2 && v_lo < v_hi) load_batch(v_lo, 0);
  // The fp32 tail on the matrix units as well (16x16x4 fp32 MFMA): wavefront w < ceil(G / 16) owns rows
  // 16 w .. 16 w + 15 of S'.  Its slice of Q_a stays in registers: the B operand of k-step s is
  // Q_a[16 w + lane % 16][4 s + lane / 16] (zero outside G x r).
  const bool tail_wave = wave * 16 < c.G;
  const int kq = lane >> 4;
  float qreg[16];
  f32x4 sp[4];                                       // S'[16 w + 4 (lane / 16) + e][16 ct + lane % 16]
#pragma unroll
  for (int x = 0; x < 16; ++x) {
    const int g = wave * 16 + n, a = 4 * x + kq;
    qreg[x] = (tail_wave && g < c.G && a < c.r) ? c.Qa[g * c.r + a] : 0.f;
  }
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) sp[ct] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int vis = v_lo; vis < v_hi; ++vis) {
    if (ROLE != 2) {
      f32x4 acc[4];
#pragma unroll
      for (int rt = 0; rt < 4; ++rt) acc[rt] = f32x4{0.f, 0.f, 0.f, 0.f};
      for (int bi = 0; bi < n_batches; ++bi) {
        const int h0 = bi * HB;
#pragma unroll
        for (int hh = 0; hh < HB; ++hh) {
          const int h = h0 + hh;
          if (h < c.Hkv) {
            // this head's slices of W^a first: their latency runs under the transposition below
            Op w[4][4];
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) {
              if (rt < c.n_rt) {
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) w[cc][rt].u = Wp[(((size_t)h * 4 + cc) * 4 + rt) * 64 + lane];
              }
            }
            Op op[4];
            if (ROLE == 0) {
#pragma unroll
              for (int cc = 0; cc < 4; ++cc) op[cc].u = buf[hh][cc];
            } else {
              // V part -> LDS (the operand needs 8 consecutive columns of one token, which the token-minor
              // layout scatters)
              uint16_t* vs = sm.enc.vstage[t];
#pragma unroll
              for (int i = 0; i < NP; ++i) ((u32x4*)vs)[(i * 4 + kgrp) * 18 + n + (n >> 3)] = buf[hh][i];
              __builtin_amdgcn_wave_barrier();
#pragma unroll
              for (int cc = 0; cc < 4; ++cc) {
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                  const int i = cc * 32 + 8 * kgrp + x, mm = i & 15;        // value column; its row in the tile
                  op[cc].s[x] = vs[(((i >> 4) * 4 + vkg) * 18 + mm + (mm >> 3)) * 8 + ve];
                }
              }
              __builtin_amdgcn_wave_barrier();                 // the next head overwrites the staging area
            }
#pragma unroll
            for (int rt = 0; rt < 4; ++rt) {
              if (rt < c.n_rt) {
#pragma unroll
                for (int cc = 0; cc < 4; ++cc)
                  acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(op[cc].h, w[cc][rt].h, acc[rt], 0, 0, 0);
              }
            }
          }
        }
        if (bi + 1 < n_batches) load_batch(vis, h0 + HB);
        else if (vis + 1 < v_hi) load_batch(vis + 1, 0);
      }
      // D[token 4 kgrp + e of the tile][column 16 rt + n]
      float (*dst)[kEncMaxGR + 1] = ROLE == 1 ? sm.enc.tail.Va : sm.enc.tail.Ka;
#pragma unroll
      for (int rt = 0; rt < 4; ++rt) {
        if (rt < c.n_rt) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int row = 16 * t + 4 * kgrp + e, pl = 32 * vis + row;      // place counted from the first group
            dst[row][rt * 16 + n] = (pl >= off0 && pl < off0 + c.C) ? acc[rt][e] : 0.f;
          }
        }
      }
    }
    __syncthreads();
    if (tail_wave) {
      // P^T = K_a Q_a^T for the two 16-token tiles: pt[t][e] = P[g = 16 w + lane % 16][token 16 t + 4 (lane / 16) + e]
      f32x4 pt[2];
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        pt[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          if (x < 4 * c.n_rt)
            pt[tt] = __builtin_amdgcn_mfma_f32_16x16x4f32(sm.enc.tail.Ka[16 * tt + n][4 * x + kq], qreg[x], pt[tt], 0, 0, 0);
        }
      }
      // S' += P V_a: k-step (t, e) contracts the tokens 16 t + 4 k + e, k = 0..3, which is what lane group
      // k holds of P in pt[t][e]: the result of the first product is the operand of the second as it is
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) {
        if (ct < c.n_rt) {
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              sp[ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(pt[tt][e], sm.enc.tail.Va[16 * tt + 4 * kq + e][16 * ct + n], sp[ct],
                                                            0, 0, 0);
          }
        }
      }
    }
    __syncthreads();
  }
  // S' into LDS, row-major G x r, for the update of S
  float* stage = &sm.enc.tail.Ka[0][0];
  if (tail_wave) {
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int g = wave * 16 + 4 * kq + e, col = 16 * ct + n;
        if (ct < c.n_rt && g < c.G && col < c.r) stage[g * c.r + col] = sp[ct][e];
      }
    }
  }
}

// Groups [v_lo, v_hi) of the chunk: their contribution to S' into LDS.  Ends with a barrier.
template <int WAVES>
__device__ inline void encode_rollout_groups(const PtDev& c, StepSmem<WAVES>& sm, int b, int s0, int v_lo, int v_hi) {
  const int wave = threadIdx.x >> 6;
  if (wave >= 4) encode_groups<WAVES, 2>(c, sm, b, s0, v_lo, v_hi);
  else if (wave & 2) encode_groups<WAVES, 1>(c, sm, b, s0, v_lo, v_hi);
  else encode_groups<WAVES, 0>(c, sm, b, s0, v_lo, v_hi);
  __syncthreads();
}

// Groups of the chunk a rollout will evict NEXT, folded ahead of time: their contribution is added to the
// rollout's pending block (c.pend), which the eviction adds to S' (encode_rollout_finish).  Only one
// workgroup per rollout does this, one group or so every few steps (see the kernel), so the sum is the same
// whatever the launch looks like.  Ends with a barrier.
template <int WAVES>
__device__ inline void encode_ahead(const PtDev& c, StepSmem<WAVES>& sm, int b, int s0, int v_lo, int v_hi) {
  constexpr int THREADS = WAVES * 64;
  encode_rollout_groups<WAVES>(c, sm, b, s0, v_lo, v_hi);
  const float* stage = &sm.enc.tail.Ka[0][0];
  const int gr = c.G * c.r;
  float* pend = c.pend + (size_t)b * gr;
  for (int idx = threadIdx.x; idx < gr; idx += THREADS) pend[idx] += stage[idx];
  if (threadIdx.x == 0) c.enc_done[b] = v_hi;
  __syncthreads();
}

// The parts' shares meet, S is updated: S <- Normalize(S + (shares in part order + what was folded ahead of
// time)).  Returns whether this workgroup is the one that updated S (with
// one part per chunk: always; otherwise the last part to arrive, which adds the parts' shares in part
// order, so that the sum does not depend on who arrived when).
// `on_the_way` is called once this workgroup's stores have been acknowledged, before the ticket is drawn: what
// the caller requests there travels while the ticket does.
template <int WAVES, typename F>
__device__ inline bool encode_rollout_finish(const PtDev& c, StepSmem<WAVES>& sm, int& sm_ticket, int b, int part,
                                             int n_parts, F on_the_way) {
  constexpr int THREADS = WAVES * 64, NX = 4096 / THREADS;
  float* stage = &sm.enc.tail.Ka[0][0];
  const int gr = c.G * c.r;
  float* pend = c.pend + (size_t)b * gr;
  float sacc[16];
  if (n_parts == 1) {
#pragma unroll
    for (int x = 0; x < NX; ++x) {
      const int idx = threadIdx.x + THREADS * x;
      sacc[x] = idx < gr ? stage[idx] + pend[idx] : 0.f;
      if (idx < gr) pend[idx] = 0.f;
    }
    if (threadIdx.x == 0) c.enc_done[b] = 0;
    on_the_way();
    __syncthreads();
    pt_state_update<THREADS>(c, b, sacc, stage, sm.enc.tail.red);
    return true;
  }
  // park this part's share (device-scope stores, as for the window splits); the last part to arrive
  // adds all of them.  Nobody else touches S[b] or the pending block in this launch, so their old values are
  // fetched now, while the stores and the ticket are on their way, whoever turns out to need them.
  float* mine = c.enc_part + ((size_t)b * c.enc_parts + part) * gr;
  for (int idx = threadIdx.x; idx < gr; idx += THREADS) st_agent1(mine + idx, stage[idx]);
  float sprev[NX], spend[NX];
#pragma unroll
  for (int x = 0; x < NX; ++x) {
    const int idx = threadIdx.x + THREADS * x;
    sprev[x] = idx < gr ? c.S[(size_t)b * gr + idx] : 0.f;
    spend[x] = idx < gr ? pend[idx] : 0.f;
  }
  wait_own_stores();
  on_the_way();
  __syncthreads();
  if (threadIdx.x == 0) sm_ticket = atomicAdd(c.tick_enc + b, 1);
  __syncthreads();
  if (sm_ticket != n_parts - 1) return false;
  if (threadIdx.x == 0) { c.tick_enc[b] = 0; c.enc_done[b] = 0; }
  const float* all = c.enc_part + (size_t)b * c.enc_parts * gr;
#pragma unroll
  for (int x = 0; x < NX; ++x) {
    const int idx = threadIdx.x + THREADS * x;
    // every part's value requested before the first is added (in part order)
    float t[PT_MAX_ENC_PARTS];
#pragma unroll
    for (int p = 0; p < PT_MAX_ENC_PARTS; ++p)
      t[p] = (idx < gr && p < n_parts) ? ld_agent1(all + (size_t)p * gr + idx) : 0.f;
    float v = 0.f;
#pragma unroll
    for (int p = 0; p < PT_MAX_ENC_PARTS; ++p) v += t[p];
    sacc[x] = (v + spend[x]) + sprev[x];
    if (idx < gr) pend[idx] = 0.f;
  }
  __syncthreads();
  pt_state_update<THREADS, false>(c, b, sacc, stage, sm.enc.tail.red);
  return true;
}

// What a step does to one rollout, from the counters it finds.  Both kinds of workgroup of a rollout
// (the attention ones and the encoding one) derive it from the same values, so they agree on who
// takes part in the arrival count below.
struct StepPlan {
  bool evicting, append_full, appending, will_select, need_ticket;
  long long base1, len1;      // the counters as the step leaves them
};
template <bool MASS>
__device__ inline StepPlan plan_step(const PtDev& c, const StepArgs& a, bool act, long long len0, long long base0) {
  StepPlan p;
  p.evicting = act && a.do_evict && (len0 - base0 == c.Wr);
  p.base1 = base0 + (p.evicting ? c.C : 0);
  p.append_full = act && a.do_append && (len0 - p.base1 >= c.Wr);
  p.appending = act && a.do_append && !p.append_full;
  p.len1 = len0 + (p.appending ? 1 : 0);
  // scored policy: the step whose append fills the ring chooses the next victims at its end
  p.will_select = MASS && p.appending && (p.len1 - p.base1 == c.Wr);
  // something must happen after every workgroup of the rollout is through: counters written in place,
  // or the choice of victims
  p.need_ticket = (a.in_place != 0 && (p.appending || p.evicting)) || p.will_select;
  return p;
}

// Arrival of one workgroup of rollout b (of `expected` in all); the last one to arrive chooses the next
// victims (scored policy, ring just filled) and writes the counters where they are (in-place mode).
template <int WAVES, bool MASS>
__device__ inline void arrive_rollout(const PtDev& c, const StepArgs& a, StepSmem<WAVES>& sm, int& sm_ticket,
                                      float* dyn_lds, int b, const StepPlan& pl, int expected) {
  if (!pl.need_ticket) return;
  // rare (once per C steps): the other workgroups' new token and score updates must be visible to the
  // one that selects, whichever XCD each ran on: device-wide release here, acquire there
  if (pl.will_select) __threadfence();
  wait_own_stores();
  __syncthreads();
  if (threadIdx.x == 0) sm_ticket = atomicAdd(c.tick_rollout + b, 1);
  __syncthreads();
  if (sm_ticket != expected - 1) return;
  if constexpr (MASS) {
    if (pl.will_select) {
      __threadfence();
      pt_scored_select<WAVES * 64>(c, b, pl.base1, dyn_lds, sm.sel);
    }
  }
  if (threadIdx.x == 0) {
    if (a.in_place) { c.len[b] = pl.len1; c.base[b] = pl.base1; }
    c.tick_rollout[b] = 0;
  }
}

// A rollout whose ring is full has its oldest chunk folded into S by its own workgroups BEFORE they walk the
// window: workgroup number `part` (< c.enc_parts) of the row takes that part of the chunk's groups.  The walk
// skips the chunk and takes the new token from the step's inputs, so it depends on nothing done here; a
// workgroup that starts its walk a few microseconds late shares the memory system with the others all the
// same and ends with them (while encoding workgroups of their own, queued behind the attention workgroups
// in the grid, got a CU only when the first attention workgroups left, and ran their chain of dependent
// memory accesses against a saturated memory system: the tail of every step of a running batch).  The last
// part to finish updates S and, the chunk's oldest slot being free at last, stores the step's new token
// there.  Ends with the workgroup's LDS free for the walk.
template <int WAVES, bool MASS, typename F>
__device__ inline void encode_part(const PtDev& c, const StepArgs& a, StepSmem<WAVES>& sm, int& sm_ticket, int b,
                                   int j_row, int s0e, int part, int n_parts, int v_lo, int v_hi, const StepPlan& pl,
                                   long long len0, F on_the_way) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 15, kgrp = lane >> 4;
  encode_rollout_groups<WAVES>(c, sm, b, s0e, v_lo, v_hi);
  if (encode_rollout_finish<WAVES>(c, sm, sm_ticket, b, part, n_parts, on_the_way)) {
    if (a.dbg_chunk) {
      const int dkv = c.Hkv * 128;
      uint16_t* dK = a.dbg_chunk + (size_t)b * 2 * c.C * dkv;
      uint16_t* dV = dK + (size_t)c.C * dkv;
      for (int idx = tid; idx < c.C * dkv; idx += WAVES * 64) {
        const int j = idx / dkv, hi = idx - j * dkv, h = hi >> 7, i = hi & 127;
        const uint16_t* src = (const uint16_t*)c.cache + (size_t)(b * c.Hkv + h) * pt_slab_elems(c.W, 128);
        int slot = s0e + j; if (slot >= c.Wr) slot -= c.Wr;
        slot += c.n_sink;
        dK[idx] = src[pt_k_off(1, c.W, 128, slot, i)];
        dV[idx] = src[pt_v_off(1, c.W, 128, slot, i)];
      }
    }
    __syncthreads();   // every read of the chunk is done: its oldest slot may take the new token
    if (pl.appending) {
      int s0 = s0e + c.C;
      if (s0 >= c.Wr) s0 -= c.Wr;
      int s_new = s0 + (int)(len0 - pl.base1);
      if (s_new >= c.Wr) s_new -= c.Wr;
      for (int h = wave; h < c.Hkv; h += WAVES) {
        Op kp[4];
        uint32_t vp[4];
        load_newest(kp, vp, a.knew, a.vnew, ((size_t)j_row * c.Hkv + h) * 128, n, kgrp);
        store_newest((uint16_t*)c.cache + (size_t)(b * c.Hkv + h) * pt_slab_elems(c.W, 128), c.W, c.n_sink + s_new, kp, vp,
                     n, kgrp);
      }
    }
    if (tid == 0 && !pl.will_select) c.selected[b] = 0;   // the chosen chunk has left
  }
  __syncthreads();     // the encoder's LDS is the walk's merge buffer
}

// An encoding workgroup of its own (launches that leave CUs free, see the kernel: c.enc_parts per row, after the
// attention workgroups in the grid): if the rollout's ring is full, the row's encoding workgroups fold the oldest
// chunk into S and then, the chunk's oldest slot being free at last, the one that finished the job
// stores the step's new token there.  The rollout's attention workgroups meanwhile walk the window
// without the chunk and take the new token from the step's inputs; nobody waits for anybody.
template <int WAVES, bool MASS>
__device__ inline void encoder_role(const PtDev& c, const StepArgs& a, StepSmem<WAVES>& sm, int& sm_ticket,
                                    float* dyn_lds, int enc_idx, const int* ids, const uint8_t* active,
                                    const long long* len_cur, const long long* base_cur) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 15, kgrp = lane >> 4;
  // a long chunk has several encoding workgroups per row: part 0 stands for the row where nothing is
  // evicted; of an evicting row's parts, the last one to finish its share does everything after it
  const int j_row = enc_idx / c.enc_parts, part = enc_idx - j_row * c.enc_parts;
  int b = j_row;
  if (ids) {
    b = ld_uniform(ids + j_row);
    if ((unsigned)b >= (unsigned)c.B) return;            // flagged by the row's attention workgroups
  }
  // counters and mask in one round trip (where nothing is full this workgroup should be gone at once)
  const uintptr_t mask_addr = (uintptr_t)(active + b);
  const uint32_t* mask_word_p = active ? (const uint32_t*)(mask_addr & ~(uintptr_t)3) : (const uint32_t*)(c.n_prompt + b);
  const StepHead head = load_step_head<8, false>(len_cur + b, base_cur + b, c.n_prompt + b, mask_word_p, c.enc_done + b, nullptr);
  const bool act = !active || ((head.mask_word >> (8 * (int)(mask_addr & 3))) & 0xffu) != 0;
  const long long len0 = head.len, base0 = head.base;
  if (len0 < base0) return;
  const StepPlan pl = plan_step<MASS>(c, a, act, len0, base0);
  if (!pl.evicting && part != 0) return;
  if (pl.evicting) {
    const int s0e = (int)(base0 % c.Wr);
    // what has not been folded ahead of time (every part reads the same count: the one that resets it is
    // the last to draw its ticket)
    const int n_vis = pt_chunk_groups(c, s0e), done = MASS ? 0 : min(max(head.enc_done, 0), n_vis), rest = n_vis - done;
    encode_rollout_groups<WAVES>(c, sm, b, s0e, done + part * rest / c.enc_parts, done + (part + 1) * rest / c.enc_parts);
    if (!encode_rollout_finish<WAVES>(c, sm, sm_ticket, b, part, c.enc_parts, []() {})) return;
    if (a.dbg_chunk) {
      const int dkv = c.Hkv * 128;
      uint16_t* dK = a.dbg_chunk + (size_t)b * 2 * c.C * dkv;
      uint16_t* dV = dK + (size_t)c.C * dkv;
      for (int idx = tid; idx < c.C * dkv; idx += WAVES * 64) {
        const int j = idx / dkv, hi = idx - j * dkv, h = hi >> 7, i = hi & 127;
        const uint16_t* src = (const uint16_t*)c.cache + (size_t)(b * c.Hkv + h) * pt_slab_elems(c.W, 128);
        int slot = s0e + j; if (slot >= c.Wr) slot -= c.Wr;
        slot += c.n_sink;
        dK[idx] = src[pt_k_off(1, c.W, 128, slot, i)];
        dV[idx] = src[pt_v_off(1, c.W, 128, slot, i)];
      }
    }
    __syncthreads();   // every read of the chunk is done: its oldest slot may take the new token
    if (pl.appending) {
      int s0 = s0e + c.C;
      if (s0 >= c.Wr) s0 -= c.Wr;
      int s_new = s0 + (int)(len0 - pl.base1);
      if (s_new >= c.Wr) s_new -= c.Wr;
      for (int h = wave; h < c.Hkv; h += WAVES) {
        Op kp[4];
        uint32_t vp[4];
        load_newest(kp, vp, a.knew, a.vnew, ((size_t)j_row * c.Hkv + h) * 128, n, kgrp);
        store_newest((uint16_t*)c.cache + (size_t)(b * c.Hkv + h) * pt_slab_elems(c.W, 128), c.W, c.n_sink + s_new, kp, vp,
                     n, kgrp);
      }
    }
    if (tid == 0 && !pl.will_select) c.selected[b] = 0;   // the chosen chunk has left
  }
  arrive_rollout<WAVES, MASS>(c, a, sm, sm_ticket, dyn_lds, b, pl, c.Hkv * c.n_splits + 1);
}

// ENC: 0 = launches that cannot evict (what the steps run while no ring can be nearly full yet: leaner);
// 1 = may evict, encoding workgroups of their own behind the attention workgroups; 2 = may evict, the rows'
// own workgroups encode before they walk.  (One instantiation per way of encoding, so that neither carries
// the other's code and registers.)
// Profiling build (-DPTENC_TIMELINE, see build.py): thread 0 of every workgroup notes the 100 MHz wall clock at
// the boundaries of the step's phases; nothing of it exists in the library proper.
#ifdef PTENC_TIMELINE
#define PT_STAMP_AT(k, who)                                                                              \
  do {                                                                                                   \
    const size_t wg_ = (size_t)blockIdx.x + (size_t)gridDim.x * blockIdx.y;                              \
    if ((who) && wg_ < (size_t)PT_TIMELINE_WGS) c.timeline[wg_ * PT_TIMELINE_SLOTS + (k)] = wall_clock64(); \
  } while (0)
#else
#define PT_STAMP_AT(k, who) ((void)0)
#endif
#define PT_STAMP(k) PT_STAMP_AT(k, threadIdx.x == 0)

template <bool NT, int WAVES, bool MASS, int ENC>
__global__ __launch_bounds__(WAVES * 64, 2) void decode_mfma_kernel(
    // what the walk cannot start without comes first, as plain scalars: the build asks for these
    // leading arguments to be preloaded into registers at wavefront launch, so the counters and the
    // first K/V group are requested without first waiting for the argument block (one round trip to
    // memory less per step)
    const int* ids, const uint8_t* active, const long long* len_cur, const long long* base_cur,
    const int* n_prompt, const void* cache_p, int n_rows, unsigned heads_and_groups, PtDev c, StepArgs a) {
  // (14 dwords can be preloaded; KV heads, window splits, groups requested ahead and W / 32 share one:
  // 8, 6, 2 and 16 bits)
  const int n_kv_heads = (int)(heads_and_groups & 0xffu), ns = (int)((heads_and_groups >> 8) & 0x3fu);
  const int ahead = (int)((heads_and_groups >> 14) & 3u);   // groups a wavefront requests before it knows the counters
  const bool ahead2 = WAVES == 4 && ahead == 2;             // (8 wavefronts: short walks)
  const int NGt = (int)(heads_and_groups >> 16), w_slots = NGt << 5;
  const int n_rollouts = c.B;
  constexpr int kWaves = WAVES;
  __shared__ StepSmem<WAVES> sm;
  __shared__ int sm_ticket;
  extern __shared__ __align__(16) float dyn_lds[];   // MASS only: parked masses
  PT_STAMP(0);

  // row j of the launch (and of q / k / v / out) is rollout b: j itself, or ids[j] for a compact list
  const int j_row = blockIdx.x / n_kv_heads, hkv = blockIdx.x - j_row * n_kv_heads, split = blockIdx.y;
  if (__builtin_expect(j_row >= n_rows, 0)) {
    // beyond the rows' workgroups: every row's encoding workgroups, if the launch carries them, then ...
    if (split != 0) return;
    const int extra = blockIdx.x - n_rows * n_kv_heads;
    if constexpr (ENC == 1) {
      if (extra < n_rows * c.enc_parts) {
        encoder_role<WAVES, MASS>(c, a, sm, sm_ticket, dyn_lds, extra, ids, active, len_cur, base_cur);
        return;
      }
    }
    // ... the one workgroup that carries counters over (compact list, two counter buffers).  A listed
    // rollout's workgroup puts its new counters into the buffer this step writes; the unlisted rollouts'
    // counters must arrive there too, unchanged.  Counters only grow between resets (which clear both
    // buffers), so "the larger of what is there and the current value" is right for listed and unlisted
    // rollouts in either order of arrival: no workgroup waits for another one.
    for (int r = threadIdx.x; r < n_rollouts; r += WAVES * 64) {
      atomicMax(c.len_nx + r, len_cur[r]);
      atomicMax(c.base_nx + r, base_cur[r]);
    }
    return;
  }
  // explicit arguments: 14 preloaded dwords, then the two blocks
  constexpr int kArgBytes = 56 + (int)sizeof(PtDev) + (int)sizeof(StepArgs);
  static_assert(sizeof(PtDev) % 8 == 0 && sizeof(StepArgs) % 8 == 0, "argument blocks are laid out back to back");
  const KernargPtr ka = (const void*)__builtin_amdgcn_kernarg_segment_ptr();
  int b = j_row;
  if (ids) {
    b = load_row_id<kArgBytes>(ids + j_row, ka);
    if ((unsigned)b >= (unsigned)n_rollouts) {            // never index with a bad id: flag it and leave
      if (threadIdx.x == 0 && hkv == 0 && split == 0) atomicOr(c.err, PTENC_DEVERR_BAD_ID);
      return;
    }
  }
  const int slab = b * n_kv_heads + hkv;           // cache slab, scratch and arrival counters go by rollout
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // The slab is W / 32 groups (question groups first, then the ring's); wavefront w of split s takes
  // groups s * WAVES + w, + n_splits * WAVES, ... whatever the counters say (softmax does not care
  // about the order of the keys), so its first group (long walks: its first two) can be requested
  // before the counters are known: the two round trips to memory run side by side instead of one
  // after the other.  Should a group turn out not to be live, what arrived is dropped (the addresses
  // are inside the slab in any case).  Two groups ahead pay on long walks (-1.1 % per step at 32 groups
  // per wavefront against -0.5 % with one); on short ones the first group's arithmetic then waits for
  // the second group's bytes as well, because the queries are requested after both (with 8 groups per
  // wavefront: -1.5 % instead of -3 %).
  const int stride = ns * kWaves;
  const int pg_first = split * kWaves + wave;
  u32x4* slab_p = (u32x4*)((uint16_t*)const_cast<void*>(cache_p) + (size_t)slab * pt_slab_elems(w_slots, 128));
  Frag fa, fb;
  if (ahead != 0 && pg_first < NGt) load_group<NT>(fa, (const u32x4*)slab_p + (size_t)pg_first * (PT_GROUP_ELEMS / 8), lane);
  if (ahead2 && pg_first + stride < NGt)
    load_group<NT>(fb, (const u32x4*)slab_p + (size_t)(pg_first + stride) * (PT_GROUP_ELEMS / 8), lane);
  const uintptr_t mask_addr = (uintptr_t)(active + b);
  const uint32_t* mask_word_p = active ? (const uint32_t*)(mask_addr & ~(uintptr_t)3) : (const uint32_t*)(n_prompt + b);
  // (the scalar loads of the counters wait for themselves only: the K/V requests above stay in flight)
  const StepHead head = ids ? load_step_head<kArgBytes, false>(len_cur + b, base_cur + b, n_prompt + b, mask_word_p, c.enc_done + b, ka)
                            : load_step_head<kArgBytes, true>(len_cur + b, base_cur + b, n_prompt + b, mask_word_p, c.enc_done + b, ka);

  const int n = lane & 15, kgrp = lane >> 4;
  const int g = c.group;
  if (head.len < head.base) return;      // counters that no sequence of calls produces: leave everything alone
  const bool act = !active || ((head.mask_word >> (8 * (int)(mask_addr & 3))) & 0xffu) != 0;

  // counters as the step finds them, and as it leaves them
  const long long len0 = head.len, base0 = head.base;
  const StepPlan pl = plan_step<MASS>(c, a, act, len0, base0);
  const bool evicting = pl.evicting, append_full = pl.append_full, appending = pl.appending;
  const long long base1 = pl.base1, len1 = pl.len1;

  // what this step attends over, as a walk over 32-slot groups: first the groups of the question
  // tokens (slots 0 .. P-1), then the ring of thinking tokens from its oldest live slot
  const int P = act ? head.n_prompt : 0;
  const int n_live = act ? (int)(len1 - base1) : 0;
  // ring-relative slots from ONE division (64-bit only when a counter has outgrown 32 bits; the walk
  // cannot start before these are known): the oldest position before this step's eviction, the oldest
  // live one after it, and the one the new token takes
  const int s0e = ((unsigned long long)base0 >> 32) == 0 ? (int)((uint32_t)base0 % (uint32_t)c.Wr) : (int)(base0 % c.Wr);
  int s0 = s0e + (evicting ? c.C : 0);
  if (s0 >= c.Wr) s0 -= c.Wr;
  int s_new = s0 + (int)(len0 - base1);
  if (s_new >= c.Wr) s_new -= c.Wr;
  const int g0 = s0 >> 5, off0 = s0 & 31;
  const int NG = c.Wr >> 5, gs = c.n_sink >> 5;
  // live groups: question group pg < gs holds slots 32 pg .. of the P question tokens; ring group r is
  // live iff it is among the nv groups from the one that holds the oldest live token on (mod NG)
  const int nv = n_live > 0 ? min(NG, (off0 + n_live + PT_GROUP_TOKENS - 1) >> 5) : 0;
  auto group_live = [&](int pg) {
    if (pg < gs) return pg * PT_GROUP_TOKENS < P;
    int d = pg - gs - g0;
    d += d < 0 ? NG : 0;
    return d < nv;
  };
  // (while a ring's live range does not wrap around its end, nothing at or beyond live_end is live: the
  // search for the next live group stops there instead of running through the dead rest of the slab)
  const int live_end = g0 + nv <= NG ? gs + g0 + nv : NGt;
  auto next_live = [&](int pg) {
    while (pg < live_end && !group_live(pg)) pg += stride;
    return pg < live_end ? pg : NGt;
  };
  // logical index of a group's first slot within its region (negative for the group that holds the
  // ring's start: process_group wraps), and that region's live count
  auto group_jg = [&](int pg) {
    if (pg < gs) return pg * PT_GROUP_TOKENS;
    const int a0 = (pg - gs) * PT_GROUP_TOKENS - s0;
    return a0 <= -PT_GROUP_TOKENS ? a0 + c.Wr : a0;
  };
  auto group_lim = [&](int pg) { return pg < gs ? P : n_live; };
  auto group_wrap = [&](int pg) { return pg < gs ? 0 : c.Wr; };
  // the group the new token goes to; the split that walks it appends for this KV head
  const int pg_new = gs + (s_new >> 5);
  const bool owner = (pg_new % stride) / kWaves == split;

  // Where the row's own workgroups encode (a launch that fills the chip), they do it before they walk.
  //   Sliding window: the chunk a rollout evicts next is known as soon as the previous one has left (its oldest
  //   C tokens), so it is folded AHEAD OF TIME, a group at a time, spread evenly over the C steps that refill
  //   the ring, into the rollout's pending block (encode_ahead), by the workgroup of KV head 0: a walk that
  //   starts a few microseconds late, once in a while.  The evicting step then only adds the pending block to
  //   S; what is not folded yet (counters set by the host, steps taken through other entry points) it folds
  //   first.  A whole chunk in the evicting step made the evicting rollout's walks late by the chunk's whole
  //   duration: with the evictions of a running batch spread over the steps, +3.5 % per step at a quarter-window chunk.
  //   Scored policy: the victims are known only when the ring is full, so the evicting step folds all of them,
  //   shared by c.enc_parts of the row's workgroups.
  // The groups requested ahead of the counters are requested again afterwards, whatever this launch's
  // setting (clamped into the slab: what the walk does not want it drops): redefined on this path, their
  // registers are free during the encoding instead of being carried across it.
  if constexpr (ENC == 2) {
    {
      int part = -1, n_parts = 1, v_lo = 0, v_hi = 0;
      bool ahead_of_time = false;
      if constexpr (MASS) {
        const int p = hkv + n_kv_heads * split;
        if (evicting && p < c.enc_parts) {
          const int n_vis = pt_chunk_groups(c, s0e);
          part = p; n_parts = c.enc_parts;
          v_lo = p * n_vis / n_parts; v_hi = (p + 1) * n_vis / n_parts;
        }
      } else if (hkv == 0 && split == 0) {
        const int n_vis = pt_chunk_groups(c, s0e), done = min(max(head.enc_done, 0), n_vis);
        if (evicting) {
          part = 0; v_lo = done; v_hi = n_vis;
        } else if (appending) {
          // after this step's append the ring holds Wr - C + j tokens: by then j / C of the next chunk's groups
          // are to be folded (all of them when the ring is full)
          const int j = n_live - (c.Wr - c.C);
          int target = j >= 1 ? (int)min((long long)n_vis, (long long)j * n_vis / c.C) : 0;
          // ... but only groups whose tokens are all in the cache already: this step's own token is not yet
          // (a chunk as long as the ring reaches up to the newest token)
          const long long have = len0 - base0;             // tokens of the ring before this step
          const int present = have >= c.C ? n_vis : (int)((have + (s0e & 31)) >> 5);
          target = min(target, present);
          if (done < target) { part = 0; v_lo = done; v_hi = target; ahead_of_time = true; }
        }
      }
      if (part >= 0) {
        if (ahead_of_time) {
          encode_ahead<WAVES>(c, sm, b, s0e, v_lo, v_hi);
          load_group<NT>(fa, (const u32x4*)slab_p + (size_t)min(pg_first, NGt - 1) * (PT_GROUP_ELEMS / 8), lane);
        } else {
          // (the first group while the parts' shares meet, once this part's own stores need no more waiting
          // for: it travels while the ticket does; both groups would not fit the registers next to the hand-over's own)
          encode_part<WAVES, MASS>(c, a, sm, sm_ticket, b, j_row, s0e, part, n_parts, v_lo, v_hi, pl, len0, [&]() {
            load_group<NT>(fa, (const u32x4*)slab_p + (size_t)min(pg_first, NGt - 1) * (PT_GROUP_ELEMS / 8), lane);
          });
        }
        load_group<NT>(fb, (const u32x4*)slab_p + (size_t)min(pg_first + stride, NGt - 1) * (PT_GROUP_ELEMS / 8), lane);
      }
    }
  }
  if (owner && appending && !evicting && !a.do_attend && wave == 0) {
    // append without attention: straight from the inputs (with attention the store happens after
    // the walk, from the registers that also patch the last group)
    Op kp[4];
    uint32_t vp[4];
    load_newest(kp, vp, a.knew, a.vnew, ((size_t)j_row * c.Hkv + hkv) * 128, n, kgrp);
    store_newest((uint16_t*)slab_p, c.W, c.n_sink + s_new, kp, vp, n, kgrp);
    if (c.scored && lane == 0) {            // a new token starts with no score
      const int slot = c.n_sink + s_new;
      c.mass[(size_t)slab * c.W + slot] = 0.f;
      if (hkv == 0) c.pos[(size_t)b * c.W + slot] = len0;
    }
  }
  if (append_full && owner && hkv == 0 && tid == 0) atomicOr(c.err, PTENC_DEVERR_APPEND_FULL);

  PT_STAMP(1);
  if (a.do_attend) {
    Acc acc;
#pragma unroll
    for (int i = 0; i < 8; ++i) acc.o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    acc.m = -INFINITY;
    acc.l = 0.f;

    bool fold = false;                     // MASS: the previous step's probabilities join the scores in this walk
    float* mass_slab = nullptr;
    {
      const bool patch = appending && owner;       // this workgroup walks the group the new token goes to
      const int p_tl = s_new & 31;
      Op kp[4];
      uint32_t vp[4];
      if (patch) load_newest(kp, vp, a.knew, a.vnew, ((size_t)j_row * c.Hkv + hkv) * 128, n, kgrp);
      Op qf[4];
      if (n < g) {
        const u32x4* qp = (const u32x4*)(a.q + ((size_t)j_row * c.Hq + hkv * g + n) * 128);
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) qf[cc].u = qp[cc * 4 + kgrp];
      } else {
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) qf[cc].u = u32x4{0u, 0u, 0u, 0u};
      }
      // the previous step's queries and statistics, if they wait to be folded into the scores
      // (saved by the step that left len == len0, in the buffer of that parity)
      bool lag = false;                    // this lane's column carries a head of the previous step
      float il = 0.f;                      // that step's 1 / sum for the lane's head
      float* park = dyn_lds;               // MASS: 32 floats per group this workgroup walks
      auto grp_ptr = [&](int pg) { return (const u32x4*)slab_p + (size_t)pg * (PT_GROUP_ELEMS / 8); };
      // where a group's 32 masses are parked: by its index in the slab
      auto park_of = [&](int pg) { return park + pg * PT_GROUP_TOKENS; };
      int i = pg_first;
      // of the two groups requested ahead of the counters, the second is of use if both are part of this walk
      bool have_next = ahead2 && i + stride < NGt && group_live(i) && group_live(i + stride);
      if (ahead == 0) {
        i = next_live(i);
        if (i < NGt) load_group<NT>(fa, grp_ptr(i), lane);
      } else if (!(i < NGt && group_live(i))) {
        // not part of this walk: what arrives is dropped
        i = next_live(i + stride);
        if (i < NGt) load_group<NT>(fa, grp_ptr(i), lane);
      }
      if constexpr (MASS) {
        // after the first group's loads are on their way: the previous step's queries into columns 8..15
        // (saved by the step that left len == len0, in the buffer of that parity; the addresses are valid
        // whether or not anything waits to be folded)
        mass_slab = c.mass + (size_t)slab * c.W;
        const long long tag = ld_scalar(c.mtag + slab);
        const int par = (int)(len0 & 1), hl = (n >= 8 && n - 8 < g) ? n - 8 : 0;
        const uint16_t* qb = c.qprev + (((size_t)par * c.B + b) * c.Hq + hkv * g + hl) * 128;
        const float* mlb = c.mlprev + (((size_t)par * c.B + b) * c.Hq + hkv * g + hl) * 2;
        u32x4 ql[4];
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) ql[cc] = ((const u32x4*)qb)[cc * 4 + kgrp];
        const float mpl = mlb[0], ill = mlb[1];
        fold = appending && tag == len0;
        lag = fold && n >= 8 && n - 8 < g;
        if (lag) {
#pragma unroll
          for (int cc = 0; cc < 4; ++cc) qf[cc].u = ql[cc];
          acc.m = mpl;                     // frozen: see process_group
          il = ill;
        }
      }
      while (i < NGt) {
        int nx = next_live(i + stride);
        if (nx < NGt && !have_next) load_group<NT>(fb, grp_ptr(nx), lane);
        have_next = false;
        if (patch && i == pg_new) patch_newest(fa, kp, vp, p_tl, n, kgrp);
        if constexpr (MASS) {
          process_group<true>(fa, qf, acc, group_jg(i), group_lim(i), group_wrap(i), c.scale_log2, kgrp, lag, il,
                              (fold && i >= gs) ? park_of(i) : nullptr, n);
        } else {
          process_group(fa, qf, acc, group_jg(i), group_lim(i), group_wrap(i), c.scale_log2, kgrp);
        }
        i = nx;
        if (i >= NGt) break;
        nx = next_live(i + stride);
        if (nx < NGt) load_group<NT>(fa, grp_ptr(nx), lane);
        if (patch && i == pg_new) patch_newest(fb, kp, vp, p_tl, n, kgrp);
        if constexpr (MASS) {
          process_group<true>(fb, qf, acc, group_jg(i), group_lim(i), group_wrap(i), c.scale_log2, kgrp, lag, il,
                              (fold && i >= gs) ? park_of(i) : nullptr, n);
        } else {
          process_group(fb, qf, acc, group_jg(i), group_lim(i), group_wrap(i), c.scale_log2, kgrp);
        }
        i = nx;
      }
      // the store of the new token rides behind the walk: its inputs arrived long ago, and the
      // chunk of an evicting step was read before anything could overwrite its oldest slot
      if (patch && wave == 0 && !evicting)
        store_newest((uint16_t*)slab_p, c.W, c.n_sink + s_new, kp, vp, n, kgrp);
      if constexpr (MASS) {
        if (patch && wave == 0) {
          // this step's queries wait for the next step, in the buffer of the parity of the length it leaves
          if (n < g) {
            u32x4* qs = (u32x4*)(c.qprev + (((size_t)(len1 & 1) * c.B + b) * c.Hq + hkv * g + n) * 128);
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) qs[cc * 4 + kgrp] = qf[cc].u;
          }
          if (hkv == 0 && lane == 0) c.pos[(size_t)b * c.W + c.n_sink + s_new] = len0;
        }
      }
    }

    PT_STAMP(2);
    PT_STAMP_AT(8 + (threadIdx.x >> 6), (threadIdx.x & 63) == 0);
    // ---- merge the 4 wavefronts through LDS ----
    acc.l += __shfl_xor(acc.l, 16, 64);
    acc.l += __shfl_xor(acc.l, 32, 64);
    if (n < g) {
      if (kgrp == 0) { sm.merge.m[wave][n] = acc.m; sm.merge.l[wave][n] = acc.l; }
#pragma unroll
      for (int i = 0; i < 8; ++i) *(f32x4*)&sm.merge.o[wave][n][16 * i + 4 * kgrp] = acc.o[i];
    }
    __syncthreads();
    PT_STAMP(3);

    if constexpr (MASS) {
      // The masses parked during the walk join the accumulators: the workgroup's threads share out the
      // slots (slot = 32 pg + token) of the ring groups this workgroup walked.
      // The token this step appended starts at zero and took no part in the previous step; question
      // tokens are not scored.  One thread adds to one accumulator once per step, so a returnless
      // hardware float add gives the same bits as load-add-store and needs no round trip; the adds
      // are on their way while the merge below runs.
      if (appending && owner && tid == 0) mass_slab[c.n_sink + s_new] = 0.f;
      if (fold) {
        // half a wavefront per group: the m-th group this workgroup walks is
        // (m / WAVES) * stride + split * WAVES + m % WAVES (wavefront w of split s takes s * WAVES + w, + stride, ...)
        const float* park = dyn_lds;
        const int l5 = tid & 31;
        constexpr int kPer = 2 * kWaves, kBatch = 4;       // groups per pass of the workgroup; passes per batch
        for (int m0 = tid >> 5; (m0 / kWaves) * stride < NGt; m0 += kBatch * kPer) {
          float add[kBatch];
          int slots[kBatch];
#pragma unroll
          for (int u = 0; u < kBatch; ++u) {     // the LDS reads of a batch together, then its adds
            const int m = m0 + u * kPer, pg = (m / kWaves) * stride + split * kWaves + (m % kWaves);
            const bool mine = pg >= gs && pg < NGt;
            slots[u] = mine ? pg * PT_GROUP_TOKENS + l5 : -1;
            add[u] = mine ? park[pg * PT_GROUP_TOKENS + l5] : 0.f;
          }
#pragma unroll
          for (int u = 0; u < kBatch; ++u) {
            int j = slots[u] - gs * PT_GROUP_TOKENS - s0;             // logical index of the slot
            j += j < 0 ? c.Wr : 0;
            if (slots[u] >= 0 && (unsigned)j < (unsigned)(n_live - 1)) unsafeAtomicAdd(mass_slab + slots[u], add[u]);
          }
        }
      }
    }

    PT_STAMP(4);
    const int qn = tid >> 4, part = tid & 15;   // 16 threads per query, 8 columns each
    const bool has_row = qn < g;
    const size_t row = (size_t)b * c.Hq + hkv * g + (has_row ? qn : 0);          // scratch row
    const size_t row_io = (size_t)j_row * c.Hq + hkv * g + (has_row ? qn : 0);   // row of out
    float M = -INFINITY, L = 0.f, o[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) o[x] = 0.f;
    if (has_row) {
#pragma unroll
      for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sm.merge.m[w][qn]);
      if (M != -INFINITY) {
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
          const float fw = __builtin_amdgcn_exp2f(sm.merge.m[w][qn] - M);
          L = fmaf(fw, sm.merge.l[w][qn], L);
          const f32x4 lo = *(const f32x4*)&sm.merge.o[w][qn][part * 8], hi = *(const f32x4*)&sm.merge.o[w][qn][part * 8 + 4];
#pragma unroll
          for (int x = 0; x < 4; ++x) { o[x] = fmaf(fw, lo[x], o[x]); o[4 + x] = fmaf(fw, hi[x], o[4 + x]); }
        }
      }
    }
    bool write_out = has_row;
    if (ns > 1) {
      // park this split's (M, L, o); the last split to arrive merges all of them in split order
      if (has_row) {
        float* po = c.partial + (row * ns + split) * (128 + 2);
        if (part == 0) st_agent2(po, M, L);
#pragma unroll
        for (int x = 0; x < 4; ++x) st_agent2(po + 2 + part * 8 + 2 * x, o[2 * x], o[2 * x + 1]);
      }
      wait_own_stores();
      __syncthreads();
      if (tid == 0) sm_ticket = atomicAdd(c.tick_slab + slab, 1);
      __syncthreads();
      PT_STAMP(6);
      const bool last = sm_ticket == ns - 1;
      write_out = has_row && last;
      if (last) {
        if (has_row) {
          const float* pp = c.partial + row * ns * (128 + 2);
          // statistics: lane `part` of the row's 16 lanes takes splits part and part + 16, all loads in
          // flight at once, then the 16 lanes exchange by shuffle
          float Ms[2], Ls[2];
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            const int s = part + 16 * j;
            Ms[j] = -INFINITY; Ls[j] = 0.f;
            if (s < ns) ld_agent2(pp + (size_t)s * 130, Ms[j], Ls[j]);
          }
          M = fmaxf(Ms[0], Ms[1]);
#pragma unroll
          for (int off = 1; off < 16; off <<= 1) M = fmaxf(M, __shfl_xor(M, off, 16));
          float fs[2];
#pragma unroll
          for (int j = 0; j < 2; ++j) fs[j] = M == -INFINITY ? 0.f : exp2f(Ms[j] - M);
          L = fs[0] * Ls[0] + fs[1] * Ls[1];
#pragma unroll
          for (int off = 1; off < 16; off <<= 1) L += __shfl_xor(L, off, 16);
#pragma unroll
          for (int x = 0; x < 8; ++x) o[x] = 0.f;
          for (int s0 = 0; s0 < ns; s0 += 4) {
            float t[4][8];
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (s0 + j < ns) {
#pragma unroll
                for (int x = 0; x < 4; ++x)
                  ld_agent2(pp + (size_t)(s0 + j) * 130 + 2 + part * 8 + 2 * x, t[j][2 * x], t[j][2 * x + 1]);
              }
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (s0 + j < ns) {
                const int s = s0 + j;
                const float f0 = __shfl(fs[0], s & 15, 16), f1 = __shfl(fs[1], s & 15, 16);
                const float fw = (s >> 4) ? f1 : f0;
#pragma unroll
                for (int x = 0; x < 8; ++x) o[x] = fmaf(fw, t[j][x], o[x]);
              }
          }
        }
        if (tid == 0) c.tick_slab[slab] = 0;
      }
    }
    if constexpr (MASS) {
      if (write_out && appending) {
        if (part == 0) {
          float* ml = c.mlprev + (((size_t)(len1 & 1) * c.B + b) * c.Hq + hkv * g + qn) * 2;
          ml[0] = M;
          ml[1] = L > 0.f ? 1.f / L : 0.f;
        }
        if (tid == 0) c.mtag[slab] = len1;
      }
    }
    if (write_out) {
      const float inv = L > 0.f ? 1.f / L : 0.f;
      Op r;
#pragma unroll
      for (int x = 0; x < 8; ++x) r.h[x] = (__bf16)(o[x] * inv);
      *(u32x4*)(a.out + row_io * 128 + part * 8) = r.u;
      if (act && n_live + P == 0 && part == 0 && qn == 0 && hkv == 0) atomicOr(c.err, PTENC_DEVERR_ATTEND_EMPTY);
    }
  }

  PT_STAMP(5);
  // ---- counters ----
  // They go to the other buffer (nobody reads that one in this kernel), so no workgroup waits for the
  // rest of its rollout; under a compact list as "the larger of what is there and mine", which commutes
  // with the carrying workgroup's update of the same entry.  With the in-place option the rollout's last
  // workgroup to arrive writes them where they are (arrive_rollout).
  const bool advancing = a.do_evict || a.do_append;
  const bool in_place = a.in_place != 0;
  if (advancing && !in_place && hkv == 0 && split == 0 && tid == 0) {
    if (a.carry) {
      atomicMax(c.len_nx + b, len1);
      atomicMax(c.base_nx + b, base1);
    } else {
      c.len_nx[b] = len1;
      c.base_nx[b] = base1;
    }
  }

  // ---- arrival count of the rollout's workgroups, where the step needs one ----
  arrive_rollout<WAVES, MASS>(c, a, sm, sm_ticket, dyn_lds, b, pl, c.Hkv * ns + ((a.do_evict && !a.enc_inline) ? 1 : 0));
}

// W^a (row-major [H_kv*128, r]) -> MFMA B operands: [head][k-chunk c][column tile rt][lane][8],
// lane = 16 * kgrp + n holding rows 128 h + 32 c + 8 kgrp + e of column 16 rt + n (zero beyond r).
__global__ void pack_weights_kernel(PtDev c, const uint16_t* __restrict__ WaK, const uint16_t* __restrict__ WaV) {
  const int h = blockIdx.x, cc = blockIdx.y >> 2, rt = blockIdx.y & 3;
  const int lane = threadIdx.x, n = lane & 15, kgrp = lane >> 4;
  const int col = rt * 16 + n;
  uint16_t* dk = (uint16_t*)c.WKp + ((((size_t)h * 4 + cc) * 4 + rt) * 64 + lane) * 8;
  uint16_t* dv = (uint16_t*)c.WVp + ((((size_t)h * 4 + cc) * 4 + rt) * 64 + lane) * 8;
  for (int e = 0; e < 8; ++e) {
    const size_t rowi = (size_t)h * 128 + cc * 32 + 8 * kgrp + e;
    dk[e] = col < c.r ? WaK[rowi * c.r + col] : (uint16_t)0;
    dv[e] = col < c.r ? WaV[rowi * c.r + col] : (uint16_t)0;
  }
}

}  // namespace

hipError_t pt_launch_pack_weights(const PtDev& c, hipStream_t s) {
  hipLaunchKernelGGL(pack_weights_kernel, dim3(c.Hkv, 16), dim3(64), 0, s, c, (const uint16_t*)c.WaK,
                     (const uint16_t*)c.WaV);
  return hipGetLastError();
}

hipError_t pt_launch_decode_mfma(const PtDev& c, bool nontemporal, int waves, bool do_evict, bool do_append, bool do_attend,
                                 const void* q, const void* k, const void* v, void* out, const uint8_t* active,
                                 void* dbg_chunk, const int* ids, int n_rows, bool in_place, hipStream_t s) {
  StepArgs a;
  a.ids = ids;
  a.in_place = in_place ? 1 : 0;
  a.carry = (ids != nullptr && !in_place) ? 1 : 0;
  a.q = (const uint16_t*)q; a.out = (uint16_t*)out;
  a.knew = (const uint16_t*)k; a.vnew = (const uint16_t*)v;
  a.active = active; a.dbg_chunk = (uint16_t*)dbg_chunk;
  a.do_evict = do_evict; a.do_append = do_append; a.do_attend = do_attend;
  // without attention there is nothing to split
  PtDev cc = c;
  if (!do_attend) cc.n_splits = 1;
  const int rows = ids ? n_rows : cc.B;
  // Who encodes an evicted chunk.  A launch of at most one workgroup per CU leaves CUs free: encoding workgroups
  // of their own, behind the attention workgroups in the grid, start at once and run beside the walks (folded into
  // the row's own workgroups the encoding would lengthen the step by its whole duration: +36 % per step
  // at the 3B shape with evictions in every step).  A launch that fills the chip has no place for them until
  // the first attention workgroups leave, and what they then do against a saturated memory system is the
  // tail of the step (+5 % at the 7B shape): there the row's own workgroups fold the chunk before they walk.
  // (8-wavefront workgroups sit one per CU, 4-wavefront ones two: 256 or 512 places; a launch within a few dozen
  // of all of them still leaves encoding workgroups nowhere to start at once)
  const long places = waves == 8 ? 256 : 448;
  a.enc_inline = cc.enc_inline_opt >= 0 ? cc.enc_inline_opt : ((long)rows * cc.Hkv * cc.n_splits > places ? 1 : 0);
  if (a.enc_inline) {
    // (scored policy only: the sliding window folds its chunks ahead of time, one workgroup per rollout)
    cc.enc_parts = cc.enc_parts_inline;
    if (cc.enc_parts > cc.Hkv * cc.n_splits) cc.enc_parts = cc.Hkv * cc.n_splits;
  }
  // one workgroup per (row, KV head, split), then the encoding workgroups if they are on their own, then the carrier
  dim3 grid(rows * cc.Hkv + ((do_evict && !a.enc_inline) ? rows * cc.enc_parts : 0) + (a.carry ? 1 : 0), cc.n_splits);
  // scores are maintained by whole steps only (append + attention) under the scored policy
  const bool mass = cc.scored && do_append && do_attend;
  // long walks request two groups ahead of the counters, short ones one (see the kernel)
  const int kw = waves == 8 ? 8 : 4;
  unsigned ahead = (kw == 4 && (cc.W / PT_GROUP_TOKENS) / (cc.n_splits * 4) >= 16) ? 2u : 1u;
  // ... and none while every ring is known to be short (a run's first steps): most of what would be
  // requested is not live yet.  (Not for launches that may be replayed, whose rings grow between replays;
  // with question tokens the first groups are theirs.)
  if (!in_place && cc.n_sink == 0) {
    const long long per_group_ahead = (long long)PT_GROUP_TOKENS * cc.n_splits * kw;   // tokens that make one more group per wavefront live
    while (ahead > 0 && 2 * cc.live_ub < per_group_ahead * ahead) --ahead;
  }
  // parked masses of every group of the slab
  const size_t park = mass ? (size_t)(cc.W / PT_GROUP_TOKENS + 2) * PT_GROUP_TOKENS * sizeof(float) : 0;
#define PT_STEP_LAUNCH(NT_, WAVES_, MASS_, ENC_)                                                                      \
  hipLaunchKernelGGL((decode_mfma_kernel<NT_, WAVES_, MASS_, ENC_>), grid, dim3(WAVES_ * 64), park, s, ids, active, \
                     cc.len, cc.base, cc.n_prompt, (const void*)cc.cache, rows,                             \
                     (unsigned)cc.Hkv | ((unsigned)cc.n_splits << 8) | (ahead << 14) |                       \
                         ((unsigned)(cc.W / PT_GROUP_TOKENS) << 16),                                                   \
                     cc, a)
#define PT_STEP_PICK_ENC(NT_, WAVES_, MASS_)                                  \
  do {                                                                       \
    if (!do_evict) PT_STEP_LAUNCH(NT_, WAVES_, MASS_, 0);                    \
    else if (a.enc_inline) PT_STEP_LAUNCH(NT_, WAVES_, MASS_, 2);            \
    else PT_STEP_LAUNCH(NT_, WAVES_, MASS_, 1);                              \
  } while (0)
#define PT_STEP_PICK_MASS(NT_, WAVES_) \
  do { if (mass) PT_STEP_PICK_ENC(NT_, WAVES_, true); else PT_STEP_PICK_ENC(NT_, WAVES_, false); } while (0)
  if (waves == 8) {
    if (nontemporal) PT_STEP_PICK_MASS(true, 8); else PT_STEP_PICK_MASS(false, 8);
  } else {
    if (nontemporal) PT_STEP_PICK_MASS(true, 4); else PT_STEP_PICK_MASS(false, 4);
  }
#undef PT_STEP_PICK_MASS
#undef PT_STEP_PICK_ENC
#undef PT_STEP_LAUNCH
  return hipGetLastError();
}
