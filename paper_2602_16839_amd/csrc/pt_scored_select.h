// Importance-based eviction, the choice: which C ring entries of a full ring leave next, and the
// exchange that brings them to the front of the ring (the heavy-hitter rule the paper's ablation on
// token dropping strategies integrates, chunked like its sliding window).  The eviction itself --
// dropping the oldest C ring places and folding them into S (Our Approach, the Delta-W equation and
// the update rule) -- is then the sliding window's, unchanged.
//
// One workgroup (THREADS = 256 or 512 threads) per rollout:
//   1. score of every eligible ring entry (all but the n_recent newest) = sum over KV heads of the
//      per-head accumulators the decode step maintains, in head order;
//   2. the C lowest, ties towards the older entry: a radix select on the float bit patterns
//      (scores are >= +0, so unsigned order is numeric order), then one ordered pass for the ties;
//   3. the survivors among the oldest C ring places trade places with the victims beyond them
//      (k-th survivor with the k-th such victim; key, value, accumulators and position tag travel
//      together), so the oldest C places hold exactly the victims and the ring stays one run.
// The pairs are disjoint, so every exchange is independent of the others.
#pragma once

#include "ptenc_internal.h"

constexpr int kSelThreads = 256;   // the stand-alone launch

struct SelSmall {
  uint32_t vmask[PT_SCORED_MAX_ELIGIBLE / 32];   // bit i: ring entry i is a victim
  int wpre[PT_SCORED_MAX_ELIGIBLE / 32];         // victims before word w
  int hist[256];
  int sh[4];
  int wsum[8];
};

// exclusive count, over the workgroup's threads in thread order, of a flag; total in *total
template <int THREADS>
__device__ inline int pt_sel_excl_count(bool flag, SelSmall& sm, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long bal = __ballot(flag);
  const int within = __popcll(bal & ((1ull << lane) - 1ull));
  __syncthreads();
  if (lane == 0) sm.wsum[wave] = __popcll(bal);
  __syncthreads();
  int before = 0, tot = 0;
  for (int w = 0; w < THREADS / 64; ++w) {
    if (w < wave) before += sm.wsum[w];
    tot += sm.wsum[w];
  }
  *total = tot;
  return before + within;
}

// Rollout b's ring is full and starts at position `base`.  `work` = LDS for max(n_el floats, n_el ints),
// n_el = Wr - n_recent: first the scores by ring index, then the two index lists of the exchanges.
// Called by all THREADS threads of a workgroup; starts and ends with a barrier.
template <int THREADS>
__device__ inline void pt_scored_select(const PtDev& c, int b, long long base, float* work, SelSmall& sm) {
  const int t = threadIdx.x;
  const int n_el = c.Wr - c.n_recent, C = c.C;
  const int s0 = (int)(base % c.Wr);
  auto slot_of = [&](int i) { int s = s0 + i; if (s >= c.Wr) s -= c.Wr; return s + c.n_sink; };
  __syncthreads();

  // ---- 1. scores ----
  for (int i0 = 0; i0 < n_el; i0 += 8 * THREADS) {       // 8 entries per thread at a time, loads in flight together
    float sc[8];
    int sl[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) { sc[u] = 0.f; sl[u] = slot_of(min(i0 + u * THREADS + t, n_el - 1)); }
    for (int h = 0; h < c.Hkv; ++h) {                     // head order: the score is reproducible
      const float* m = c.mass + (size_t)(b * c.Hkv + h) * c.W;
      float x[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) x[u] = m[sl[u]];
#pragma unroll
      for (int u = 0; u < 8; ++u) sc[u] += x[u];
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
      if (i0 + u * THREADS + t < n_el) work[i0 + u * THREADS + t] = sc[u];
  }
  for (int w = t; w < PT_SCORED_MAX_ELIGIBLE / 32; w += THREADS) sm.vmask[w] = 0u;
  __syncthreads();

  // ---- 2. the C-th smallest bit pattern, one byte at a time from the top ----
  uint32_t prefix = 0u, pmask = 0u;
  int k = C;                                            // still to take among the entries matching prefix
  for (int shift = 24; shift >= 0; shift -= 8) {
    if (t < 256) sm.hist[t] = 0;
    __syncthreads();
    for (int i = t; i < n_el; i += THREADS) {
      const uint32_t bits = __float_as_uint(work[i]);
      if ((bits & pmask) == prefix) atomicAdd(&sm.hist[(bits >> shift) & 255u], 1);
    }
    __syncthreads();
    if (t < 64) {
      // the first digit whose cumulative count reaches k: lane l holds digits 4 l .. 4 l + 3
      const int h0 = sm.hist[4 * t], h1 = sm.hist[4 * t + 1], h2 = sm.hist[4 * t + 2], h3 = sm.hist[4 * t + 3];
      const int mine = h0 + h1 + h2 + h3;
      int incl = mine;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (t >= o) incl += v;
      }
      const int before = incl - mine;
      if (before < k && incl >= k) {                      // exactly one lane (k >= 1, the total is >= k)
        int cum = before, dgt = 4 * t;
        if (cum + h0 < k) { cum += h0; ++dgt; if (cum + h1 < k) { cum += h1; ++dgt; if (cum + h2 < k) { cum += h2; ++dgt; } } }
        sm.sh[0] = dgt;
        sm.sh[1] = k - cum;
      }
    }
    __syncthreads();
    prefix |= (uint32_t)sm.sh[0] << shift;
    pmask |= 255u << shift;
    k = sm.sh[1];
    __syncthreads();
  }
  // prefix = the threshold pattern; k >= 1 of the entries equal to it are taken, oldest first
  int eq_seen = 0;
  for (int i0 = 0; i0 < n_el; i0 += THREADS) {
    const int i = i0 + t;
    const uint32_t bits = i < n_el ? __float_as_uint(work[i]) : 0xffffffffu;
    const bool eq = i < n_el && bits == prefix;
    int tot;
    const int rank = eq_seen + pt_sel_excl_count<THREADS>(eq, sm, &tot);
    if (i < n_el && (bits < prefix || (eq && rank < k))) atomicOr(&sm.vmask[i >> 5], 1u << (i & 31));
    eq_seen += tot;
  }
  __syncthreads();
  if (t < 64) {
    // victims before each 32-entry word: lane l takes words l, l + 64, ... in turn, carrying the running total
    int carry = 0;
    for (int w0 = 0; w0 < (n_el + 31) / 32; w0 += 64) {
      const int w = w0 + t;
      const int cnt = w < (n_el + 31) / 32 ? __popc(sm.vmask[w]) : 0;
      int incl = cnt;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int v = __shfl_up(incl, o, 64);
        if (t >= o) incl += v;
      }
      if (w < (n_el + 31) / 32) sm.wpre[w] = carry + incl - cnt;
      carry += __shfl(incl, 63, 64);
    }
  }
  __syncthreads();
  auto is_victim = [&](int i) { return i < n_el && ((sm.vmask[i >> 5] >> (i & 31)) & 1u); };
  auto victims_before = [&](int i) {   // victims among ring entries [0, i), i <= n_el
    const int w = i >> 5;
    return (w < (n_el + 31) / 32 ? sm.wpre[w] + __popc(sm.vmask[w] & ((1u << (i & 31)) - 1u))
                                 : sm.wpre[w - 1] + __popc(sm.vmask[w - 1]));
  };
  // what leaves, by position, in ring order (before anything trades places)
  for (int i = t; i < n_el; i += THREADS)
    if (is_victim(i)) c.victims[(size_t)b * C + victims_before(i)] = c.pos[(size_t)b * c.W + slot_of(i)];
  const int v_head = victims_before(min(C, n_el));      // victims inside the oldest chunk
  __syncthreads();                                      // scores are dead from here on: `work` holds the pairs

  // ---- 3. survivors of the oldest chunk <-> victims beyond it ----
  const int n_mv = C - v_head;
  int* mv_a = (int*)work;                               // k-th survivor of the oldest chunk
  int* mv_b = mv_a + n_el / 2 + 1;                      // k-th victim beyond it (n_mv <= n_el / 2)
  for (int i = t; i < n_el; i += THREADS) {
    if (i < C && !is_victim(i)) mv_a[i - victims_before(i)] = i;
    if (i >= C && is_victim(i)) mv_b[victims_before(i) - v_head] = i;
  }
  __syncthreads();
  // a token of one KV head = 16 key pieces of 16 bytes + 128 value elements (token-minor, one per
  // 16-byte piece of the group's V part).  Exchanged in batches: all loads of a batch, then its stores,
  // with enough of them in flight per thread that the exchange of a whole chunk takes a few round trips
  // to memory (keys: 8 pieces per thread and batch; values: 32 elements).
  uint16_t* cache = (uint16_t*)c.cache;
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  auto pair_slabs = [&](int mv, int h, int& sa, int& sb) {
    sa = slot_of(mv_a[mv]); sb = slot_of(mv_b[mv]);
    return (size_t)(b * c.Hkv + h) * pt_slab_elems(c.W, 128);
  };
  {
    constexpr int NB = 8;
    const int n_items = n_mv * c.Hkv * 16;
    for (int i0 = 0; i0 < n_items; i0 += THREADS * NB) {
      u32x4 ka[NB], kb[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int idx = i0 + u * THREADS + t;
        if (idx < n_items) {
          const int it = idx & 15, mh = idx >> 4, mv = mh / c.Hkv, h = mh - mv * c.Hkv;
          int sa, sb;
          const size_t so = pair_slabs(mv, h, sa, sb);
          ka[u] = *(const u32x4*)(cache + so + pt_k_off(1, c.W, 128, sa, it * 8));
          kb[u] = *(const u32x4*)(cache + so + pt_k_off(1, c.W, 128, sb, it * 8));
        }
      }
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int idx = i0 + u * THREADS + t;
        if (idx < n_items) {
          const int it = idx & 15, mh = idx >> 4, mv = mh / c.Hkv, h = mh - mv * c.Hkv;
          int sa, sb;
          const size_t so = pair_slabs(mv, h, sa, sb);
          *(u32x4*)(cache + so + pt_k_off(1, c.W, 128, sa, it * 8)) = kb[u];
          *(u32x4*)(cache + so + pt_k_off(1, c.W, 128, sb, it * 8)) = ka[u];
        }
      }
    }
  }
  {
    constexpr int NB = 32;
    const int n_items = n_mv * c.Hkv * 128;
    for (int i0 = 0; i0 < n_items; i0 += THREADS * NB) {
      uint16_t va[NB], vb[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int idx = i0 + u * THREADS + t;
        if (idx < n_items) {
          const int i = idx & 127, mh = idx >> 7, mv = mh / c.Hkv, h = mh - mv * c.Hkv;
          int sa, sb;
          const size_t so = pair_slabs(mv, h, sa, sb);
          va[u] = cache[so + pt_v_off(1, c.W, 128, sa, i)];
          vb[u] = cache[so + pt_v_off(1, c.W, 128, sb, i)];
        }
      }
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int idx = i0 + u * THREADS + t;
        if (idx < n_items) {
          const int i = idx & 127, mh = idx >> 7, mv = mh / c.Hkv, h = mh - mv * c.Hkv;
          int sa, sb;
          const size_t so = pair_slabs(mv, h, sa, sb);
          cache[so + pt_v_off(1, c.W, 128, sa, i)] = vb[u];
          cache[so + pt_v_off(1, c.W, 128, sb, i)] = va[u];
        }
      }
    }
  }
  for (int idx = t; idx < n_mv * (c.Hkv + 1); idx += THREADS) {
    const int mv = idx / (c.Hkv + 1), h = idx - mv * (c.Hkv + 1);
    const int sa = slot_of(mv_a[mv]), sb = slot_of(mv_b[mv]);
    if (h < c.Hkv) {
      float* m = c.mass + (size_t)(b * c.Hkv + h) * c.W;
      const float x = m[sa], y = m[sb];
      m[sa] = y; m[sb] = x;
    } else {
      long long* p = c.pos + (size_t)b * c.W;
      const long long x = p[sa], y = p[sb];
      p[sa] = y; p[sb] = x;
    }
  }
  if (t == 0) c.selected[b] = 1;
  __syncthreads();
}
