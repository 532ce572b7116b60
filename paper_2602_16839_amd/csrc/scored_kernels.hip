// Importance-based eviction: when a rollout's ring is full, the C tokens with the lowest
// accumulated attention probability leave instead of the C oldest (the heavy-hitter rule the paper's
// ablation on token dropping strategies integrates, chunked like its sliding window).
//
// This kernel only CHOOSES them and brings them to the front of the ring; the decode step that
// follows then evicts "the oldest chunk" exactly as under the sliding window and folds it into S
// with the same encoder (Our Approach, the Delta-W equation and the update rule).
// One workgroup per rollout (bf16, head_dim 128, tiled cache only), in this order:
//   1. score of every eligible ring entry (all but the n_recent newest) = sum over KV heads of the
//      per-head accumulators the decode step maintains, in head order;
//   2. the C lowest, ties towards the older entry: a radix select on the float bit patterns
//      (scores are >= +0, so unsigned order is numeric order), then one ordered pass for the ties;
//   3. the survivors among the oldest C ring places trade places with the victims beyond them
//      (k-th survivor with the k-th such victim; key, value, accumulators and position tag travel
//      together), so the oldest C places hold exactly the victims and the ring stays one run.
// The pairs are disjoint, so every exchange is independent of the others.
#include "ptenc_internal.h"

namespace {

constexpr int kThreads = 256;

struct ScoredSmem {
  union {
    float sc[PT_SCORED_MAX_ELIGIBLE];            // phase 1-2: scores by ring index
    int moves[2][PT_SCORED_MAX_ELIGIBLE / 2];    // phase 3: the two ring indices of every exchange
  } u;
  uint32_t vmask[PT_SCORED_MAX_ELIGIBLE / 32];   // bit i: ring entry i is a victim
  int wpre[PT_SCORED_MAX_ELIGIBLE / 32];         // victims before word w
  int hist[256];
  int sh[4];
  int wsum[kThreads / 64];
};

// exclusive count, over the workgroup's threads in thread order, of a flag; total in *total
__device__ inline int block_excl_count(bool flag, ScoredSmem& sm, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long bal = __ballot(flag);
  const int within = __popcll(bal & ((1ull << lane) - 1ull));
  __syncthreads();
  if (lane == 0) sm.wsum[wave] = __popcll(bal);
  __syncthreads();
  int before = 0, tot = 0;
  for (int w = 0; w < kThreads / 64; ++w) {
    if (w < wave) before += sm.wsum[w];
    tot += sm.wsum[w];
  }
  *total = tot;
  return before + within;
}

__global__ __launch_bounds__(kThreads) void scored_select_kernel(PtDev c, const uint8_t* __restrict__ active,
                                                                const int* __restrict__ ids) {
  __shared__ ScoredSmem sm;
  const int t = threadIdx.x;
  int b = blockIdx.x;
  if (ids) {
    b = ids[blockIdx.x];
    if ((unsigned)b >= (unsigned)c.B) {
      if (t == 0) atomicOr(c.err, PTENC_DEVERR_BAD_ID);
      return;
    }
  }
  if (active && !active[b]) return;
  const long long len = c.len[b], base = c.base[b];
  if (len - base != c.Wr) return;                       // not full: nothing leaves
  const int n_el = c.Wr - c.n_recent, C = c.C;
  const int s0 = (int)(base % c.Wr);
  auto slot_of = [&](int i) { int s = s0 + i; if (s >= c.Wr) s -= c.Wr; return s + c.n_sink; };

  // ---- 1. scores ----
  for (int i = t; i < n_el; i += kThreads) {
    const int slot = slot_of(i);
    float s = 0.f;
    for (int h = 0; h < c.Hkv; ++h) s += c.mass[(size_t)(b * c.Hkv + h) * c.W + slot];
    sm.u.sc[i] = s;
  }
  for (int w = t; w < PT_SCORED_MAX_ELIGIBLE / 32; w += kThreads) sm.vmask[w] = 0u;
  __syncthreads();

  // ---- 2. the C-th smallest bit pattern, one byte at a time from the top ----
  uint32_t prefix = 0u, pmask = 0u;
  int k = C;                                            // still to take among the entries matching prefix
  for (int shift = 24; shift >= 0; shift -= 8) {
    sm.hist[t] = 0;
    __syncthreads();
    for (int i = t; i < n_el; i += kThreads) {
      const uint32_t bits = __float_as_uint(sm.u.sc[i]);
      if ((bits & pmask) == prefix) atomicAdd(&sm.hist[(bits >> shift) & 255u], 1);
    }
    __syncthreads();
    if (t == 0) {
      int cum = 0, dgt = 255;
      for (int x = 0; x < 256; ++x) {
        if (cum + sm.hist[x] >= k) { dgt = x; break; }
        cum += sm.hist[x];
      }
      sm.sh[0] = dgt;
      sm.sh[1] = k - cum;
    }
    __syncthreads();
    prefix |= (uint32_t)sm.sh[0] << shift;
    pmask |= 255u << shift;
    k = sm.sh[1];
    __syncthreads();
  }
  // prefix = the threshold pattern; k >= 1 of the entries equal to it are taken, oldest first
  int eq_seen = 0;
  for (int i0 = 0; i0 < n_el; i0 += kThreads) {
    const int i = i0 + t;
    const uint32_t bits = i < n_el ? __float_as_uint(sm.u.sc[i]) : 0xffffffffu;
    const bool eq = i < n_el && bits == prefix;
    int tot;
    const int rank = eq_seen + block_excl_count(eq, sm, &tot);
    if (i < n_el && (bits < prefix || (eq && rank < k))) atomicOr(&sm.vmask[i >> 5], 1u << (i & 31));
    eq_seen += tot;
  }
  __syncthreads();
  if (t == 0) {
    int cum = 0;
    for (int w = 0; w < (n_el + 31) / 32; ++w) { sm.wpre[w] = cum; cum += __popc(sm.vmask[w]); }
  }
  __syncthreads();
  auto is_victim = [&](int i) { return i < n_el && ((sm.vmask[i >> 5] >> (i & 31)) & 1u); };
  auto victims_before = [&](int i) {   // victims among ring entries [0, i), i <= n_el
    const int w = i >> 5;
    return (w < (n_el + 31) / 32 ? sm.wpre[w] + __popc(sm.vmask[w] & ((1u << (i & 31)) - 1u))
                                 : sm.wpre[w - 1] + __popc(sm.vmask[w - 1]));
  };
  // what leaves, by position, in ring order (before anything trades places)
  for (int i = t; i < n_el; i += kThreads)
    if (is_victim(i)) c.victims[(size_t)b * C + victims_before(i)] = c.pos[(size_t)b * c.W + slot_of(i)];
  const int v_head = victims_before(min(C, n_el));      // victims inside the oldest chunk
  __syncthreads();                                      // scores are dead from here on: sm.u holds the pairs

  // ---- 3. survivors of the oldest chunk <-> victims beyond it ----
  const int n_mv = C - v_head;
  for (int i = t; i < n_el; i += kThreads) {
    if (i < C && !is_victim(i)) sm.u.moves[0][i - victims_before(i)] = i;            // k-th survivor
    if (i >= C && is_victim(i)) sm.u.moves[1][victims_before(i) - v_head] = i;       // k-th victim beyond
  }
  __syncthreads();
  // a token of one KV head = 16 key pieces of 16 bytes + 128 value elements (token-minor): 144 items,
  // exchanged in batches of loads followed by stores so that the round trips overlap
  uint16_t* cache = (uint16_t*)c.cache;
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  const int n_items = n_mv * c.Hkv * 144;
  for (int i0 = 0; i0 < n_items; i0 += kThreads * 4) {
    u32x4 ka[4], kb[4];
    uint16_t va[4], vb[4];
    size_t oa[4], ob[4];
    int kind[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int idx = i0 + u * kThreads + t;
      kind[u] = -1;
      if (idx < n_items) {
        const int mv = idx / (c.Hkv * 144), rem = idx - mv * (c.Hkv * 144);
        const int h = rem / 144, it = rem - h * 144;
        const int sa = slot_of(sm.u.moves[0][mv]), sb = slot_of(sm.u.moves[1][mv]);
        const size_t so = (size_t)(b * c.Hkv + h) * pt_slab_elems(c.W, 128);
        if (it < 16) {
          kind[u] = 0;
          oa[u] = so + pt_k_off(1, c.W, 128, sa, it * 8);
          ob[u] = so + pt_k_off(1, c.W, 128, sb, it * 8);
          ka[u] = *(const u32x4*)(cache + oa[u]);
          kb[u] = *(const u32x4*)(cache + ob[u]);
        } else {
          kind[u] = 1;
          oa[u] = so + pt_v_off(1, c.W, 128, sa, it - 16);
          ob[u] = so + pt_v_off(1, c.W, 128, sb, it - 16);
          va[u] = cache[oa[u]];
          vb[u] = cache[ob[u]];
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (kind[u] == 0) { *(u32x4*)(cache + oa[u]) = kb[u]; *(u32x4*)(cache + ob[u]) = ka[u]; }
      else if (kind[u] == 1) { cache[oa[u]] = vb[u]; cache[ob[u]] = va[u]; }
    }
  }
  for (int idx = t; idx < n_mv * (c.Hkv + 1); idx += kThreads) {
    const int mv = idx / (c.Hkv + 1), h = idx - mv * (c.Hkv + 1);
    const int sa = slot_of(sm.u.moves[0][mv]), sb = slot_of(sm.u.moves[1][mv]);
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
}

}  // namespace

hipError_t pt_launch_scored_select(const PtDev& c, const uint8_t* active, const int* ids, int n_rows, hipStream_t s) {
  hipLaunchKernelGGL(scored_select_kernel, dim3(ids ? n_rows : c.B), dim3(kThreads), 0, s, c, active, ids);
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
