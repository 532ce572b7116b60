// The plain-ALU step prologue of one rollout -- [evict the oldest chunk of a full window and fold it
// into S] (Our Approach, the Delta-W equation and the update rule) then [append the new k, v]
// (Notation and Preliminaries, decode-stage equation) -- as a routine for one workgroup of kEncThreads
// threads, shared by the stand-alone prologue kernel and the single-launch plain decode step.
#pragma once

#include "pt_encode_alu.h"

template <typename T>
struct CacheChunk {   // the C oldest live thinking tokens of rollout b, logical order
  const T* cache; int b, Hkv, d, W, tiled, s0, n_sink, Wr;
  __device__ float get(int which, int tok, int kk) const {
    int slot = s0 + tok; if (slot >= Wr) slot -= Wr;
    slot += n_sink;
    const int h = kk / d, i = kk - h * d;
    const T* slab = cache + (size_t)(b * Hkv + h) * pt_slab_elems(W, d);
    const size_t off = which == 0 ? pt_k_off(tiled, W, d, slot, i) : pt_v_off(tiled, W, d, slot, i);
    return pt_ld<T>(slab + off);
  }
};

// j_row = row of knew / vnew (and of ids, if given); the counters go to the other buffer pair, or in place.
template <typename T>
__device__ inline void pt_step_prologue(EncSmem& sm, const PtDev& c, int j_row, int do_evict, int do_append,
                                        const T* __restrict__ knew, const T* __restrict__ vnew,
                                        const uint8_t* __restrict__ active, T* dbg_chunk,
                                        const int* __restrict__ ids, int in_place) {
  const int t = threadIdx.x;
  int b = j_row;
  if (ids) {
    b = ids[j_row];
    if ((unsigned)b >= (unsigned)c.B) {
      if (t == 0) atomicOr(c.err, PTENC_DEVERR_BAD_ID);
      return;
    }
  }
  const long long len = c.len[b];
  long long base = c.base[b];
  long long len1 = len;
  const int dkv = c.Hkv * c.d;
  T* cache = (T*)c.cache;
  const bool act = !active || active[b];

  if (act && do_evict && len - base == c.Wr) {
    CacheChunk<T> src{cache, b, c.Hkv, c.d, c.W, c.tiled, (int)(base % c.Wr), c.n_sink, c.Wr};
    float sacc[16];
    T* dbg = dbg_chunk ? dbg_chunk + (size_t)b * 2 * c.C * dkv : nullptr;
    encode_chunk<T>(sm, src, c.C, dkv, c.G, c.r, c.Qa, (const T*)c.WaK, (const T*)c.WaV, dbg, sacc);
    // S <- Normalize(S + S')   (Our Approach, the update rule)
    pt_state_update<kEncThreads>(c, b, sacc, &sm.Ws[0][0], sm.tail.red);
    base += c.C;
    __syncthreads();   // every read of the evicted slots is done before the append below
  }

  if (act && do_append) {
    if (len - base >= c.Wr) {
      if (t == 0) atomicOr(c.err, PTENC_DEVERR_APPEND_FULL);
    } else {
      const int slot = c.n_sink + (int)(len % c.Wr);
      for (int idx = t; idx < dkv; idx += kEncThreads) {
        const int h = idx / c.d, i = idx - h * c.d;
        T* slab = cache + (size_t)(b * c.Hkv + h) * pt_slab_elems(c.W, c.d);
        const size_t src = (size_t)j_row * dkv + idx;
        slab[pt_k_off(c.tiled, c.W, c.d, slot, i)] = knew[src];
        slab[pt_v_off(c.tiled, c.W, c.d, slot, i)] = vnew[src];
      }
      len1 = len + 1;
    }
  }
  // counters go to the other buffer, for every rollout, changed or not; with a compact list (which
  // would leave the unlisted rollouts out) they are written in place: this workgroup is the only
  // one that touches rollout b in this kernel
  if (t == 0) {
    if (in_place) { c.len[b] = len1; c.base[b] = base; }
    else { c.len_nx[b] = len1; c.base_nx[b] = base; }
  }
}

