// Internal definitions shared by the host API and the gfx950 kernels of libptenc.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ptenc.h"

// ------------------------------------------------------------------------------------------
// Device-visible view of a context (passed to kernels by value).
// ------------------------------------------------------------------------------------------
struct PtDev {
  int B, Hq, Hkv, d, W, C, G, r;
  int n_sink;         // slots 0 .. n_sink-1 of every slab hold question tokens (kept for good)
  int Wr;             // W - n_sink: capacity of the ring of thinking tokens behind them
  int group;          // H_q / H_kv
  int dtype;          // ptenc_dtype
  int tiled;          // 1: bf16 d=128 MFMA-tiled cache layout, 0: row-major
  int norm_mode;
  int n_splits;
  float norm_eps;
  float scale_log2;   // softmax scale * log2(e): scores live in the base-2 domain
  void* cache;
  float* S;           // [B, G, r]
  float* Qa;          // [G, r]
  float* S0;          // [G, r]
  long long* len;     // [B]  counters as the next kernel finds them
  long long* base;    // [B]
  long long* len_nx;  // [B]  where a kernel that advances the counters writes them (all rollouts,
  long long* base_nx; //      changed or not); the host swaps the pairs after such a launch
  int* n_prompt;      // [B]  question tokens held in the reserved slots
  int* err;           // sticky error word
  float* partial;     // [rows][n_splits][2 + d]: (m, l, unnormalised out) per window split
  const void* WaK;    // [H_kv*d, r] borrowed
  const void* WaV;    // [H_kv*d, r] borrowed
  // MFMA path only
  int n_rt;           // ceil(r / 16): 16-column tiles of the latent space
  int* tick_rollout;  // [B]      arrival counters, zero between kernels
  int* tick_slab;     // [B*H_kv]
  int* tick_enc;      // [B]      (the parts of a long chunk's encoding)
  int enc_parts;      // workgroups that share one rollout's chunk (1 unless the chunk is long): encoding workgroups
                      //   of their own
  int enc_parts_inline; // the same where the row's own workgroups encode before they walk (capped by their number)
  int enc_inline_opt;   // -1: the launch decides by its size who encodes; 0 / 1: forced (PTENC_OPT_ENCODE_INLINE)
  float* enc_part;    // [B][enc_parts][G*r] their partial S', in the scratch buffer after `partial`
  float* pend;        // [B][G*r] what has been folded ahead of time of the chunk the rollout evicts next (the
                      //   sliding window's next chunk is known C steps before it leaves); added to S' by the eviction
  int* enc_done;      // [B] how many of that chunk's 32-token groups `pend` holds (0 after every eviction)
  void* WKp;          // W^a_K, W^a_V repacked as MFMA B operands: [H_kv][4][4][64 lanes][8] bf16
  void* WVp;
  // importance-based eviction (MFMA path only)
  int scored;         // 1: an eviction takes the lowest-scored tokens instead of the oldest
  int n_recent;       // most recent ring entries an eviction never takes
  float* mass;        // [B*H_kv][W] by physical slot: attention probability the token has received from
                      //   this KV head's query heads, all folded steps summed
  long long* pos;     // [B][W] by physical slot: position (append index) of the token stored there
  long long* victims; // [B][C] positions the rollout's last eviction took, ring order (-1: none yet)
  uint16_t* qprev;    // [2][B][H_q][128] the latest step's queries, buffer = parity of the length it left
  float* mlprev;      // [2][B][H_q][2]   that step's softmax maximum (base-2 domain) and 1 / sum
  long long* mtag;    // [B*H_kv] the length that step left (its data waits to be folded); -1: none
  int* selected;      // [B] 1: the ring is full and its next victims already sit in its oldest C places
  // host side only (travels with the launch parameters): upper bound on the live thinking tokens of the
  // fullest ring, this launch's append included (appends since the last full reset or ptenc_set_counters)
  long long live_ub;
#ifdef PTENC_TIMELINE
  // profiling build only (see build.py): wall-clock stamps of the step kernel's phases, PT_TIMELINE_SLOTS per
  // workgroup, at the end of the state block
  long long* timeline;
#endif
};

#ifdef PTENC_TIMELINE
constexpr int PT_TIMELINE_SLOTS = 16;      // per workgroup: 0 entry, 1 walk begins, 2 walk ends, 3 wavefronts merged,
                                           //   4 scores folded, 5 result out, 6 split ticket taken, 8.. walk end of wavefront w
constexpr int PT_TIMELINE_WGS = 8192;      // workgroups (x + grid.x * y) that have room
#endif

struct ptenc_ctx {
  ptenc_config cfg;
  PtDev dev;
  size_t cache_bytes, state_bytes, scratch_bytes;
  int encoder_set;
  int opt_splits;        // 0 = heuristic
  int opt_force_generic;
  int opt_nontemporal;   // -1 = heuristic, 0, 1
  int nontemporal;       // resolved
  int opt_waves;         // 0 = heuristic, 4, 8
  int opt_enc_parts;     // 0 = heuristic, 1..PT_MAX_ENC_PARTS
  int opt_enc_inline;    // -1 = heuristic, 0, 1
  int opt_in_place;      // 1 = counters are updated in place (no buffer rotation on the host)
  int opt_policy;        // 0 sliding window, 1 scored
  int opt_recent;        // -1 = default
  int select_stale;      // scored policy: a ring may be full without a valid selection (see ptenc_api.hip)
  int swaps;             // how often the two counter buffers have changed roles (parity = which is current)
  int waves;             // resolved: wavefronts per workgroup of the MFMA kernel
  int attn_kernel;       // 0 generic, 1 mfma
  int encode_kernel;     // 0 generic, 1 mfma
};

// ------------------------------------------------------------------------------------------
// Physical cache layout.
//
// The cache is an array of slabs, one per (rollout b, KV head h): slab = b * H_kv + h, each of
// 2 * W * d elements, W slots.  Slots 0 .. n_sink-1 hold the rollout's question tokens (token j in
// slot j); thinking-token position p lives in slot n_sink + p mod (W - n_sink).
//
// Row-major layout (fp32, or bf16 shapes the MFMA kernel does not take):
//   K[slot][i] at slot * d + i,  V[slot][i] at W * d + slot * d + i.
//
// Tiled layout (bf16, d = 128, W % 32 == 0): the slab is W/32 groups of 32 consecutive slots;
// a group is 16 KiB = [K tile 0 | K tile 1 | V], each part ordered so that one 16-byte load
// per lane of a 64-wide wavefront is both a contiguous 1 KiB read and an MFMA 16x16x32 bf16
// operand (lane = 16 * kgrp + row holds 8 consecutive contraction elements):
//   K tile t (slots 16t .. 16t+15 of the group), 2048 elements:
//       element ((c * 4 + kgrp) * 16 + m) * 8 + e  =  K[slot 16t + m][i = 32c + 8 kgrp + e]
//   V part, 4096 elements, transposed so that the contraction runs over tokens:
//       element ((it * 4 + kgrp) * 16 + m) * 8 + e  =  V[slot tl][i = 16 it + m],
//       tl = (e / 4) * 16 + 4 * kgrp + (e % 4)
//   (tl's order matches the register order in which the score MFMA leaves the 32 tokens of a
//    group in each lane, so the probabilities feed the second MFMA without any lane exchange).
// ------------------------------------------------------------------------------------------
#define PT_GROUP_TOKENS 32
#define PT_MAX_ENC_PARTS 8  /* workgroups that may share the encoding of one evicted chunk */
#define PT_GROUP_ELEMS 8192      // 32 tokens * 128 * 2 (K and V)

__host__ __device__ inline size_t pt_slab_elems(int W, int d) { return (size_t)2 * W * d; }

__host__ __device__ inline size_t pt_k_off(int tiled, int W, int d, int slot, int i) {
  (void)W;   // same signature as pt_v_off, whose row-major form needs it
  if (!tiled) return (size_t)slot * d + i;
  const int grp = slot >> 5, tl = slot & 31;
  const int t = tl >> 4, m = tl & 15;
  const int c = i >> 5, kgrp = (i & 31) >> 3, e = i & 7;
  return (size_t)grp * PT_GROUP_ELEMS + t * 2048 + (((c * 4 + kgrp) * 16 + m) * 8 + e);
}

__host__ __device__ inline size_t pt_v_off(int tiled, int W, int d, int slot, int i) {
  if (!tiled) return (size_t)W * d + (size_t)slot * d + i;
  const int grp = slot >> 5, tl = slot & 31;
  const int it = i >> 4, m = i & 15;
  const int kgrp = (tl & 15) >> 2, e = ((tl >> 4) << 2) | (tl & 3);
  return (size_t)grp * PT_GROUP_ELEMS + 4096 + (((it * 4 + kgrp) * 16 + m) * 8 + e);
}

// ------------------------------------------------------------------------------------------
// bf16 <-> fp32 (round to nearest even; NaN stays NaN)
// ------------------------------------------------------------------------------------------
__host__ __device__ inline float pt_bf16_to_f32(uint16_t h) {
  union { uint32_t u; float f; } x;
  x.u = (uint32_t)h << 16;
  return x.f;
}

__host__ __device__ inline uint16_t pt_f32_to_bf16(float f) {
  union { uint32_t u; float f; } x;
  x.f = f;
  if ((x.u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x.u >> 16) | 0x40u);
  const uint32_t lsb = (x.u >> 16) & 1u;
  x.u += 0x7fffu + lsb;
  return (uint16_t)(x.u >> 16);
}

template <typename T> __device__ inline float pt_ld(const T* p);
template <> __device__ inline float pt_ld<float>(const float* p) { return *p; }
template <> __device__ inline float pt_ld<uint16_t>(const uint16_t* p) { return pt_bf16_to_f32(*p); }

template <typename T> __device__ inline void pt_st(T* p, float v);
template <> __device__ inline void pt_st<float>(float* p, float v) { *p = v; }
template <> __device__ inline void pt_st<uint16_t>(uint16_t* p, float v) { *p = pt_f32_to_bf16(v); }

// Host bookkeeping of a decode step whose launch the context did not issue itself (the replay of
// a recorded graph): the counter buffers change roles, the fill bound grows (ptenc_api.hip).
void pt_ctx_stepped_by_replay(ptenc_ctx* ctx);
// Before a step is recorded for replay: it may run at any later time, so it must carry the eviction machinery.
void pt_ctx_assume_full(ptenc_ctx* ctx);
// Scored policy: the stand-alone choice of victims, if the context's state asks for one (a launch, no
// allocation); a replay does this first, because a recorded step cannot.
hipError_t pt_ctx_refresh_selection(ptenc_ctx* ctx, hipStream_t s);

// ------------------------------------------------------------------------------------------
// Launchers implemented in the kernel files (host side, return hipError_t).
// ------------------------------------------------------------------------------------------
hipError_t pt_launch_reset(const PtDev& c, const uint8_t* mask, bool clear_err, hipStream_t s);
hipError_t pt_launch_step_prologue(const PtDev& c, bool do_evict, bool do_append,
                                   const void* k, const void* v, const uint8_t* active, void* dbg_chunk,
                                   const int* ids, int n_rows, bool in_place, hipStream_t s);
hipError_t pt_launch_gather(const PtDev& c, void* K, void* V, hipStream_t s);
hipError_t pt_launch_prefill(const PtDev& c, const void* k, const void* v, int p_max, const int* ids, const int* lens,
                             int n_rows, hipStream_t s);
hipError_t pt_launch_encoder_init(const PtDev& c, const void* qg, const void* WaQ, const void* kg,
                                  const void* vg, hipStream_t s);
hipError_t pt_launch_attn_generic(const PtDev& c, const void* q, void* out, const uint8_t* active,
                                  const int* ids, int n_rows, hipStream_t s);
hipError_t pt_launch_step_generic(const PtDev& c, const void* q, const void* k, const void* v, void* out,
                                  const uint8_t* active, hipStream_t s);
hipError_t pt_launch_combine(const PtDev& c, void* out, const uint8_t* active, hipStream_t s);
hipError_t pt_launch_apply_delta(const PtDev& c, const void* x, const void* At, const void* Bt, void* y, int d_in,
                                 int d_out, const uint8_t* active, const int* ids, int n_rows, hipStream_t s);
hipError_t pt_launch_pack_weights(const PtDev& c, hipStream_t s);
hipError_t pt_launch_decode_mfma(const PtDev& c, bool nontemporal, int waves, bool do_evict, bool do_append, bool do_attend,
                                 const void* q, const void* k, const void* v, void* out, const uint8_t* active,
                                 void* dbg_chunk, const int* ids, int n_rows, bool in_place, hipStream_t s);
// importance-based eviction (scored_kernels.hip)
hipError_t pt_launch_scored_select(const PtDev& c, const uint8_t* active, const int* ids, int n_rows, hipStream_t s);
hipError_t pt_launch_scores_get(const PtDev& c, float* d_score, long long* d_pos, hipStream_t s);
hipError_t pt_launch_scores_set(const PtDev& c, const float* d_score, hipStream_t s);
#define PT_SCORED_MAX_ELIGIBLE 12288   // eligible ring entries the selection can rank (48 KiB of LDS)
