/*
 * ptenc -- bounded-cache rollout decode for Progressive Thought Encoding on one MI355X (gfx950).
 *
 * One context = one attention layer decoding B independent rollouts.  Per rollout the library
 * keeps a KV cache of W token slots -- n_sink slots reserved for the rollout's question tokens,
 * which are never evicted, and a ring of W - n_sink slots for thinking tokens -- two counters
 * (len = thinking tokens appended, base = thinking tokens evicted; live positions are
 * [base, len), position p lives in slot n_sink + p mod (W - n_sink)) and the fixed-size context
 * state S (G x r, fp32).
 *
 * The calls follow the paper's problem statement:
 *   - a cache policy that prunes the KV cache online during decoding, so that every token is
 *     generated from a pruned context (Challenges for Efficient RL Training, the rollout
 *     distribution under cache policy D);
 *   - the decode step extends the cache by the new k, v first and then lets the query attend
 *     over it, its own key included (Notation and Preliminaries, decode-stage equation);
 *   - when the cache is full the earliest thinking tokens are evicted as a chunk and folded
 *     into the context state: S' = ((q_g W^a_Q)(K_e W^a_K)^T)(V_e W^a_V), then
 *     S <- Normalize(S + S') (Our Approach, the Delta-W equation and the update rule); S starts
 *     from the same contraction applied to the global tokens' own k_g, v_g (same section);
 *   - question tokens stay in the cache for good and only thinking tokens slide (Our Approach,
 *     "The selection of D during training"; the response-length analysis quotes a cache of
 *     768 = 512 sink tokens + 256 in the sliding window).
 *
 * Conventions for every entry point
 *   - All "d_" pointers are DEVICE pointers, all "h_" pointers are HOST pointers.
 *   - Ownership: every device buffer is allocated and freed by the caller.  The library
 *     allocates only the small host-side context.  d_cache, d_state and d_scratch must be
 *     256-byte aligned, at least as large as ptenc_query_sizes reports, and must outlive the
 *     context.  Encoder parameters are read during ptenc_set_encoder and ptenc_evict_encode /
 *     ptenc_decode_step; W^a_K and W^a_V are borrowed until the next ptenc_set_encoder.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous on that stream and never synchronise, except ptenc_get_counters,
 *     ptenc_get_state and ptenc_poll_error, which synchronise the stream they are given.
 *   - Errors: every function returns a ptenc_status and never throws or aborts.  Problems the
 *     host can see (NULL pointer, bad configuration, unsupported value, HIP failure) return a
 *     code at once and leave all state untouched.  Misuse only the device can see (append to a
 *     full window, attention of an active rollout with an empty window) sets a bit in a sticky
 *     device error word, skips the offending rollout, and is reported by ptenc_poll_error.
 *   - Masks: d_active is uint8[B] or NULL (= all active).  A rollout with d_active[b] == 0 is
 *     untouched by append / evict and its rows of `out` are written as zeros.
 *   - Element type: q, k, v, out, the cache and the encoder parameters all have cfg.dtype.
 *     Scores, softmax statistics, accumulators and S are fp32.
 *   - The state block is the library's: change counters and S only through ptenc_reset,
 *     ptenc_set_counters and ptenc_set_state (the host side keeps a bound on how full the fullest
 *     ring can be and launches steps without the eviction machinery while none can be full; a
 *     ring filled behind its back shows up as PTENC_DEVERR_APPEND_FULL).
 *   - Overlapping calls on one context from different streams race; serialise them.
 *   - The scratch block only carries what workgroups of ONE launch hand to each other (the window
 *     splits' partial results, the shares of a chunk's encoding); nothing in it outlives a launch,
 *     so contexts whose launches never overlap may share one block (the layers of a ptenc_stack do).
 *   - HIP graphs: every decode entry point only launches kernels (no allocation, copy or memset),
 *     so it can be captured; set PTENC_OPT_COUNTERS_IN_PLACE first, and give the graph fixed
 *     input / output buffers that are refilled between replays.
 */
#ifndef PTENC_H
#define PTENC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PTENC_OK = 0,
  PTENC_ERR_INVALID_ARG = 1,
  PTENC_ERR_STATE = 2,        /* call order: e.g. evict_encode before set_encoder */
  PTENC_ERR_UNSUPPORTED = 3,
  PTENC_ERR_HIP = 4,
  PTENC_ERR_NOMEM = 5,
  PTENC_ERR_TOO_LARGE = 6     /* ptenc_decode_step_noalloc: more scratch needed than the built-in block holds */
} ptenc_status;

typedef enum { PTENC_F32 = 0, PTENC_BF16 = 1 } ptenc_dtype;

/* Normalize in S <- Normalize(S + S') is not defined by the paper; the default treats the
 * state as one object: X / max(||X||_F, eps).  ROW_L2 divides each of the G rows by its own
 * 2-norm; NONE is the identity (the plain linear-attention state). */
typedef enum { PTENC_NORM_FROBENIUS = 0, PTENC_NORM_ROW_L2 = 1, PTENC_NORM_NONE = 2 } ptenc_norm;

/* Bits of the sticky device error word. */
enum { PTENC_DEVERR_APPEND_FULL = 1, PTENC_DEVERR_ATTEND_EMPTY = 2, PTENC_DEVERR_BAD_ID = 4 };

/* Tunables for ptenc_set_option. */
typedef enum {
  PTENC_OPT_SPLITS = 0,       /* window splits per (rollout, KV head); 1..PTENC_MAX_SPLITS; 0 = heuristic */
  PTENC_OPT_FORCE_GENERIC = 1,/* 1 = use the plain ALU attention kernel even where the MFMA one applies */
  PTENC_OPT_NONTEMPORAL = 2,  /* K/V stream with non-temporal loads: 1 / 0; -1 = heuristic (on when the cache
                                 exceeds the memory-side cache) */
  PTENC_OPT_WAVES = 3,        /* wavefronts per workgroup of the MFMA kernel: 4, or 8 (taken only with at most
                                 8 query heads per KV head); 0 = heuristic */
  PTENC_OPT_COUNTERS_IN_PLACE = 4, /* 1 = steps update len / base in place instead of alternating between two
                                 buffers on the host.  Needed when a step is captured into a HIP graph and
                                 replayed (the alternation would be frozen into the graph); costs one extra
                                 arrival counter per rollout and step.  Default 0. */
  PTENC_OPT_EVICT_POLICY = 5, /* ptenc_policy: which tokens an eviction takes.  Set it before the first step after
                                 a reset (scores are kept only while it is PTENC_POLICY_SCORED). */
  PTENC_OPT_RECENT = 6,       /* scored policy: the n most recent ring entries are never taken; 0 .. W - n_sink - C;
                                 -1 = default (half the ring, at most W - n_sink - C) */
  PTENC_OPT_ENCODE_PARTS = 7, /* MFMA path: workgroups that share the encoding of one rollout's evicted chunk, each
                                 a contiguous range of its 32-token groups, their shares of S' added in range
                                 order; 1..8; 0 = heuristic (one per 64 tokens of the chunk, at most 8).  S
                                 depends on it in the last bits only (fp32 summation order). */
  PTENC_OPT_ENCODE_INLINE = 8 /* MFMA path: who folds evicted chunks into S.  0: encoding workgroups of their own,
                                 launched behind the attention workgroups, fold the whole chunk in the evicting
                                 step (right where the launch leaves CUs free).  1: the rollout's own workgroups
                                 do it before they walk the window -- under the sliding window one 32-token group
                                 at a time, ahead of time, spread over the steps that refill the ring, so that the
                                 evicting step only adds what is pending (right where the launch fills the
                                 chip).  -1 = heuristic by launch size (default).  S depends on it in the last
                                 bits only. */
} ptenc_option;

/* Which tokens leave when the sliding part of the cache is full.
 * SLIDING: the C oldest thinking tokens (Our Approach, "The selection of D during training").
 * SCORED:  importance-based token dropping (Ablation Study and Discussion, "Integration with inference-time token
 *          dropping strategy": the paper finds it more accurate but 37 % slower in rollouts and leaves an
 *          efficient integration open).  Here the score is the heavy-hitter one -- the attention
 *          probability a token has received, summed over decode steps and over all query heads -- and
 *          it is a by-product of ptenc_decode_step: the probabilities of a step are recomputed, from
 *          that step's saved queries and softmax statistics, while the NEXT step of the rollout streams
 *          the same keys, so they join the scores one step late and cost no extra pass over the cache.
 *          When the ring is full, the C lowest-scored entries among all but the PTENC_OPT_RECENT most
 *          recent ones are chosen (ties: the older ring entry first); the survivors among the oldest C
 *          ring places trade places with the chosen entries beyond them, so that the oldest C places hold
 *          exactly the chosen tokens, which then leave and are encoded into S exactly as a sliding chunk
 *          is, and the ring stays one contiguous run (attention does not depend on the order of the
 *          cache; d_dbg_chunk of ptenc_evict_encode lists them in the order of those places).
 *          Question tokens are never scored or taken.  With
 *          PTENC_OPT_RECENT = W - n_sink - C the policy is the sliding window.
 *          Needs the MFMA path (bf16, head_dim 128, W and n_sink multiples of 32), at most 8 query heads
 *          per KV head and at most 12288
 *          eligible entries; else PTENC_ERR_UNSUPPORTED.  Scores advance only through
 *          ptenc_decode_step / ptenc_decode_run / ptenc_decode_step_ids / ptenc_decode_run_ids (a
 *          separate ptenc_decode_attn leaves them alone); ptenc_set_counters accepts only empty
 *          windows.  The step whose append fills a ring chooses the next victims at its own end, so a run of
 *          decode steps needs no extra launch; a ring filled by a bare ptenc_cache_append, or re-scored by
 *          ptenc_set_scores, gets a stand-alone selection launch from the next call that may evict. */
typedef enum { PTENC_POLICY_SLIDING = 0, PTENC_POLICY_SCORED = 1 } ptenc_policy;

#define PTENC_MAX_SPLITS 32

typedef struct {
  int32_t batch;          /* B rollouts */
  int32_t n_q_heads;      /* H_q */
  int32_t n_kv_heads;     /* H_kv, divides H_q */
  int32_t head_dim;       /* d, 1..256 */
  int32_t window;         /* W cache slots per rollout, question tokens included */
  int32_t chunk;          /* C tokens evicted at once, 1 <= C <= W - n_sink */
  int32_t n_sink;         /* slots reserved for permanently retained question tokens, 0 <= n_sink < W */
  int32_t n_global;       /* G global tokens, 1..64 */
  int32_t rank;           /* r latent width, 1..64 */
  int32_t dtype;          /* ptenc_dtype */
  int32_t norm_mode;      /* ptenc_norm */
  float norm_eps;         /* 0 => 1e-12 */
  float softmax_scale;    /* 0 => 1/sqrt(head_dim) (Notation and Preliminaries, attention equation) */
} ptenc_config;

typedef struct ptenc_ctx ptenc_ctx; /* opaque, host side */

/* Bytes the caller must provide for the cache, the state block and the scratch block. */
ptenc_status ptenc_query_sizes(const ptenc_config* cfg, size_t* cache_bytes, size_t* state_bytes,
                               size_t* scratch_bytes);

/* Validates cfg and binds the caller's device buffers.  Touches no device memory: call
 * ptenc_set_encoder and ptenc_reset before decoding. */
ptenc_status ptenc_create(const ptenc_config* cfg, void* d_cache, void* d_state, void* d_scratch,
                          ptenc_ctx** out);
ptenc_status ptenc_destroy(ptenc_ctx* ctx);

ptenc_status ptenc_set_option(ptenc_ctx* ctx, int32_t option, int32_t value);

/* Encoder parameters (row-major, cfg.dtype): q_g [G, H_q*d], W^a_Q [H_q*d, r], W^a_K and W^a_V
 * [H_kv*d, r], k_g and v_g [G, H_kv*d] (both NULL => S_0 = 0, the zero-initialised ablation).
 * Computes Q_a = q_g W^a_Q and S_0 = (Q_a (k_g W^a_K)^T)(v_g W^a_V) on the device (Our Approach,
 * initialisation with learnable global tokens).  S_0 is not normalised. */
ptenc_status ptenc_set_encoder(ptenc_ctx* ctx, const void* d_qg, const void* d_WaQ, const void* d_WaK,
                               const void* d_WaV, const void* d_kg, const void* d_vg, void* stream);

/* len = base = 0, no question tokens, and S = S_0 for the rollouts selected by d_mask (uint8[B], NULL = all);
 * clears the error word when d_mask is NULL.  Cache contents are left as they are (dead slots
 * are never read). */
ptenc_status ptenc_reset(ptenc_ctx* ctx, const uint8_t* d_mask, void* stream);

/* Question tokens of every rollout into its reserved slots (bulk append): d_k, d_v are
 * [B, p_max, H_kv, d] of cfg.dtype, h_prompt_len is a HOST array of B lengths, each
 * 0 <= len <= min(n_sink, p_max); rollout b's tokens 0 .. len-1 are taken, replacing whatever
 * question tokens it held.  They are attended to at every step and never evicted or encoded.
 * Synchronises the stream (the host array is consumed before return). */
ptenc_status ptenc_prefill(ptenc_ctx* ctx, const void* d_k, const void* d_v, const int32_t* h_prompt_len,
                           int32_t p_max, void* stream);

/* The same for a list of rollouts only (a rollout engine that recycles finished rollouts: ptenc_reset
 * with a mask, then this): d_k, d_v are [n, p_max, H_kv, d], row j belongs to rollout d_ids[j] (DEVICE
 * int32[n], distinct) and has h_prompt_len[j] tokens (HOST array of n lengths).  Rollouts not listed
 * keep their question tokens.  An id outside 0 .. B-1 sets PTENC_DEVERR_BAD_ID and is skipped.
 * n = 0 does nothing.  Synchronises the stream. */
ptenc_status ptenc_prefill_ids(ptenc_ctx* ctx, const void* d_k, const void* d_v, const int32_t* d_ids,
                               const int32_t* h_prompt_len, int32_t n, int32_t p_max, void* stream);
ptenc_status ptenc_get_prompt_len(ptenc_ctx* ctx, int32_t* h_prompt_len, void* stream);

/* Writes k, v [B, H_kv, d] of every active rollout to the ring slot of position len, then len += 1
 * (Notation and Preliminaries: the cache is extended by k_{t+1}, v_{t+1} before attending). */
ptenc_status ptenc_cache_append(ptenc_ctx* ctx, const void* d_k, const void* d_v,
                                const uint8_t* d_active, void* stream);

/* out[b, h] = softmax(q[b, h] . K_live / sqrt(d)) V_live over rollout b's question tokens and live positions,
 * query head h reading KV head h / (H_q / H_kv); q and out are [B, H_q, d]
 * (Notation and Preliminaries, attention equation, restricted to the pruned context). */
ptenc_status ptenc_decode_attn(ptenc_ctx* ctx, const void* d_q, void* d_out, const uint8_t* d_active,
                               void* stream);

/* For every active rollout whose ring is full (len - base == W - n_sink): takes its C oldest
 * positions [base, base + C), oldest first, folds them into S as defined above, and
 * base += C.  Other rollouts are untouched.  d_dbg_chunk is NULL, or [B, 2, C, H_kv*d] of
 * cfg.dtype receiving K_e (index 0) and V_e (index 1) of each evicting rollout in logical
 * order (rows of rollouts that did not evict are left untouched). */
ptenc_status ptenc_evict_encode(ptenc_ctx* ctx, const uint8_t* d_active, void* d_dbg_chunk, void* stream);

/* One decode step: evict_encode, cache_append, decode_attn, in this order. */
ptenc_status ptenc_decode_step(ptenc_ctx* ctx, const void* d_q, const void* d_k, const void* d_v,
                               void* d_out, const uint8_t* d_active, void* stream);

/* ptenc_decode_step for callers that cannot allocate or hand over a scratch block of their own choosing:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same result, but what the step's workgroups hand to each other (the window splits' partial results,
 * the encoding workgroups' shares of S') goes through a block built into the library -- a fixed array of
 * PTENC_NOALLOC_SCRATCH_BYTES in device memory, one copy per GPU, held until the process ends --
 * instead of the d_scratch given to ptenc_create (which is not touched).  The call allocates and
 * frees nothing and only launches kernels.
 *   - Limit: with the context's current plan (window splits, encoding workgroups per chunk) the step needs
 *     B * H_q * n_splits * (d + 2) * 4  +  B * enc_parts * G * r * 4  bytes (each part rounded up to 256);
 *     beyond PTENC_NOALLOC_SCRATCH_BYTES the call returns PTENC_ERR_TOO_LARGE and does nothing.  (All of the
 *     benchmark shapes fit: the 7B-shaped layer needs 6 MiB, the 8B-shaped one 8.5 MiB.)
 *   - The block keeps the last call's contents; nothing in it has to start at zero (every word a launch
 *     reads from it was written earlier in the same launch), so nothing is cleared.
 *   - Every context on a GPU shares that GPU's block: calls whose kernels may overlap on one GPU (different
 *     streams, no ordering between them) race on it.  Calls on one stream, or ordered by events, are safe.
 *   - The block's address is looked up once per GPU, by the first ptenc_decode_step_noalloc issued with
 *     that GPU current (the library has no initialisation call); the GPU that `stream` belongs to must be
 *     the current one during every call.  A failed look-up returns PTENC_ERR_HIP. */
#define PTENC_NOALLOC_SCRATCH_BYTES (16u << 20)
ptenc_status ptenc_decode_step_noalloc(ptenc_ctx* ctx, const void* d_q, const void* d_k, const void* d_v,
                                       void* d_out, const uint8_t* d_active, void* stream);

/* n_steps decode steps from step-major buffers: q and out [n_steps, B, H_q, d], k and v
 * [n_steps, B, H_kv, d], d_active NULL or uint8 [n_steps, B].  Same result as n_steps calls of
 * ptenc_decode_step; the loop runs on the host without synchronising.  n_steps = 0 does nothing and
 * accepts NULL buffers. */
ptenc_status ptenc_decode_run(ptenc_ctx* ctx, const void* d_q, const void* d_k, const void* d_v,
                              void* d_out, const uint8_t* d_active, int64_t n_steps, void* stream);

/* One decode step for a compact list of rollouts (a rollout engine drops finished rollouts from its
 * batch instead of masking them): d_ids is int32[n] on the DEVICE, distinct rollout indices in
 * [0, B); q and out are [n, H_q, d], k and v [n, H_kv, d], row j belonging to rollout d_ids[j].
 * Rollouts not listed are untouched.  Same result per listed rollout as ptenc_decode_step.  An id
 * out of range sets PTENC_DEVERR_BAD_ID and its row is skipped; duplicate ids race.  0 <= n <= B. */
ptenc_status ptenc_decode_step_ids(ptenc_ctx* ctx, const void* d_q, const void* d_k, const void* d_v,
                                   void* d_out, const int32_t* d_ids, int32_t n, void* stream);

/* n_steps such steps from concatenated buffers: step t uses rows h_row_offsets[t] ..
 * h_row_offsets[t+1]-1 of q, k, v, out and d_ids (h_row_offsets: HOST int64[n_steps + 1],
 * non-decreasing, starting at 0).  The loop runs on the host without synchronising. */
ptenc_status ptenc_decode_run_ids(ptenc_ctx* ctx, const void* d_q, const void* d_k, const void* d_v,
                                  void* d_out, const int32_t* d_ids, const int64_t* h_row_offsets,
                                  int64_t n_steps, void* stream);

/* The context state used as a per-rollout low-rank weight delta (Our Approach: Delta-W = A S B,
 * theta' = theta + Delta-W; which projections receive it is the caller's choice):
 *     y[j] += ((x[j] A) S_b) B        for every row j, b = j (or d_ids[j])
 * x is [rows, d_in], y [rows, d_out] (updated in place), both cfg.dtype; A (d_in x G) is given
 * transposed, d_At [G, d_in]; B (r x d_out) is given transposed, d_Bt [d_out, r]; fp32
 * accumulation.  rows = B with d_ids NULL (d_active may mask rollouts: their rows of y are left
 * as they are), else rows = n with rollout ids as in ptenc_decode_step_ids. */
ptenc_status ptenc_apply_delta(ptenc_ctx* ctx, const void* d_x, const void* d_At, const void* d_Bt, void* d_y,
                               int32_t d_in, int32_t d_out, const uint8_t* d_active, const int32_t* d_ids, int32_t n,
                               void* stream);

/* Counters to / from host arrays of B int64 each.  set_counters requires
 * 0 <= base <= len <= base + W - n_sink for every rollout (used for resume and rotation tests).
 * It also drops whatever a rollout had folded ahead of time of its next chunk (PTENC_OPT_ENCODE_INLINE): the
 * next eviction then folds the whole chunk itself, and S may differ in the last bits from a run whose
 * counters were never rewritten (a resume from cache + S + counters is bit-identical where chunks are
 * folded by encoding workgroups of their own, equal to rounding otherwise). */
ptenc_status ptenc_get_counters(ptenc_ctx* ctx, int64_t* h_len, int64_t* h_base, void* stream);
ptenc_status ptenc_set_counters(ptenc_ctx* ctx, const int64_t* h_len, const int64_t* h_base, void* stream);

/* S to / from a host array [B, G, r] fp32. */
ptenc_status ptenc_get_state(ptenc_ctx* ctx, float* h_S, void* stream);
ptenc_status ptenc_set_state(ptenc_ctx* ctx, const float* h_S, void* stream);

/* Q_a [G, r] and S_0 [G, r] (fp32) as computed by ptenc_set_encoder; either may be NULL. */
ptenc_status ptenc_get_encoder_state(ptenc_ctx* ctx, float* h_Qa, float* h_S0, void* stream);

/* Everything a rollout attends over, in logical order (question tokens, then live positions oldest
 * first) into d_K, d_V [B, H_kv, W, d] of cfg.dtype; the remaining rows are zero-filled.
 * Debug / checkpoint helper. */
ptenc_status ptenc_gather_window(ptenc_ctx* ctx, void* d_K, void* d_V, void* stream);

/* Element offset, within d_cache, of element i of the key (which = 0) or value (which = 1) of
 * KV head h of rollout b stored in ring slot `slot`.  Documents the physical layout for tests
 * that poison or inspect raw slots. */
ptenc_status ptenc_cache_offset(ptenc_ctx* ctx, int32_t b, int32_t h, int32_t slot, int32_t i,
                                int32_t which, size_t* elem_offset);

/* Scored policy only (else PTENC_ERR_STATE).
 * ptenc_get_scores: the folded scores (float [B][W]) and the positions (int64 [B][W], position = the
 *   token's 0-based append index within its rollout) of the live ring entries, in ring order, oldest
 *   ring entry first; entries past the live count read 0 and -1.  Either output may be NULL.  Device
 *   pointers; asynchronous.
 * ptenc_set_scores: overwrites the scores of the live ring entries (same layout) and drops the
 *   probabilities of the latest step that were still waiting to be folded.  A full ring has had its
 *   victims chosen and brought to its oldest places already: ring order is what that left, and the
 *   next call that may evict chooses again from the new scores, in that order.
 * ptenc_get_victims: the positions of every rollout's latest choice of victims (int64 [B][C], ring
 *   order; -1 where none was made since the reset).  The choice is made when a ring fills and carried
 *   out by the rollout's next step, so after an evicting step this names what that step took -- unless
 *   the step refilled the ring (C = 1), in which case it already names what leaves next.  Host
 *   pointer; synchronises. */
ptenc_status ptenc_get_scores(ptenc_ctx* ctx, float* d_score, int64_t* d_pos, void* stream);
ptenc_status ptenc_set_scores(ptenc_ctx* ctx, const float* d_score, void* stream);
ptenc_status ptenc_get_victims(ptenc_ctx* ctx, int64_t* h_pos, void* stream);

/* Reads and returns the sticky device error word (does not clear it; ptenc_reset(NULL) does). */
ptenc_status ptenc_poll_error(ptenc_ctx* ctx, int32_t* h_flags, void* stream);

/* Which kernels this context runs: *attn_kernel = 0 plain ALU, 1 MFMA tiled; *n_splits = window
 * splits in use; *encode_kernel likewise. Any pointer may be NULL. */
ptenc_status ptenc_get_plan(ptenc_ctx* ctx, int32_t* attn_kernel, int32_t* n_splits, int32_t* encode_kernel);

/* ---- Multi-layer driver -------------------------------------------------------------------------
 * A stack is L contexts with one configuration -- the L attention layers of one model decoding the
 * same B rollouts (Experimental Setup, Models: the evaluated models are stacks of identical attention layers,
 * each with its own KV cache; the rollout stage pays the bounded-cache step once per layer and
 * token).  d_cache and d_state hold L consecutive per-layer slices of the sizes ptenc_query_sizes
 * reports (layer l starts at l times that size); d_scratch is ONE layer's scratch, shared, which is
 * safe because the layers of a stack run in stream order -- all calls on a stack and on its
 * layers must be issued to one stream, or be serialised by the caller.  Layers are created with
 * non-temporal K/V loads when the L caches together exceed the memory-side cache.  Everything per layer (ptenc_set_encoder, ptenc_prefill,
 * ptenc_get_state, ...) goes through the borrowed context ptenc_stack_layer returns; it dies with
 * the stack. */
typedef struct ptenc_stack ptenc_stack; /* opaque, host side */
#define PTENC_MAX_LAYERS 1024

ptenc_status ptenc_stack_query_sizes(const ptenc_config* cfg, int32_t n_layers, size_t* cache_bytes,
                                     size_t* state_bytes, size_t* scratch_bytes);
ptenc_status ptenc_stack_create(const ptenc_config* cfg, int32_t n_layers, void* d_cache, void* d_state,
                                void* d_scratch, ptenc_stack** out);
ptenc_status ptenc_stack_destroy(ptenc_stack* stack);
ptenc_status ptenc_stack_layer(ptenc_stack* stack, int32_t layer, ptenc_ctx** out);
/* ptenc_reset of every layer. */
ptenc_status ptenc_stack_reset(ptenc_stack* stack, const uint8_t* d_mask, void* stream);

/* One decode step of every layer, in layer order: ptenc_decode_step(layer l, h_q[l], h_k[l], h_v[l],
 * h_out[l], d_active).  h_q, h_k, h_v, h_out are HOST arrays of L DEVICE pointers (a model computes
 * layer l's q, k, v from layer l-1's output, so they live in per-layer buffers anyway); shapes per
 * layer as for ptenc_decode_step.  Stops at the first layer that returns an error and returns it. */
ptenc_status ptenc_stack_decode_step(ptenc_stack* stack, const void* const* h_q, const void* const* h_k,
                                     const void* const* h_v, void* const* h_out, const uint8_t* d_active,
                                     void* stream);

/* Records one ptenc_stack_decode_step over the given buffers into HIP graphs kept by the stack
 * (replacing earlier ones); nothing is executed.  (Two recordings, one for either role assignment of
 * the layers' two counter buffers: replays and eager steps can be mixed freely.  Stepping a single
 * layer of the stack on its own in between leaves the layers in disagreement: PTENC_ERR_STATE from
 * the next recording or replay until the others have been stepped too.)  The pointers are frozen
 * into the graphs: refill the same buffers between replays.  Every layer's encoder must be set (else PTENC_ERR_STATE).
 * The recording uses a stream of the library's own, so the caller's stream can be the default one.
 * A graph holds whatever kernel plan the layers had when it was recorded: record again after
 * ptenc_set_option. */
ptenc_status ptenc_stack_graph_capture(ptenc_stack* stack, const void* const* h_q, const void* const* h_k,
                                       const void* const* h_v, void* const* h_out, const uint8_t* d_active);
/* Replays the recorded step on `stream` (PTENC_ERR_STATE if none was recorded): one call = one
 * decode step of all layers.  Allocates nothing. */
ptenc_status ptenc_stack_graph_launch(ptenc_stack* stack, void* stream);

/* Calibration helpers (no context needed): a plain streaming read of `bytes` (whole 16 KiB units,
 * a multiple of 16384 is read; d_sink is 4 bytes that are practically never written) and a
 * plain copy of `bytes` (multiple of 16), each on n_blocks workgroups of 256 threads.  They
 * measure the HBM rate a kernel with no arithmetic reaches, and scale the profiler's byte
 * counters.  Pointers are device pointers, 16-byte aligned. */
ptenc_status ptenc_util_stream_read(const void* d_src, size_t bytes, void* d_sink, int32_t n_blocks, void* stream);
/* The same read with non-temporal loads, as the decode kernel streams K and V. */
ptenc_status ptenc_util_stream_read_nt(const void* d_src, size_t bytes, void* d_sink, int32_t n_blocks, void* stream);
ptenc_status ptenc_util_copy(void* d_dst, const void* d_src, size_t bytes, int32_t n_blocks, void* stream);

const char* ptenc_status_string(ptenc_status s);

#ifdef __cplusplus
}
#endif
#endif /* PTENC_H */
