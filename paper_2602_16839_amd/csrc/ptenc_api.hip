// Host side of libptenc: argument checks, context bookkeeping, kernel launches.
#include <math.h>
#include <mutex>
#include <new>
#include <stdlib.h>
#include <string.h>

#include "ptenc_internal.h"

// The built-in scratch block of ptenc_decode_step_noalloc: what the caller's d_scratch is to ptenc_decode_step
// (window splits' partial results, encoding workgroups' shares of S'), for callers that cannot provide or
// allocate one.  Every GPU the library runs on holds its own copy until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; kernels get the resolved device address.
static __device__ __align__(256) unsigned char scratch[PTENC_NOALLOC_SCRATCH_BYTES];

namespace {

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// device address of `scratch` on each GPU, resolved once per device with that device current
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

hipError_t builtin_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

struct StateLayout {
  size_t S, Qa, S0, len, base, len2, base2, n_prompt, err, tick_rollout, tick_slab, tick_enc, WKp, WVp;
  size_t mass, pos, victims, qprev, mlprev, mtag, selected;   // importance-based eviction
  size_t pend, enc_done, total;
#ifdef PTENC_TIMELINE
  size_t timeline;
#endif
};

StateLayout state_layout(const ptenc_config& c) {
  StateLayout L;
  size_t off = 0;
  const size_t gr = (size_t)c.n_global * c.rank * sizeof(float);
  L.S = off;    off = align256(off + gr * c.batch);
  L.Qa = off;   off = align256(off + gr);
  L.S0 = off;   off = align256(off + gr);
  L.len = off;  off = align256(off + sizeof(long long) * c.batch);
  L.base = off; off = align256(off + sizeof(long long) * c.batch);
  L.len2 = off;  off = align256(off + sizeof(long long) * c.batch);
  L.base2 = off; off = align256(off + sizeof(long long) * c.batch);
  L.n_prompt = off; off = align256(off + sizeof(int) * c.batch);
  L.err = off;  off = align256(off + sizeof(int));
  L.tick_rollout = off; off = align256(off + sizeof(int) * c.batch);
  L.tick_slab = off;    off = align256(off + sizeof(int) * c.batch * c.n_kv_heads);
  L.tick_enc = off;     off = align256(off + sizeof(int) * c.batch);
  const size_t packed = (size_t)c.n_kv_heads * 4 * 4 * 64 * 8 * 2;   // MFMA operand form of W^a_K / W^a_V
  L.WKp = off;  off = align256(off + packed);
  L.WVp = off;  off = align256(off + packed);
  const size_t slabs = (size_t)c.batch * c.n_kv_heads, rows = (size_t)c.batch * c.n_q_heads;
  L.mass = off;    off = align256(off + slabs * c.window * sizeof(float));
  L.pos = off;     off = align256(off + (size_t)c.batch * c.window * sizeof(long long));
  L.victims = off; off = align256(off + (size_t)c.batch * c.chunk * sizeof(long long));
  L.qprev = off;   off = align256(off + 2 * rows * c.head_dim * 2);
  L.mlprev = off;  off = align256(off + 2 * rows * 2 * sizeof(float));
  L.mtag = off;    off = align256(off + slabs * sizeof(long long));
  L.selected = off; off = align256(off + (size_t)c.batch * sizeof(int));
  L.pend = off;     off = align256(off + gr * c.batch);
  L.enc_done = off; off = align256(off + (size_t)c.batch * sizeof(int));
#ifdef PTENC_TIMELINE
  L.timeline = off; off = align256(off + (size_t)PT_TIMELINE_WGS * PT_TIMELINE_SLOTS * sizeof(long long));
#endif
  L.total = off;
  return L;
}

ptenc_status check_config(const ptenc_config* c) {
  if (!c) return PTENC_ERR_INVALID_ARG;
  if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1) return PTENC_ERR_INVALID_ARG;
  if (c->n_q_heads % c->n_kv_heads != 0) return PTENC_ERR_INVALID_ARG;
  if (c->window < 1 || c->n_sink < 0 || c->n_sink >= c->window) return PTENC_ERR_INVALID_ARG;
  if (c->chunk < 1 || c->chunk > c->window - c->n_sink) return PTENC_ERR_INVALID_ARG;
  if (c->n_global < 1 || c->rank < 1) return PTENC_ERR_INVALID_ARG;
  if (c->dtype != PTENC_F32 && c->dtype != PTENC_BF16) return PTENC_ERR_INVALID_ARG;
  if (c->norm_mode < PTENC_NORM_FROBENIUS || c->norm_mode > PTENC_NORM_NONE) return PTENC_ERR_INVALID_ARG;
  if (!(c->norm_eps >= 0.f) || !(c->softmax_scale >= 0.f) || isinf(c->softmax_scale)) return PTENC_ERR_INVALID_ARG;
  if (c->head_dim > 256 || c->n_global > 64 || c->rank > 64) return PTENC_ERR_UNSUPPORTED;
  if ((size_t)c->batch * c->n_q_heads > 0x7fffffffu / PTENC_MAX_SPLITS) return PTENC_ERR_UNSUPPORTED;
  return PTENC_OK;
}

size_t elem_bytes(int dtype) { return dtype == PTENC_F32 ? 4 : 2; }

size_t partial_bytes(const ptenc_config& c) {
  return align256((size_t)c.batch * c.n_q_heads * PTENC_MAX_SPLITS * (c.head_dim + 2) * sizeof(float));
}

// A chunk is encoded by several workgroups, each a contiguous range of its 32-token groups (one workgroup takes
// about 4.5 us per group; every further part costs a hand-over through memory).  Encoding workgroups of their
// own (launches that leave CUs free) take about two groups each.  Where the row's own workgroups encode before
// they walk, a part delays one walk by its whole duration, and what the delay costs the step depends on how
// much earlier than the step's last workgroup that walk would have ended: measured at the 7B shape with the
// evictions of a running batch spread over the steps, per chunk size the best count was one part per four
// groups (C = 128: 1 part +0.4 % per step, 2 parts +2.2 %; C = 512: 1, 2, 4 parts +8.7, +4.8, +2.2 %).
int enc_parts_for(const ptenc_config& c, bool inline_mode) {
  const int e = c.chunk / (inline_mode ? 128 : 64);
  return e < 1 ? 1 : (e > PT_MAX_ENC_PARTS ? PT_MAX_ENC_PARTS : e);
}
size_t enc_part_bytes(const ptenc_config& c) {
  return align256((size_t)c.batch * PT_MAX_ENC_PARTS * c.n_global * c.rank * sizeof(float));
}

bool mfma_attn_applies(const ptenc_config& c) {
  return c.dtype == PTENC_BF16 && c.head_dim == 128 && c.window % 32 == 0 && c.n_sink % 32 == 0 &&
         c.n_q_heads / c.n_kv_heads <= 16 &&
         c.n_kv_heads <= 0xff && c.window / 32 <= 0xffff;        // (they share one kernel argument)
}

// Window splits.  Splitting a (rollout, KV head) row over several workgroups costs a round trip
// through memory for the partial results; it pays while the launch has fewer workgroups than the
// chip has CUs.  Measured on MI355X (2 KV heads, windows of 1024, 2048 and 4096, both interfaces): from
// 60 rows up the best count is the largest one that keeps rows x splits within about 240 workgroups
// (one split from 121 rows), below that about 128 workgroups; never fewer than 256 tokens per split.
// Two refinements for the MFMA kernel, whose wavefronts take whole 32-token groups: a count that deals
// the groups unevenly (32 groups to 3 x 8 wavefronts: some get two, the step lasts as long as if all did)
// gives way to the next count that deals them evenly: a larger one if the launch stays within 224
// workgroups, else a smaller one if the busiest wavefront has no more groups under it than under the
// uneven count (otherwise the uneven count stays: 64 groups to 3 x 8 wavefronts is 3 at most, against 4
// under two splits, and measures best); and 96 to 128 rows, which fill up to half the chip, are split
// in two only when each wavefront still keeps 8 groups or more (112 rows at a window of 4096: 38 us
// against 48; at 2048 and below one split is 0-6 % faster).
int heuristic_splits(const ptenc_ctx* x, long n_rollouts) {
  const ptenc_config& c = x->cfg;
  const long rows = n_rollouts * (x->attn_kernel ? c.n_kv_heads : c.n_q_heads);
  long want = rows >= 60 ? 240 / rows : (128 + rows - 1) / rows;
  long cap = (c.window - c.n_sink) / 256;
  if (cap < 1) cap = 1;
  if (cap > PTENC_MAX_SPLITS) cap = PTENC_MAX_SPLITS;
  if (want > cap) want = cap;
  if (want < 1) want = 1;
  if (x->attn_kernel) {
    const long ng = (c.window - c.n_sink) / PT_GROUP_TOKENS;
    const long waves = (rows * want <= 256 && x->dev.group <= 8 && x->opt_waves != 4) ? 8 : 4;
    auto even = [&](long s) { return ng % (s * waves) == 0; };
    if (want > 1 && !even(want)) {
      long up = want + 1, down = want - 1;
      while (up <= cap && !even(up)) ++up;
      while (down > 1 && !even(down)) --down;
      const auto longest = [&](long s) { return (ng + s * waves - 1) / (s * waves); };
      if (up <= cap && rows * up <= 224) want = up;
      else if (longest(down) == longest(want)) want = down;
    }
    if (rows >= 96 && rows <= 128 && cap >= 2) want = ng / (2 * waves) >= 8 ? 2 : 1;
  }
  return (int)want;
}

// 8 wavefronts per workgroup need the query group to fit 8 rows of the merge buffer; measured
// worth ~3 % when there is at most one workgroup per CU, a loss of as much when there are more
int pick_waves(const ptenc_ctx* x, long n_rollouts, int splits) {
  const long wgs = n_rollouts * x->cfg.n_kv_heads * splits;
  const int want = x->opt_waves ? x->opt_waves : (wgs <= 256 ? 8 : 4);
  return (want == 8 && x->dev.group <= 8) ? 8 : 4;
}

// most recent ring entries the scored policy protects: the caller's value, else half the ring,
// never so many that fewer than a chunk stay eligible
int resolved_recent(const ptenc_ctx* x) {
  const int Wr = x->dev.Wr, C = x->dev.C;
  int r = x->opt_recent >= 0 ? x->opt_recent : Wr / 2;
  if (r > Wr - C) r = Wr - C;
  return r;
}

void replan(ptenc_ctx* x) {
  x->attn_kernel = (x->dev.tiled && !x->opt_force_generic) ? 1 : 0;
  x->dev.scored = (x->opt_policy == PTENC_POLICY_SCORED && x->attn_kernel == 1) ? 1 : 0;
  x->dev.n_recent = resolved_recent(x);
  x->encode_kernel = x->attn_kernel;
  x->dev.enc_parts = x->opt_enc_parts > 0 ? x->opt_enc_parts : enc_parts_for(x->cfg, false);
  x->dev.enc_parts_inline = x->opt_enc_parts > 0 ? x->opt_enc_parts : enc_parts_for(x->cfg, true);
  x->dev.enc_inline_opt = x->opt_enc_inline;
  x->dev.n_splits = x->opt_splits > 0 ? x->opt_splits : heuristic_splits(x, x->cfg.batch);
  x->waves = pick_waves(x, x->cfg.batch, x->dev.n_splits);
  // a cache that fits the 256 MiB memory-side cache is better served by ordinary loads
  x->nontemporal = x->opt_nontemporal >= 0 ? x->opt_nontemporal : (x->cache_bytes > ((size_t)192 << 20) ? 1 : 0);
}

inline hipStream_t S(void* s) { return (hipStream_t)s; }

// after a launch that advanced the counters: the buffer it wrote becomes the current one
ptenc_status advanced(ptenc_ctx* x, hipError_t e) {
  if (e != hipSuccess) return PTENC_ERR_HIP;
  if (x->opt_in_place) return PTENC_OK;
  long long* t = x->dev.len; x->dev.len = x->dev.len_nx; x->dev.len_nx = t;
  t = x->dev.base; x->dev.base = x->dev.base_nx; x->dev.base_nx = t;
  ++x->swaps;
  return PTENC_OK;
}
inline ptenc_status hip_status(hipError_t e) { return e == hipSuccess ? PTENC_OK : PTENC_ERR_HIP; }

// Launches that may evict carry the eviction machinery (encoding workgroups for every row, or the code with which
// the rows' own workgroups encode).  While no ring can be full yet (the host
// keeps an upper bound on the fullest one: appends since the last full reset or ptenc_set_counters),
// steps are launched without it; should the bound ever be wrong, the
// append on the full ring sets PTENC_DEVERR_APPEND_FULL instead of going unnoticed.  Steps that may be
// replayed from a graph (counters in place) always carry it.
// (A ring that is within a chunk of full already has groups of its next chunk folded ahead of time by the
// steps that fill it, which is part of the same machinery.)
bool may_evict(const ptenc_ctx* x) { return x->opt_in_place != 0 || x->dev.live_ub >= x->dev.Wr - x->dev.C; }
void appended_one(ptenc_ctx* x) { if (x->dev.live_ub < x->dev.Wr) ++x->dev.live_ub; }

// Scored policy: a decode step chooses the next victims itself when its append fills a ring.  A ring
// can also fill up, or lose its selection, in ways that step does not see (a bare ptenc_cache_append,
// ptenc_set_scores, a change of policy); the next call that may evict then runs the stand-alone
// selection first, over every rollout (choosing early for one that sits this call out is harmless).
hipError_t refresh_selection(ptenc_ctx* x, hipStream_t s) {
  if (!x->dev.scored || !x->select_stale) return hipSuccess;
  x->select_stale = 0;
  return pt_launch_scored_select(x->dev, nullptr, nullptr, 0, s);
}

}  // namespace

void pt_ctx_stepped_by_replay(ptenc_ctx* ctx) {
  appended_one(ctx);
  (void)advanced(ctx, hipSuccess);
}

void pt_ctx_assume_full(ptenc_ctx* ctx) { ctx->dev.live_ub = ctx->dev.Wr; }

hipError_t pt_ctx_refresh_selection(ptenc_ctx* ctx, hipStream_t s) { return refresh_selection(ctx, s); }

extern "C" {

ptenc_status ptenc_query_sizes(const ptenc_config* cfg, size_t* cache_bytes, size_t* state_bytes,
                               size_t* scratch_bytes) {
  ptenc_status st = check_config(cfg);
  if (st != PTENC_OK) return st;
  if (cache_bytes)
    *cache_bytes = align256((size_t)cfg->batch * cfg->n_kv_heads * pt_slab_elems(cfg->window, cfg->head_dim) *
                            elem_bytes(cfg->dtype));
  if (state_bytes) *state_bytes = state_layout(*cfg).total;
  if (scratch_bytes)
    *scratch_bytes = partial_bytes(*cfg) + enc_part_bytes(*cfg);
  return PTENC_OK;
}

ptenc_status ptenc_create(const ptenc_config* cfg, void* d_cache, void* d_state, void* d_scratch,
                          ptenc_ctx** out) {
  if (!out) return PTENC_ERR_INVALID_ARG;
  *out = nullptr;
  ptenc_status st = check_config(cfg);
  if (st != PTENC_OK) return st;
  if (!d_cache || !d_state || !d_scratch) return PTENC_ERR_INVALID_ARG;
  if (((uintptr_t)d_cache | (uintptr_t)d_state | (uintptr_t)d_scratch) & 255) return PTENC_ERR_INVALID_ARG;
  ptenc_ctx* x = new (std::nothrow) ptenc_ctx;
  if (!x) return PTENC_ERR_NOMEM;
  memset(x, 0, sizeof(*x));
  x->cfg = *cfg;
  if (x->cfg.norm_eps == 0.f) x->cfg.norm_eps = 1e-12f;
  ptenc_query_sizes(cfg, &x->cache_bytes, &x->state_bytes, &x->scratch_bytes);
  x->opt_nontemporal = -1;
  x->opt_enc_inline = -1;
  const StateLayout L = state_layout(*cfg);
  char* sp = (char*)d_state;
  PtDev& d = x->dev;
  d.B = cfg->batch; d.Hq = cfg->n_q_heads; d.Hkv = cfg->n_kv_heads; d.d = cfg->head_dim;
  d.W = cfg->window; d.C = cfg->chunk; d.G = cfg->n_global; d.r = cfg->rank;
  d.n_sink = cfg->n_sink; d.Wr = cfg->window - cfg->n_sink;
  d.group = cfg->n_q_heads / cfg->n_kv_heads;
  d.dtype = cfg->dtype;
  d.tiled = mfma_attn_applies(*cfg) ? 1 : 0;
  d.norm_mode = cfg->norm_mode;
  d.norm_eps = x->cfg.norm_eps;
  const double scale = cfg->softmax_scale > 0.f ? (double)cfg->softmax_scale : 1.0 / sqrt((double)cfg->head_dim);
  d.scale_log2 = (float)(scale * 1.4426950408889634074);
  d.cache = d_cache;
  d.S = (float*)(sp + L.S); d.Qa = (float*)(sp + L.Qa); d.S0 = (float*)(sp + L.S0);
  d.len = (long long*)(sp + L.len); d.base = (long long*)(sp + L.base); d.err = (int*)(sp + L.err);
  d.len_nx = (long long*)(sp + L.len2); d.base_nx = (long long*)(sp + L.base2);
  d.n_prompt = (int*)(sp + L.n_prompt);
  d.partial = (float*)d_scratch;
  d.WaK = nullptr; d.WaV = nullptr;
  d.n_rt = (cfg->rank + 15) / 16;
  d.tick_rollout = (int*)(sp + L.tick_rollout); d.tick_slab = (int*)(sp + L.tick_slab);
  d.tick_enc = (int*)(sp + L.tick_enc);
  d.enc_part = (float*)((char*)d_scratch + partial_bytes(*cfg));
  d.WKp = sp + L.WKp; d.WVp = sp + L.WVp;
  d.scored = 0; d.n_recent = 0;
  d.mass = (float*)(sp + L.mass); d.pos = (long long*)(sp + L.pos); d.victims = (long long*)(sp + L.victims);
  d.qprev = (uint16_t*)(sp + L.qprev); d.mlprev = (float*)(sp + L.mlprev);
  d.mtag = (long long*)(sp + L.mtag);
  d.selected = (int*)(sp + L.selected);
  d.pend = (float*)(sp + L.pend); d.enc_done = (int*)(sp + L.enc_done);
#ifdef PTENC_TIMELINE
  d.timeline = (long long*)(sp + L.timeline);
#endif
  x->select_stale = 1;
  x->opt_recent = -1;
  x->dev.live_ub = d.Wr;       // nothing is known about the counters the state block holds
  replan(x);
  *out = x;
  return PTENC_OK;
}

#ifdef PTENC_TIMELINE
// profiling build only: where in the state block the step kernel's phase stamps are
extern "C" ptenc_status ptenc_timeline_region(const ptenc_config* cfg, size_t* offset, size_t* bytes, int* slots_per_workgroup) {
  if (check_config(cfg) != PTENC_OK || !offset || !bytes || !slots_per_workgroup) return PTENC_ERR_INVALID_ARG;
  *offset = state_layout(*cfg).timeline;
  *bytes = (size_t)PT_TIMELINE_WGS * PT_TIMELINE_SLOTS * sizeof(long long);
  *slots_per_workgroup = PT_TIMELINE_SLOTS;
  return PTENC_OK;
}
#endif

ptenc_status ptenc_destroy(ptenc_ctx* ctx) {
  if (!ctx) return PTENC_ERR_INVALID_ARG;
  delete ctx;
  return PTENC_OK;
}

ptenc_status ptenc_set_option(ptenc_ctx* ctx, int32_t option, int32_t value) {
  if (!ctx) return PTENC_ERR_INVALID_ARG;
  switch (option) {
    case PTENC_OPT_SPLITS:
      if (value < 0 || value > PTENC_MAX_SPLITS) return PTENC_ERR_INVALID_ARG;
      ctx->opt_splits = value;
      break;
    case PTENC_OPT_NONTEMPORAL:
      if (value < -1 || value > 1) return PTENC_ERR_INVALID_ARG;
      ctx->opt_nontemporal = value;
      break;
    case PTENC_OPT_ENCODE_PARTS:
      if (value < 0 || value > PT_MAX_ENC_PARTS) return PTENC_ERR_INVALID_ARG;
      ctx->opt_enc_parts = value;
      break;
    case PTENC_OPT_ENCODE_INLINE:
      if (value < -1 || value > 1) return PTENC_ERR_INVALID_ARG;
      ctx->opt_enc_inline = value;
      break;
    case PTENC_OPT_WAVES:
      if (value != 0 && value != 4 && value != 8) return PTENC_ERR_INVALID_ARG;
      ctx->opt_waves = value;
      break;
    case PTENC_OPT_COUNTERS_IN_PLACE:
      if (value != 0 && value != 1) return PTENC_ERR_INVALID_ARG;
      ctx->opt_in_place = value;
      break;
    case PTENC_OPT_FORCE_GENERIC:
      if (value != 0 && value != 1) return PTENC_ERR_INVALID_ARG;
      if (value == 1 && ctx->opt_policy == PTENC_POLICY_SCORED) return PTENC_ERR_UNSUPPORTED;
      ctx->opt_force_generic = value;
      break;
    case PTENC_OPT_EVICT_POLICY:
      if (value != PTENC_POLICY_SLIDING && value != PTENC_POLICY_SCORED) return PTENC_ERR_INVALID_ARG;
      if (value == PTENC_POLICY_SCORED) {
        // the scores are a by-product of the MFMA step kernel, and the selection ranks in LDS
        // (its spare MFMA columns carry the previous step's queries: at most 8 query heads per KV head)
        if (!ctx->dev.tiled || ctx->opt_force_generic || ctx->dev.group > 8) return PTENC_ERR_UNSUPPORTED;
        if (ctx->dev.Wr - resolved_recent(ctx) > PT_SCORED_MAX_ELIGIBLE) return PTENC_ERR_UNSUPPORTED;
      }
      ctx->opt_policy = value;
      ctx->select_stale = 1;
      break;
    case PTENC_OPT_RECENT:
      if (value < -1 || (value >= 0 && value > ctx->dev.Wr - ctx->dev.C)) return PTENC_ERR_INVALID_ARG;
      if (ctx->opt_policy == PTENC_POLICY_SCORED && value >= 0 && ctx->dev.Wr - value > PT_SCORED_MAX_ELIGIBLE)
        return PTENC_ERR_UNSUPPORTED;
      ctx->opt_recent = value;
      break;
    default:
      return PTENC_ERR_INVALID_ARG;
  }
  replan(ctx);
  return PTENC_OK;
}

ptenc_status ptenc_get_plan(ptenc_ctx* ctx, int32_t* attn_kernel, int32_t* n_splits, int32_t* encode_kernel) {
  if (!ctx) return PTENC_ERR_INVALID_ARG;
  if (attn_kernel) *attn_kernel = ctx->attn_kernel;
  if (n_splits) *n_splits = ctx->dev.n_splits;
  if (encode_kernel) *encode_kernel = ctx->encode_kernel;
  return PTENC_OK;
}

ptenc_status ptenc_set_encoder(ptenc_ctx* ctx, const void* d_qg, const void* d_WaQ, const void* d_WaK,
                               const void* d_WaV, const void* d_kg, const void* d_vg, void* stream) {
  if (!ctx || !d_qg || !d_WaQ || !d_WaK || !d_WaV) return PTENC_ERR_INVALID_ARG;
  if ((d_kg == nullptr) != (d_vg == nullptr)) return PTENC_ERR_INVALID_ARG;
  PtDev d = ctx->dev;
  d.WaK = d_WaK; d.WaV = d_WaV;
  hipError_t e = pt_launch_encoder_init(d, d_qg, d_WaQ, d_kg, d_vg, S(stream));
  if (e != hipSuccess) return PTENC_ERR_HIP;
  if (d.tiled) {
    e = pt_launch_pack_weights(d, S(stream));
    if (e != hipSuccess) return PTENC_ERR_HIP;
  }
  ctx->dev = d;
  ctx->encoder_set = 1;
  return PTENC_OK;
}

ptenc_status ptenc_reset(ptenc_ctx* ctx, const uint8_t* d_mask, void* stream) {
  if (!ctx) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  if (!d_mask) ctx->dev.live_ub = 0;        // every ring is empty (a masked reset leaves the other rings as they are)
  return hip_status(pt_launch_reset(ctx->dev, d_mask, d_mask == nullptr, S(stream)));
}

ptenc_status ptenc_prefill(ptenc_ctx* ctx, const void* d_k, const void* d_v, const int32_t* h_prompt_len,
                           int32_t p_max, void* stream) {
  if (!ctx || !d_k || !d_v || !h_prompt_len || p_max < 1) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  for (int b = 0; b < ctx->cfg.batch; ++b)
    if (h_prompt_len[b] < 0 || h_prompt_len[b] > ctx->cfg.n_sink || h_prompt_len[b] > p_max) return PTENC_ERR_INVALID_ARG;
  if (hipMemcpyAsync(ctx->dev.n_prompt, h_prompt_len, sizeof(int) * ctx->cfg.batch, hipMemcpyHostToDevice, S(stream)) !=
      hipSuccess)
    return PTENC_ERR_HIP;
  if (ctx->cfg.n_sink > 0) {
    hipError_t e = pt_launch_prefill(ctx->dev, d_k, d_v, p_max, nullptr, nullptr, 0, S(stream));
    if (e != hipSuccess) return PTENC_ERR_HIP;
  }
  // the host array may be pageable and reused by the caller right after return
  return hip_status(hipStreamSynchronize(S(stream)));
}

ptenc_status ptenc_prefill_ids(ptenc_ctx* ctx, const void* d_k, const void* d_v, const int32_t* d_ids,
                               const int32_t* h_prompt_len, int32_t n, int32_t p_max, void* stream) {
  if (!ctx || n < 0 || n > ctx->cfg.batch) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  if (n == 0) return PTENC_OK;
  if (!d_k || !d_v || !d_ids || !h_prompt_len || p_max < 1) return PTENC_ERR_INVALID_ARG;
  for (int j = 0; j < n; ++j)
    if (h_prompt_len[j] < 0 || h_prompt_len[j] > ctx->cfg.n_sink || h_prompt_len[j] > p_max) return PTENC_ERR_INVALID_ARG;
  if (ctx->cfg.n_sink == 0) return PTENC_OK;            // no reserved slots: every length is 0
  // the lengths travel through the head of the scratch buffer (idle between launches)
  int* d_lens = (int*)ctx->dev.partial;
  if (hipMemcpyAsync(d_lens, h_prompt_len, sizeof(int) * n, hipMemcpyHostToDevice, S(stream)) != hipSuccess)
    return PTENC_ERR_HIP;
  if (pt_launch_prefill(ctx->dev, d_k, d_v, p_max, d_ids, d_lens, n, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  // the host array may be pageable and reused by the caller right after return
  return hip_status(hipStreamSynchronize(S(stream)));
}

ptenc_status ptenc_get_prompt_len(ptenc_ctx* ctx, int32_t* h_prompt_len, void* stream) {
  if (!ctx || !h_prompt_len) return PTENC_ERR_INVALID_ARG;
  if (hipMemcpyAsync(h_prompt_len, ctx->dev.n_prompt, sizeof(int) * ctx->cfg.batch, hipMemcpyDeviceToHost, S(stream)) !=
      hipSuccess)
    return PTENC_ERR_HIP;
  return hip_status(hipStreamSynchronize(S(stream)));
}

ptenc_status ptenc_cache_append(ptenc_ctx* ctx, const void* d_k, const void* d_v, const uint8_t* d_active,
                                void* stream) {
  if (!ctx || !d_k || !d_v) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  if (ctx->attn_kernel == 1 && (((uintptr_t)d_k | (uintptr_t)d_v) & 15)) return PTENC_ERR_INVALID_ARG;
  ctx->select_stale = 1;   // a bare append may fill a ring without choosing its victims
  appended_one(ctx);
  if (ctx->attn_kernel == 1) {
    return advanced(ctx, pt_launch_decode_mfma(ctx->dev, ctx->nontemporal != 0, ctx->waves, false, true, false, nullptr, d_k, d_v,
                                               nullptr, d_active, nullptr, nullptr, 0, ctx->opt_in_place != 0, S(stream)));
  }
  return advanced(ctx, pt_launch_step_prologue(ctx->dev, false, true, d_k, d_v, d_active, nullptr, nullptr, 0,
                                               ctx->opt_in_place != 0, S(stream)));
}

ptenc_status ptenc_evict_encode(ptenc_ctx* ctx, const uint8_t* d_active, void* d_dbg_chunk, void* stream) {
  if (!ctx) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  if (refresh_selection(ctx, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  if (ctx->attn_kernel == 1)
    return advanced(ctx, pt_launch_decode_mfma(ctx->dev, ctx->nontemporal != 0, ctx->waves, true, false, false, nullptr, nullptr,
                                               nullptr, nullptr, d_active, d_dbg_chunk, nullptr, 0, ctx->opt_in_place != 0, S(stream)));
  return advanced(ctx, pt_launch_step_prologue(ctx->dev, true, false, nullptr, nullptr, d_active, d_dbg_chunk,
                                               nullptr, 0, ctx->opt_in_place != 0, S(stream)));
}

ptenc_status ptenc_decode_attn(ptenc_ctx* ctx, const void* d_q, void* d_out, const uint8_t* d_active,
                               void* stream) {
  if (!ctx || !d_q || !d_out) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  if (ctx->attn_kernel == 1) {
    if (((uintptr_t)d_q | (uintptr_t)d_out) & 15) return PTENC_ERR_INVALID_ARG;
    return hip_status(pt_launch_decode_mfma(ctx->dev, ctx->nontemporal != 0, ctx->waves, false, false, true, d_q, nullptr,
                                            nullptr, d_out, d_active, nullptr, nullptr, 0, false, S(stream)));
  }
  return hip_status(pt_launch_attn_generic(ctx->dev, d_q, d_out, d_active, nullptr, 0, S(stream)));
}

ptenc_status ptenc_decode_step(ptenc_ctx* ctx, const void* d_q, const void* d_k, const void* d_v, void* d_out,
                               const uint8_t* d_active, void* stream) {
  if (!ctx || !d_q || !d_k || !d_v || !d_out) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  if (ctx->attn_kernel == 1) {
    if (((uintptr_t)d_q | (uintptr_t)d_out | (uintptr_t)d_k | (uintptr_t)d_v) & 15) return PTENC_ERR_INVALID_ARG;
    if (refresh_selection(ctx, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
    const bool ev = may_evict(ctx);
    appended_one(ctx);
    return advanced(ctx, pt_launch_decode_mfma(ctx->dev, ctx->nontemporal != 0, ctx->waves, ev, true, true, d_q, d_k,
                                               d_v, d_out, d_active, nullptr, nullptr, 0, ctx->opt_in_place != 0, S(stream)));
  }
  appended_one(ctx);
  // small problems are bound by launches: the whole plain step as one (needs the two counter buffers:
  // its attention workgroups read the pair the prologue workgroup does not write)
  if (!ctx->opt_in_place && (long)ctx->cfg.batch * ctx->cfg.n_q_heads * ctx->dev.n_splits <= 2048) {
    if (advanced(ctx, pt_launch_step_generic(ctx->dev, d_q, d_k, d_v, d_out, d_active, S(stream))) != PTENC_OK)
      return PTENC_ERR_HIP;
    return ctx->dev.n_splits > 1 ? hip_status(pt_launch_combine(ctx->dev, d_out, d_active, S(stream))) : PTENC_OK;
  }
  if (advanced(ctx, pt_launch_step_prologue(ctx->dev, true, true, d_k, d_v, d_active, nullptr, nullptr, 0,
                                            ctx->opt_in_place != 0, S(stream))) != PTENC_OK)
    return PTENC_ERR_HIP;
  return ptenc_decode_attn(ctx, d_q, d_out, d_active, stream);
}

// What one step of this context hands between workgroups through the scratch block, with the plan in use:
// the window splits' partial results, then the encoding workgroups' shares of S'.
static size_t step_scratch_bytes(const ptenc_ctx* x, size_t* enc_off) {
  const ptenc_config& c = x->cfg;
  const size_t part = align256((size_t)c.batch * c.n_q_heads * x->dev.n_splits * (c.head_dim + 2) * sizeof(float));
  const size_t enc = align256((size_t)c.batch * x->dev.enc_parts * c.n_global * c.rank * sizeof(float));
  if (enc_off) *enc_off = part;
  return part + enc;
}

ptenc_status ptenc_decode_step_noalloc(ptenc_ctx* ctx, const void* d_q, const void* d_k, const void* d_v, void* d_out,
                                       const uint8_t* d_active, void* stream) {
  if (!ctx || !d_q || !d_k || !d_v || !d_out) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  size_t enc_off = 0;
  if (step_scratch_bytes(ctx, &enc_off) > (size_t)PTENC_NOALLOC_SCRATCH_BYTES) return PTENC_ERR_TOO_LARGE;
  void* sp = nullptr;
  if (builtin_scratch(&sp) != hipSuccess) return PTENC_ERR_HIP;
  // the same step on the built-in block: the kernels take the block's address as they take the caller's
  float* const partial0 = ctx->dev.partial;
  float* const enc0 = ctx->dev.enc_part;
  ctx->dev.partial = (float*)sp;
  ctx->dev.enc_part = (float*)((char*)sp + enc_off);
  const ptenc_status st = ptenc_decode_step(ctx, d_q, d_k, d_v, d_out, d_active, stream);
  ctx->dev.partial = partial0;
  ctx->dev.enc_part = enc0;
  return st;
}

ptenc_status ptenc_decode_step_ids(ptenc_ctx* ctx, const void* d_q, const void* d_k, const void* d_v, void* d_out,
                                   const int32_t* d_ids, int32_t n, void* stream) {
  if (!ctx || n < 0 || n > ctx->cfg.batch) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  if (n == 0) return PTENC_OK;
  if (!d_q || !d_k || !d_v || !d_out || !d_ids) return PTENC_ERR_INVALID_ARG;
  // the plan follows the number of rollouts actually decoded
  PtDev d = ctx->dev;
  d.n_splits = ctx->opt_splits > 0 ? ctx->opt_splits : heuristic_splits(ctx, n);
  if (ctx->attn_kernel == 1) {
    if (((uintptr_t)d_q | (uintptr_t)d_out | (uintptr_t)d_k | (uintptr_t)d_v) & 15) return PTENC_ERR_INVALID_ARG;
    if (refresh_selection(ctx, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
    // listed rollouts advance into the other counter buffer, the rest are carried over to it (or, with
    // counters in place, the rollout's last workgroup writes them where they are)
    // what this launch streams is the listed rollouts' share of the cache: once that fits the memory-side
    // cache, ordinary loads (which allocate there) serve the next step better than non-temporal ones
    bool nt = ctx->nontemporal != 0;
    if (ctx->opt_nontemporal < 0) nt = ctx->cache_bytes / (size_t)ctx->cfg.batch * (size_t)n > ((size_t)192 << 20);
    const bool ev = may_evict(ctx);
    appended_one(ctx);
    return advanced(ctx, pt_launch_decode_mfma(d, nt, pick_waves(ctx, n, d.n_splits), ev, true, true,
                                               d_q, d_k, d_v, d_out, nullptr, nullptr, d_ids, n, ctx->opt_in_place != 0,
                                               S(stream)));
  }
  appended_one(ctx);
  hipError_t e = pt_launch_step_prologue(d, true, true, d_k, d_v, nullptr, nullptr, d_ids, n, true, S(stream));
  if (e != hipSuccess) return PTENC_ERR_HIP;
  return hip_status(pt_launch_attn_generic(d, d_q, d_out, nullptr, d_ids, n, S(stream)));
}

ptenc_status ptenc_decode_run_ids(ptenc_ctx* ctx, const void* d_q, const void* d_k, const void* d_v, void* d_out,
                                  const int32_t* d_ids, const int64_t* h_row_offsets, int64_t n_steps, void* stream) {
  if (!ctx || !h_row_offsets || n_steps < 0 || h_row_offsets[0] != 0) return PTENC_ERR_INVALID_ARG;
  const ptenc_config& c = ctx->cfg;
  for (int64_t t = 0; t < n_steps; ++t) {
    const int64_t n = h_row_offsets[t + 1] - h_row_offsets[t];
    if (n < 0 || n > c.batch) return PTENC_ERR_INVALID_ARG;
  }
  const size_t es = elem_bytes(c.dtype);
  const size_t qb = (size_t)c.n_q_heads * c.head_dim * es, kb = (size_t)c.n_kv_heads * c.head_dim * es;
  for (int64_t t = 0; t < n_steps; ++t) {
    const int64_t r0 = h_row_offsets[t], n = h_row_offsets[t + 1] - r0;
    if (n == 0) continue;
    if (!d_q || !d_k || !d_v || !d_out || !d_ids) return PTENC_ERR_INVALID_ARG;
    ptenc_status st = ptenc_decode_step_ids(ctx, (const char*)d_q + r0 * qb, (const char*)d_k + r0 * kb,
                                            (const char*)d_v + r0 * kb, (char*)d_out + r0 * qb, d_ids + r0, (int32_t)n,
                                            stream);
    if (st != PTENC_OK) return st;
  }
  return PTENC_OK;
}

ptenc_status ptenc_apply_delta(ptenc_ctx* ctx, const void* d_x, const void* d_At, const void* d_Bt, void* d_y,
                               int32_t d_in, int32_t d_out, const uint8_t* d_active, const int32_t* d_ids, int32_t n,
                               void* stream) {
  if (!ctx || !d_x || !d_At || !d_Bt || !d_y || d_in < 1 || d_out < 1) return PTENC_ERR_INVALID_ARG;
  if (d_ids && (n < 0 || n > ctx->cfg.batch)) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  if (d_ids && n == 0) return PTENC_OK;
  return hip_status(pt_launch_apply_delta(ctx->dev, d_x, d_At, d_Bt, d_y, d_in, d_out, d_active, d_ids, n, S(stream)));
}

ptenc_status ptenc_decode_run(ptenc_ctx* ctx, const void* d_q, const void* d_k, const void* d_v, void* d_out,
                              const uint8_t* d_active, int64_t n_steps, void* stream) {
  if (!ctx || n_steps < 0) return PTENC_ERR_INVALID_ARG;
  if (n_steps == 0) return PTENC_OK;          // nothing to do: the buffers may be empty (NULL)
  if (!d_q || !d_k || !d_v || !d_out) return PTENC_ERR_INVALID_ARG;
  const ptenc_config& c = ctx->cfg;
  const size_t es = elem_bytes(c.dtype);
  const size_t qb = (size_t)c.batch * c.n_q_heads * c.head_dim * es;
  const size_t kb = (size_t)c.batch * c.n_kv_heads * c.head_dim * es;
  for (int64_t t = 0; t < n_steps; ++t) {
    ptenc_status st = ptenc_decode_step(ctx, (const char*)d_q + t * qb, (const char*)d_k + t * kb,
                                        (const char*)d_v + t * kb, (char*)d_out + t * qb,
                                        d_active ? d_active + t * c.batch : nullptr, stream);
    if (st != PTENC_OK) return st;
  }
  return PTENC_OK;
}

ptenc_status ptenc_get_counters(ptenc_ctx* ctx, int64_t* h_len, int64_t* h_base, void* stream) {
  if (!ctx || !h_len || !h_base) return PTENC_ERR_INVALID_ARG;
  const size_t n = sizeof(long long) * ctx->cfg.batch;
  if (hipMemcpyAsync(h_len, ctx->dev.len, n, hipMemcpyDeviceToHost, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  if (hipMemcpyAsync(h_base, ctx->dev.base, n, hipMemcpyDeviceToHost, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  return hip_status(hipStreamSynchronize(S(stream)));
}

ptenc_status ptenc_set_counters(ptenc_ctx* ctx, const int64_t* h_len, const int64_t* h_base, void* stream) {
  if (!ctx || !h_len || !h_base) return PTENC_ERR_INVALID_ARG;
  for (int b = 0; b < ctx->cfg.batch; ++b)
    if (h_base[b] < 0 || h_len[b] < h_base[b] || h_len[b] - h_base[b] > ctx->dev.Wr) return PTENC_ERR_INVALID_ARG;
  if (ctx->dev.scored) {
    // live tokens would need scores and position tags that nobody supplies: only empty windows may be re-based
    for (int b = 0; b < ctx->cfg.batch; ++b)
      if (h_len[b] != h_base[b]) return PTENC_ERR_UNSUPPORTED;
    if (hipMemsetAsync(ctx->dev.mtag, 0xff, sizeof(long long) * ctx->cfg.batch * ctx->cfg.n_kv_heads, S(stream)) != hipSuccess)
      return PTENC_ERR_HIP;
    // a choice of victims made for the old contents does not hold for what fills the ring next
    if (hipMemsetAsync(ctx->dev.selected, 0, sizeof(int) * ctx->cfg.batch, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
    ctx->select_stale = 1;
  }
  // whatever was folded ahead of time belongs to the old counters' next chunk
  if (hipMemsetAsync(ctx->dev.enc_done, 0, sizeof(int) * ctx->cfg.batch, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  if (hipMemsetAsync(ctx->dev.pend, 0, sizeof(float) * ctx->cfg.batch * ctx->cfg.n_global * ctx->cfg.rank, S(stream)) != hipSuccess)
    return PTENC_ERR_HIP;
  ctx->dev.live_ub = 0;
  for (int b = 0; b < ctx->cfg.batch; ++b)
    if (h_len[b] - h_base[b] > ctx->dev.live_ub) ctx->dev.live_ub = h_len[b] - h_base[b];
  const size_t n = sizeof(long long) * ctx->cfg.batch;
  if (hipMemcpyAsync(ctx->dev.len, h_len, n, hipMemcpyHostToDevice, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  if (hipMemcpyAsync(ctx->dev.base, h_base, n, hipMemcpyHostToDevice, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  // the other buffer too: a compact-list step merges into it by maximum, and the new values may be lower
  if (hipMemcpyAsync(ctx->dev.len_nx, h_len, n, hipMemcpyHostToDevice, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  if (hipMemcpyAsync(ctx->dev.base_nx, h_base, n, hipMemcpyHostToDevice, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  // the host arrays may be pageable and reused by the caller right after return
  return hip_status(hipStreamSynchronize(S(stream)));
}

ptenc_status ptenc_get_state(ptenc_ctx* ctx, float* h_S, void* stream) {
  if (!ctx || !h_S) return PTENC_ERR_INVALID_ARG;
  const size_t n = sizeof(float) * ctx->cfg.batch * ctx->cfg.n_global * ctx->cfg.rank;
  if (hipMemcpyAsync(h_S, ctx->dev.S, n, hipMemcpyDeviceToHost, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  return hip_status(hipStreamSynchronize(S(stream)));
}

ptenc_status ptenc_set_state(ptenc_ctx* ctx, const float* h_S, void* stream) {
  if (!ctx || !h_S) return PTENC_ERR_INVALID_ARG;
  const size_t n = sizeof(float) * ctx->cfg.batch * ctx->cfg.n_global * ctx->cfg.rank;
  if (hipMemcpyAsync(ctx->dev.S, h_S, n, hipMemcpyHostToDevice, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  return hip_status(hipStreamSynchronize(S(stream)));
}

ptenc_status ptenc_get_encoder_state(ptenc_ctx* ctx, float* h_Qa, float* h_S0, void* stream) {
  if (!ctx) return PTENC_ERR_INVALID_ARG;
  if (!ctx->encoder_set) return PTENC_ERR_STATE;
  const size_t n = sizeof(float) * ctx->cfg.n_global * ctx->cfg.rank;
  if (h_Qa && hipMemcpyAsync(h_Qa, ctx->dev.Qa, n, hipMemcpyDeviceToHost, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  if (h_S0 && hipMemcpyAsync(h_S0, ctx->dev.S0, n, hipMemcpyDeviceToHost, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  return hip_status(hipStreamSynchronize(S(stream)));
}

ptenc_status ptenc_get_scores(ptenc_ctx* ctx, float* d_score, int64_t* d_pos, void* stream) {
  if (!ctx || (!d_score && !d_pos)) return PTENC_ERR_INVALID_ARG;
  if (!ctx->dev.scored) return PTENC_ERR_STATE;
  return hip_status(pt_launch_scores_get(ctx->dev, d_score, (long long*)d_pos, S(stream)));
}

ptenc_status ptenc_set_scores(ptenc_ctx* ctx, const float* d_score, void* stream) {
  if (!ctx || !d_score) return PTENC_ERR_INVALID_ARG;
  if (!ctx->dev.scored) return PTENC_ERR_STATE;
  ctx->select_stale = 1;
  return hip_status(pt_launch_scores_set(ctx->dev, d_score, S(stream)));
}

ptenc_status ptenc_get_victims(ptenc_ctx* ctx, int64_t* h_pos, void* stream) {
  if (!ctx || !h_pos) return PTENC_ERR_INVALID_ARG;
  if (!ctx->dev.scored) return PTENC_ERR_STATE;
  const size_t n = sizeof(long long) * ctx->cfg.batch * ctx->cfg.chunk;
  if (hipMemcpyAsync(h_pos, ctx->dev.victims, n, hipMemcpyDeviceToHost, S(stream)) != hipSuccess) return PTENC_ERR_HIP;
  return hip_status(hipStreamSynchronize(S(stream)));
}

ptenc_status ptenc_gather_window(ptenc_ctx* ctx, void* d_K, void* d_V, void* stream) {
  if (!ctx || !d_K || !d_V) return PTENC_ERR_INVALID_ARG;
  return hip_status(pt_launch_gather(ctx->dev, d_K, d_V, S(stream)));
}

ptenc_status ptenc_cache_offset(ptenc_ctx* ctx, int32_t b, int32_t h, int32_t slot, int32_t i, int32_t which,
                                size_t* elem_offset) {
  if (!ctx || !elem_offset) return PTENC_ERR_INVALID_ARG;
  const ptenc_config& c = ctx->cfg;
  if (b < 0 || b >= c.batch || h < 0 || h >= c.n_kv_heads || slot < 0 || slot >= c.window || i < 0 ||
      i >= c.head_dim || (which != 0 && which != 1))
    return PTENC_ERR_INVALID_ARG;
  const size_t slab = (size_t)(b * c.n_kv_heads + h) * pt_slab_elems(c.window, c.head_dim);
  *elem_offset = slab + (which == 0 ? pt_k_off(ctx->dev.tiled, c.window, c.head_dim, slot, i)
                                    : pt_v_off(ctx->dev.tiled, c.window, c.head_dim, slot, i));
  return PTENC_OK;
}

ptenc_status ptenc_poll_error(ptenc_ctx* ctx, int32_t* h_flags, void* stream) {
  if (!ctx || !h_flags) return PTENC_ERR_INVALID_ARG;
  if (hipMemcpyAsync(h_flags, ctx->dev.err, sizeof(int), hipMemcpyDeviceToHost, S(stream)) != hipSuccess)
    return PTENC_ERR_HIP;
  return hip_status(hipStreamSynchronize(S(stream)));
}

const char* ptenc_status_string(ptenc_status s) {
  switch (s) {
    case PTENC_OK: return "ok";
    case PTENC_ERR_INVALID_ARG: return "invalid argument";
    case PTENC_ERR_STATE: return "call out of order (encoder not set)";
    case PTENC_ERR_UNSUPPORTED: return "unsupported configuration";
    case PTENC_ERR_HIP: return "HIP runtime error";
    case PTENC_ERR_NOMEM: return "out of host memory";
    case PTENC_ERR_TOO_LARGE: return "the configuration needs more scratch than the built-in block holds";
  }
  return "unknown status";
}

}  // extern "C"
