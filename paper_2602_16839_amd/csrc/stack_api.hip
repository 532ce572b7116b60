// Multi-layer driver: L attention layers of one model decoding the same B rollouts, one context
// per layer over slices of three caller-owned buffers, and one decode step of the whole stack
// either as L launches or as a replay of a HIP graph that holds them.
//
// Every layer keeps its own bounded cache, counters and context state (the paper's models have
// one KV cache and one adapted projection per layer: Experimental Setup, Models); the
// layers of a step run one after another on one stream, so they share a single scratch buffer.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "ptenc.h"
#include "ptenc_internal.h"

// A step reads one pair of counter buffers and writes the other, and the host swaps their roles after
// every step; a recorded step has its pair frozen in.  So the stack records the step twice, once for
// either assignment, and a replay takes the recording that matches the layers' current one: replays and
// eager steps can then be mixed freely and no step needs its counters updated in place.
struct ptenc_stack {
  std::vector<ptenc_ctx*> layers;
  hipStream_t capture_stream = nullptr;
  hipGraph_t graph[2] = {nullptr, nullptr};          // by parity of the layers' swap count when the step starts
  hipGraphExec_t exec[2] = {nullptr, nullptr};
};

namespace {

void drop_graph(ptenc_stack* s) {
  for (int p = 0; p < 2; ++p) {
    if (s->exec[p]) { (void)hipGraphExecDestroy(s->exec[p]); s->exec[p] = nullptr; }
    if (s->graph[p]) { (void)hipGraphDestroy(s->graph[p]); s->graph[p] = nullptr; }
  }
}

// the layers' common swap parity, or -1 if a layer was stepped on its own and they disagree
int common_parity(const ptenc_stack* s) {
  const int p = s->layers[0]->swaps & 1;
  for (const ptenc_ctx* x : s->layers)
    if ((x->swaps & 1) != p) return -1;
  return p;
}

ptenc_status launch_layers(ptenc_stack* s, const void* const* h_q, const void* const* h_k, const void* const* h_v,
                           void* const* h_out, const uint8_t* d_active, void* stream) {
  for (size_t l = 0; l < s->layers.size(); ++l) {
    ptenc_status st = ptenc_decode_step(s->layers[l], h_q[l], h_k[l], h_v[l], h_out[l], d_active, stream);
    if (st != PTENC_OK) return st;
  }
  return PTENC_OK;
}

}  // namespace

extern "C" {

ptenc_status ptenc_stack_query_sizes(const ptenc_config* cfg, int32_t n_layers, size_t* cache_bytes,
                                     size_t* state_bytes, size_t* scratch_bytes) {
  if (n_layers < 1 || n_layers > PTENC_MAX_LAYERS) return PTENC_ERR_INVALID_ARG;
  size_t cb = 0, sb = 0, xb = 0;
  ptenc_status st = ptenc_query_sizes(cfg, &cb, &sb, &xb);
  if (st != PTENC_OK) return st;
  if (cache_bytes) *cache_bytes = cb * (size_t)n_layers;
  if (state_bytes) *state_bytes = sb * (size_t)n_layers;
  if (scratch_bytes) *scratch_bytes = xb;
  return PTENC_OK;
}

ptenc_status ptenc_stack_create(const ptenc_config* cfg, int32_t n_layers, void* d_cache, void* d_state,
                                void* d_scratch, ptenc_stack** out) {
  if (!out) return PTENC_ERR_INVALID_ARG;
  *out = nullptr;
  size_t cb = 0, sb = 0, xb = 0;
  ptenc_status st = ptenc_stack_query_sizes(cfg, n_layers, &cb, &sb, &xb);
  if (st != PTENC_OK) return st;
  cb /= (size_t)n_layers;
  sb /= (size_t)n_layers;
  ptenc_stack* s = new (std::nothrow) ptenc_stack;
  if (!s) return PTENC_ERR_NOMEM;
  for (int l = 0; l < n_layers; ++l) {
    ptenc_ctx* x = nullptr;
    st = ptenc_create(cfg, (char*)d_cache + cb * l, (char*)d_state + sb * l, d_scratch, &x);
    // the layers' caches together decide whether the memory-side cache can hold the stream
    if (st == PTENC_OK && cb * (size_t)n_layers > ((size_t)192 << 20)) st = ptenc_set_option(x, PTENC_OPT_NONTEMPORAL, 1);
    if (x) s->layers.push_back(x);
    if (st != PTENC_OK) {
      (void)ptenc_stack_destroy(s);
      return st;
    }
  }
  *out = s;
  return PTENC_OK;
}

ptenc_status ptenc_stack_destroy(ptenc_stack* s) {
  if (!s) return PTENC_ERR_INVALID_ARG;
  drop_graph(s);
  if (s->capture_stream) (void)hipStreamDestroy(s->capture_stream);
  for (ptenc_ctx* x : s->layers) (void)ptenc_destroy(x);
  delete s;
  return PTENC_OK;
}

ptenc_status ptenc_stack_layer(ptenc_stack* s, int32_t layer, ptenc_ctx** out) {
  if (!s || !out || layer < 0 || (size_t)layer >= s->layers.size()) return PTENC_ERR_INVALID_ARG;
  *out = s->layers[layer];
  return PTENC_OK;
}

ptenc_status ptenc_stack_reset(ptenc_stack* s, const uint8_t* d_mask, void* stream) {
  if (!s) return PTENC_ERR_INVALID_ARG;
  for (ptenc_ctx* x : s->layers) {
    ptenc_status st = ptenc_reset(x, d_mask, stream);
    if (st != PTENC_OK) return st;
  }
  return PTENC_OK;
}

ptenc_status ptenc_stack_decode_step(ptenc_stack* s, const void* const* h_q, const void* const* h_k,
                                     const void* const* h_v, void* const* h_out, const uint8_t* d_active,
                                     void* stream) {
  if (!s || !h_q || !h_k || !h_v || !h_out) return PTENC_ERR_INVALID_ARG;
  return launch_layers(s, h_q, h_k, h_v, h_out, d_active, stream);
}

ptenc_status ptenc_stack_graph_capture(ptenc_stack* s, const void* const* h_q, const void* const* h_k,
                                       const void* const* h_v, void* const* h_out, const uint8_t* d_active) {
  if (!s || !h_q || !h_k || !h_v || !h_out) return PTENC_ERR_INVALID_ARG;
  for (size_t l = 0; l < s->layers.size(); ++l) {
    if (!h_q[l] || !h_k[l] || !h_v[l] || !h_out[l]) return PTENC_ERR_INVALID_ARG;
    if (!s->layers[l]->encoder_set) return PTENC_ERR_STATE;
  }
  drop_graph(s);
  const int p0 = common_parity(s);
  if (p0 < 0) return PTENC_ERR_STATE;
  // a stream of the library's own (default priority) records the launches; nothing runs on it
  if (!s->capture_stream && hipStreamCreateWithFlags(&s->capture_stream, hipStreamNonBlocking) != hipSuccess)
    return PTENC_ERR_HIP;
  // (a pending stand-alone choice of victims stays pending: a recording runs nothing, so it must not
  // take the request away, and a replay sees to it before the recorded step)
  std::vector<int> stale(s->layers.size());
  for (size_t l = 0; l < s->layers.size(); ++l) {
    pt_ctx_assume_full(s->layers[l]);
    stale[l] = s->layers[l]->select_stale;
    s->layers[l]->select_stale = 0;
  }
  auto restore_stale = [&]() {
    for (size_t l = 0; l < s->layers.size(); ++l) s->layers[l]->select_stale = stale[l];
  };
  // two recordings: the step as it would run now, and as it would run after it (each recording swaps the
  // host's buffer roles like a real step does, so after both the layers are as they were)
  for (int rec = 0; rec < 2; ++rec) {
    const int p = p0 ^ rec;
    if (hipStreamBeginCapture(s->capture_stream, hipStreamCaptureModeThreadLocal) != hipSuccess) {
      drop_graph(s);
      restore_stale();
      return PTENC_ERR_HIP;
    }
    ptenc_status st = launch_layers(s, h_q, h_k, h_v, h_out, d_active, s->capture_stream);
    hipGraph_t g = nullptr;
    hipError_t e = hipStreamEndCapture(s->capture_stream, &g);   // always ends the capture
    if (st != PTENC_OK || e != hipSuccess || !g) {
      if (g) (void)hipGraphDestroy(g);
      // layers that were launched have swapped: bring everybody back to the starting assignment
      for (ptenc_ctx* x : s->layers)
        if ((x->swaps & 1) != p0) pt_ctx_stepped_by_replay(x);
      drop_graph(s);
      restore_stale();
      return st != PTENC_OK ? st : PTENC_ERR_HIP;
    }
    s->graph[p] = g;
    if (hipGraphInstantiate(&s->exec[p], g, nullptr, nullptr, 0) != hipSuccess) {
      s->exec[p] = nullptr;
      for (ptenc_ctx* x : s->layers)
        if ((x->swaps & 1) != p0) pt_ctx_stepped_by_replay(x);
      drop_graph(s);
      restore_stale();
      return PTENC_ERR_HIP;
    }
  }
  restore_stale();
  return PTENC_OK;
}

ptenc_status ptenc_stack_graph_launch(ptenc_stack* s, void* stream) {
  if (!s) return PTENC_ERR_INVALID_ARG;
  const int p = common_parity(s);
  if (p < 0 || !s->exec[p]) return PTENC_ERR_STATE;
  for (ptenc_ctx* x : s->layers)
    if (pt_ctx_refresh_selection(x, (hipStream_t)stream) != hipSuccess) return PTENC_ERR_HIP;
  if (hipGraphLaunch(s->exec[p], (hipStream_t)stream) != hipSuccess) return PTENC_ERR_HIP;
  for (ptenc_ctx* x : s->layers) pt_ctx_stepped_by_replay(x);
  return PTENC_OK;
}

}  // extern "C"
