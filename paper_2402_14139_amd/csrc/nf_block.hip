// Block-level entry points of libnf (include/nf.h): the Worker loop of Algorithm 2 over the
// batches and layers of one block, and the forward-only sweep that fills the next block's
// activation cache (NeuroFlux, arXiv 2402.14139, "Efficient Forward Propagation via Prefetching
// and Adaptive Batching").  Host code only: every step is one of the single-layer entry points
// (nf_cache_read, nf_local_step, nf_layer_fwd, nf_cache_write) enqueued in the paper's order.
// Everything is validated before the first enqueue.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <mutex>
#include <vector>

#include "../../include/nf.h"

namespace nf {
bool prof_active();  // nf_api.hip: true between nf_prof_begin and nf_prof_end
}

// One captured block pass (nf_block_graph_create): the instantiated graph and the device it lives on.
struct nf_block_graph {
  hipGraphExec_t exec;
  int device;
};

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct BlockPlan {
  std::vector<size_t> y_off;  // emitted batch of every layer
  std::vector<int64_t> y_elems;
  size_t xin_off[2], lab_off[2];
  size_t layer_ws_off, layer_ws_bytes;
  size_t total;
  int64_t se_in, se_out;
};

// Shapes, chaining and shortcut wiring of the block, and its workspace plan at batch size B.
// mode: what the caller is going to run -- forward sweeps only, training passes (heads with
// gradient buffers), or early-exit evaluation (heads without gradient buffers).
enum PlanMode { PLAN_FWD = 0, PLAN_TRAIN = 1, PLAN_EVAL = 2 };
int32_t plan_block(const nf_block *blk, int32_t B, int32_t B_last, PlanMode mode, BlockPlan *pl) {
  if (!blk) return NF_ERR_NULL;
  if (blk->n_layers <= 0 || blk->n_layers > 1024) return NF_ERR_BAD_DESC;
  if (!blk->layers || !blk->p) return NF_ERR_NULL;
  const bool train = mode == PLAN_TRAIN, heads = mode != PLAN_FWD;
  if (heads && (!blk->aux || !blk->ap)) return NF_ERR_NULL;
  if (train && (!blk->gp || !blk->ga)) return NF_ERR_NULL;
  if (B <= 0 || B > 65535 || B_last <= 0 || B_last > B) return NF_ERR_BAD_DESC;
  const int n = blk->n_layers;
  pl->y_off.assign(n, 0);
  pl->y_elems.assign(n, 0);
  size_t off = 0, lws = 0;
  const nf_layer_desc &d0 = blk->layers[0];
  pl->se_in = (int64_t)d0.C_in * d0.H_in * d0.W_in;
  if (pl->se_in <= 0) return NF_ERR_BAD_DESC;
  for (int b = 0; b < 2; ++b) {
    pl->xin_off[b] = off, off += up((size_t)B * pl->se_in * sizeof(float));
    pl->lab_off[b] = off, off += up((size_t)B * sizeof(int32_t));
  }
  for (int l = 0; l < n; ++l) {
    const nf_layer_desc *d = &blk->layers[l];
    const nf_aux_desc *a = heads ? &blk->aux[l] : nullptr;
    int32_t Hp = 0, Wp = 0;
    int32_t rc = nf_layer_out_dims(d, nullptr, nullptr, &Hp, &Wp);
    if (rc) return rc;
    size_t need = 0, need_last = 0;
    if ((rc = nf_workspace_bytes(d, a, B, &need))) return rc;
    if ((rc = nf_workspace_bytes(d, a, B_last, &need_last))) return rc;
    lws = std::max(lws, std::max(need, need_last));
    if (l > 0) {
      const nf_layer_desc &q = blk->layers[l - 1];
      int32_t qh = 0, qw = 0;
      (void)nf_layer_out_dims(&q, nullptr, nullptr, &qh, &qw);
      if (d->C_in != q.C_out || d->H_in != qh || d->W_in != qw) return NF_ERR_BAD_DESC;
    }
    const int src = blk->skip_src ? blk->skip_src[l] : -1;
    if (d->skip_kind != 0) {
      if (src < 0 || src > l) return NF_ERR_BAD_DESC;
      const nf_layer_desc &q = blk->layers[src];  // the shortcut is this layer's input tensor
      if (d->skip_C != q.C_in || d->skip_H != q.H_in || d->skip_W != q.W_in) return NF_ERR_BAD_DESC;
    }
    // parameter pointers
    const nf_layer_params &p = blk->p[l];
    if (!p.W || !p.b || (d->skip_kind == 2 && !p.Wp)) return NF_ERR_NULL;
    if (!aligned16(p.W) || !aligned16(p.b) || (d->skip_kind == 2 && !aligned16(p.Wp))) return NF_ERR_BAD_DESC;
    // every pointer a per-layer call would reject is rejected here, before anything is enqueued
    if (heads) {
      const nf_aux_params &s = blk->ap[l];
      if (!s.Wa || !s.ba || !s.Wf || !s.bf) return NF_ERR_NULL;
      if (!aligned16(s.Wa) || !aligned16(s.ba) || !aligned16(s.Wf) || !aligned16(s.bf)) return NF_ERR_BAD_DESC;
    }
    if (train) {
      const nf_layer_params &g = blk->gp[l];
      const nf_aux_params &s = blk->ga[l];
      if (!g.W || !g.b || (d->skip_kind == 2 && !g.Wp)) return NF_ERR_NULL;
      if (!s.Wa || !s.ba || !s.Wf || !s.bf) return NF_ERR_NULL;
      if (!aligned16(g.W) || !aligned16(g.b) || (d->skip_kind == 2 && !aligned16(g.Wp))) return NF_ERR_BAD_DESC;
      if (!aligned16(s.Wa) || !aligned16(s.ba) || !aligned16(s.Wf) || !aligned16(s.bf)) return NF_ERR_BAD_DESC;
    }
    pl->y_elems[l] = (int64_t)d->C_out * Hp * Wp;
    pl->y_off[l] = off, off += up((size_t)B * pl->y_elems[l] * sizeof(float));
  }
  pl->se_out = pl->y_elems[n - 1];
  pl->layer_ws_off = off, pl->layer_ws_bytes = lws, off += up(lws);
  pl->total = off;
  return NF_OK;
}

inline float *at(void *ws, size_t off) { return reinterpret_cast<float *>(static_cast<char *>(ws) + off); }

// Input tensor of layer l inside the block for the batch held in double-buffer slot `slot`.
inline const float *input_of(const BlockPlan &pl, void *ws, int l, int slot) {
  return l == 0 ? at(ws, pl.xin_off[slot]) : at(ws, pl.y_off[l - 1]);
}

// Four events per device for the prefetch hand-shake, created once and kept for the process.
struct PrefetchEvents {
  hipEvent_t fork, ready[2], done[2];
};
std::mutex g_ev_mutex;
std::vector<std::pair<int, PrefetchEvents>> g_ev;

int32_t prefetch_events(PrefetchEvents *out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return NF_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_ev_mutex);
  for (auto &e : g_ev)
    if (e.first == dev) return *out = e.second, NF_OK;
  PrefetchEvents pe;
  hipEvent_t *all[5] = {&pe.fork, &pe.ready[0], &pe.ready[1], &pe.done[0], &pe.done[1]};
  for (hipEvent_t *e : all)
    if (hipEventCreateWithFlags(e, hipEventDisableTiming) != hipSuccess) return NF_ERR_DEVICE;
  g_ev.emplace_back(dev, pe);
  *out = pe;
  return NF_OK;
}

#define NF_HIP(call) \
  if ((call) != hipSuccess) return NF_ERR_DEVICE

}  // namespace

extern "C" {

int32_t nf_block_workspace_bytes(const nf_block *blk, int32_t B, size_t *out) {
  if (!out) return NF_ERR_NULL;
  BlockPlan pl;
  // the heads are part of the plan whenever the block carries them
  const PlanMode mode = (blk && blk->aux && blk->ap) ? ((blk->gp && blk->ga) ? PLAN_TRAIN : PLAN_EVAL) : PLAN_FWD;
  const int32_t rc = plan_block(blk, B, B, mode, &pl);
  if (rc) return rc;
  *out = pl.total;
  return NF_OK;
}

int32_t nf_block_train_epoch(const nf_block *blk, const nf_sgd_desc *s, int32_t B, int64_t n_items,
                             const float *cache, const int32_t *cache_labels, int64_t capacity,
                             const int64_t *idx, float *losses, void *ws, size_t ws_bytes, void *stream,
                             void *prefetch_stream) {
  if (!blk || !s || !cache || !cache_labels || !losses) return NF_ERR_NULL;
  if (n_items <= 0 || capacity <= 0 || B <= 0) return NF_ERR_BAD_DESC;
  if (!idx && n_items > capacity) return NF_ERR_CACHE_RANGE;
  const int64_t n_batches = (n_items + B - 1) / B;
  const int32_t B_last = (int32_t)(n_items - (n_batches - 1) * B);
  BlockPlan pl;
  int32_t rc = plan_block(blk, B, B_last, PLAN_TRAIN, &pl);
  if (rc) return rc;
  if (s->momentum != 0.f) {
    if (!blk->vp || !blk->va) return NF_ERR_NULL;
    for (int l = 0; l < blk->n_layers; ++l) {
      const nf_layer_params &v = blk->vp[l];
      const nf_aux_params &u = blk->va[l];
      if (!v.W || !v.b || (blk->layers[l].skip_kind == 2 && !v.Wp) || !u.Wa || !u.ba || !u.Wf || !u.bf)
        return NF_ERR_NULL;
      if (!aligned16(v.W) || !aligned16(v.b) || (blk->layers[l].skip_kind == 2 && !aligned16(v.Wp)) ||
          !aligned16(u.Wa) || !aligned16(u.ba) || !aligned16(u.Wf) || !aligned16(u.bf))
        return NF_ERR_BAD_DESC;
    }
  }
  if (!aligned16(cache)) return NF_ERR_BAD_DESC;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & (ALIGN - 1)) || ws_bytes < pl.total) return NF_ERR_WORKSPACE;
  if (prefetch_stream == stream) prefetch_stream = nullptr;

  hipStream_t st = static_cast<hipStream_t>(stream), pf = static_cast<hipStream_t>(prefetch_stream);
  PrefetchEvents ev;
  if (pf) {
    if ((rc = prefetch_events(&ev))) return rc;
    NF_HIP(hipEventRecord(ev.fork, st));  // the cache may have been produced on `stream`
    NF_HIP(hipStreamWaitEvent(pf, ev.fork, 0));
  }
  // A HIP error after the fork: whatever was enqueued on the prefetch stream is joined back into
  // `stream` before the call returns, so that `stream` alone still orders everything the call did.
  auto fail = [&](int32_t code) -> int32_t {
    if (pf && hipEventRecord(ev.ready[0], pf) == hipSuccess) (void)hipStreamWaitEvent(st, ev.ready[0], 0);
    return code;
  };
  auto read_batch = [&](int64_t j, hipStream_t on) -> int32_t {
    const int slot = (int)(j & 1);
    const int32_t nb = j == n_batches - 1 ? B_last : B;
    return nf_cache_read(cache, cache_labels, capacity, pl.se_in, idx ? 0 : j * B, idx ? idx + j * B : nullptr, nb,
                         at(ws, pl.xin_off[slot]), reinterpret_cast<int32_t *>(at(ws, pl.lab_off[slot])), on);
  };
  if (pf) {
    if ((rc = read_batch(0, pf))) return fail(rc);
    if (hipEventRecord(ev.ready[0], pf) != hipSuccess) return fail(NF_ERR_DEVICE);
  }
  const int n = blk->n_layers;
  for (int64_t j = 0; j < n_batches; ++j) {
    const int slot = (int)(j & 1);
    const int32_t nb = j == n_batches - 1 ? B_last : B;
    if (pf) {
      if (j + 1 < n_batches) {
        // slot of batch j+1 was last used by batch j-1
        if (j >= 1 && hipStreamWaitEvent(pf, ev.done[slot ^ 1], 0) != hipSuccess) return fail(NF_ERR_DEVICE);
        if ((rc = read_batch(j + 1, pf))) return fail(rc);
        if (hipEventRecord(ev.ready[slot ^ 1], pf) != hipSuccess) return fail(NF_ERR_DEVICE);
      }
      if (hipStreamWaitEvent(st, ev.ready[slot], 0) != hipSuccess) return fail(NF_ERR_DEVICE);
    } else {
      if ((rc = read_batch(j, st))) return fail(rc);
    }
    const int32_t *lab = reinterpret_cast<const int32_t *>(at(ws, pl.lab_off[slot]));
    for (int l = 0; l < n; ++l) {
      const nf_layer_desc *d = &blk->layers[l];
      const float *x = input_of(pl, ws, l, slot);
      const float *xs = d->skip_kind ? input_of(pl, ws, blk->skip_src[l], slot) : nullptr;
      rc = nf_local_step(d, &blk->aux[l], s, nb, x, xs, lab, &blk->p[l], &blk->ap[l], &blk->gp[l], &blk->ga[l],
                         blk->vp ? &blk->vp[l] : nullptr, blk->va ? &blk->va[l] : nullptr, at(ws, pl.y_off[l]),
                         losses + j * n + l, at(ws, pl.layer_ws_off), pl.layer_ws_bytes, st);
      if (rc) return fail(rc);
    }
    if (pf && j + 2 < n_batches && hipEventRecord(ev.done[slot], st) != hipSuccess) return fail(NF_ERR_DEVICE);
  }
  return NF_OK;
}

int32_t nf_block_graph_create(const nf_block *blk, const nf_sgd_desc *s, int32_t B, int64_t n_items,
                              const float *cache, const int32_t *cache_labels, int64_t capacity,
                              const int64_t *idx, float *losses, void *ws, size_t ws_bytes, nf_block_graph **out) {
  if (!out) return NF_ERR_NULL;
  *out = nullptr;
  // event pairs around every launch cannot be part of a graph
  if (nf::prof_active()) return NF_ERR_UNSUPPORTED;
  int dev = 0;
  NF_HIP(hipGetDevice(&dev));
  // a stream of its own for the capture (default priority), gone again before the call returns
  hipStream_t cs = nullptr;
  NF_HIP(hipStreamCreateWithFlags(&cs, hipStreamNonBlocking));
  if (hipStreamBeginCapture(cs, hipStreamCaptureModeThreadLocal) != hipSuccess) {
    (void)hipStreamDestroy(cs);
    return NF_ERR_DEVICE;
  }
  // validation happens in here, before the first enqueue: an argument error leaves an empty capture
  const int32_t rc = nf_block_train_epoch(blk, s, B, n_items, cache, cache_labels, capacity, idx, losses, ws, ws_bytes,
                                          cs, nullptr);
  hipGraph_t graph = nullptr;
  const hipError_t ec = hipStreamEndCapture(cs, &graph);  // always: a stream must not be left capturing
  (void)hipStreamDestroy(cs);
  if (rc != NF_OK || ec != hipSuccess || !graph) {
    if (graph) (void)hipGraphDestroy(graph);
    return rc != NF_OK ? rc : NF_ERR_DEVICE;
  }
  hipGraphExec_t exec = nullptr;
  const hipError_t ei = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (ei != hipSuccess || !exec) return NF_ERR_DEVICE;
  *out = new nf_block_graph{exec, dev};
  return NF_OK;
}

int32_t nf_block_graph_launch(nf_block_graph *g, void *stream) {
  if (!g) return NF_ERR_NULL;
  int dev = 0;
  NF_HIP(hipGetDevice(&dev));
  if (dev != g->device) return NF_ERR_BAD_DESC;
  NF_HIP(hipGraphLaunch(g->exec, static_cast<hipStream_t>(stream)));
  return NF_OK;
}

int32_t nf_block_graph_destroy(nf_block_graph *g) {
  if (!g) return NF_OK;
  const hipError_t e = hipGraphExecDestroy(g->exec);
  delete g;
  return e == hipSuccess ? NF_OK : NF_ERR_DEVICE;
}

int32_t nf_block_fill_cache(const nf_block *blk, int32_t B, int64_t n_items, const float *cache_in,
                            const int32_t *labels_in, int64_t capacity_in, float *cache_out, int32_t *labels_out,
                            int64_t capacity_out, void *ws, size_t ws_bytes, void *stream) {
  if (!blk || !cache_in || !labels_in || !cache_out || !labels_out) return NF_ERR_NULL;
  if (n_items <= 0 || capacity_in <= 0 || capacity_out <= 0 || B <= 0) return NF_ERR_BAD_DESC;
  if (n_items > capacity_in || n_items > capacity_out) return NF_ERR_CACHE_RANGE;
  const int64_t n_batches = (n_items + B - 1) / B;
  const int32_t B_last = (int32_t)(n_items - (n_batches - 1) * B);
  BlockPlan pl;
  int32_t rc = plan_block(blk, B, B_last, PLAN_FWD, &pl);
  if (rc) return rc;
  if (!aligned16(cache_in) || !aligned16(cache_out)) return NF_ERR_BAD_DESC;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & (ALIGN - 1)) || ws_bytes < pl.total) return NF_ERR_WORKSPACE;
  const int n = blk->n_layers;
  for (int64_t j = 0; j < n_batches; ++j) {
    const int32_t nb = j == n_batches - 1 ? B_last : B;
    int32_t *lab = reinterpret_cast<int32_t *>(at(ws, pl.lab_off[0]));
    if ((rc = nf_cache_read(cache_in, labels_in, capacity_in, pl.se_in, j * B, nullptr, nb, at(ws, pl.xin_off[0]), lab,
                            stream)))
      return rc;
    for (int l = 0; l < n; ++l) {
      const nf_layer_desc *d = &blk->layers[l];
      const float *xs = d->skip_kind ? input_of(pl, ws, blk->skip_src[l], 0) : nullptr;
      if ((rc = nf_layer_fwd(d, nb, input_of(pl, ws, l, 0), xs, &blk->p[l], at(ws, pl.y_off[l]),
                             at(ws, pl.layer_ws_off), pl.layer_ws_bytes, stream)))
        return rc;
    }
    if ((rc = nf_cache_write(cache_out, labels_out, capacity_out, pl.se_out, j * B, nb, at(ws, pl.y_off[n - 1]), lab,
                             stream)))
      return rc;
  }
  return NF_OK;
}

int32_t nf_block_evaluate(const nf_block *blk, int32_t exit_layer, int32_t B, int64_t n_items, const float *cache,
                          const int32_t *cache_labels, int64_t capacity, int32_t *pred_out, int32_t *n_correct,
                          void *ws, size_t ws_bytes, void *stream) {
  if (!blk || !cache || !pred_out) return NF_ERR_NULL;
  if ((cache_labels == nullptr) != (n_correct == nullptr)) return NF_ERR_NULL;  // both, or plain prediction
  if (n_items <= 0 || capacity <= 0 || B <= 0) return NF_ERR_BAD_DESC;
  if (n_items > capacity) return NF_ERR_CACHE_RANGE;
  if (exit_layer < 0 || exit_layer >= blk->n_layers) return NF_ERR_BAD_DESC;
  const int64_t n_batches = (n_items + B - 1) / B;
  const int32_t B_last = (int32_t)(n_items - (n_batches - 1) * B);
  BlockPlan pl;
  int32_t rc = plan_block(blk, B, B_last, PLAN_EVAL, &pl);
  if (rc) return rc;
  if (!aligned16(cache)) return NF_ERR_BAD_DESC;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & (ALIGN - 1)) || ws_bytes < pl.total) return NF_ERR_WORKSPACE;
  for (int64_t j = 0; j < n_batches; ++j) {
    const int32_t nb = j == n_batches - 1 ? B_last : B;
    int32_t *lab = cache_labels ? reinterpret_cast<int32_t *>(at(ws, pl.lab_off[0])) : nullptr;
    if ((rc = nf_cache_read(cache, cache_labels, capacity, pl.se_in, j * B, nullptr, nb, at(ws, pl.xin_off[0]), lab,
                            stream)))
      return rc;
    for (int l = 0; l <= exit_layer; ++l) {
      const nf_layer_desc *d = &blk->layers[l];
      const float *xs = d->skip_kind ? input_of(pl, ws, blk->skip_src[l], 0) : nullptr;
      if ((rc = nf_layer_fwd(d, nb, input_of(pl, ws, l, 0), xs, &blk->p[l], at(ws, pl.y_off[l]),
                             at(ws, pl.layer_ws_off), pl.layer_ws_bytes, stream)))
        return rc;
    }
    // the exit's head; the count of correct predictions accumulates over the batches
    if ((rc = nf_aux_predict(&blk->layers[exit_layer], &blk->aux[exit_layer], nb, at(ws, pl.y_off[exit_layer]), lab,
                             &blk->ap[exit_layer], pred_out + j * B, n_correct, j > 0, nullptr,
                             at(ws, pl.layer_ws_off), pl.layer_ws_bytes, stream)))
      return rc;
  }
  return NF_OK;
}

}  // extern "C"
