// Layer-wise preloading of chunk-caches (Sec. 3.4.2, Eq. (12), Algorithm 2): while the GPU works on
// layer i, the chunk-caches of the next layers travel from host memory into an HBM read buffer on
// a copy stream of their own.
//
// Host-side runtime only: one copy stream, one "loaded" event and one "released" event per layer.
// The read buffer is a ring of slots in device memory owned by the caller; layer j uses slot
// j mod n_slots, so its copy is ordered behind the release of layer j - n_slots (the previous
// tenant of the slot).  The compute stream never blocks the host: acquire() makes it wait for the
// layer's event on the GPU (hipStreamWaitEvent), release() records the event that frees the slot.
#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

#include "common.h"

struct cc_preloader {
  int n_layers = 0, depth = 0, n_slots = 0;
  int issued = 0;                       // layers 0 .. issued-1 have their copies enqueued
  hipStream_t copy_stream = nullptr;
  struct Layer {
    const void* src = nullptr;          // pinned host memory
    void* dst = nullptr;                // slot in the caller's device read buffer
    size_t bytes = 0;
    hipEvent_t loaded = nullptr, released = nullptr;
    bool released_recorded = false;
  };
  std::vector<Layer> layers;
  std::vector<int32_t> log;             // order in which copies were enqueued (for inspection)
};

namespace {

// Algorithm 2's inner loop before layer i is computed: every layer up to min(i + depth, L - 1)
// (0-based) must have been asked for.
int last_wanted(const cc_preloader* p, int layer) { return std::min(layer + p->depth, p->n_layers - 1); }

int enqueue_up_to(cc_preloader* p, int last) {
  while (p->issued <= last) {
    const int j = p->issued;
    cc_preloader::Layer& l = p->layers[j];
    if (l.bytes > 0 && (l.src == nullptr || l.dst == nullptr)) return CC_ERR_INVALID_ARG;
    const int prev = j - p->n_slots;    // previous tenant of the slot
    if (prev >= 0) {
      if (!p->layers[prev].released_recorded) return CC_ERR_INVALID_ARG;   // caller skipped a release
      if (hipStreamWaitEvent(p->copy_stream, p->layers[prev].released, 0) != hipSuccess) return CC_ERR_HIP;
    }
    if (l.bytes > 0 &&
        hipMemcpyAsync(l.dst, l.src, l.bytes, hipMemcpyHostToDevice, p->copy_stream) != hipSuccess)
      return CC_ERR_HIP;
    if (hipEventRecord(l.loaded, p->copy_stream) != hipSuccess) return CC_ERR_HIP;
    p->log.push_back(j);
    p->issued = j + 1;
  }
  return CC_OK;
}

}  // namespace

extern "C" {

int32_t cc_preload_depth(int32_t n_layers, double t_prefill, double t_load) {
  if (n_layers <= 0 || !(t_prefill >= 0.0) || !(t_load >= 0.0) || !std::isfinite(t_prefill) ||
      !std::isfinite(t_load))
    return CC_ERR_INVALID_ARG;
  if (t_load <= 0.0 || t_prefill >= t_load) return 1;       // loading hides behind one layer of compute
  const double lp = (n_layers - 1) * (1.0 - t_prefill / t_load) + 1.0;
  const int32_t depth = static_cast<int32_t>(std::ceil(lp - 1e-9));
  return std::max<int32_t>(1, std::min<int32_t>(depth, n_layers));
}

int cc_preloader_create(cc_preloader** out, int32_t n_layers, int32_t depth, int32_t n_slots) {
  if (out == nullptr) return CC_ERR_INVALID_ARG;
  *out = nullptr;
  // a slot ring shorter than depth + 1 would make the copies of Algorithm 2's window wait for
  // layers that have not been computed yet
  if (n_layers <= 0 || depth < 1 || n_slots < std::min(depth + 1, n_layers)) return CC_ERR_INVALID_ARG;
  cc_preloader* p = new (std::nothrow) cc_preloader();
  if (p == nullptr) return CC_ERR_INVALID_ARG;
  p->n_layers = n_layers;
  p->depth = depth;
  p->n_slots = n_slots;
  p->layers.resize(n_layers);
  bool ok = hipStreamCreateWithFlags(&p->copy_stream, hipStreamNonBlocking) == hipSuccess;
  for (int j = 0; ok && j < n_layers; ++j) {
    ok = hipEventCreateWithFlags(&p->layers[j].loaded, hipEventDisableTiming) == hipSuccess &&
         hipEventCreateWithFlags(&p->layers[j].released, hipEventDisableTiming) == hipSuccess;
  }
  if (!ok) {
    cc_preloader_destroy(p);
    return CC_ERR_HIP;
  }
  *out = p;
  return CC_OK;
}

void cc_preloader_destroy(cc_preloader* p) {
  if (p == nullptr) return;
  if (p->copy_stream != nullptr) (void)hipStreamSynchronize(p->copy_stream);
  for (auto& l : p->layers) {
    if (l.loaded != nullptr) (void)hipEventDestroy(l.loaded);
    if (l.released != nullptr) (void)hipEventDestroy(l.released);
  }
  if (p->copy_stream != nullptr) (void)hipStreamDestroy(p->copy_stream);
  delete p;
}

int cc_preloader_set_layer(cc_preloader* p, int32_t layer, const void* host_src, void* dev_dst, size_t bytes) {
  if (p == nullptr || layer < 0 || layer >= p->n_layers || layer < p->issued) return CC_ERR_INVALID_ARG;
  if (bytes > 0 && (host_src == nullptr || dev_dst == nullptr)) return CC_ERR_INVALID_ARG;
  p->layers[layer].src = host_src;
  p->layers[layer].dst = dev_dst;
  p->layers[layer].bytes = bytes;
  return CC_OK;
}

int cc_preloader_acquire(cc_preloader* p, int32_t layer, void* compute_stream) {
  if (p == nullptr || layer < 0 || layer >= p->n_layers) return CC_ERR_INVALID_ARG;
  const int st = enqueue_up_to(p, last_wanted(p, layer));
  if (st != CC_OK) return st;
  if (hipStreamWaitEvent(static_cast<hipStream_t>(compute_stream), p->layers[layer].loaded, 0) != hipSuccess)
    return CC_ERR_HIP;
  return CC_OK;
}

int cc_preloader_release(cc_preloader* p, int32_t layer, void* compute_stream) {
  if (p == nullptr || layer < 0 || layer >= p->n_layers || layer >= p->issued) return CC_ERR_INVALID_ARG;
  if (hipEventRecord(p->layers[layer].released, static_cast<hipStream_t>(compute_stream)) != hipSuccess)
    return CC_ERR_HIP;
  p->layers[layer].released_recorded = true;
  return CC_OK;
}

int32_t cc_preloader_issued(const cc_preloader* p, int32_t* order, int32_t capacity) {
  if (p == nullptr) return CC_ERR_INVALID_ARG;
  const int32_t n = static_cast<int32_t>(p->log.size());
  if (order != nullptr)
    for (int32_t i = 0; i < std::min(n, capacity); ++i) order[i] = p->log[i];
  return n;
}

}  // extern "C"
