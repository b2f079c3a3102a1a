// K modules as concurrent HIP streams on one GPU (Algorithm 1 of arXiv 1804.10574: the K
// backward passes of one iteration run in parallel). The pipeline owns the tensors the
// modules exchange: h[k] (output of module k, input of k+1) and a two-slot mailbox per edge
// for the error gradient that module k+1 hands to module k for the NEXT iteration
// (Figure 2). Every cross-module dependency is a stream wait on an event, so running all
// modules on one stream gives bit-identical results.
#include "../../include/ddg.h"
#include "ddg_kernels.h"

#include <hip/hip_runtime_api.h>

#include <string>
#include <vector>

struct ddg_pipeline {
  int K = 0;
  std::vector<ddg_module*> mods;
  std::vector<hipStream_t> streams;
  std::vector<void*> h;                 // h[k], k = 1..K-1 (index k)
  std::vector<void*> mail[2];           // mail[slot][k]: df/dh_k, k = 1..K-1
  std::vector<long> mail_iter[2];       // iteration the slot content belongs to
  std::vector<size_t> h_elems;
  std::vector<int> dtype;
  std::vector<hipEvent_t> fwd_done;     // [k] recorded after module k's forward
  std::vector<hipEvent_t> bwd_done[2];  // [t%2][k] recorded after module k's backward+update
  hipEvent_t input_free = nullptr;
  long t = 0;
  bool dry = false;
  float* scratch_f32 = nullptr; size_t scratch_elems = 0;
};

extern "C" {

static ddg_status pfail(ddg_status s) { return s; }

ddg_status ddg_pipeline_destroy(ddg_pipeline* p) {
  if (!p) return DDG_OK;
  if (!p->dry) {
    for (hipStream_t s : p->streams) (void)hipStreamSynchronize(s);
    for (size_t k = 0; k < p->h.size(); ++k) if (p->h[k]) (void)hipFree(p->h[k]);
    for (int sl = 0; sl < 2; ++sl) {
      for (void* q : p->mail[sl]) if (q) (void)hipFree(q);
      for (hipEvent_t e : p->bwd_done[sl]) if (e) (void)hipEventDestroy(e);
    }
    for (hipEvent_t e : p->fwd_done) if (e) (void)hipEventDestroy(e);
    if (p->scratch_f32) (void)hipFree(p->scratch_f32);
  }
  for (ddg_module* m : p->mods) ddg_module_destroy(m);
  delete p;
  return DDG_OK;
}

ddg_status ddg_pipeline_create(const ddg_module_desc* descs, int K, void* const* streams, ddg_pipeline** out) {
  if (!out || !descs || K < 1) return DDG_ERR_INVALID_ARG;
  *out = nullptr;
  ddg_pipeline* p = new ddg_pipeline();
  p->K = K;
  p->dry = descs[0].dry_run != 0;
  p->mods.assign(K + 1, nullptr);
  p->streams.assign(K + 1, nullptr);
  p->h.assign(K + 1, nullptr);
  p->h_elems.assign(K + 1, 0);
  p->dtype.assign(K + 1, 0);
  p->fwd_done.assign(K + 1, nullptr);
  for (int sl = 0; sl < 2; ++sl) {
    p->mail[sl].assign(K + 1, nullptr);
    p->mail_iter[sl].assign(K + 1, -1);
    p->bwd_done[sl].assign(K + 1, nullptr);
  }
  for (int k = 1; k <= K; ++k) {
    ddg_module_desc d = descs[k - 1];
    if (d.K != K || d.k != k) { ddg_pipeline_destroy(p); return DDG_ERR_INVALID_ARG; }
    d.stream = streams ? streams[k - 1] : nullptr;
    p->streams[k] = (hipStream_t)d.stream;
    ddg_status st = ddg_module_create(&d, &p->mods[k]);
    if (st != DDG_OK) { ddg_pipeline_destroy(p); return st; }
    p->dtype[k] = d.compute;
    int c, hh, ww;
    ddg_out_shape(p->mods[k], &c, &hh, &ww);
    p->h_elems[k] = (size_t)d.batch * c * hh * ww;
    if (k > 1) {
      // module k's input must be module k-1's output
      if ((size_t)d.batch * d.in_c * d.in_h * d.in_w != p->h_elems[k - 1] || d.compute != p->dtype[k - 1]) {
        ddg_pipeline_destroy(p);
        return DDG_ERR_SHAPE;
      }
    }
    if (p->h_elems[k] > p->scratch_elems) p->scratch_elems = p->h_elems[k];
  }
  if (!p->dry) {
    for (int k = 1; k <= K; ++k) {
      const size_t bytes = p->h_elems[k] * ddg::dtype_size(p->dtype[k]);
      if (k < K) {
        if (hipMalloc(&p->h[k], bytes) != hipSuccess || hipMalloc(&p->mail[0][k], bytes) != hipSuccess ||
            hipMalloc(&p->mail[1][k], bytes) != hipSuccess) { ddg_pipeline_destroy(p); return DDG_ERR_OOM; }
      }
      if (hipEventCreateWithFlags(&p->fwd_done[k], hipEventDisableTiming) != hipSuccess ||
          hipEventCreateWithFlags(&p->bwd_done[0][k], hipEventDisableTiming) != hipSuccess ||
          hipEventCreateWithFlags(&p->bwd_done[1][k], hipEventDisableTiming) != hipSuccess) {
        ddg_pipeline_destroy(p); return DDG_ERR_DEVICE;
      }
    }
    if (hipMalloc((void**)&p->scratch_f32, p->scratch_elems * sizeof(float)) != hipSuccess) { ddg_pipeline_destroy(p); return DDG_ERR_OOM; }
  }
  else {
    // dry run: nothing is dereferenced; hand the modules a non-null, aligned placeholder
    for (int k = 1; k < K; ++k) { p->h[k] = (void*)4096; p->mail[0][k] = (void*)4096; p->mail[1][k] = (void*)4096; }
  }
  *out = p;
  return DDG_OK;
}

ddg_module* ddg_pipeline_module(ddg_pipeline* p, int k) { return (p && k >= 1 && k <= p->K) ? p->mods[k] : nullptr; }

ddg_status ddg_pipeline_step(ddg_pipeline* p, const void* x, const int32_t* labels, float lr, float* loss_out) {
  if (!p || !x || !labels) return DDG_ERR_INVALID_ARG;
  const int K = p->K;
  const long t = p->t;
  const int cur = (int)(t & 1), prev = cur ^ 1;
  // forward, k = 1..K in turn (Section 3.1)
  for (int k = 1; k <= K; ++k) {
    if (!p->dry) {
      if (k > 1) if (hipStreamWaitEvent(p->streams[k], p->fwd_done[k - 1], 0) != hipSuccess) return DDG_ERR_DEVICE;
      // h[k] is still being read by module k+1's forward of the previous iteration
      if (k < K && t > 0) if (hipStreamWaitEvent(p->streams[k], p->fwd_done[k + 1], 0) != hipSuccess) return DDG_ERR_DEVICE;
    }
    ddg_status st = ddg_forward(p->mods[k], t, k == 1 ? x : p->h[k - 1], k < K ? p->h[k] : nullptr);
    if (st != DDG_OK) return pfail(st);
    if (!p->dry) if (hipEventRecord(p->fwd_done[k], p->streams[k]) != hipSuccess) return DDG_ERR_DEVICE;
  }
  // backward + update: the K modules are independent within one iteration
  for (int k = 1; k <= K; ++k) {
    const long s = t - K + k;
    if (!p->dry && s >= 0 && t > 0) {
      // read-after-write: the error gradient for iteration s was written by module k+1 during t-1
      if (k < K) if (hipStreamWaitEvent(p->streams[k], p->bwd_done[prev][k + 1], 0) != hipSuccess) return DDG_ERR_DEVICE;
      // write-after-read: slot `cur` of mailbox k-1 was read by module k-1 during t-1
      if (k > 1) if (hipStreamWaitEvent(p->streams[k], p->bwd_done[prev][k - 1], 0) != hipSuccess) return DDG_ERR_DEVICE;
    }
    const void* din = (k < K) ? p->mail[prev][k] : nullptr;
    void* dout = (k > 1) ? p->mail[cur][k - 1] : nullptr;
    int did = 0;
    ddg_status st = ddg_backward_delayed(p->mods[k], t, (s >= 0) ? din : nullptr, k == K ? labels : nullptr,
                                         dout, k == K ? loss_out : nullptr, &did);
    if (st != DDG_OK) return pfail(st);
    if (k > 1) p->mail_iter[cur][k - 1] = did ? s : -1;
    st = ddg_update(p->mods[k], t, lr);
    if (st != DDG_OK) return pfail(st);
    if (!p->dry) if (hipEventRecord(p->bwd_done[cur][k], p->streams[k]) != hipSuccess) return DDG_ERR_DEVICE;
  }
  p->t = t + 1;
  return DDG_OK;
}

ddg_status ddg_pipeline_sync(ddg_pipeline* p) {
  if (!p) return DDG_ERR_INVALID_ARG;
  if (p->dry) return DDG_OK;
  for (int k = 1; k <= p->K; ++k) if (hipStreamSynchronize(p->streams[k]) != hipSuccess) return DDG_ERR_DEVICE;
  return DDG_OK;
}

static ddg_status fetch_f32(ddg_pipeline* p, const void* dev, size_t elems, int dtype, float* host_dst) {
  if (hipDeviceSynchronize() != hipSuccess) return DDG_ERR_DEVICE;
  if (ddg::to_f32_launch(dev, p->scratch_f32, elems, dtype, nullptr) != hipSuccess) return DDG_ERR_DEVICE;
  if (hipMemcpy(host_dst, p->scratch_f32, elems * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) return DDG_ERR_DEVICE;
  return DDG_OK;
}

ddg_status ddg_pipeline_get_h(ddg_pipeline* p, int k, float* host_dst) {
  if (!p || !host_dst || k < 1 || k >= p->K) return DDG_ERR_INVALID_ARG;
  if (p->dry) return DDG_OK;
  return fetch_f32(p, p->h[k], p->h_elems[k], p->dtype[k], host_dst);
}

ddg_status ddg_pipeline_get_delta(ddg_pipeline* p, int k, float* host_dst, long* iteration) {
  if (!p || k < 1 || k >= p->K) return DDG_ERR_INVALID_ARG;
  // the slot written during the last completed iteration
  const int slot = (int)((p->t - 1) & 1);
  const long it = (p->t > 0) ? p->mail_iter[slot][k] : -1;
  if (iteration) *iteration = it;
  if (it < 0 || !host_dst || p->dry) return DDG_OK;
  return fetch_f32(p, p->mail[slot][k], p->h_elems[k], p->dtype[k], host_dst);
}

}  // extern "C"
