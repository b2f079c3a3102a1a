// K modules as concurrent HIP streams on one GPU (Algorithm 1 of arXiv 1804.10574: the K
// backward passes of one iteration run in parallel). The pipeline owns the tensors the
// modules exchange: h[k] (output of module k, input of k+1) and a two-slot mailbox per edge
// for the error gradient that module k+1 hands to module k for the NEXT iteration
// (Figure 2). Every cross-module dependency is a stream wait on an event, so running all
// modules on one stream gives bit-identical results.
#include "../../include/ddg.h"
#include "ddg_kernels.h"
#include "ddg_internal.h"

#include <cstdlib>
#include <map>

#include <hip/hip_runtime_api.h>

#include <string>
#include <vector>

// Host-side model of what orders the streams. Every stream carries a vector clock; recording an
// event keeps the recording stream's clock, waiting for it merges that clock into the waiter's.
// A step declares which tensors each call reads and writes and on which stream; an access that is
// not ordered after the last write of the tensor (for a write: also after every read since) is
// a hazard that the events do not cover. Runs in dry-run pipelines (no device work) and, with
// DDG_CHECK_ORDER=1, beside the real calls.
struct OrderModel {
  struct Acc { int s; long v; };
  struct Buf { Acc w{-1, 0}; std::vector<Acc> r; };
  std::vector<std::vector<long>> clk;           // [stream][stream]
  std::map<int, std::vector<long>> ev;          // event id -> clock at its last record
  std::map<std::string, Buf> bufs;
  std::string msg;                              // first hazard found
  long waits = 0, drop = -1;                    // test hook: the wait with this running number is ignored
  void init(int nstreams) { clk.assign(nstreams, std::vector<long>(nstreams, 0)); }
  bool before(const Acc& a, int s) const { return a.s < 0 || clk[s][a.s] >= a.v; }
  void record(int eid, int s) { ev[eid] = clk[s]; }
  void wait(int s, int eid) {
    if (waits++ == drop) return;
    auto it = ev.find(eid);
    if (it == ev.end()) return;                 // never recorded: the wait returns at once
    for (size_t i = 0; i < clk[s].size(); ++i) if (it->second[i] > clk[s][i]) clk[s][i] = it->second[i];
  }
  void host_sync() {                            // the host waited for every stream
    std::vector<long> m(clk.size(), 0);
    for (auto& c : clk) for (size_t i = 0; i < c.size(); ++i) if (c[i] > m[i]) m[i] = c[i];
    for (auto& c : clk) c = m;
  }
  void op(int s, long t, const char* what, const std::vector<std::string>& reads, const std::vector<std::string>& writes) {
    clk[s][s] += 1;
    const Acc me{s, clk[s][s]};
    auto hazard = [&](const char* kind, const std::string& b, const Acc& a) {
      if (msg.empty())
        msg = std::string(kind) + " hazard at iteration " + std::to_string(t) + ": " + what + " on stream " + std::to_string(s) +
              " touches " + b + " unordered with an access on stream " + std::to_string(a.s);
    };
    for (const std::string& b : reads) {
      Buf& q = bufs[b];
      if (!before(q.w, s)) hazard("read-after-write", b, q.w);
      q.r.push_back(me);
    }
    for (const std::string& b : writes) {
      Buf& q = bufs[b];
      if (!before(q.w, s)) hazard("write-after-write", b, q.w);
      for (const Acc& a : q.r) if (!before(a, s)) hazard("write-after-read", b, a);
      q.w = me; q.r.clear();
    }
  }
};

struct ddg_pipeline {
  int K = 0;
  OrderModel order;
  bool check_order = false;
  std::vector<int> sid_f, sid_b;        // logical stream numbers of module k's forward / backward stream
  bool stale = false;
  std::vector<ddg_module*> mods;
  std::vector<hipStream_t> streams;     // [k] backward / update stream of module k
  std::vector<hipStream_t> fstreams;    // [k] forward stream (== streams[k] unless the module has its own)
  std::vector<void*> h;                 // h[k], k = 1..K-1 (index k), for even iterations
  std::vector<void*> h_odd;             // the same for odd iterations: the producer of iteration t+1
                                        // need not wait for the consumer of iteration t
  std::vector<void*> mail[2];           // mail[slot][k]: df/dh_k, k = 1..K-1
  std::vector<long> mail_iter[2];       // iteration the slot content belongs to
  std::vector<size_t> h_elems;
  std::vector<int> dtype;
  std::vector<hipEvent_t> fwd_done[2];  // [t%2][k] recorded after module k's forward
  std::vector<hipEvent_t> bwd_done[2];  // [t%2][k] recorded after module k's backward+update
  hipEvent_t input_free = nullptr;
  long t = 0;
  bool dry = false;
  float* scratch_f32 = nullptr; size_t scratch_elems = 0;
  // HIP-graph replay of each module's forward and backward+update call (steady state only).
  // A call's launches depend on t only through the ring slot (period K-k+1) and the mailbox
  // slot (period 2), so one graph per residue of t modulo their least common multiple.
  bool graphs = true;
  std::vector<int> period;                                  // [k]
  std::vector<std::map<int, hipGraphExec_t>> gfwd, gbwd, gupd;   // [k][t mod period]
  void* xin = nullptr;            // staged network input (stable address for the graphs)
  int32_t* labels_dev = nullptr;  // staged labels
  float* loss_dev = nullptr;      // loss of the last iteration
  float* lr_dev = nullptr;        // step size read by the update kernels
  float lr_host = -1.f;
  size_t x_bytes = 0;
  int batch = 0;
};

namespace {
int gcd_i(int a, int b) { return b ? gcd_i(b, a % b) : a; }

// Capture what `fn` enqueues on `s` into an executable graph.
template <class F>
ddg_status capture(hipStream_t s, hipGraphExec_t* exec, F fn) {
  if (hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal) != hipSuccess) return DDG_ERR_DEVICE;
  ddg_status st = fn();
  hipGraph_t g = nullptr;
  hipError_t e = hipStreamEndCapture(s, &g);
  if (st != DDG_OK) { if (g) (void)hipGraphDestroy(g); return st; }
  if (e != hipSuccess || !g) return DDG_ERR_DEVICE;
  e = hipGraphInstantiate(exec, g, nullptr, nullptr, 0);
  (void)hipGraphDestroy(g);
  return e == hipSuccess ? DDG_OK : DDG_ERR_DEVICE;
}
}  // namespace

extern "C" {

static ddg_status pfail(ddg_status s) { return s; }

ddg_status ddg_pipeline_destroy(ddg_pipeline* p) {
  if (!p) return DDG_OK;
  if (!p->dry) {
    for (hipStream_t s : p->streams) (void)hipStreamSynchronize(s);
    for (hipStream_t s : p->fstreams) if (s) (void)hipStreamSynchronize(s);
    for (size_t k = 0; k < p->h.size(); ++k) if (p->h[k]) (void)hipFree(p->h[k]);
    for (size_t k = 0; k < p->h_odd.size(); ++k) if (p->h_odd[k]) (void)hipFree(p->h_odd[k]);
    for (int sl = 0; sl < 2; ++sl) {
      for (void* q : p->mail[sl]) if (q) (void)hipFree(q);
      for (hipEvent_t e : p->bwd_done[sl]) if (e) (void)hipEventDestroy(e);
    }
    for (int sl = 0; sl < 2; ++sl) for (hipEvent_t e : p->fwd_done[sl]) if (e) (void)hipEventDestroy(e);
    if (p->scratch_f32) (void)hipFree(p->scratch_f32);
    for (auto& mp : p->gfwd) for (auto& kv : mp) (void)hipGraphExecDestroy(kv.second);
    for (auto& mp : p->gbwd) for (auto& kv : mp) (void)hipGraphExecDestroy(kv.second);
    for (auto& mp : p->gupd) for (auto& kv : mp) (void)hipGraphExecDestroy(kv.second);
    if (p->xin) (void)hipFree(p->xin);
    if (p->labels_dev) (void)hipFree(p->labels_dev);
    if (p->loss_dev) (void)hipFree(p->loss_dev);
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
  p->h_odd.assign(K + 1, nullptr);
  p->h_elems.assign(K + 1, 0);
  p->dtype.assign(K + 1, 0);
  p->fstreams.assign(K + 1, nullptr);
  p->sid_f.assign(K + 1, 0);
  p->sid_b.assign(K + 1, 0);
  p->order.init(2 * K + 1);
  p->stale = descs[0].stale_jacobian != 0;
  {
    const char* env = getenv("DDG_CHECK_ORDER");
    p->check_order = p->dry || (env && env[0] == '1');
  }
  for (int sl = 0; sl < 2; ++sl) {
    p->fwd_done[sl].assign(K + 1, nullptr);
    p->mail[sl].assign(K + 1, nullptr);
    p->mail_iter[sl].assign(K + 1, -1);
    p->bwd_done[sl].assign(K + 1, nullptr);
  }
  for (int k = 1; k <= K; ++k) {
    ddg_module_desc d = descs[k - 1];
    if (d.K != K || d.k != k) { ddg_pipeline_destroy(p); return DDG_ERR_INVALID_ARG; }
    d.stream = streams ? streams[k - 1] : nullptr;
    if (!streams) d.forward_stream = nullptr;
    ddg_status st = ddg_module_create(&d, &p->mods[k]);
    if (st != DDG_OK) { ddg_pipeline_destroy(p); return st; }
    // logical stream numbers for the ordering model: 0 when everything runs on one stream
    p->sid_b[k] = streams ? k : 0;
    const bool own_fwd = streams && !d.stale_jacobian && d.forward_stream && d.forward_stream != d.stream && K - k > 0;
    p->sid_f[k] = own_fwd ? K + k : p->sid_b[k];
    if (!p->dry) {
      ddg_internal_streams(p->mods[k], &p->fstreams[k], &p->streams[k]);
      ddg_internal_external_sync(p->mods[k], true);
    }
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
        if (hipMalloc(&p->h[k], bytes) != hipSuccess || hipMalloc(&p->h_odd[k], bytes) != hipSuccess ||
            hipMalloc(&p->mail[0][k], bytes) != hipSuccess ||
            hipMalloc(&p->mail[1][k], bytes) != hipSuccess) { ddg_pipeline_destroy(p); return DDG_ERR_OOM; }
      }
      if (hipEventCreateWithFlags(&p->fwd_done[0][k], hipEventDisableTiming) != hipSuccess ||
          hipEventCreateWithFlags(&p->fwd_done[1][k], hipEventDisableTiming) != hipSuccess ||
          hipEventCreateWithFlags(&p->bwd_done[0][k], hipEventDisableTiming) != hipSuccess ||
          hipEventCreateWithFlags(&p->bwd_done[1][k], hipEventDisableTiming) != hipSuccess) {
        ddg_pipeline_destroy(p); return DDG_ERR_DEVICE;
      }
    }
    if (hipMalloc((void**)&p->scratch_f32, p->scratch_elems * sizeof(float)) != hipSuccess) { ddg_pipeline_destroy(p); return DDG_ERR_OOM; }
    p->batch = descs[0].batch;
    p->x_bytes = (size_t)descs[0].batch * descs[0].in_c * descs[0].in_h * descs[0].in_w * ddg::dtype_size(descs[0].compute);
    void* sc = nullptr;
    if (hipMalloc(&p->xin, p->x_bytes) != hipSuccess || hipMalloc((void**)&p->labels_dev, p->batch * sizeof(int32_t)) != hipSuccess ||
        hipMalloc(&sc, 2 * sizeof(float)) != hipSuccess) { ddg_pipeline_destroy(p); return DDG_ERR_OOM; }
    p->loss_dev = (float*)sc; p->lr_dev = p->loss_dev + 1;
    const char* env = getenv("DDG_NO_GRAPH");
    if (env && env[0] == '1') p->graphs = false;
    if (!streams) p->graphs = false;   // the default stream cannot be captured
    p->period.assign(K + 1, 1);
    p->gfwd.resize(K + 1); p->gbwd.resize(K + 1); p->gupd.resize(K + 1);
    for (int k = 1; k <= K; ++k) {
      const int nslots = K - k + 1;
      p->period[k] = nslots * 2 / gcd_i(nslots, 2);
      ddg_internal_lr_from(p->mods[k], p->lr_dev);
    }
  }
  else {
    // dry run: nothing is dereferenced; hand the modules a non-null, aligned placeholder
    for (int k = 1; k < K; ++k) { p->h[k] = (void*)4096; p->h_odd[k] = (void*)4096; p->mail[0][k] = (void*)4096; p->mail[1][k] = (void*)4096; }
  }
  *out = p;
  return DDG_OK;
}

ddg_module* ddg_pipeline_module(ddg_pipeline* p, int k) { return (p && k >= 1 && k <= p->K) ? p->mods[k] : nullptr; }

ddg_status ddg_pipeline_set_graphs(ddg_pipeline* p, int on) {
  if (!p) return DDG_ERR_INVALID_ARG;
  p->graphs = on != 0;
  return DDG_OK;
}

ddg_status ddg_pipeline_set_optimizer(ddg_pipeline* p, int kind, float beta1, float beta2, float eps) {
  if (!p) return DDG_ERR_INVALID_ARG;
  for (int k = 1; k <= p->K; ++k) {
    const ddg_status st = ddg_set_optimizer(p->mods[k], kind, beta1, beta2, eps);
    if (st != DDG_OK) return st;
  }
  // graphs captured with the other update kernel must not be replayed; a replay may still be
  // running on the streams, so wait for them before the executables go
  {
    const ddg_status st = ddg_pipeline_sync(p);
    if (st != DDG_OK) return st;
  }
  for (int k = 1; k <= p->K; ++k) {
    for (auto& kv : p->gupd[k]) if (kv.second) (void)hipGraphExecDestroy(kv.second);
    p->gupd[k].clear();
  }
  return DDG_OK;
}

ddg_status ddg_pipeline_set_bn_momentum(ddg_pipeline* p, float rho) {
  if (!p) return DDG_ERR_INVALID_ARG;
  for (int k = 1; k <= p->K; ++k) {
    const ddg_status st = ddg_set_bn_momentum(p->mods[k], rho);
    if (st != DDG_OK) return st;
  }
  return DDG_OK;
}

// Evaluation of the whole network between iterations. Module k writes into the buffer that
// iteration p->t will overwrite anyway (the one ddg_pipeline_get_h does not read); modules run
// one after the other, each waited for.
ddg_status ddg_pipeline_forward_eval(ddg_pipeline* p, const void* x, const int32_t* labels, float* loss_out,
                                     float* logits_out) {
  if (!p || !x) return DDG_ERR_INVALID_ARG;
  if (p->dry) return DDG_OK;
  ddg_status st = ddg_pipeline_sync(p);
  if (st != DDG_OK) return st;
  const void* in = x;
  for (int k = 1; k <= p->K; ++k) {
    void* out = (k < p->K) ? ((p->t & 1) ? p->h_odd[k] : p->h[k]) : nullptr;
    st = ddg_forward_eval(p->mods[k], in, out, k == p->K ? labels : nullptr, k == p->K ? loss_out : nullptr,
                          k == p->K ? logits_out : nullptr);
    if (st != DDG_OK) return st;
    st = ddg_module_sync(p->mods[k]);
    if (st != DDG_OK) return st;
    in = out;
  }
  return DDG_OK;
}

ddg_status ddg_pipeline_step(ddg_pipeline* p, const void* x, const int32_t* labels, float lr, float* loss_out) {
  if (!p || !x || !labels) return DDG_ERR_INVALID_ARG;
  const int K = p->K;
  const long t = p->t;
  const int cur = (int)(t & 1), prev = cur ^ 1;
  bool use_graph = !p->dry && p->graphs && t >= K;   // steady state: every module has a gradient
  if (use_graph) for (int k = 1; k <= K; ++k) if (ddg_internal_profiling(p->mods[k])) use_graph = false;
#define DDG_P(expr) do { if ((expr) != hipSuccess) return DDG_ERR_DEVICE; } while (0)
  // Every wait and record goes through these two, so that the ordering model sees exactly the
  // dependencies the streams get. Event numbers: fwd_done[sl][k] = sl*(K+1)+k, bwd_done after them.
  OrderModel& om = p->order;
  const bool model = p->check_order;
  auto ev_f = [&](int sl, int k) { return sl * (K + 1) + k; };
  auto ev_b = [&](int sl, int k) { return 2 * (K + 1) + sl * (K + 1) + k; };
  auto wait_f = [&](int sid, hipStream_t s, int sl, int k) -> hipError_t {
    if (model) om.wait(sid, ev_f(sl, k));
    return p->dry ? hipSuccess : hipStreamWaitEvent(s, p->fwd_done[sl][k], 0); };
  auto wait_b = [&](int sid, hipStream_t s, int sl, int k) -> hipError_t {
    if (model) om.wait(sid, ev_b(sl, k));
    return p->dry ? hipSuccess : hipStreamWaitEvent(s, p->bwd_done[sl][k], 0); };
  auto nm = [](const char* base, int a, long b = -1) {
    std::string r = std::string(base) + std::to_string(a);
    if (b >= 0) r += "/" + std::to_string(b);
    return r; };
  if (!p->dry) {
    // stage the caller's tensors at stable addresses; the step size lives in device memory
    DDG_P(ddg::copy_launch(x, p->xin, p->x_bytes, p->fstreams[1]));
    DDG_P(ddg::copy_launch(labels, p->labels_dev, p->batch * sizeof(int32_t), p->streams[K]));
    if (lr != p->lr_host) {
      // every module's update of the previous iteration must have read the old value
      for (int k = 1; k <= K; ++k) DDG_P(hipStreamSynchronize(p->streams[k]));
      DDG_P(ddg::set_scalar_launch(p->lr_dev, lr, p->streams[1]));
      DDG_P(hipStreamSynchronize(p->streams[1]));
      p->lr_host = lr;
    }
  }
  if (model) {
    om.op(p->sid_f[1], t, "the copy of the network input", {}, {"xin"});
    om.op(p->sid_b[K], t, "the copy of the labels", {}, {"labels"});
  }
  const void* x_in = p->dry ? x : p->xin;
  const int32_t* lab = p->dry ? labels : p->labels_dev;
  // Runs `call` on stream s: eagerly, or as a captured graph (captured at the first use of this
  // residue of t, replayed afterwards while the module only advances its host-side state).
  auto run = [&](int k, hipStream_t s, std::map<int, hipGraphExec_t>& cache, auto call) -> ddg_status {
    if (!use_graph) return call();
    const int v = (int)(t % p->period[k]);
    auto it = cache.find(v);
    ddg_status st;
    if (it == cache.end()) {
      hipGraphExec_t ex = nullptr;
      st = capture(s, &ex, call);
      if (st != DDG_OK) return st;
      it = cache.emplace(v, ex).first;
    } else {
      ddg_internal_skip_launches(p->mods[k], true);
      st = call();
      ddg_internal_skip_launches(p->mods[k], false);
      if (st != DDG_OK) return st;
    }
    return hipGraphLaunch(it->second, s) == hipSuccess ? DDG_OK : DDG_ERR_DEVICE;
  };
  // forward, k = 1..K in turn (Section 3.1), each on its module's forward stream
  for (int k = 1; k <= K; ++k) {
    hipStream_t fs = p->dry ? nullptr : p->fstreams[k];
    const int sf = p->sid_f[k];
    const bool split = sf != p->sid_b[k];
    if (k > 1) DDG_P(wait_f(sf, fs, cur, k - 1));
    // this iteration's h[k] buffer was last read by module k+1's forward two iterations ago
    // (the event of this parity still carries that record: module k+1 re-records it later)
    if (k < K && t > 1) DDG_P(wait_f(sf, fs, cur, k + 1));
    // a forward stream of its own: the weights of update(t-1), and the ring slot that
    // backward(t-1) read, come from the module's other stream
    if (split && t > 0) DDG_P(wait_b(sf, fs, prev, k));
    if (model) {
      // what ddg_forward(t) of module k touches (delay d, ring of d+1 slots)
      const int d = K - k, n = d + 1;
      std::vector<std::string> rd{k == 1 ? std::string("xin") : nm("h", cur, k - 1), nm("w", k)}, wr{nm("ring", k, t % n)};
      if (k < K) wr.push_back(nm("h", cur, k));
      if (p->stale) { wr.push_back(nm("tape", k, t % n)); wr.push_back(nm("wsnap", k, t % n)); }
      else if (split) wr.push_back(nm("fbuf", k));
      else {
        wr.push_back(nm("tape", k));
        if (d > 0 && t >= d) rd.push_back(nm("ring", k, (t - d) % n));   // paired with the re-forward
      }
      om.op(sf, t, "forward", rd, wr);
    }
    ddg_status st = run(k, fs, p->gfwd[k], [&]() {
      std::vector<void*>& hb = cur ? p->h_odd : p->h;
      return ddg_forward(p->mods[k], t, k == 1 ? x_in : hb[k - 1], k < K ? hb[k] : nullptr); });
    if (st != DDG_OK) return st;
    if (model) om.record(ev_f(cur, k), sf);
    if (!p->dry) DDG_P(hipEventRecord(p->fwd_done[cur][k], fs));
  }
  // backward + update: the K modules are independent within one iteration
  for (int k = 1; k <= K; ++k) {
    const long s = t - K + k;
    hipStream_t bs = p->dry ? nullptr : p->streams[k];
    const int sb = p->sid_b[k];
    const bool split = p->sid_f[k] != sb;
    if (s >= 0 && t > 0) {
      // read-after-write: the error gradient for iteration s was written by module k+1 during t-1
      if (k < K) DDG_P(wait_b(sb, bs, prev, k + 1));
      // write-after-read: slot `cur` of mailbox k-1 was read by module k-1 during t-1
      if (k > 1) DDG_P(wait_b(sb, bs, prev, k - 1));
      // the stored input of iteration s <= t-1 was written by the forward stream
      if (split) DDG_P(wait_f(sb, bs, prev, k));
    }
    const void* din = (k < K) ? p->mail[prev][k] : nullptr;
    void* dout = (k > 1) ? p->mail[cur][k - 1] : nullptr;
    int did = 0;
    if (model && s >= 0) {
      const int d = K - k, n = d + 1;
      std::vector<std::string> rd{nm("ring", k, s % n), nm("w", k)}, wr{nm("g", k)};
      rd.push_back(k < K ? nm("mail", prev, k) : std::string("labels"));
      if (k > 1) wr.push_back(nm("mail", cur, k - 1));
      if (k == K) wr.push_back("loss");
      if (p->stale) { rd.push_back(nm("tape", k, s % n)); rd.push_back(nm("wsnap", k, s % n)); }
      else if (split) wr.push_back(nm("tape", k));          // re-forwards on this stream, then reads it
      else rd.push_back(nm("tape", k));
      om.op(sb, t, "backward", rd, wr);
    }
    ddg_status st = run(k, bs, p->gbwd[k], [&]() {
      return ddg_backward_delayed(p->mods[k], t, (s >= 0) ? din : nullptr, k == K ? lab : nullptr, dout,
                                  k == K ? (p->dry ? loss_out : p->loss_dev) : nullptr, &did); });
    if (st != DDG_OK) return st;
    if (k > 1) p->mail_iter[cur][k - 1] = did ? s : -1;
    // the update overwrites the weights that this iteration's forward pass reads
    if (split) DDG_P(wait_f(sb, bs, cur, k));
    if (model && s >= 0) om.op(sb, t, "update", {nm("g", k)}, {nm("w", k)});
    st = run(k, bs, p->gupd[k], [&]() { return ddg_update(p->mods[k], t, lr); });
    if (st != DDG_OK) return st;
    if (model && k == K && loss_out && s >= 0) om.op(sb, t, "the copy of the loss", {"loss"}, {});
    if (!p->dry) {
      if (k == K && loss_out && s >= 0) DDG_P(ddg::copy_launch(p->loss_dev, loss_out, sizeof(float), bs));
    }
    if (model) om.record(ev_b(cur, k), sb);
    if (!p->dry) DDG_P(hipEventRecord(p->bwd_done[cur][k], bs));
  }
#undef DDG_P
  p->t = t + 1;
  if (model && !om.msg.empty()) {
    ddg_internal_set_error(om.msg.c_str());
    return DDG_ERR_STATE;
  }
  return DDG_OK;
}

// Test hooks of the ordering model (not part of the C boundary): the number of waits the model
// has seen, and the running number of a wait it is to ignore.
long ddg_internal_pipeline_waits(const ddg_pipeline* p) { return p ? p->order.waits : -1; }
void ddg_internal_pipeline_drop_wait(ddg_pipeline* p, long n) { if (p) p->order.drop = n; }

ddg_status ddg_pipeline_sync(ddg_pipeline* p) {
  if (!p) return DDG_ERR_INVALID_ARG;
  if (p->check_order) p->order.host_sync();
  if (p->dry) return DDG_OK;
  for (int k = 1; k <= p->K; ++k) {
    if (hipStreamSynchronize(p->streams[k]) != hipSuccess) return DDG_ERR_DEVICE;
    if (p->fstreams[k] != p->streams[k] && hipStreamSynchronize(p->fstreams[k]) != hipSuccess) return DDG_ERR_DEVICE;
  }
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
  // the buffer written during the last completed iteration
  return fetch_f32(p, ((p->t - 1) & 1) ? p->h_odd[k] : p->h[k], p->h_elems[k], p->dtype[k], host_dst);
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

long ddg_pipeline_time(const ddg_pipeline* p) { return p ? p->t : -1; }

ddg_status ddg_pipeline_set_time(ddg_pipeline* p, long t) {
  if (!p || t < 0) return DDG_ERR_INVALID_ARG;
  ddg_status st = ddg_pipeline_sync(p);
  if (st != DDG_OK) return st;
  for (int k = 1; k <= p->K; ++k) {
    st = ddg_set_time(p->mods[k], t);
    if (st != DDG_OK) return st;
  }
  p->t = t;
  for (int sl = 0; sl < 2; ++sl) for (int k = 1; k < p->K; ++k) p->mail_iter[sl][k] = -1;
  return DDG_OK;
}

size_t ddg_pipeline_mail_bytes(const ddg_pipeline* p, int k) {
  return (p && k >= 1 && k < p->K) ? p->h_elems[k] * ddg::dtype_size(p->dtype[k]) : 0;
}

ddg_status ddg_pipeline_get_mail(ddg_pipeline* p, int k, void* host_dst, long* iteration) {
  if (!p || k < 1 || k >= p->K) return DDG_ERR_INVALID_ARG;
  // the slot written during the last completed iteration is the one the next iteration reads
  const int slot = (int)((p->t - 1) & 1);
  const long it = (p->t > 0) ? p->mail_iter[slot][k] : -1;
  if (iteration) *iteration = it;
  if (it < 0 || !host_dst || p->dry) return DDG_OK;
  const ddg_status st = ddg_pipeline_sync(p);
  if (st != DDG_OK) return st;
  return hipMemcpy(host_dst, p->mail[slot][k], ddg_pipeline_mail_bytes(p, k), hipMemcpyDeviceToHost) == hipSuccess
             ? DDG_OK : DDG_ERR_DEVICE;
}

ddg_status ddg_pipeline_set_mail(ddg_pipeline* p, int k, const void* host_src, long iteration) {
  if (!p || k < 1 || k >= p->K || !host_src || iteration < 0 || p->t < 1) return DDG_ERR_INVALID_ARG;
  // module k reads it during iteration p->t as the gradient of iteration p->t - K + k
  if (iteration != p->t - 1 - p->K + (k + 1)) return DDG_ERR_INVALID_ARG;
  const int slot = (int)((p->t - 1) & 1);
  p->mail_iter[slot][k] = iteration;
  if (p->dry) return DDG_OK;
  const ddg_status st = ddg_pipeline_sync(p);
  if (st != DDG_OK) return st;
  return hipMemcpy(p->mail[slot][k], host_src, ddg_pipeline_mail_bytes(p, k), hipMemcpyHostToDevice) == hipSuccess
             ? DDG_OK : DDG_ERR_DEVICE;
}

}  // extern "C"
