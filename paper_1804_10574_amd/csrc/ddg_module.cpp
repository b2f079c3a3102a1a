// Host side of the DDG module-step library: builds a launch plan for one module G(k)
// (Section 3 of arXiv 1804.10574), keeps its input ring (delay K-k), and implements the
// C boundary declared in include/ddg.h. All arithmetic happens in the HIP kernels; this
// file only validates, allocates and enqueues.
#include "../../include/ddg.h"
#include "ddg_kernels.h"
#include "ddg_internal.h"

#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

using namespace ddg;

thread_local ddg::ProfEvents ddg::g_prof_events;

static thread_local std::string g_err;
static ddg_status fail(ddg_status st, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return st;
}

// One kind per kernel (the three convolution passes: the generic kernel, then one kind per
// instance of the LDS-tiled kernel, in the order 16, 32, 64 channels); "family.instance" names.
enum ProfKind {
  PK_CONV_FPROP = 0, PK_CONV_FPROP_T16, PK_CONV_FPROP_T32, PK_CONV_FPROP_T64,
  PK_CONV_DGRAD, PK_CONV_DGRAD_T16, PK_CONV_DGRAD_T32, PK_CONV_DGRAD_T64,
  PK_CONV_WGRAD, PK_CONV_WGRAD_T16, PK_CONV_WGRAD_T32, PK_CONV_WGRAD_T64,
  // a launch that carries an input-gradient kernel and the weight gradient of the unit above
  PK_BWD_PAIR_T16, PK_BWD_PAIR_T32, PK_BWD_PAIR_T64, PK_BWD_PAIR = PK_BWD_PAIR_T16 - 1,
  // the GEMM-class kernels of the wide layers
  PK_CONV_FPROP_WIDE = PK_BWD_PAIR_T64 + 1, PK_CONV_DGRAD_WIDE, PK_CONV_WGRAD_WIDE,
  PK_CONV_WGRAD_S2,   // the LDS-tiled weight gradient of the stride-2 layers between stages
  PK_WGRAD_REDUCE, PK_BN_FINALIZE, PK_BN_APPLY,
  PK_BN_BWD_REDUCE, PK_BN_BWD_FINALIZE, PK_BN_BWD_APPLY, PK_HEAD, PK_SGD, PK_PACK, PK_COPY, PK_ADAM, PK_BN_RUNNING, PK_COUNT
};
static const char* kProfNames[PK_COUNT] = {
  "conv_fprop.generic", "conv_fprop.tiled_c16_w32", "conv_fprop.tiled_c32_w16", "conv_fprop.tiled_c64_w8",
  "conv_dgrad.generic", "conv_dgrad.tiled_c16_w32", "conv_dgrad.tiled_c32_w16", "conv_dgrad.tiled_c64_w8",
  "conv_wgrad.generic", "conv_wgrad.tiled_c16_w32", "conv_wgrad.tiled_c32_w16", "conv_wgrad.tiled_c64_w8",
  "conv_bwd_pair.tiled_c16_w32", "conv_bwd_pair.tiled_c32_w16", "conv_bwd_pair.tiled_c64_w8",
  "conv_fprop.wide", "conv_dgrad.wide", "conv_wgrad.wide", "conv_wgrad.tiled_stride2",
  "wgrad_reduce", "bn_finalize", "bn_apply",
  "bn_bwd_reduce", "bn_bwd_finalize", "bn_bwd_apply", "head", "sgd", "pack_weights", "copy", "adam", "bn_running"};

struct Unit {  // convolution + batch normalisation
  int cin = 0, cout = 0, R = 0, stride = 1, pad = 0;
  int N = 0, H = 0, W = 0, P = 0, Q = 0;
  size_t ow = 0, og = 0, ob = 0;
  void* wpack_f = nullptr;
  void* wpack_d = nullptr;      // input-gradient operand (stale-Jacobian mode: one per ring slot)
  size_t wpack_d_bytes = 0;
  void* z = nullptr;
  float* mean = nullptr;   // mean, invstd, scale, shift, coef[3C] in one allocation
  float* invstd = nullptr;
  float* scale = nullptr;
  float* shift = nullptr;
  float* coef = nullptr;
  ConvArgs fprop{}, dgrad{};
  WgradArgs wg{};
  bool has_dgrad = false;
  int wg_tiled_rows = 0;   // > 0: the LDS-tiled bf16 weight-gradient kernel covers this layer
  int tiled_grid = 0;      // > 0: the LDS-tiled conv kernel covers this layer (forward and dgrad)
  float* wg_partial = nullptr;  // this layer's weight-gradient partial tiles (kept until the update)
  float* fstat = nullptr;       // partial rows of the forward statistics [group][fcap][2][cout]
  float* bstat = nullptr;       // partial rows of the BN-backward sums [brows][2][cout]
  int fcap = 0;                 // rows reserved per group in fstat
  int frows = 0;                // rows written by the last forward conv (per group)
  // consumers finalise the partial rows themselves (their reduction is built for these widths)
  float *rmean = nullptr, *rvar = nullptr;     // running estimates for evaluation
  float *escale = nullptr, *eshift = nullptr;  // evaluation-time scale and shift derived from them
  bool wide_f = false, wide_d = false;   // the GEMM-class kernel runs the forward conv / the input gradient
  int wide_splits = 0;                   // > 0: the GEMM-class weight-gradient kernel, this many pixel slices
  bool small_c() const { return cout == 16 || cout == 32 || cout == 64; }
  int tiled_instance() const { return cin == 16 ? 1 : cin == 32 ? 2 : 3; }   // offset of a tiled kernel's profile kind
  size_t out_elems() const { return (size_t)N * P * Q * cout; }
  size_t in_elems() const { return (size_t)N * H * W * cin; }
  // Group g of the forward buffers. Group 0 is the tape the backward pass reads; a module that
  // runs the forward pass of the current minibatch together with the re-forward of the delayed
  // one keeps a second group right behind the first (conv output, statistics rows, vectors).
  int vec_stride() const { return 7 * cout; }   // floats from a group's mean to the next group's
};

struct Blk {
  int kind = 0;
  std::vector<Unit> u;
  int nmain = 0;
  bool proj = false;
  std::vector<void*> act;  // post-ReLU outputs of the main units except the last
  void* y = nullptr;       // block output
  size_t y_elems = 0;
  // head
  size_t ofcw = 0, ofcb = 0;
  int C = 0, HW = 0;
  float *pooled = nullptr, *dlogits = nullptr, *loss_n = nullptr;
};

struct ddg_module {
  ddg_module_desc d{};
  std::vector<ddg_block_desc> blocks_desc;
  std::vector<Blk> blocks;
  // Second set of forward buffers (conv outputs, statistics, block outputs) for the forward pass
  // on the current minibatch when it runs on its own stream next to the delayed backward.
  std::vector<Blk> fblocks;
  hipStream_t stream = nullptr;    // the stream the call being executed enqueues on
  hipStream_t bstream = nullptr;   // backward / update stream (desc.stream)
  hipStream_t fstream = nullptr;   // forward stream (== bstream unless two_streams)
  bool two_streams = false;
  bool external_sync = false;      // a pipeline orders the two streams; the module records/waits nothing
  hipEvent_t ev_fwd[2] = {nullptr, nullptr};   // forward(t) done, by parity of t
  hipEvent_t ev_upd = nullptr;                 // last update (or parameter load) done
  int delay = 0, nslots = 1;
  int groups = 1;                  // forward buffer groups (2: paired forward, see run_forward_pair;
                                   // K-k+1 in stale-Jacobian mode: one tape per ring slot)
  bool stale = false;              // Eq. 6-7 literally: tapes and weight snapshots per ring slot
  float* theta_snap = nullptr;     // stale: [nslots][nparams] weights as of each kept forward
  const float* theta_bwd = nullptr;   // the weights the backward pass reads (theta, or a snapshot)
  std::vector<PackDesc*> pack_descs_d;   // stale: per-slot tables of the input-gradient operands
  int n_pack_d = 0;
  int out_c = 0, out_h = 0, out_w = 0;
  size_t nparams = 0, in_elems = 0, out_elems = 0, max_act = 0;
  size_t esz = 4;
  float *theta = nullptr, *vel = nullptr, *grad = nullptr;
  // optimizer: momentum SGD, or Adam (Algorithm 2) with the first moment in vel
  int opt = DDG_OPT_SGD;
  float beta1 = 0.9f, beta2 = 0.999f, adam_eps = 1e-8f;
  float* mom2 = nullptr;           // Adam: second moment
  double* adam_pw = nullptr;       // Adam: beta1^n, beta2^n (device)
  long nupd = 0;                   // Adam: updates executed so far (n)
  std::vector<void*> ring;
  void *Ga = nullptr, *Gb = nullptr, *D1 = nullptr, *D2 = nullptr, *D3 = nullptr;
  // dz buffers: units alternate between D1 and D1b, so that the weight gradient of a unit can
  // run one launch late, beside the input-gradient kernel of the unit below
  void* D1b = nullptr; int dz_flip = 0;
  struct PendingWgrad {
    bool on = false; const Unit* u = nullptr;
    const void* x = nullptr; const float* xsc = nullptr; const float* xsh = nullptr; const void* dz = nullptr;
  } pend_w;
  bool defer_wgrad = true;         // DDG_NO_BWD_PAIR=1 switches the deferred weight gradient off
  bool no_defer = false;           // DDG_NO_DEFER=1: every residual block runs its own normalise-add-ReLU pass
  bool premasked = true;           // DDG_NO_PREMASK=1: readers of a stored masked gradient apply the mask again
  bool wide_below = true;          // DDG_NO_WIDE_BELOW=1: wide input-gradient kernels leave the sums of the layer below to a reduction pass
  // Evaluation: running batch-norm estimates, flat per conv unit in parameter order (mean[C],
  // variance[C]), followed in the same allocation by the evaluation scale/shift vectors; one
  // table of layer descriptors per group of forward buffers (the statistics the estimates
  // follow are those of the group that held the current minibatch), plus one for the forward
  // stream's own buffers.
  float* running = nullptr; size_t nrunning = 0;
  float bn_rho = 0.1f;
  std::vector<RunDesc*> run_descs; RunDesc* run_descs_f = nullptr; int n_run = 0, run_max_c = 0;
  int32_t* zero_labels = nullptr;  // head modules: labels for an evaluation without labels
  bool eval_mode = false;          // the forward helpers normalise with the evaluation vectors
  float* ws_stat = nullptr; size_t ws_stat_elems = 0;
  PackDesc* pack_descs = nullptr; int n_pack = 0;     // device tables for the whole-module kernels
  unsigned pack_max = 0;                              // largest packed operand (elements)
  WredDesc* wred_descs = nullptr; int n_wred = 0; int wred_max = 0;   // wred_max: largest Cout*Jp
  std::vector<void*> allocs;
  size_t bytes = 0;
  // state
  long t_next = 0;
  int phase = 0;  // 0: expect forward, 1: expect backward, 2: expect update
  bool has_grad = false;
  bool tape_is_current = false;  // saved activations belong to forward(t) with current weights
  ddg_status sticky = DDG_OK;
  bool skip = false;               // advance state only (a captured graph is replayed instead)
  const float* lr_dev = nullptr;   // step size in device memory, if set
  // profiling
  bool prof = false;
  struct Ev { int kind; hipEvent_t a, b; bool bracket; };
  std::vector<Ev> evs;
  long prof_n[PK_COUNT] = {0};
  double prof_ms[PK_COUNT] = {0};
  double prof_bytes[PK_COUNT] = {0};
  double prof_empty_ms = 0.0;      // mean length of an empty event bracket, subtracted per launch
  double prof_flops[PK_COUNT] = {0};
};

namespace {

bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

ddg_status dev_alloc(ddg_module* m, void** p, size_t bytes) {
  *p = nullptr;
  if (m->d.dry_run || bytes == 0) return DDG_OK;
  bytes = (bytes + 255) & ~(size_t)255;
  hipError_t e = hipMalloc(p, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(e == hipErrorOutOfMemory ? DDG_ERR_OOM : DDG_ERR_DEVICE, "hipMalloc(%zu): %s", bytes,
                hipGetErrorString(e));
  }
  m->allocs.push_back(*p);
  m->bytes += bytes;
  return DDG_OK;
}

// Times one launch when profiling, and books the launch's algorithmic work: bytes = every
// tensor the kernel must read once plus every tensor it must write once, in the storage type;
// flops = 2*M*N*K of a convolution pass. Single-kernel families arm an event pair that the
// launch itself stamps with the kernel's begin and end; families of several kernels are
// bracketed by two stream markers instead.
struct Launch {
  ddg_module* m; int kind; hipEvent_t a = nullptr, b = nullptr; bool bracket = false;
  Launch(ddg_module* m_, int kind_, double bytes = 0.0, double flops = 0.0) : m(m_), kind(kind_) {
    if (m->prof) {
      m->prof_bytes[kind] += bytes; m->prof_flops[kind] += flops;
      (void)hipEventCreate(&a); (void)hipEventCreate(&b);
      bracket = (kind == PK_HEAD || kind == PK_BN_BWD_REDUCE);
      if (bracket) (void)hipEventRecord(a, m->stream);
      else { g_prof_events.a = a; g_prof_events.b = b; g_prof_events.armed = true; }
    }
  }
  ~Launch() {
    if (m->prof) {
      if (bracket) (void)hipEventRecord(b, m->stream);
      const bool launched = bracket || !g_prof_events.armed;
      g_prof_events.armed = false;
      if (launched) m->evs.push_back({kind, a, b, bracket});
      else { (void)hipEventDestroy(a); (void)hipEventDestroy(b); }
    }
  }
};

#define DDG_TRY(expr)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) {                                                                 \
      m->sticky = DDG_ERR_DEVICE;                                                           \
      return fail(DDG_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e_));                  \
    }                                                                                       \
  } while (0)

#define DDG_OKAY(expr)                          \
  do {                                          \
    ddg_status s_ = (expr);                     \
    if (s_ != DDG_OK) return s_;                \
  } while (0)

int out_dim(int h, int stride) { return (h - 1) / stride + 1; }

// ---- plan ---------------------------------------------------------------------------------

ddg_status validate(const ddg_module_desc* d) {
  if (!d) return fail(DDG_ERR_INVALID_ARG, "desc is null");
  if (d->K < 1 || d->k < 1 || d->k > d->K) return fail(DDG_ERR_INVALID_ARG, "need 1 <= k <= K (K=%d k=%d)", d->K, d->k);
  if (d->compute != DDG_F32 && d->compute != DDG_BF16) return fail(DDG_ERR_INVALID_ARG, "compute must be DDG_F32 or DDG_BF16");
  if (d->batch < 1 || d->in_c < 1 || d->in_h < 1 || d->in_w < 1) return fail(DDG_ERR_SHAPE, "input shape must be positive");
  if (d->num_blocks < 1 || !d->blocks) return fail(DDG_ERR_INVALID_ARG, "module needs at least one block");
  if (!(d->momentum >= 0.f && d->momentum < 1.f)) return fail(DDG_ERR_INVALID_ARG, "momentum must be in [0,1)");
  if (!(d->weight_decay >= 0.f)) return fail(DDG_ERR_INVALID_ARG, "weight_decay must be >= 0");
  if (!(d->bn_eps > 0.f)) return fail(DDG_ERR_INVALID_ARG, "bn_eps must be > 0");
  int c = d->in_c, h = d->in_h, w = d->in_w;
  for (int i = 0; i < d->num_blocks; ++i) {
    const ddg_block_desc& b = d->blocks[i];
    if (b.kind < DDG_BLOCK_STEM || b.kind > DDG_BLOCK_HEAD) return fail(DDG_ERR_INVALID_ARG, "block %d: unknown kind %d", i, b.kind);
    if (b.cin != c) return fail(DDG_ERR_SHAPE, "block %d: cin=%d but the incoming tensor has %d channels", i, b.cin, c);
    if (b.kind == DDG_BLOCK_HEAD) {
      if (i != d->num_blocks - 1) return fail(DDG_ERR_SHAPE, "the head must be the last block");
      if (d->num_classes < 2) return fail(DDG_ERR_SHAPE, "a head needs num_classes >= 2");
      if (d->k != d->K) return fail(DDG_ERR_SHAPE, "only the last module (k == K) may end in the head");
      continue;
    }
    if (b.stride != 1 && b.stride != 2) return fail(DDG_ERR_SHAPE, "block %d: stride must be 1 or 2", i);
    if (!is_pow2(b.cout) || b.cout < 16) return fail(DDG_ERR_SHAPE, "block %d: cout=%d must be a power of two >= 16", i, b.cout);
    if (b.kind == DDG_BLOCK_BOTTLENECK && (!is_pow2(b.cmid) || b.cmid < 16))
      return fail(DDG_ERR_SHAPE, "block %d: cmid=%d must be a power of two >= 16", i, b.cmid);
    if (b.kind != DDG_BLOCK_STEM) {
      if (!is_pow2(b.cin) || b.cin < 16) return fail(DDG_ERR_SHAPE, "block %d: cin=%d must be a power of two >= 16", i, b.cin);
      if ((b.stride != 1 || b.cin != b.cout) && !b.projection)
        return fail(DDG_ERR_SHAPE, "block %d: stride/channel change needs a projection shortcut", i);
    } else if (b.cin > 1024) {
      return fail(DDG_ERR_SHAPE, "block %d: stem cin too large", i);
    }
    c = b.cout; h = out_dim(h, b.stride); w = out_dim(w, b.stride);
  }
  const bool has_head = d->blocks[d->num_blocks - 1].kind == DDG_BLOCK_HEAD;
  if (has_head != (d->num_classes > 0)) return fail(DDG_ERR_SHAPE, "num_classes > 0 iff the last block is the head");
  if ((size_t)d->batch * d->in_h * d->in_w * (size_t)(c > d->in_c ? c : d->in_c) > ((size_t)1 << 31) - 1)
    return fail(DDG_ERR_SHAPE, "tensor too large for 32-bit pixel indexing");
  return DDG_OK;
}

void add_unit(Blk& b, size_t& off, int ci, int co, int R, int st, int N, int H, int W) {
  Unit u;
  u.cin = ci; u.cout = co; u.R = R; u.stride = st; u.pad = (R == 3) ? 1 : 0;
  u.N = N; u.H = H; u.W = W; u.P = out_dim(H, st); u.Q = out_dim(W, st);
  u.ow = off; off += (size_t)co * ci * R * R;
  u.og = off; off += co;
  u.ob = off; off += co;
  b.u.push_back(u);
}

ddg_status build_plan(ddg_module* m) {
  const ddg_module_desc& d = m->d;
  const int dt = d.compute;
  m->esz = dtype_size(dt);
  size_t off = 0;
  int c = d.in_c, h = d.in_h, w = d.in_w;
  const int N = d.batch;
  // A module with a delay runs forward(t) and the re-forward of iteration t-K+k in the same
  // launches (same weights, two minibatches): second group of forward buffers.
  auto env_on = [](const char* name) { const char* e = getenv(name); return e && e[0] == '1'; };
  const bool no_pair = env_on("DDG_NO_PAIR");
  m->no_defer = env_on("DDG_NO_DEFER");
  m->premasked = !env_on("DDG_NO_PREMASK");
  m->wide_below = getenv("DDG_NO_WIDE_BELOW") == nullptr;
  const int no_lds32 = env_on("DDG_NO_LDS32") ? 1 : 0;
  m->stale = d.stale_jacobian != 0 && d.K - d.k > 0;
  m->groups = m->stale ? (d.K - d.k + 1) : ((d.K - d.k > 0 && !m->two_streams && !no_pair) ? 2 : 1);
  m->in_elems = (size_t)N * h * w * c;
  m->max_act = m->in_elems;
  for (int i = 0; i < d.num_blocks; ++i) {
    const ddg_block_desc& bd = m->blocks_desc[i];
    Blk b;
    b.kind = bd.kind;
    b.proj = bd.projection != 0;
    if (bd.kind == DDG_BLOCK_HEAD) {
      b.C = c; b.HW = h * w;
      b.ofcw = off; off += (size_t)d.num_classes * c;
      b.ofcb = off; off += d.num_classes;
      m->blocks.push_back(b);
      continue;
    }
    if (bd.kind == DDG_BLOCK_STEM) {
      add_unit(b, off, bd.cin, bd.cout, 3, bd.stride, N, h, w); b.nmain = 1;
    } else if (bd.kind == DDG_BLOCK_BASIC) {
      add_unit(b, off, bd.cin, bd.cout, 3, bd.stride, N, h, w);
      add_unit(b, off, bd.cout, bd.cout, 3, 1, N, b.u[0].P, b.u[0].Q); b.nmain = 2;
      if (b.proj) add_unit(b, off, bd.cin, bd.cout, 1, bd.stride, N, h, w);
    } else {
      add_unit(b, off, bd.cin, bd.cmid, 1, 1, N, h, w);
      add_unit(b, off, bd.cmid, bd.cmid, 3, bd.stride, N, h, w);
      add_unit(b, off, bd.cmid, bd.cout, 1, 1, N, b.u[1].P, b.u[1].Q); b.nmain = 3;
      if (b.proj) add_unit(b, off, bd.cin, bd.cout, 1, bd.stride, N, h, w);
    }
    const bool first_block = (i == 0);
    for (size_t ui = 0; ui < b.u.size(); ++ui) {
      Unit& u = b.u[ui];
      // the gradient w.r.t. the module input is needed unless this is module 1
      const bool reads_module_input = first_block && (ui == 0 || (int)ui == b.nmain);
      u.has_dgrad = !(reads_module_input && d.k == 1);
      if (u.has_dgrad && (u.cin % 16 != 0))
        return fail(DDG_ERR_SHAPE, "block %d: input gradient needs cin %% 16 == 0 (cin=%d)", i, u.cin);
      if (u.out_elems() > m->max_act) m->max_act = u.out_elems();
      if (u.in_elems() > m->max_act) m->max_act = u.in_elems();
      // forward
      ConvArgs& f = u.fprop;
      f.N = N; f.IH = u.H; f.IW = u.W; f.IC = u.cin; f.OH = u.P; f.OW = u.Q; f.OC = u.cout;
      f.R = u.R; f.stride = u.stride; f.pad = u.pad; f.ntaps = u.R * u.R;
      f.M = N * u.P * u.Q; f.dgrad = 0; f.dtype = dt;
      size_t ne = conv_wpack_elems(u.cin, u.cout, u.R, dt, &f.log2cp, &f.ksteps);
      DDG_OKAY(dev_alloc(m, &u.wpack_f, ne * m->esz));
      conv_plan(f);
      u.tiled_grid = (dt == DDG_F32 && no_lds32) ? 0 : conv_tiled_grid(N, u.H, u.W, u.cin, u.cout, u.R, u.stride, dt);
      if (u.tiled_grid > 0) f.grid_x = u.tiled_grid;   // the generic kernel never runs this layer
      u.wide_f = conv_wide_ok(u.cin, u.cout, u.R, u.stride, dt) && !getenv("DDG_NO_WIDE");
      u.wide_d = u.has_dgrad && conv_wide_ok(u.cout, u.cin, u.R, u.stride, dt) && !getenv("DDG_NO_WIDE");
      if (u.wide_f) f.grid_x = conv_wide_rows(f.M);
      u.fcap = f.grid_x;
      u.frows = u.fcap;    // what the forward conv of this layer writes (the same every time)
      size_t st_e = (size_t)f.grid_x * 2 * u.cout;
      if (st_e > m->ws_stat_elems) m->ws_stat_elems = st_e;
      { void* sp = nullptr;
        DDG_OKAY(dev_alloc(m, &sp, m->groups * st_e * sizeof(float)));
        u.fstat = (float*)sp;
        // backward rows come from bn_bwd_reduce (its own grid) or from the tiled input-gradient
        // kernel of the layer above (at most conv_tiled_max_grid() workgroups)
        int brows = bn_bwd_grid(u.out_elems(), u.cout, dt);
        if (conv_tiled_max_grid() > brows) brows = conv_tiled_max_grid();
        // (or from the GEMM-class input-gradient kernel above: one row per 64 pixels)
        if (u.cout % 128 == 0 && conv_wide_rows(N * u.P * u.Q) > brows) brows = conv_wide_rows(N * u.P * u.Q);
        DDG_OKAY(dev_alloc(m, &sp, (size_t)brows * 2 * u.cout * sizeof(float)));
        u.bstat = (float*)sp; }
      // input gradient
      if (u.has_dgrad) {
        ConvArgs& g = u.dgrad;
        g.N = N; g.IH = u.P; g.IW = u.Q; g.IC = u.cout; g.OH = u.H; g.OW = u.W; g.OC = u.cin;
        g.R = u.R; g.stride = u.stride; g.pad = u.pad; g.ntaps = u.R * u.R;
        g.M = N * u.H * u.W; g.dgrad = 1; g.dtype = dt;
        ne = conv_wpack_elems(u.cout, u.cin, u.R, dt, &g.log2cp, &g.ksteps);
        u.wpack_d_bytes = (ne * m->esz + 255) & ~(size_t)255;
        DDG_OKAY(dev_alloc(m, &u.wpack_d, (m->stale ? (size_t)(d.K - d.k + 1) : 1) * u.wpack_d_bytes));
        conv_plan(g);
      }
      // weight gradient
      WgradArgs& wgd = u.wg;
      wgd.N = N; wgd.H = u.H; wgd.W = u.W; wgd.Cin = u.cin; wgd.P = u.P; wgd.Q = u.Q; wgd.Cout = u.cout;
      wgd.R = u.R; wgd.stride = u.stride; wgd.pad = u.pad; wgd.M = N * u.P * u.Q; wgd.dtype = dt;
      wgrad_plan(wgd);
      u.wg_tiled_rows = (dt == DDG_F32 && no_lds32) ? 0 : wgrad_tiled_rows(N, u.H, u.W, u.cin, u.cout, u.R, u.stride, dt);
      if (u.wg_tiled_rows > 0) wgd.msplit = u.wg_tiled_rows;  // the reduce kernel sums this many rows
      if (wgrad_wide_ok(u.cin, u.cout, u.R, u.stride, dt) && !getenv("DDG_NO_WIDE")) {
        u.wide_splits = wgrad_wide_splits(wgd.M, u.cin, u.cout, u.R);
        wgd.msplit = u.wide_splits;
      }
      { void* wp = nullptr;
        DDG_OKAY(dev_alloc(m, &wp, wgrad_partial_elems(wgd) * sizeof(float)));
        u.wg_partial = (float*)wp; }
      const int bg = bn_bwd_grid(u.out_elems(), u.cout, dt);
      st_e = (size_t)bg * 2 * u.cout;
      if (st_e > m->ws_stat_elems) m->ws_stat_elems = st_e;
      // saved tensors and per-channel vectors
      DDG_OKAY(dev_alloc(m, &u.z, m->groups * u.out_elems() * m->esz));
      void* pc = nullptr;
      DDG_OKAY(dev_alloc(m, &pc, (size_t)7 * m->groups * u.cout * sizeof(float)));
      u.mean = (float*)pc; u.invstd = u.mean + u.cout; u.scale = u.invstd + u.cout;
      u.shift = u.scale + u.cout; u.coef = u.shift + u.cout;
    }
    for (int ui = 0; ui + 1 < b.nmain; ++ui) {
      // the activation between two units is materialised only if the consumer cannot derive
      // it from the producer's conv output while loading
      void* a = nullptr;
      const Unit& cons = b.u[ui + 1];
      // the consumer's forward conv and weight gradient both transform while staging (the wide
      // kernels read final scale/shift vectors, which a producer with more than 64 channels has)
      const bool on_load = cons.tiled_grid > 0 || (cons.wide_f && cons.wide_splits > 0 && !b.u[ui].small_c());
      if (!on_load) DDG_OKAY(dev_alloc(m, &a, m->groups * b.u[ui].out_elems() * m->esz));
      b.act.push_back(a);
    }
    b.y_elems = b.u[b.nmain - 1].out_elems();
    DDG_OKAY(dev_alloc(m, &b.y, m->groups * b.y_elems * m->esz));
    c = bd.cout; h = out_dim(h, bd.stride); w = out_dim(w, bd.stride);
    m->blocks.push_back(b);
  }
  m->out_c = c; m->out_h = h; m->out_w = w;
  m->out_elems = (size_t)N * h * w * c;
  m->nparams = off;
  if (d.num_classes > 0) {
    Blk& hb = m->blocks.back();
    void* p = nullptr;
    DDG_OKAY(dev_alloc(m, &p, ((size_t)N * hb.C + (size_t)N * d.num_classes + N) * sizeof(float)));
    hb.pooled = (float*)p; hb.dlogits = hb.pooled + (size_t)N * hb.C; hb.loss_n = hb.dlogits + (size_t)N * d.num_classes;
  }
  void* p = nullptr;
  DDG_OKAY(dev_alloc(m, &p, 4 * m->nparams * sizeof(float) + 2 * sizeof(double)));
  m->theta = (float*)p; m->vel = m->theta + m->nparams; m->grad = m->vel + m->nparams;
  m->mom2 = m->grad + m->nparams;
  m->adam_pw = (double*)((char*)p + ((4 * m->nparams * sizeof(float) + 7) & ~(size_t)7));
  m->delay = d.K - d.k;
  m->nslots = m->delay + 1;
  m->ring.resize(m->nslots, nullptr);
  for (int s = 0; s < m->nslots; ++s) DDG_OKAY(dev_alloc(m, &m->ring[s], m->in_elems * m->esz));
  DDG_OKAY(dev_alloc(m, &m->Ga, m->max_act * m->esz));
  DDG_OKAY(dev_alloc(m, &m->Gb, m->max_act * m->esz));
  DDG_OKAY(dev_alloc(m, &m->D1, m->max_act * m->esz));
  DDG_OKAY(dev_alloc(m, &m->D1b, m->max_act * m->esz));
  if (const char* e = getenv("DDG_NO_BWD_PAIR")) m->defer_wgrad = !(e[0] == '1');
  DDG_OKAY(dev_alloc(m, &m->D2, m->max_act * m->esz));
  DDG_OKAY(dev_alloc(m, &m->D3, m->max_act * m->esz));
  DDG_OKAY(dev_alloc(m, &p, m->ws_stat_elems * sizeof(float)));
  m->ws_stat = (float*)p;
  // device tables: one entry per packed operand / per layer
  // (stale-Jacobian mode: the input-gradient operands are packed per ring slot when a forward
  // pass is kept, from tables of their own; the main table then holds the forward operands only)
  std::vector<PackDesc> pd;
  std::vector<std::vector<PackDesc>> pdd(m->stale ? m->nslots : 0);
  std::vector<WredDesc> wd;
  for (Blk& b : m->blocks)
    for (Unit& u : b.u) {
      for (int mode = 0; mode < 2; ++mode) {
        if (mode == 1 && !u.has_dgrad) continue;
        PackDesc d{};
        const int md = mode == 0 ? 0 : ((u.tiled_grid > 0 || u.wide_d) ? 2 : 1);
        const int kc = md ? u.cout : u.cin, nc = md ? u.cin : u.cout;
        d.W = m->theta + u.ow; d.wpack = mode == 0 ? u.wpack_f : u.wpack_d;
        d.Cout = u.cout; d.Cin = u.cin; d.R = u.R; d.mode = md;
        d.total = (unsigned)conv_wpack_elems(kc, nc, u.R, dt, &d.log2cp, &d.ksteps);
        d.OCB = nc / 16;
        if (d.total > m->pack_max) m->pack_max = d.total;
        if (mode == 1 && m->stale) {
          for (int j = 0; j < m->nslots; ++j) { d.wpack = (char*)u.wpack_d + (size_t)j * u.wpack_d_bytes; pdd[j].push_back(d); }
        } else {
          pd.push_back(d);
        }
      }
      WredDesc w{};
      w.partial = u.wg_partial; w.dW = m->grad + u.ow; w.rows = u.wg.msplit; w.Cout = u.cout; w.Cin = u.cin;
      w.R = u.R; w.log2cp = u.wg.log2cp; w.Jp = u.wg.JB * 16;
      wd.push_back(w);
      if (w.Cout * w.Jp > m->wred_max) m->wred_max = w.Cout * w.Jp;
    }
  m->n_pack = (int)pd.size(); m->n_wred = (int)wd.size();
  if (!d.dry_run && m->n_pack) {
    DDG_OKAY(dev_alloc(m, &p, pd.size() * sizeof(PackDesc)));
    m->pack_descs = (PackDesc*)p;
    DDG_OKAY(dev_alloc(m, &p, wd.size() * sizeof(WredDesc)));
    m->wred_descs = (WredDesc*)p;
    if (hipMemcpy(m->pack_descs, pd.data(), pd.size() * sizeof(PackDesc), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(m->wred_descs, wd.data(), wd.size() * sizeof(WredDesc), hipMemcpyHostToDevice) != hipSuccess)
      return fail(DDG_ERR_DEVICE, "copying the layer tables failed");
    for (size_t j = 0; j < pdd.size(); ++j) {
      m->n_pack_d = (int)pdd[j].size();
      if (!m->n_pack_d) break;
      DDG_OKAY(dev_alloc(m, &p, pdd[j].size() * sizeof(PackDesc)));
      m->pack_descs_d.push_back((PackDesc*)p);
      if (hipMemcpy(p, pdd[j].data(), pdd[j].size() * sizeof(PackDesc), hipMemcpyHostToDevice) != hipSuccess)
        return fail(DDG_ERR_DEVICE, "copying the layer tables failed");
    }
  }
  if (m->stale && !d.dry_run) {
    DDG_OKAY(dev_alloc(m, &p, (size_t)m->nslots * m->nparams * sizeof(float)));
    m->theta_snap = (float*)p;
  }
  m->theta_bwd = m->theta;
  if (!d.dry_run) {
    hipError_t e = hipMemsetAsync(m->theta, 0, 4 * m->nparams * sizeof(float), m->stream);
    if (e == hipSuccess) {
      const double one[2] = {1.0, 1.0};   // beta^0
      e = hipMemcpy(m->adam_pw, one, sizeof one, hipMemcpyHostToDevice);
    }
    if (e != hipSuccess) return fail(DDG_ERR_DEVICE, "hipMemsetAsync: %s", hipGetErrorString(e));
  }
  return DDG_OK;
}

// ---- enqueue helpers ---------------------------------------------------------------------

ddg_status pack_all(ddg_module* m) {
  Launch L(m, PK_PACK);
  DDG_TRY(pack_all_launch(m->pack_descs, m->n_pack, m->d.compute, m->stream, m->pack_max));
  return DDG_OK;
}

// The LDS-tiled kernels for the module's operand type (same arguments for both).
static hipError_t conv_tiled_any(const ddg_module* m, const void* in, const float* scale, const float* shift,
                                 const BnRows* in_rows, const void* wpack, void* out, const ConvStat& st, const void* add_g,
                                 const void* add_mask, int N, int H, int W, int C, int grid, hipStream_t s,
                                 const void* res = nullptr, void* y_out = nullptr, int groups = 1, int vec_stride = 0,
                                 const WgradFuse* apply = nullptr, const WgradPair* pair = nullptr) {
  if (m->d.compute == DDG_BF16)
    return conv_tiled_launch(in, scale, shift, in_rows, wpack, out, st, add_g, add_mask, N, H, W, C, grid, s, res, y_out,
                             groups, vec_stride, apply, pair);
  return conv_tiled_f32_launch(in, scale, shift, in_rows, wpack, out, st, add_g, add_mask, N, H, W, C, grid, s, res, y_out,
                               groups, vec_stride, apply, pair);
}
static hipError_t wgrad_tiled_any(const ddg_module* m, const void* x, const float* scale, const float* shift, const void* dz,
                                  const WgradFuse* fuse, float* partial, int N, int H, int W, int C, int rows, hipStream_t s,
                                  int Cout = 0, int R = 3, int stride = 1) {
  if (m->d.compute == DDG_BF16) return wgrad_tiled_launch(x, scale, shift, dz, fuse, partial, N, H, W, C, rows, s, Cout, R, stride);
  if ((Cout != 0 && Cout != C) || R != 3 || stride != 1) return hipErrorInvalidValue;
  return wgrad_tiled_f32_launch(x, scale, shift, dz, fuse, partial, N, H, W, C, rows, s);
}

// Algorithmic work of one convolution pass over unit u.
double conv_flops(const Unit& u) { return 2.0 * u.N * u.P * u.Q * (double)u.cout * u.cin * u.R * u.R; }
double wbytes(const ddg_module* m, const Unit& u) { return (double)u.cout * u.cin * u.R * u.R * m->esz; }

// Pointer to group g of a forward buffer whose groups are `bytes` apart.
static inline const void* grp(const void* p, size_t bytes, int g) { return p ? (const char*)p + (size_t)g * bytes : nullptr; }
static inline void* grp(void* p, size_t bytes, int g) { return p ? (char*)p + (size_t)g * bytes : nullptr; }

// The forward statistics of u (group g) as partial rows for a consuming kernel.
BnRows fwd_rows(ddg_module* m, Unit& u, int g = 0) {
  BnRows r{};
  r.partial = u.fstat + (size_t)g * u.fcap * 2 * u.cout; r.rows = u.frows;
  r.gamma = m->theta + u.og; r.beta = m->theta + u.ob;
  r.count = (float)((size_t)u.N * u.P * u.Q); r.eps = m->d.bn_eps;
  const int vo = g * u.vec_stride();
  r.mean = u.mean + vo; r.invstd = u.invstd + vo; r.scale = u.scale + vo; r.shift = u.shift + vo;
  return r;
}

// conv of one unit: in -> u.z plus partial rows of its batch statistics. For 16/32/64 channels
// the consumer of the BN output derives mean/invstd/scale/shift from the rows (and stores
// them); wider layers get a finalise launch here. `src`, if given, is the unit whose BN + ReLU
// produces this conv's input from `in` while loading (LDS-tiled kernel only). With `res` the
// input is the output of the residual block before, relu(bn(in) + res), which the kernel also
// stores to y_store: that block's separate normalise-add-ReLU pass is absorbed.
// Groups: the launch covers G minibatches starting with group g (G = 2 needs g = 0 and the
// tiled kernel); in, res and y_store point at group g, whose successors follow contiguously.
ddg_status unit_forward(ddg_module* m, Unit& u, const void* in, Unit* src, const void* res = nullptr,
                        void* y_store = nullptr, int G = 1, int g = 0) {
  if (res && !(u.tiled_grid > 0 && src)) return fail(DDG_ERR_STATE, "internal: residual input needs the tiled kernel");
  if (G > 1 && !(u.tiled_grid > 0 && g == 0 && G <= m->groups)) return fail(DDG_ERR_STATE, "internal: grouped launch needs the tiled kernel");
  void* z = grp(u.z, u.out_elems() * m->esz, g);
  float* fstat = u.fstat + (size_t)g * u.fcap * 2 * u.cout;
  const int vo = g * u.vec_stride();
  if (u.tiled_grid > 0) {
    u.frows = u.tiled_grid;
    ConvStat st{};
    st.mode = 1; st.partial = fstat;
    BnRows ir{};
    const bool from_rows = src && src->small_c() && !m->eval_mode;
    if (from_rows) ir = fwd_rows(m, *src, g);
    const int svo = src ? g * src->vec_stride() : 0;
    const float* ssc = !src ? nullptr : (m->eval_mode ? src->escale : src->scale + svo);
    const float* ssh = !src ? nullptr : (m->eval_mode ? src->eshift : src->shift + svo);
    Launch L(m, PK_CONV_FPROP + u.tiled_instance(),
             G * (((res ? 3.0 : 1.0) * u.in_elems() + u.out_elems()) * (double)m->esz) + wbytes(m, u), G * conv_flops(u));
    DDG_TRY(conv_tiled_any(m, in, (src && !from_rows) ? ssc : nullptr, (src && !from_rows) ? ssh : nullptr,
                              from_rows ? &ir : nullptr, u.wpack_f, z, st, nullptr, nullptr, G * u.N, u.H, u.W,
                              u.cin, G * u.tiled_grid, m->stream, res, y_store, G, src ? src->vec_stride() : 0));
  } else {
    if (src && !u.wide_f) return fail(DDG_ERR_STATE, "internal: generic conv needs a materialised input");
    if (u.wide_f) {
      u.frows = conv_wide_rows(u.N * u.P * u.Q);
      const int svo = src ? g * src->vec_stride() : 0;   // (a wide producer's vectors are final: it ran its finalise launch)
      Launch L(m, PK_CONV_FPROP_WIDE, (u.in_elems() + u.out_elems()) * (double)m->esz + wbytes(m, u), conv_flops(u));
      DDG_TRY(conv_wide_launch(in, u.wpack_f, z, fstat, nullptr, nullptr, u.N, u.H, u.W, u.cin, u.cout, u.R, m->stream,
                               !src ? nullptr : (m->eval_mode ? src->escale : src->scale + svo),
                               !src ? nullptr : (m->eval_mode ? src->eshift : src->shift + svo)));
    } else {
      ConvArgs a = u.fprop;
      conv_plan(a);
      u.frows = a.grid_x;
      a.in = in; a.wpack = u.wpack_f; a.out = z; a.stat_partial = fstat; a.add_g = nullptr; a.add_mask = nullptr;
      Launch L(m, PK_CONV_FPROP, (u.in_elems() + u.out_elems()) * (double)m->esz + wbytes(m, u), conv_flops(u));
      DDG_TRY(conv_launch(a, m->stream));
    }
  }
  if (!u.small_c() && !m->eval_mode) {   // (evaluation normalises with the running estimates)
    Launch L(m, PK_BN_FINALIZE);
    DDG_TRY(bn_finalize_launch(fstat, u.frows, u.cout, m->theta + u.og, m->theta + u.ob,
                               (float)((size_t)u.N * u.P * u.Q), m->d.bn_eps, u.mean + vo, u.invstd + vo, u.scale + vo,
                               u.shift + vo, m->stream));
  }
  return DDG_OK;
}

// y = relu(bn(u.z) [+ shortcut]) for group g; the shortcut is `res` itself or, with ru, bn(ru->z)
// of a projection unit. res and y point at group g.
ddg_status apply_bn(ddg_module* m, Unit& u, const void* res, Unit* ru, void* y, int g = 0) {
  BnRows zr{}, rr{};
  const bool zrows = u.small_c() && !m->eval_mode, rrows = ru && ru->small_c() && !m->eval_mode;
  if (zrows) zr = fwd_rows(m, u, g);
  if (rrows) rr = fwd_rows(m, *ru, g);
  const int vo = g * u.vec_stride(), rvo = ru ? g * ru->vec_stride() : 0;
  Launch L(m, PK_BN_APPLY, ((res || ru) ? 3.0 : 2.0) * u.out_elems() * m->esz);
  const bool ev = m->eval_mode;
  DDG_TRY(bn_apply_launch(grp(u.z, u.out_elems() * m->esz, g), ev ? u.escale : u.scale + vo, ev ? u.eshift : u.shift + vo,
                          zrows ? &zr : nullptr,
                          ru ? grp(ru->z, ru->out_elems() * m->esz, g) : res, !ru ? nullptr : (ev ? ru->escale : ru->scale + rvo),
                          !ru ? nullptr : (ev ? ru->eshift : ru->shift + rvo), rrows ? &rr : nullptr, y, u.out_elems(), u.cout, 1,
                          m->d.compute, m->stream));
  return DDG_OK;
}

// One block, one group, nothing deferred: x -> y.
ddg_status block_forward(ddg_module* m, Blk& b, const void* x, void* y, int g) {
  const void* cur = x;
  Unit* src = nullptr;   // pending relu(bn(.)) of `cur`
  for (int i = 0; i < b.nmain; ++i) {
    Unit& u = b.u[i];
    DDG_OKAY(unit_forward(m, u, cur, src, nullptr, nullptr, 1, g));
    src = nullptr;
    if (i + 1 < b.nmain) {
      if (b.act[i]) {
        void* act = grp(b.act[i], u.out_elems() * m->esz, g);
        DDG_OKAY(apply_bn(m, u, nullptr, nullptr, act, g));
        cur = act;
      } else {
        cur = grp(u.z, u.out_elems() * m->esz, g); src = &u;   // the next conv applies BN + ReLU while loading
      }
    }
  }
  Unit& ul = b.u[b.nmain - 1];
  if (b.kind == DDG_BLOCK_STEM) return apply_bn(m, ul, nullptr, nullptr, y, g);
  if (b.proj) {
    Unit& up = b.u[b.nmain];
    DDG_OKAY(unit_forward(m, up, x, nullptr, nullptr, nullptr, 1, g));
    return apply_bn(m, ul, nullptr, &up, y, g);
  }
  return apply_bn(m, ul, x, nullptr, y, g);
}

// The same conv for the two minibatches of a paired forward pass (groups 0 and 1) in one launch
// where the kernel can: the tiled kernel when the two inputs lie one group apart, the generic
// and the GEMM-class kernels always (they take a second set of pointers).
ddg_status unit_forward_two(ddg_module* m, Unit& u, const void* in0, const void* in1, Unit* src) {
  if (u.tiled_grid > 0) {
    if ((const char*)in1 == (const char*)in0 + u.in_elems() * m->esz) return unit_forward(m, u, in0, src, nullptr, nullptr, 2, 0);
    DDG_OKAY(unit_forward(m, u, in0, src, nullptr, nullptr, 1, 0));
    return unit_forward(m, u, in1, src, nullptr, nullptr, 1, 1);
  }
  if (src && !u.wide_f) return fail(DDG_ERR_STATE, "internal: generic conv needs a materialised input");
  void* z1 = grp(u.z, u.out_elems() * m->esz, 1);
  float* fstat1 = u.fstat + (size_t)u.fcap * 2 * u.cout;
  const double bytes = 2.0 * ((u.in_elems() + u.out_elems()) * (double)m->esz) + wbytes(m, u);
  if (u.wide_f) {
    u.frows = conv_wide_rows(u.N * u.P * u.Q);
    const int sv = src ? src->vec_stride() : 0;
    ConvWideSecond sec{in1, z1, fstat1, src ? src->scale + sv : nullptr, src ? src->shift + sv : nullptr};
    Launch L(m, PK_CONV_FPROP_WIDE, bytes, 2.0 * conv_flops(u));
    DDG_TRY(conv_wide_launch(in0, u.wpack_f, u.z, u.fstat, nullptr, nullptr, u.N, u.H, u.W, u.cin, u.cout, u.R, m->stream,
                             src ? src->scale : nullptr, src ? src->shift : nullptr, &sec));
  } else {
    ConvArgs a = u.fprop;
    conv_plan(a);
    u.frows = a.grid_x;
    a.in = in0; a.wpack = u.wpack_f; a.out = u.z; a.stat_partial = u.fstat; a.add_g = nullptr; a.add_mask = nullptr;
    a.in_b = in1; a.out_b = z1; a.stat_partial_b = fstat1;
    Launch L(m, PK_CONV_FPROP, bytes, 2.0 * conv_flops(u));
    DDG_TRY(conv_launch(a, m->stream));
  }
  if (!u.small_c()) {
    Launch L(m, PK_BN_FINALIZE);
    DDG_TRY(bn_finalize_launch(u.fstat, u.frows, u.cout, m->theta + u.og, m->theta + u.ob,
                               (float)((size_t)u.N * u.P * u.Q), m->d.bn_eps, u.mean, u.invstd, u.scale, u.shift, m->stream,
                               fstat1, u.mean + u.vec_stride()));
  }
  return DDG_OK;
}

// y = relu(bn(u.z) [+ shortcut]) for both groups in one launch (see apply_bn).
ddg_status apply_bn_two(ddg_module* m, Unit& u, const void* res0, const void* res1, Unit* ru, void* y0, void* y1) {
  const int V = m->d.compute == DDG_BF16 ? 8 : 4;
  if ((256 * V) % u.cout != 0) {   // not covered by the two-set kernel
    DDG_OKAY(apply_bn(m, u, res0, ru, y0, 0));
    return apply_bn(m, u, res1, ru, y1, 1);
  }
  BnApplySet st[2];
  const bool zrows = u.small_c(), rrows = ru && ru->small_c();
  for (int g = 0; g < 2; ++g) {
    BnApplySet& q = st[g];
    q = BnApplySet{};
    const int vo = g * u.vec_stride(), rvo = ru ? g * ru->vec_stride() : 0;
    q.z = grp(u.z, u.out_elems() * m->esz, g); q.scale = u.scale + vo; q.shift = u.shift + vo;
    if (zrows) q.zrows = fwd_rows(m, u, g);
    q.res = ru ? grp(ru->z, ru->out_elems() * m->esz, g) : (g ? res1 : res0);
    q.rscale = ru ? ru->scale + rvo : nullptr; q.rshift = ru ? ru->shift + rvo : nullptr;
    if (rrows) q.rrows = fwd_rows(m, *ru, g);
    q.y = g ? y1 : y0;
  }
  Launch L(m, PK_BN_APPLY, 2.0 * ((res0 || ru) ? 3.0 : 2.0) * u.out_elems() * m->esz);
  hipError_t e = hipSuccess;
  if (!bn_apply_pair_launch(st[0], st[1], u.out_elems(), u.cout, 1, m->d.compute, m->stream, &e))
    return fail(DDG_ERR_STATE, "internal: two-set normalisation not covered");
  DDG_TRY(e);
  return DDG_OK;
}

// One block for both groups of a paired forward pass, nothing deferred: (x0, x1) -> (y0, y1).
ddg_status block_forward_two(ddg_module* m, Blk& b, const void* x0, const void* x1, void* y0, void* y1) {
  const void* c0 = x0; const void* c1 = x1;
  Unit* src = nullptr;   // pending relu(bn(.)) of the current tensors
  for (int i = 0; i < b.nmain; ++i) {
    Unit& u = b.u[i];
    DDG_OKAY(unit_forward_two(m, u, c0, c1, src));
    src = nullptr;
    if (i + 1 < b.nmain) {
      if (b.act[i]) {
        void* a0 = b.act[i]; void* a1 = grp(b.act[i], u.out_elems() * m->esz, 1);
        DDG_OKAY(apply_bn_two(m, u, nullptr, nullptr, nullptr, a0, a1));
        c0 = a0; c1 = a1;
      } else {
        c0 = u.z; c1 = grp(u.z, u.out_elems() * m->esz, 1); src = &u;
      }
    }
  }
  Unit& ul = b.u[b.nmain - 1];
  if (b.kind == DDG_BLOCK_STEM) return apply_bn_two(m, ul, nullptr, nullptr, nullptr, y0, y1);
  if (b.proj) {
    Unit& up = b.u[b.nmain];
    DDG_OKAY(unit_forward_two(m, up, x0, x1, nullptr));
    return apply_bn_two(m, ul, nullptr, nullptr, &up, y0, y1);
  }
  return apply_bn_two(m, ul, x0, x1, nullptr, y0, y1);
}

// An identity block of the LDS-tiled shapes, whose convs can take two groups in one launch and
// whose first conv can absorb the normalise-add-ReLU of the block before.
static bool tiled_identity_block(const Blk& b) {
  return b.kind == DDG_BLOCK_BASIC && !b.proj && b.nmain == 2 && b.u[0].tiled_grid > 0 && b.u[1].tiled_grid > 0 &&
         b.u[0].cin == b.u[0].cout;
}

// Paired forward: the stored minibatch in0 goes through group 0 (the tape the backward pass
// reads), the current minibatch in1 through group 1 (only its last block output, out1, is
// kept). Both use the same weights, so wherever a block is of the tiled identity kind and its
// input lies in the module's own two-group buffers, one launch serves both minibatches (each
// with its own batch statistics); other blocks run once per group.
ddg_status run_forward_pair(ddg_module* m, std::vector<Blk>& blocks, const void* in0, const void* in1, void* out1) {
  const int nres = (int)blocks.size() - (m->d.num_classes > 0 ? 1 : 0);
  const bool no_defer = m->no_defer;
  const void* x0 = in0; const void* x1 = in1;
  struct { Unit* u = nullptr; const void* res = nullptr; void* y = nullptr; } pend;   // group-0 pointers
  for (int bi = 0; bi < nres; ++bi) {
    Blk& b = blocks[bi];
    const bool last = bi == nres - 1;
    void* y0 = b.y;
    void* y1 = last ? out1 : grp(b.y, b.y_elems * m->esz, 1);
    // both groups' inputs are contiguous from the second block on
    const bool both = bi >= 1 && tiled_identity_block(b);
    if (!both) {
      if (pend.u) return fail(DDG_ERR_STATE, "internal: deferred block output without a consumer");
      DDG_OKAY(block_forward_two(m, b, x0, x1, y0, y1));
    } else {
      Unit& u0 = b.u[0]; Unit& u1 = b.u[1];
      if (pend.u) {
        DDG_OKAY(unit_forward(m, u0, pend.u->z, pend.u, pend.res, pend.y, 2, 0));
        x0 = pend.y; x1 = grp(pend.y, b.y_elems * m->esz, 1);   // materialised by that launch (same shape as this block's)
        pend.u = nullptr;
      } else {
        DDG_OKAY(unit_forward(m, u0, x0, nullptr, nullptr, nullptr, 2, 0));
      }
      DDG_OKAY(unit_forward(m, u1, u0.z, &u0, nullptr, nullptr, 2, 0));
      const bool defer = !no_defer && !last && bi + 1 < nres && tiled_identity_block(blocks[bi + 1]) &&
                         blocks[bi + 1].u[0].cin == u1.cout && blocks[bi + 1].u[0].H == u1.P && blocks[bi + 1].u[0].W == u1.Q;
      if (defer) { pend.u = &u1; pend.res = x0; pend.y = y0; }
      else DDG_OKAY(apply_bn_two(m, u1, x0, x1, nullptr, y0, y1));
    }
    x0 = y0; x1 = y1;
  }
  return DDG_OK;
}

// Forward through all residual blocks. `final_out`, if given, receives the last block's
// output instead of the module's own buffer (used when the tape is not needed).
ddg_status run_forward(ddg_module* m, std::vector<Blk>& blocks, const void* in, void* final_out) {
  const void* x = in;
  const int nres = (int)blocks.size() - (m->d.num_classes > 0 ? 1 : 0);
  // An identity block followed by another identity block of the same shape does not run its
  // own normalise-add-ReLU pass: the next block's first conv forms y = relu(bn(z) + x) while
  // loading and stores it (`pend` carries what that conv needs).
  const bool no_defer = m->no_defer;
  struct { Unit* u = nullptr; const void* res = nullptr; void* y = nullptr; } pend;
  for (int bi = 0; bi < nres; ++bi) {
    Blk& b = blocks[bi];
    void* yout = (bi == nres - 1 && final_out) ? final_out : b.y;
    const void* cur = x;
    Unit* src = nullptr;   // pending relu(bn(.)) of `cur`
    const void* res_in = nullptr;
    void* y_store = nullptr;
    if (pend.u) {
      cur = pend.u->z; src = pend.u; res_in = pend.res; y_store = pend.y;
      x = pend.y;          // materialised by this block's first conv
      pend.u = nullptr;
    }
    for (int i = 0; i < b.nmain; ++i) {
      Unit& u = b.u[i];
      DDG_OKAY(unit_forward(m, u, cur, src, i == 0 ? res_in : nullptr, i == 0 ? y_store : nullptr));
      src = nullptr;
      if (i + 1 < b.nmain) {
        if (b.act[i]) {
          DDG_OKAY(apply_bn(m, u, nullptr, nullptr, b.act[i]));
          cur = b.act[i];
        } else {
          cur = u.z; src = &u;   // the next conv applies BN + ReLU while loading
        }
      }
    }
    Unit& ul = b.u[b.nmain - 1];
    if (b.kind == DDG_BLOCK_STEM) {
      DDG_OKAY(apply_bn(m, ul, nullptr, nullptr, yout));
    } else if (b.proj) {
      Unit& up = b.u[b.nmain];
      DDG_OKAY(unit_forward(m, up, x, nullptr));
      DDG_OKAY(apply_bn(m, ul, nullptr, &up, yout));
    } else {
      bool defer = false;
      if (!no_defer && bi + 1 < nres && b.kind == DDG_BLOCK_BASIC && ul.tiled_grid > 0) {
        const Blk& nb = blocks[bi + 1];
        defer = nb.kind == DDG_BLOCK_BASIC && !nb.proj && nb.u[0].tiled_grid > 0 && nb.u[0].cin == ul.cout &&
                nb.u[0].H == ul.P && nb.u[0].W == ul.Q;
      }
      if (defer) { pend.u = &ul; pend.res = x; pend.y = yout; }
      else DDG_OKAY(apply_bn(m, ul, x, nullptr, yout));
    }
    x = yout;
  }
  return DDG_OK;
}

// What the BN-backward sums of a unit need: its ReLU mask and the tensors they read.
struct BelowBn {
  const Unit* u = nullptr;           // the conv+BN unit whose backward comes next
  const void* mask = nullptr;        // its ReLU was active where mask*mscale+mshift > 0
  const float* mscale = nullptr;
  const float* mshift = nullptr;
};

// Launches the weight gradient a unit left for later (plain: its dz is in memory by now).
ddg_status flush_pending_wgrad(ddg_module* m) {
  if (!m->pend_w.on) return DDG_OK;
  const ddg_module::PendingWgrad w = m->pend_w;
  m->pend_w.on = false;
  const Unit& u = *w.u;
  Launch L(m, PK_CONV_WGRAD + u.tiled_instance(), (u.in_elems() + (double)u.out_elems()) * m->esz + wbytes(m, u) * 4.0 / m->esz,
           conv_flops(u));
  DDG_TRY(wgrad_tiled_any(m, w.x, w.xsc, w.xsh, w.dz, nullptr, u.wg_partial, u.N, u.H, u.W, u.cin, u.wg_tiled_rows,
                             m->stream));
  return DDG_OK;
}

// BN backward + weight gradient (+ input gradient) of one unit.
//   dy: gradient w.r.t. the ReLU output that follows this unit's BN; the ReLU was active where
//       mask > 0 (or mask*mscale+mshift > 0); mask == null: no ReLU in between
//   stats_rows > 0: the partial rows (sum g, sum g*xhat) of this unit are already in the
//       statistics workspace, written by the kernel that produced dy (that many rows)
//   x_in: the unit's conv input, or with x_scale the tensor it derives from by relu(x*s+t)
//   dx: where the input gradient goes (null: not needed); add_g/add_mask: optional term added
//       to dx in the same kernel
//   below: if given and the input-gradient kernel supports it, that kernel also forms the
//       BN-backward sums of the unit below from dx and stores dx multiplied by that unit's ReLU
//       mask; *below_rows > 0 reports that it did (the readers of dx then pass mask = null)
ddg_status unit_backward(ddg_module* m, Unit& u, const void* dy, const void* mask, const float* mscale,
                         const float* mshift, int stats_rows, const void* x_in, const float* x_scale,
                         const float* x_shift, void* dz_buf, void* dx, const void* add_g, const void* add_mask,
                         const BelowBn* below, int* below_rows) {
  const int dt = m->d.compute;
  const size_t E = u.out_elems();
  if (below_rows) *below_rows = 0;
  dz_buf = m->dz_flip ? m->D1b : m->D1;   // not the buffer a pending weight gradient reads
  m->dz_flip ^= 1;
  if (stats_rows <= 0) {
    stats_rows = bn_bwd_grid(E, u.cout, dt);
    Launch L(m, PK_BN_BWD_REDUCE, (mask && mask != u.z ? 3.0 : 2.0) * E * m->esz);
    DDG_TRY(bn_bwd_reduce_launch(dy, mask, mscale, mshift, u.z, u.mean, u.invstd, u.bstat, E, u.cout, dt, m->stream));
  }
  BnBwdRows br{};
  br.partial = u.bstat; br.rows = stats_rows; br.gamma = m->theta_bwd + u.og; br.mean = u.mean; br.invstd = u.invstd;
  br.count = (float)((size_t)u.N * u.P * u.Q); br.dgamma = m->grad + u.og; br.dbeta = m->grad + u.ob;
  if (m->defer_wgrad && u.wg_tiled_rows > 0 && u.tiled_grid > 0 && dx && dx != dy) {   // (a halo kernel cannot work in place)
    // The input-gradient kernel forms dz = BN-backward(dy) while staging (coefficients from the
    // rows), stores it, convolves it, and forms the sums of the unit below in its epilogue. The
    // weight gradient of this unit then needs nothing but dz and the input: it runs one launch
    // late, in the same launch as the next unit's input-gradient kernel.
    WgradFuse f{};
    f.dy = dy; f.mask = mask; f.mscale = mscale; f.mshift = mshift; f.z = u.z; f.coef = nullptr; f.rows = &br;
    f.dz_out = dz_buf;
    ConvStat st{};
    double extra = (add_g ? (add_mask ? 2.0 : 1.0) : 0.0);
    if (below && below->u) {
      st.mode = 2; st.partial = below->u->bstat;
      st.mask = below->mask; st.mscale = below->mscale; st.mshift = below->mshift;
      st.z = below->u->z; st.zmean = below->u->mean; st.zinvstd = below->u->invstd;
      if (below_rows) *below_rows = u.tiled_grid;
      extra += (below->mask == below->u->z) ? 1.0 : 2.0;
    }
    // a pending weight gradient of the same shape rides in this launch
    const ddg_module::PendingWgrad pw = m->pend_w;
    const bool ride = pw.on && pw.u->cin == u.cin && pw.u->W == u.W && pw.u->H == u.H && pw.u->N == u.N;
    if (!ride) DDG_OKAY(flush_pending_wgrad(m));
    {
      // reads dy, z (and the mask tensor if it is a different one) and the weights, writes dz and
      // dx; plus the shortcut term and what the sums of the unit below read; plus, for a weight
      // gradient that rides along, its input and dz read and its partial tiles written
      double bytes = ((mask && mask != u.z ? 4.0 : 3.0) * E + (1.0 + extra) * u.in_elems()) * m->esz + wbytes(m, u);
      double flops = conv_flops(u);
      WgradPair wp{};
      if (ride) {
        wp.x = pw.x; wp.scale = pw.xsc; wp.shift = pw.xsh; wp.dz = pw.dz; wp.partial = pw.u->wg_partial; wp.rows = pw.u->wg_tiled_rows;
        bytes += (pw.u->in_elems() + (double)pw.u->out_elems()) * m->esz + wbytes(m, *pw.u) * 4.0 / m->esz;
        flops += conv_flops(*pw.u);
        m->pend_w.on = false;
      }
      Launch L(m, (ride ? PK_BWD_PAIR : PK_CONV_DGRAD) + u.tiled_instance(), bytes, flops);
      DDG_TRY(conv_tiled_any(m, dy, nullptr, nullptr, nullptr, u.wpack_d, dx, st, add_g, add_mask, u.N, u.H, u.W,
                                u.cin, u.tiled_grid, m->stream, nullptr, nullptr, 1, 0, &f, ride ? &wp : nullptr));
    }
    m->pend_w.on = true; m->pend_w.u = &u; m->pend_w.x = x_in; m->pend_w.xsc = x_scale; m->pend_w.xsh = x_shift;
    m->pend_w.dz = dz_buf;
    return DDG_OK;
  }
  DDG_OKAY(flush_pending_wgrad(m));
  WgradArgs w = u.wg;
  w.x = x_in; w.dz = dz_buf; w.partial = u.wg_partial; w.dW = m->grad + u.ow;
  if (u.wg_tiled_rows > 0) {
    // one kernel: dz = BN-backward(dy) formed while staging (coefficients from the rows),
    // written to dz_buf for the input gradient, and contracted with the input for dW
    WgradFuse f{};
    f.dy = dy; f.mask = mask; f.mscale = mscale; f.mshift = mshift; f.z = u.z; f.coef = nullptr; f.rows = &br;
    f.dz_out = dz_buf;
    // reads x, dy, z (and the mask tensor if it is a different one), writes dz and dW
    Launch L(m, u.stride == 2 ? PK_CONV_WGRAD_S2 : PK_CONV_WGRAD + u.tiled_instance(),
             (u.in_elems() + (mask && mask != u.z ? 4.0 : 3.0) * E) * m->esz + wbytes(m, u) * 4.0 / m->esz, conv_flops(u));
    DDG_TRY(wgrad_tiled_any(m, x_in, x_scale, x_shift, nullptr, &f, u.wg_partial, u.N, u.H, u.W, u.cin,
                               u.wg_tiled_rows, m->stream, u.cout, u.R, u.stride));
  } else {
    if (u.small_c()) {
      // the apply kernel derives dgamma, dbeta and its coefficients from the rows
      Launch L(m, PK_BN_BWD_APPLY, (mask && mask != u.z ? 4.0 : 3.0) * E * m->esz);
      DDG_TRY(bn_bwd_apply_launch(dy, mask, mscale, mshift, u.z, nullptr, &br, dz_buf, E, u.cout, dt, m->stream));
    } else {
      { Launch L(m, PK_BN_BWD_FINALIZE);
        DDG_TRY(bn_bwd_finalize_launch(u.bstat, stats_rows, u.cout, m->theta_bwd + u.og, u.mean, u.invstd,
                                       (float)((size_t)u.N * u.P * u.Q), m->grad + u.og, m->grad + u.ob, u.coef, m->stream)); }
      Launch L(m, PK_BN_BWD_APPLY, (mask && mask != u.z ? 4.0 : 3.0) * E * m->esz);
      DDG_TRY(bn_bwd_apply_launch(dy, mask, mscale, mshift, u.z, u.coef, nullptr, dz_buf, E, u.cout, dt, m->stream));
    }
    if (x_scale && u.wide_splits == 0) return fail(DDG_ERR_STATE, "internal: generic weight gradient needs a materialised input");
    Launch L(m, u.wide_splits > 0 ? PK_CONV_WGRAD_WIDE : PK_CONV_WGRAD,
             (u.in_elems() + E) * (double)m->esz + wbytes(m, u) * 4.0 / m->esz, conv_flops(u));
    if (u.wide_splits > 0)
      DDG_TRY(wgrad_wide_launch(x_in, dz_buf, u.wg_partial, u.N, u.H, u.W, u.cin, u.cout, u.R, u.wide_splits, m->stream,
                                x_scale, x_shift));
    else
      DDG_TRY(wgrad_launch(w, m->stream));
  }
  if (dx) {
    // reads dz and the weights, writes dx; plus the shortcut term (and its mask), plus the mask
    // and conv output of the layer below when its BN-backward sums are formed here
    const bool wide_below = u.tiled_grid == 0 && u.wide_d && below && below->u && below->u->cout == u.cin &&
                            m->d.compute == DDG_BF16 && m->wide_below;
    const bool fuse_below = (u.tiled_grid > 0 && below && below->u) || wide_below;
    double extra = (add_g ? (add_mask ? 2.0 : 1.0) : 0.0);
    if (fuse_below) extra += (below->mask == below->u->z) ? 1.0 : 2.0;
    Launch L(m, u.tiled_grid > 0 ? PK_CONV_DGRAD + u.tiled_instance() : (u.wide_d ? PK_CONV_DGRAD_WIDE : PK_CONV_DGRAD),
             (E + (1.0 + extra) * u.in_elems()) * m->esz + wbytes(m, u), conv_flops(u));
    if (u.tiled_grid == 0 && u.wide_d) {
      ConvStat st{};
      if (wide_below) {
        st.mode = 2; st.partial = below->u->bstat;
        st.mask = below->mask; st.mscale = below->mscale; st.mshift = below->mshift;
        st.z = below->u->z; st.zmean = below->u->mean; st.zinvstd = below->u->invstd;
        if (below_rows) *below_rows = conv_wide_rows(u.N * u.H * u.W);
      }
      DDG_TRY(conv_wide_launch(dz_buf, u.wpack_d, dx, nullptr, add_g, add_mask, u.N, u.P, u.Q, u.cout, u.cin, u.R, m->stream,
                               nullptr, nullptr, nullptr, wide_below ? &st : nullptr));
    } else if (u.tiled_grid > 0) {
      ConvStat st{};
      if (below && below->u) {
        st.mode = 2; st.partial = below->u->bstat;
        st.mask = below->mask; st.mscale = below->mscale; st.mshift = below->mshift;
        st.z = below->u->z; st.zmean = below->u->mean; st.zinvstd = below->u->invstd;
        if (below_rows) *below_rows = u.tiled_grid;
      }
      DDG_TRY(conv_tiled_any(m, dz_buf, nullptr, nullptr, nullptr, u.wpack_d, dx, st, add_g, add_mask, u.N, u.H, u.W,
                                u.cin, u.tiled_grid, m->stream));
    } else {
      ConvArgs a = u.dgrad;
      a.in = dz_buf; a.wpack = u.wpack_d; a.out = dx; a.stat_partial = nullptr;
      a.add_g = add_g; a.add_mask = add_mask;
      DDG_TRY(conv_launch(a, m->stream));
    }
  }
  return DDG_OK;
}

// Backward through the tape held in `blocks` (the module's own, or a ring slot's view of them).
// dtop: gradient at the module output (null with a head).
ddg_status run_backward(ddg_module* m, std::vector<Blk>& blocks, const void* in, const void* dtop,
                        const int32_t* labels, void* delta_out, float* loss_out) {
  const int dt = m->d.compute;
  const bool head = m->d.num_classes > 0;
  const int nres = (int)blocks.size() - (head ? 1 : 0);
  const void* dy = dtop;
  if (head) {
    Blk& hb = blocks.back();
    HeadArgs a{};
    // a module that is the head alone (a split point after the last conv layer) reads its
    // stored input and hands the gradient straight to delta_out
    a.h = nres > 0 ? blocks[nres - 1].y : in; a.fcw = m->theta + hb.ofcw; a.fcb = m->theta + hb.ofcb; a.labels = labels;
    a.pooled = hb.pooled; a.dlogits = hb.dlogits; a.loss_n = hb.loss_n; a.loss_out = loss_out;
    a.dfcw = m->grad + hb.ofcw; a.dfcb = m->grad + hb.ofcb; a.dh = nres > 0 ? m->Ga : delta_out;
    a.N = m->d.batch; a.HW = hb.HW; a.C = hb.C; a.classes = m->d.num_classes; a.dtype = dt;
    Launch L(m, PK_HEAD);
    DDG_TRY(head_launch(a, m->stream));
    dy = m->Ga;
  }
  void* gnext = (dy == m->Ga) ? m->Gb : m->Ga;  // where this block's input gradient goes
  int top_rows = 0;   // > 0: the BN sums of this block's last unit are already in the workspace
  // DDG_NO_PREMASK=1 (timing experiments): readers apply the ReLU mask again (same result, the old traffic)
  const bool premasked = m->premasked;
  for (int bi = nres - 1; bi >= 0; --bi) {
    Blk& b = blocks[bi];
    const void* x = (bi == 0) ? in : blocks[bi - 1].y;
    const bool want_dx = (bi > 0) || (m->d.k > 1);
    void* dx_dst = nullptr;
    if (want_dx) dx_dst = (bi == 0) ? delta_out : gnext;
    // the BN whose backward follows this block's input gradient: the last main unit of the
    // block below (its ReLU mask is that block's output)
    BelowBn below_blk;
    if (bi > 0) {
      Blk& pb = blocks[bi - 1];
      below_blk.u = &pb.u[pb.nmain - 1];
      below_blk.mask = pb.y;
    }
    int next_top_rows = 0;
    // the ReLU mask of this block's output: already applied to dy by the kernel that produced
    // it, if that kernel also formed the sums (top_rows > 0)
    const void* ymask = (top_rows > 0 && premasked) ? nullptr : b.y;
    if (b.kind == DDG_BLOCK_STEM) {
      DDG_OKAY(unit_backward(m, b.u[0], dy, ymask, nullptr, nullptr, top_rows, x, nullptr, nullptr, m->D1,
                             dx_dst, nullptr, nullptr, bi > 0 ? &below_blk : nullptr, &next_top_rows));
    } else {
      // shortcut term of the input gradient
      const void* add_g = nullptr; const void* add_mask = nullptr;
      if (b.proj) {
        Unit& up = b.u[b.nmain];
        DDG_OKAY(unit_backward(m, up, dy, ymask, nullptr, nullptr, 0, x, nullptr, nullptr, m->D1,
                               want_dx ? m->D3 : nullptr, nullptr, nullptr, nullptr, nullptr));
        if (want_dx) add_g = m->D3;
      } else if (want_dx) {
        add_g = dy; add_mask = ymask;
      }
      const void* d = dy; const void* mask = ymask;
      const float *msc = nullptr, *msh = nullptr;
      int stats_rows = top_rows;
      for (int i = b.nmain - 1; i >= 0; --i) {
        Unit& u = b.u[i];
        // the unit's input: the block input, a materialised activation, or the previous unit's
        // conv output with its BN + ReLU applied on the fly
        const void* uin = x; const float *xsc = nullptr, *xsh = nullptr;
        BelowBn below;
        if (i > 0) {
          if (b.act[i - 1]) uin = b.act[i - 1];
          else { uin = b.u[i - 1].z; xsc = b.u[i - 1].scale; xsh = b.u[i - 1].shift; }
          below.u = &b.u[i - 1]; below.mask = uin; below.mscale = xsc; below.mshift = xsh;
        } else {
          below = below_blk;
        }
        void* udx = (i > 0) ? m->D2 : dx_dst;
        int done = 0;
        DDG_OKAY(unit_backward(m, u, d, mask, msc, msh, stats_rows, uin, xsc, xsh, m->D1, udx,
                               i == 0 ? add_g : nullptr, i == 0 ? add_mask : nullptr,
                               (udx && below.u) ? &below : nullptr, &done));
        if (i > 0) {
          d = m->D2; mask = uin; msc = xsc; msh = xsh; stats_rows = done;
          if (done > 0 && premasked) { mask = nullptr; msc = nullptr; msh = nullptr; }   // D2 is masked already
        } else {
          next_top_rows = done;
        }
      }
    }
    top_rows = next_top_rows;
    if (bi > 0) { dy = gnext; gnext = (gnext == m->Ga) ? m->Gb : m->Ga; }
  }
  return flush_pending_wgrad(m);
}

// The module's blocks with every forward buffer (conv outputs, statistics rows, per-channel
// vectors, activations, block outputs) and the input-gradient operand moved to group / ring
// slot g: what a kept forward pass of that slot wrote, and what its backward pass reads.
std::vector<Blk> group_view(ddg_module* m, int g) {
  std::vector<Blk> v = m->blocks;
  for (Blk& b : v) {
    if (b.kind == DDG_BLOCK_HEAD) continue;
    for (size_t i = 0; i < b.u.size(); ++i) {
      Unit& u = b.u[i];
      u.z = grp(u.z, u.out_elems() * m->esz, g);
      u.fstat += (size_t)g * u.fcap * 2 * u.cout;
      const int vo = g * u.vec_stride();
      u.mean += vo; u.invstd += vo; u.scale += vo; u.shift += vo; u.coef += vo;
      if (u.wpack_d) u.wpack_d = (char*)u.wpack_d + (size_t)g * u.wpack_d_bytes;
    }
    for (size_t i = 0; i < b.act.size(); ++i) b.act[i] = grp(b.act[i], b.u[i].out_elems() * m->esz, g);
    b.y = grp(b.y, b.y_elems * m->esz, g);
  }
  return v;
}

// Second set of forward buffers: same plan and packed weights, own conv outputs, statistics
// and block outputs, so that the forward pass on the current minibatch and the re-forward of
// the delayed one can be in flight at the same time.
ddg_status build_forward_shadow(ddg_module* m) {
  m->fblocks = m->blocks;
  for (Blk& b : m->fblocks) {
    if (b.kind == DDG_BLOCK_HEAD) continue;
    for (Unit& u : b.u) {
      void* p = nullptr;
      DDG_OKAY(dev_alloc(m, &p, u.out_elems() * m->esz)); u.z = p;
      DDG_OKAY(dev_alloc(m, &p, (size_t)u.fprop.grid_x * 2 * u.cout * sizeof(float))); u.fstat = (float*)p;
      DDG_OKAY(dev_alloc(m, &p, (size_t)7 * u.cout * sizeof(float)));
      u.mean = (float*)p; u.invstd = u.mean + u.cout; u.scale = u.invstd + u.cout;
      u.shift = u.scale + u.cout; u.coef = u.shift + u.cout;
    }
    for (size_t i = 0; i < b.act.size(); ++i)
      if (b.act[i]) DDG_OKAY(dev_alloc(m, &b.act[i], b.u[i].out_elems() * m->esz));
    DDG_OKAY(dev_alloc(m, &b.y, b.y_elems * m->esz));
  }
  for (int i = 0; i < 2; ++i)
    if (hipEventCreateWithFlags(&m->ev_fwd[i], hipEventDisableTiming) != hipSuccess) return fail(DDG_ERR_DEVICE, "event");
  if (hipEventCreateWithFlags(&m->ev_upd, hipEventDisableTiming) != hipSuccess) return fail(DDG_ERR_DEVICE, "event");
  return DDG_OK;
}

// Running batch-norm estimates (start: mean 0, variance 1), the evaluation vectors, and the
// per-group tables of layer descriptors for the kernels that maintain them.
ddg_status build_running_tables(ddg_module* m) {
  size_t sum_c = 0;
  for (const Blk& b : m->blocks) for (const Unit& u : b.u) { sum_c += u.cout; ++m->n_run; if (u.cout > m->run_max_c) m->run_max_c = u.cout; }
  m->nrunning = 2 * sum_c;
  if (m->d.dry_run || m->n_run == 0) return DDG_OK;
  void* p = nullptr;
  DDG_OKAY(dev_alloc(m, &p, 4 * sum_c * sizeof(float)));
  m->running = (float*)p;
  std::vector<float> init(4 * sum_c, 0.f);
  size_t off = 0;
  auto assign = [&](std::vector<Blk>& blocks) {
    size_t o = 0;
    for (Blk& b : blocks) for (Unit& u : b.u) {
      u.rmean = m->running + o; u.rvar = u.rmean + u.cout;
      u.escale = m->running + 2 * sum_c + o; u.eshift = u.escale + u.cout;
      o += 2 * (size_t)u.cout;
    }
  };
  assign(m->blocks);
  if (m->two_streams) assign(m->fblocks);
  for (const Blk& b : m->blocks) for (const Unit& u : b.u) {
    for (int c = 0; c < u.cout; ++c) init[off + u.cout + c] = 1.f;
    off += 2 * (size_t)u.cout;
  }
  if (hipMemcpy(m->running, init.data(), init.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess)
    return fail(DDG_ERR_DEVICE, "initialising the running estimates failed");
  auto table = [&](const std::vector<Blk>& blocks, RunDesc** out) -> ddg_status {
    std::vector<RunDesc> t;
    for (const Blk& b : blocks) for (const Unit& u : b.u) {
      RunDesc r{};
      r.mean = u.mean; r.invstd = u.invstd; r.gamma = m->theta + u.og; r.beta = m->theta + u.ob;
      r.rmean = u.rmean; r.rvar = u.rvar; r.escale = u.escale; r.eshift = u.eshift;
      r.C = u.cout; r.count = (float)((size_t)u.N * u.P * u.Q); r.eps = m->d.bn_eps;
      t.push_back(r);
    }
    void* q = nullptr;
    DDG_OKAY(dev_alloc(m, &q, t.size() * sizeof(RunDesc)));
    if (hipMemcpy(q, t.data(), t.size() * sizeof(RunDesc), hipMemcpyHostToDevice) != hipSuccess)
      return fail(DDG_ERR_DEVICE, "copying the layer tables failed");
    *out = (RunDesc*)q;
    return DDG_OK;
  };
  for (int g = 0; g < m->groups; ++g) {
    RunDesc* t = nullptr;
    DDG_OKAY(table(group_view(m, g), &t));
    m->run_descs.push_back(t);
  }
  if (m->two_streams) DDG_OKAY(table(m->fblocks, &m->run_descs_f));
  if (m->d.num_classes > 0) {
    DDG_OKAY(dev_alloc(m, &p, (size_t)m->d.batch * sizeof(int32_t)));
    m->zero_labels = (int32_t*)p;
    if (hipMemset(p, 0, (size_t)m->d.batch * sizeof(int32_t)) != hipSuccess) return fail(DDG_ERR_DEVICE, "hipMemset failed");
  }
  return DDG_OK;
}

ddg_status sync_streams(ddg_module* m) {
  DDG_TRY(hipStreamSynchronize(m->bstream));
  if (m->two_streams) DDG_TRY(hipStreamSynchronize(m->fstream));
  return DDG_OK;
}

ddg_status check_handle(const ddg_module* m) {
  if (!m) return fail(DDG_ERR_INVALID_ARG, "module handle is null");
  if (m->sticky != DDG_OK) return fail(m->sticky, "module is in a failed state after an earlier device error");
  return DDG_OK;
}

}  // namespace

// ---- C boundary ------------------------------------------------------------------------------

extern "C" {

const char* ddg_last_error(void) { return g_err.c_str(); }
const char* ddg_version(void) { return "ddg-mi355x 0.1 (gfx950)"; }

ddg_status ddg_module_create(const ddg_module_desc* desc, ddg_module** out) {
  if (!out) return fail(DDG_ERR_INVALID_ARG, "out is null");
  *out = nullptr;
  DDG_OKAY(validate(desc));
  ddg_module* m = new ddg_module();
  m->d = *desc;
  m->blocks_desc.assign(desc->blocks, desc->blocks + desc->num_blocks);
  m->d.blocks = m->blocks_desc.data();
  m->bstream = (hipStream_t)desc->stream;
  m->fstream = m->bstream;
  m->stream = m->bstream;
  m->two_streams = !desc->stale_jacobian && desc->forward_stream && desc->forward_stream != desc->stream && (desc->K - desc->k) > 0 &&
                   !desc->dry_run;
  if (m->two_streams) m->fstream = (hipStream_t)desc->forward_stream;
  ddg_status st = build_plan(m);
  if (st == DDG_OK && m->two_streams) st = build_forward_shadow(m);
  if (st == DDG_OK) st = build_running_tables(m);
  if (st != DDG_OK) {
    for (void* p : m->allocs) (void)hipFree(p);
    delete m;
    return st;
  }
  *out = m;
  return DDG_OK;
}

ddg_status ddg_module_destroy(ddg_module* m) {
  if (!m) return DDG_OK;
  if (!m->d.dry_run) {
    (void)hipStreamSynchronize(m->bstream);
    if (m->two_streams) (void)hipStreamSynchronize(m->fstream);
    for (int i = 0; i < 2; ++i) if (m->ev_fwd[i]) (void)hipEventDestroy(m->ev_fwd[i]);
    if (m->ev_upd) (void)hipEventDestroy(m->ev_upd);
    for (auto& e : m->evs) { (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b); }
    for (void* p : m->allocs) (void)hipFree(p);
  }
  delete m;
  return DDG_OK;
}

size_t ddg_param_count(const ddg_module* m) { return m ? m->nparams : 0; }
size_t ddg_device_bytes(const ddg_module* m) { return m ? m->bytes : 0; }

ddg_status ddg_out_shape(const ddg_module* m, int* c, int* h, int* w) {
  if (!m) return fail(DDG_ERR_INVALID_ARG, "module handle is null");
  if (c) *c = m->out_c;
  if (h) *h = m->out_h;
  if (w) *w = m->out_w;
  return DDG_OK;
}

ddg_status ddg_set_params(ddg_module* m, const float* src, int is_device) {
  DDG_OKAY(check_handle(m));
  if (!src) return fail(DDG_ERR_INVALID_ARG, "src is null");
  if (m->d.dry_run) return DDG_OK;
  m->stream = m->bstream;
  DDG_OKAY(sync_streams(m));   // nothing may still be reading the old weights
  if (is_device) {
    Launch L(m, PK_COPY);
    DDG_TRY(copy_launch(src, m->theta, m->nparams * sizeof(float), m->stream));
  } else {
    DDG_TRY(hipMemcpy(m->theta, src, m->nparams * sizeof(float), hipMemcpyHostToDevice));
  }
  m->tape_is_current = false;
  DDG_OKAY(pack_all(m));
  if (m->two_streams) DDG_TRY(hipStreamSynchronize(m->bstream));   // visible to the forward stream
  return DDG_OK;
}

ddg_status ddg_set_velocity(ddg_module* m, const float* src, int is_device) {
  DDG_OKAY(check_handle(m));
  if (!src) return fail(DDG_ERR_INVALID_ARG, "src is null");
  if (m->d.dry_run) return DDG_OK;
  m->stream = m->bstream;
  if (is_device) {
    Launch L(m, PK_COPY);
    DDG_TRY(copy_launch(src, m->vel, m->nparams * sizeof(float), m->stream));
  } else {
    DDG_TRY(hipStreamSynchronize(m->bstream));
    DDG_TRY(hipMemcpy(m->vel, src, m->nparams * sizeof(float), hipMemcpyHostToDevice));
  }
  return DDG_OK;
}

ddg_status ddg_set_moment2(ddg_module* m, const float* src, int is_device) {
  DDG_OKAY(check_handle(m));
  if (!src) return fail(DDG_ERR_INVALID_ARG, "src is null");
  if (m->d.dry_run) return DDG_OK;
  m->stream = m->bstream;
  if (is_device) {
    Launch L(m, PK_COPY);
    DDG_TRY(copy_launch(src, m->mom2, m->nparams * sizeof(float), m->stream));
  } else {
    DDG_TRY(hipStreamSynchronize(m->bstream));
    DDG_TRY(hipMemcpy(m->mom2, src, m->nparams * sizeof(float), hipMemcpyHostToDevice));
  }
  return DDG_OK;
}

ddg_status ddg_set_optimizer(ddg_module* m, int kind, float beta1, float beta2, float eps) {
  DDG_OKAY(check_handle(m));
  if (kind != DDG_OPT_SGD && kind != DDG_OPT_ADAM) return fail(DDG_ERR_INVALID_ARG, "unknown optimizer kind %d", kind);
  if (kind == DDG_OPT_ADAM && !(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f && eps >= 0.f))
    return fail(DDG_ERR_INVALID_ARG, "Adam needs 0 <= beta1, beta2 < 1 and eps >= 0");
  if (m->phase != 0) return fail(DDG_ERR_STATE, "the optimizer can only change between iterations");
  const bool betas_changed = kind == DDG_OPT_ADAM && (beta1 != m->beta1 || beta2 != m->beta2);
  m->opt = kind;
  if (kind == DDG_OPT_ADAM) { m->beta1 = beta1; m->beta2 = beta2; m->adam_eps = eps; }
  if (betas_changed) return ddg_set_update_count(m, m->nupd);   // beta^n for the new betas
  return DDG_OK;
}

ddg_status ddg_set_update_count(ddg_module* m, long n) {
  DDG_OKAY(check_handle(m));
  if (n < 0) return fail(DDG_ERR_INVALID_ARG, "update count must be >= 0");
  m->nupd = n;
  if (m->d.dry_run) return DDG_OK;
  DDG_OKAY(sync_streams(m));
  // beta^n as the update kernels form it, one multiplication per executed update, so that a
  // restored count continues a run bit for bit (beyond 10^8 updates: the closed form)
  double pw[2] = {1.0, 1.0};
  if (n <= 100000000L) {
    for (long i = 0; i < n; ++i) { pw[0] *= (double)m->beta1; pw[1] *= (double)m->beta2; }
  } else {
    pw[0] = std::pow((double)m->beta1, (double)n); pw[1] = std::pow((double)m->beta2, (double)n);
  }
  DDG_TRY(hipMemcpy(m->adam_pw, pw, sizeof pw, hipMemcpyHostToDevice));
  return DDG_OK;
}

long ddg_get_update_count(const ddg_module* m) { return m ? m->nupd : 0; }

static ddg_status get_vec(ddg_module* m, const float* dev, float* host_dst) {
  DDG_OKAY(check_handle(m));
  if (!host_dst) return fail(DDG_ERR_INVALID_ARG, "host_dst is null");
  if (m->d.dry_run) { memset(host_dst, 0, m->nparams * sizeof(float)); return DDG_OK; }
  DDG_OKAY(sync_streams(m));
  DDG_TRY(hipMemcpy(host_dst, dev, m->nparams * sizeof(float), hipMemcpyDeviceToHost));
  return DDG_OK;
}
ddg_status ddg_get_params(ddg_module* m, float* host_dst) { return get_vec(m, m ? m->theta : nullptr, host_dst); }
ddg_status ddg_get_velocity(ddg_module* m, float* host_dst) { return get_vec(m, m ? m->vel : nullptr, host_dst); }
ddg_status ddg_get_moment2(ddg_module* m, float* host_dst) { return get_vec(m, m ? m->mom2 : nullptr, host_dst); }
ddg_status ddg_get_grad(ddg_module* m, float* host_dst, int* valid) {
  DDG_OKAY(get_vec(m, m ? m->grad : nullptr, host_dst));
  if (valid) *valid = m->has_grad ? 1 : 0;
  return DDG_OK;
}

ddg_status ddg_forward(ddg_module* m, long t, const void* h_in, void* h_out) {
  DDG_OKAY(check_handle(m));
  if (m->phase != 0) return fail(DDG_ERR_STATE, "ddg_forward(t=%ld) called while iteration %ld is unfinished (phase %d)", t, m->t_next, m->phase);
  if (t != m->t_next) return fail(DDG_ERR_STATE, "ddg_forward expected t=%ld, got %ld", m->t_next, t);
  if (!h_in) return fail(DDG_ERR_INVALID_ARG, "h_in is null");
  const bool head = m->d.num_classes > 0;
  if (!head && !h_out) return fail(DDG_ERR_INVALID_ARG, "h_out is null");
  if (((uintptr_t)h_in & 15) || ((uintptr_t)h_out & 15)) return fail(DDG_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
  m->phase = 1;
  if (m->d.dry_run) return DDG_OK;
  // paired: this call also re-forwards the minibatch of iteration t - delay (same weights)
  const bool paired = !m->stale && m->groups == 2 && t >= m->delay;
  if (m->skip) { m->tape_is_current = (m->delay == 0) || paired; return DDG_OK; }
  m->stream = m->fstream;
  const bool self_sync = m->two_streams && !m->external_sync;
  // the forward stream needs the weights of update(t-1) and the ring slot that backward(t-1) read
  if (self_sync) DDG_TRY(hipStreamWaitEvent(m->fstream, m->ev_upd, 0));
  void* slot = m->ring[t % m->nslots];
  { Launch L(m, PK_COPY, 2.0 * m->in_elems * m->esz); DDG_TRY(copy_launch(h_in, slot, m->in_elems * m->esz, m->stream)); }
  // A module with delay > 0 re-forwards before its backward, so this pass need not keep a
  // tape and writes straight to h_out; the last module keeps the tape for its own backward.
  // the running estimates follow the batch statistics of this pass on minibatch t
  const RunDesc* run_table = nullptr;
  if (m->stale) {
    // keep this pass: its tape, the weights it used and their input-gradient operands
    const int g = (int)(t % m->nslots);
    if (m->n_run) run_table = m->run_descs[g];
    std::vector<Blk> tape = group_view(m, g);
    { Launch L(m, PK_COPY, 2.0 * m->nparams * sizeof(float));
      DDG_TRY(copy_launch(m->theta, m->theta_snap + (size_t)g * m->nparams, m->nparams * sizeof(float), m->stream)); }
    if (m->n_pack_d) { Launch L(m, PK_PACK); DDG_TRY(pack_all_launch(m->pack_descs_d[g], m->n_pack_d, m->d.compute, m->stream, m->pack_max)); }
    DDG_OKAY(run_forward(m, tape, slot, nullptr));
    m->tape_is_current = false;
    const Blk& lb = tape[tape.size() - 1];
    Launch L(m, PK_COPY, 2.0 * m->out_elems * m->esz);
    DDG_TRY(copy_launch(lb.y, h_out, m->out_elems * m->esz, m->stream));
  } else if (paired) {
    DDG_OKAY(run_forward_pair(m, m->blocks, m->ring[(t - m->delay) % m->nslots], slot, h_out));
    m->tape_is_current = true;    // group 0 holds the tape of iteration t - delay
    if (m->n_run) run_table = m->run_descs[1];   // group 1 held minibatch t
  } else if (m->delay > 0) {
    DDG_OKAY(run_forward(m, m->two_streams ? m->fblocks : m->blocks, slot, h_out));
    m->tape_is_current = false;
    if (m->n_run) run_table = m->two_streams ? m->run_descs_f : m->run_descs[0];
  } else {
    DDG_OKAY(run_forward(m, m->blocks, slot, nullptr));
    m->tape_is_current = true;
    if (h_out) {
      Launch L(m, PK_COPY);
      DDG_TRY(copy_launch(m->blocks[m->blocks.size() - (head ? 2 : 1)].y, h_out, m->out_elems * m->esz, m->stream));
    }
    if (m->n_run) run_table = m->run_descs[0];
  }
  if (run_table && m->bn_rho > 0.f) {
    Launch L(m, PK_BN_RUNNING);
    DDG_TRY(running_update_launch(run_table, m->n_run, m->run_max_c, m->bn_rho, m->stream));
  }
  if (m->delay > 0 && !m->stale && !paired && self_sync) DDG_TRY(hipEventRecord(m->ev_fwd[t & 1], m->fstream));
  return DDG_OK;
}

ddg_status ddg_set_bn_momentum(ddg_module* m, float rho) {
  DDG_OKAY(check_handle(m));
  if (!(rho >= 0.f && rho <= 1.f)) return fail(DDG_ERR_INVALID_ARG, "the weight of the newest batch statistic must lie in [0, 1]");
  if (m->t_next != 0) return fail(DDG_ERR_STATE, "the weight can only be set before the first iteration");
  m->bn_rho = rho;
  return DDG_OK;
}

int ddg_ring_slots(const ddg_module* m) { return m ? m->nslots : 0; }
size_t ddg_ring_slot_bytes(const ddg_module* m) { return m ? m->in_elems * m->esz : 0; }

static ddg_status ring_slot_ok(ddg_module* m, int slot, const void* host) {
  DDG_OKAY(check_handle(m));
  if (!host) return fail(DDG_ERR_INVALID_ARG, "host buffer is null");
  if (slot < 0 || slot >= m->nslots) return fail(DDG_ERR_INVALID_ARG, "ring slot %d outside [0, %d)", slot, m->nslots);
  if (m->phase != 0) return fail(DDG_ERR_STATE, "the ring can only be read or written between iterations");
  if (m->stale) return fail(DDG_ERR_STATE, "stale-Jacobian mode keeps forward passes that a checkpoint does not hold");
  return DDG_OK;
}

ddg_status ddg_get_ring_slot(ddg_module* m, int slot, void* host_dst) {
  DDG_OKAY(ring_slot_ok(m, slot, host_dst));
  if (m->d.dry_run) return DDG_OK;
  DDG_OKAY(sync_streams(m));
  DDG_TRY(hipMemcpy(host_dst, m->ring[slot], m->in_elems * m->esz, hipMemcpyDeviceToHost));
  return DDG_OK;
}

ddg_status ddg_set_ring_slot(ddg_module* m, int slot, const void* host_src) {
  DDG_OKAY(ring_slot_ok(m, slot, host_src));
  if (m->d.dry_run) return DDG_OK;
  DDG_OKAY(sync_streams(m));
  DDG_TRY(hipMemcpy(m->ring[slot], host_src, m->in_elems * m->esz, hipMemcpyHostToDevice));
  return DDG_OK;
}

ddg_status ddg_set_time(ddg_module* m, long t) {
  DDG_OKAY(check_handle(m));
  if (t < 0) return fail(DDG_ERR_INVALID_ARG, "iteration must be >= 0");
  if (m->phase != 0) return fail(DDG_ERR_STATE, "the time can only be set between iterations");
  if (m->stale) return fail(DDG_ERR_STATE, "stale-Jacobian mode keeps forward passes that a checkpoint does not hold");
  if (!m->d.dry_run) DDG_OKAY(sync_streams(m));
  m->t_next = t;
  m->tape_is_current = false;
  m->has_grad = false;
  return DDG_OK;
}

long ddg_get_time(const ddg_module* m) { return m ? m->t_next : -1; }

size_t ddg_running_count(const ddg_module* m) { return m ? m->nrunning : 0; }

ddg_status ddg_get_running(ddg_module* m, float* host_dst) {
  DDG_OKAY(check_handle(m));
  if (!host_dst) return fail(DDG_ERR_INVALID_ARG, "destination is null");
  if (m->d.dry_run || m->nrunning == 0) return DDG_OK;
  DDG_OKAY(sync_streams(m));
  DDG_TRY(hipMemcpy(host_dst, m->running, m->nrunning * sizeof(float), hipMemcpyDeviceToHost));
  return DDG_OK;
}

ddg_status ddg_set_running(ddg_module* m, const float* host_src) {
  DDG_OKAY(check_handle(m));
  if (!host_src) return fail(DDG_ERR_INVALID_ARG, "source is null");
  if (m->d.dry_run || m->nrunning == 0) return DDG_OK;
  DDG_OKAY(sync_streams(m));
  DDG_TRY(hipMemcpy(m->running, host_src, m->nrunning * sizeof(float), hipMemcpyHostToDevice));
  return DDG_OK;
}

// The evaluation forward through `blocks` (the module's own forward buffers, or a view of them
// whose buffers lie elsewhere); hs: the head's per-sample scratch.
struct HeadScratch { float* pooled; float* dlogits; float* loss_n; };
static ddg_status eval_forward(ddg_module* m, std::vector<Blk>& blocks, const HeadScratch& hs, const void* h_in,
                               void* h_out, const int32_t* labels, float* loss_out, float* logits_out) {
  const bool head = m->d.num_classes > 0;
  m->stream = m->bstream;
  if (m->n_run) DDG_TRY(eval_vectors_launch(m->run_descs[0], m->n_run, m->run_max_c, m->stream));
  const int nres = (int)blocks.size() - (head ? 1 : 0);
  m->eval_mode = true;
  ddg_status st = DDG_OK;
  if (nres > 0) st = run_forward(m, blocks, h_in, head ? nullptr : h_out);
  m->eval_mode = false;
  DDG_OKAY(st);
  if (head) {
    Blk& hb = blocks.back();
    HeadArgs a{};
    a.h = nres > 0 ? blocks[nres - 1].y : h_in; a.fcw = m->theta + hb.ofcw; a.fcb = m->theta + hb.ofcb;
    a.labels = labels ? labels : m->zero_labels;
    a.pooled = hs.pooled; a.dlogits = hs.dlogits; a.loss_n = hs.loss_n; a.loss_out = loss_out;
    a.dfcw = nullptr; a.dfcb = nullptr; a.dh = nullptr; a.logits_out = logits_out;
    a.N = m->d.batch; a.HW = hb.HW; a.C = hb.C; a.classes = m->d.num_classes; a.dtype = m->d.compute;
    DDG_TRY(head_launch(a, m->stream));
  }
  return DDG_OK;
}

static ddg_status eval_args_ok(ddg_module* m, const void* h_in, void* h_out, const int32_t* labels, float* loss_out) {
  DDG_OKAY(check_handle(m));
  const bool head = m->d.num_classes > 0;
  if (!h_in) return fail(DDG_ERR_INVALID_ARG, "h_in is null");
  if (!head && !h_out) return fail(DDG_ERR_INVALID_ARG, "h_out is null");
  if (head && loss_out && !labels) return fail(DDG_ERR_INVALID_ARG, "the loss needs labels");
  if (((uintptr_t)h_in & 15) || ((uintptr_t)h_out & 15)) return fail(DDG_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
  if (m->phase != 0) return fail(DDG_ERR_STATE, "evaluation runs between iterations (after ddg_update, before the next ddg_forward)");
  return DDG_OK;
}

ddg_status ddg_forward_eval(ddg_module* m, const void* h_in, void* h_out, const int32_t* labels, float* loss_out,
                            float* logits_out) {
  DDG_OKAY(eval_args_ok(m, h_in, h_out, labels, loss_out));
  if (m->stale) return fail(DDG_ERR_STATE, "no evaluation forward in stale-Jacobian mode: every set of forward buffers holds a kept tape");
  if (m->d.dry_run) return DDG_OK;
  m->tape_is_current = false;     // the forward buffers of group 0 now hold this pass
  HeadScratch hs{};
  if (m->d.num_classes > 0) { const Blk& hb = m->blocks.back(); hs.pooled = hb.pooled; hs.dlogits = hb.dlogits; hs.loss_n = hb.loss_n; }
  return eval_forward(m, m->blocks, hs, h_in, h_out, labels, loss_out, logits_out);
}

// Bytes of static scratch the evaluation forward of this module needs, and (base != null) a view
// of the module's blocks whose forward buffers lie in it. Layout: two slots for block outputs
// (block i writes slot i mod 2: the output of block i-1 is the last one read when block i+1's
// first conv forms the output of block i), then two regions for the conv outputs, statistics
// rows and activations of a block (block i uses region i mod 2: the last conv output of block i
// is read while the first conv of block i+1 writes its own), then the head's per-sample vectors.
static size_t static_eval_layout(const ddg_module* m, char* base, std::vector<Blk>* view, HeadScratch* hs) {
  auto up = [](size_t b) { return (b + 255) & ~(size_t)255; };
  size_t ymax = 0, zmax = 0;
  for (const Blk& b : m->blocks) {
    if (b.kind == DDG_BLOCK_HEAD) continue;
    size_t zb = 0;
    for (const Unit& u : b.u) zb += up(u.out_elems() * m->esz) + up((size_t)u.fcap * 2 * u.cout * sizeof(float));
    for (size_t i = 0; i < b.act.size(); ++i) if (b.act[i]) zb += up(b.u[i].out_elems() * m->esz);
    if (zb > zmax) zmax = zb;
    if (up(b.y_elems * m->esz) > ymax) ymax = up(b.y_elems * m->esz);
  }
  size_t total = 2 * ymax + 2 * zmax;
  const size_t head_off = total;
  if (m->d.num_classes > 0) {
    const Blk& hb = m->blocks.back();
    total += up(((size_t)m->d.batch * hb.C + (size_t)m->d.batch * m->d.num_classes + m->d.batch) * sizeof(float));
  }
  if (!base) return total;
  *view = m->blocks;
  int bi = 0;
  for (Blk& b : *view) {
    if (b.kind == DDG_BLOCK_HEAD) continue;
    b.y = base + (size_t)(bi & 1) * ymax;
    char* p = base + 2 * ymax + (size_t)(bi & 1) * zmax;
    for (Unit& u : b.u) {
      u.z = p; p += up(u.out_elems() * m->esz);
      u.fstat = (float*)p; p += up((size_t)u.fcap * 2 * u.cout * sizeof(float));
    }
    for (size_t i = 0; i < b.act.size(); ++i) if (b.act[i]) { b.act[i] = p; p += up(b.u[i].out_elems() * m->esz); }
    ++bi;
  }
  if (m->d.num_classes > 0) {
    const Blk& hb = m->blocks.back();
    hs->pooled = (float*)(base + head_off);
    hs->dlogits = hs->pooled + (size_t)m->d.batch * hb.C;
    hs->loss_n = hs->dlogits + (size_t)m->d.batch * m->d.num_classes;
  }
  return total;
}

ddg_status ddg_forward_eval_static(ddg_module* m, const void* h_in, void* h_out, const int32_t* labels,
                                   float* loss_out, float* logits_out) {
  DDG_OKAY(eval_args_ok(m, h_in, h_out, labels, loss_out));
  const size_t need = static_eval_layout(m, nullptr, nullptr, nullptr);
  if (need > DDG_STATIC_SCRATCH_BYTES)
    return fail(DDG_ERR_SHAPE, "this module's evaluation forward needs %zu bytes of scratch; the static scratch holds %zu",
                need, (size_t)DDG_STATIC_SCRATCH_BYTES);
  if (m->d.dry_run) return DDG_OK;
  void* base = nullptr; size_t have = 0;
  DDG_TRY(static_scratch(&base, &have));
  std::vector<Blk> view;
  HeadScratch hs{};
  static_eval_layout(m, (char*)base, &view, &hs);
  // every buffer in the scratch is written before it is read (conv outputs and statistics rows
  // by the conv launches, block outputs by the launch that forms them, the head's vectors by the
  // head kernel), so nothing of an earlier call's contents has to be cleared
  return eval_forward(m, view, hs, h_in, h_out, labels, loss_out, logits_out);
}

ddg_status ddg_backward_delayed(ddg_module* m, long t, const void* delta_in, const int32_t* labels,
                                void* delta_out, float* loss_out, int* did_backward) {
  DDG_OKAY(check_handle(m));
  if (m->phase != 1 || t != m->t_next) return fail(DDG_ERR_STATE, "ddg_backward_delayed(t=%ld) must follow ddg_forward(t=%ld)", t, m->t_next);
  const bool head = m->d.num_classes > 0;
  const long s = t - m->d.K + m->d.k;
  if (s >= 0) {
    if (head && (!labels || delta_in)) return fail(DDG_ERR_INVALID_ARG, "the head module takes labels and no delta_in");
    if (!head && !delta_in) return fail(DDG_ERR_INVALID_ARG, "delta_in is null");
    if (m->d.k > 1 && !delta_out) return fail(DDG_ERR_INVALID_ARG, "delta_out is null (k > 1)");
    if (((uintptr_t)delta_in & 15) || ((uintptr_t)delta_out & 15)) return fail(DDG_ERR_INVALID_ARG, "tensors must be 16-byte aligned");
  }
  m->phase = 2;
  m->has_grad = (s >= 0);
  if (did_backward) *did_backward = m->has_grad ? 1 : 0;
  if (s < 0 || m->d.dry_run) return DDG_OK;
  if (m->skip) { m->tape_is_current = false; return DDG_OK; }
  m->stream = m->bstream;
  // the stored input of iteration s <= t-1 was written by the forward stream
  if (m->two_streams && !m->external_sync && t > 0) DDG_TRY(hipStreamWaitEvent(m->bstream, m->ev_fwd[(t - 1) & 1], 0));
  void* slot = m->ring[s % m->nslots];
  if (!m->tape_is_current && !m->stale) DDG_OKAY(run_forward(m, m->blocks, slot, nullptr));
  m->tape_is_current = false;
  if (m->stale) {
    // the tape and the weights of iteration s (Eq. 6-7 as printed)
    const int g = (int)(s % m->nslots);
    std::vector<Blk> tape = group_view(m, g);
    m->theta_bwd = m->theta_snap + (size_t)g * m->nparams;
    const ddg_status st = run_backward(m, tape, slot, delta_in, labels, m->d.k > 1 ? delta_out : nullptr, loss_out);
    m->theta_bwd = m->theta;
    DDG_OKAY(st);
  } else {
    DDG_OKAY(run_backward(m, m->blocks, slot, delta_in, labels, m->d.k > 1 ? delta_out : nullptr, loss_out));
  }
  // every layer's weight-gradient partials -> g (one launch for the module, fixed order)
  Launch L(m, PK_WGRAD_REDUCE, (double)m->nparams * 4.0);
  DDG_TRY(wgrad_reduce_all_launch(m->wred_descs, m->n_wred, m->wred_max, m->stream));
  return DDG_OK;
}

ddg_status ddg_update(ddg_module* m, long t, float lr) {
  DDG_OKAY(check_handle(m));
  if (m->phase != 2 || t != m->t_next) return fail(DDG_ERR_STATE, "ddg_update(t=%ld) must follow ddg_backward_delayed(t=%ld)", t, m->t_next);
  m->phase = 0;
  m->t_next = t + 1;
  if (m->has_grad && m->opt == DDG_OPT_ADAM) m->nupd += 1;   // also while a captured graph does the work
  if (!m->has_grad || m->d.dry_run || m->skip) return DDG_OK;
  m->stream = m->bstream;
  const bool self_sync = m->two_streams && !m->external_sync;
  // the forward pass of this iteration must have finished reading the weights
  if (self_sync) DDG_TRY(hipStreamWaitEvent(m->bstream, m->ev_fwd[t & 1], 0));
  if (m->opt == DDG_OPT_ADAM) {
    { Launch L(m, PK_ADAM); DDG_TRY(adam_advance_launch(m->adam_pw, m->beta1, m->beta2, m->stream)); }
    Launch L(m, PK_ADAM, (double)m->nparams * 28.0);   // w, m, v read and written, g read
    DDG_TRY(adam_launch(m->theta, m->vel, m->mom2, m->grad, m->nparams, lr, m->lr_dev, m->beta1, m->beta2,
                        m->adam_eps, m->d.weight_decay, m->adam_pw, m->stream));
  } else {
    Launch L(m, PK_SGD, (double)m->nparams * 20.0);
    DDG_TRY(sgd_launch(m->theta, m->vel, m->grad, m->nparams, lr, m->lr_dev, m->d.momentum, m->d.weight_decay, m->stream));
  }
  DDG_OKAY(pack_all(m));
  if (self_sync) DDG_TRY(hipEventRecord(m->ev_upd, m->bstream));
  return DDG_OK;
}

ddg_status ddg_module_sync(ddg_module* m) {
  DDG_OKAY(check_handle(m));
  if (m->d.dry_run) return DDG_OK;
  return sync_streams(m);
}

void ddg_internal_skip_launches(ddg_module* m, bool skip) { m->skip = skip; }
void ddg_internal_external_sync(ddg_module* m, bool on) { m->external_sync = on; }
void ddg_internal_streams(ddg_module* m, hipStream_t* fwd, hipStream_t* bwd) { *fwd = m->fstream; *bwd = m->bstream; }
void ddg_internal_lr_from(ddg_module* m, const float* lr_dev) { m->lr_dev = lr_dev; }
bool ddg_internal_profiling(const ddg_module* m) { return m->prof; }
void ddg_internal_set_error(const char* msg) { g_err = msg ? msg : ""; }

int ddg_profile_kinds(void) { return PK_COUNT; }
const char* ddg_profile_kind_name(int kind) { return (kind >= 0 && kind < PK_COUNT) ? kProfNames[kind] : ""; }

static ddg_status prof_collect(ddg_module* m) {
  if (m->evs.empty()) return DDG_OK;
  DDG_OKAY(sync_streams(m));
  for (auto& e : m->evs) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, e.a, e.b) == hipSuccess) {
      const double d = (double)ms - (e.bracket ? m->prof_empty_ms : 0.0);
      m->prof_n[e.kind] += 1; m->prof_ms[e.kind] += d > 0.0 ? d : 0.0;
    }
    (void)hipEventDestroy(e.a); (void)hipEventDestroy(e.b);
  }
  m->evs.clear();
  return DDG_OK;
}

ddg_status ddg_profile_enable(ddg_module* m, int on) {
  DDG_OKAY(check_handle(m));
  if (m->d.dry_run) return DDG_OK;
  DDG_OKAY(prof_collect(m));
  m->prof = on != 0;
  if (m->prof) {
    // An event bracket around nothing still has a length (the two records are processed one
    // after the other); measure it so that it can be taken off every bracketed launch.
    DDG_OKAY(sync_streams(m));
    const int reps = 32;
    hipEvent_t a[reps], b[reps];
    for (int i = 0; i < reps; ++i) {
      DDG_TRY(hipEventCreate(&a[i])); DDG_TRY(hipEventCreate(&b[i]));
      DDG_TRY(hipEventRecord(a[i], m->bstream)); DDG_TRY(hipEventRecord(b[i], m->bstream));
    }
    DDG_TRY(hipStreamSynchronize(m->bstream));
    double sum = 0.0;
    for (int i = 0; i < reps; ++i) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, a[i], b[i]) == hipSuccess) sum += ms;
      (void)hipEventDestroy(a[i]); (void)hipEventDestroy(b[i]);
    }
    m->prof_empty_ms = sum / reps;
  }
  return DDG_OK;
}

ddg_status ddg_profile_read(ddg_module* m, int kind, long* launches, double* total_ms, double* bytes,
                            double* flops) {
  DDG_OKAY(check_handle(m));
  if (kind < 0 || kind >= PK_COUNT) return fail(DDG_ERR_INVALID_ARG, "kind out of range");
  if (!m->d.dry_run) DDG_OKAY(prof_collect(m));
  if (launches) *launches = m->prof_n[kind];
  if (total_ms) *total_ms = m->prof_ms[kind];
  if (bytes) *bytes = m->prof_bytes[kind];
  if (flops) *flops = m->prof_flops[kind];
  return DDG_OK;
}

ddg_status ddg_profile_reset(ddg_module* m) {
  DDG_OKAY(check_handle(m));
  if (!m->d.dry_run) DDG_OKAY(prof_collect(m));
  for (int i = 0; i < PK_COUNT; ++i) { m->prof_n[i] = 0; m->prof_ms[i] = 0; m->prof_bytes[i] = 0; m->prof_flops[i] = 0; }
  return DDG_OK;
}

}  // extern "C"
