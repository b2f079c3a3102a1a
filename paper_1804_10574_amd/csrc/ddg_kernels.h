// Host-side launch interface of the HIP kernels. Every launcher validates nothing:
// the module code checks shapes before it builds a plan.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

namespace ddg {

// Per-launch timing for the measurement pass: when a pair of events is armed, the next kernel
// launch hands them to the runtime, which stamps them with that kernel's own begin and end
// times (what a kernel trace shows), not with the time two extra stream markers are processed.
struct ProfEvents { hipEvent_t a = nullptr, b = nullptr; bool armed = false; };
extern thread_local ProfEvents g_prof_events;
#define DDG_LAUNCH(kernel, grid, block, shmem, stream, ...)                                        \
  do {                                                                                             \
    if (ddg::g_prof_events.armed) {                                                                \
      ddg::g_prof_events.armed = false;                                                            \
      hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, ddg::g_prof_events.a,              \
                            ddg::g_prof_events.b, 0, __VA_ARGS__);                                 \
    } else {                                                                                       \
      hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);                         \
    }                                                                                              \
  } while (0)

enum DType { F32 = 0, BF16 = 1 };
inline size_t dtype_size(int dt) { return dt == BF16 ? 2 : 4; }
inline int mma_kv(int dt) { return dt == BF16 ? 8 : 4; }

// Partial rows of a batch-norm reduction that the consuming kernel finalises itself
// (partial == nullptr: the per-channel vectors are already final).
struct BnRows {        // forward: rows [rows][2][C] of (sum, sum of squares)
  const float* partial; int rows;
  const float* gamma; const float* beta; float count, eps;
  float* mean; float* invstd; float* scale; float* shift;   // written by workgroup 0
};
struct BnBwdRows {     // backward: rows of (sum g, sum g*xhat)
  const float* partial; int rows;
  const float* gamma; const float* mean; const float* invstd; float count;
  float* dgamma; float* dbeta;                              // written by workgroup 0
};

// Implicit-GEMM convolution on the matrix cores. One kernel serves the forward
// convolution and the gradient w.r.t. the input:
//   fprop: out[n,oh,ow,:] = sum_taps in[n, oh*st+r-pad, ow*st+s-pad, :] . W
//   dgrad: out[n,ih,iw,:] = sum_taps in[n, (ih+pad-r)/st, (iw+pad-s)/st, :] . W^T  (only when divisible)
// `in` has IC channels (the contraction), `out` has OC channels.
struct ConvArgs {
  const void* in;
  const void* wpack;        // packed operand, see pack_weights
  void* out;
  float* stat_partial;      // fprop only: [grid_x][2][OC] per-workgroup sum / sum of squares, or null
  // optional second minibatch in the same launch (forward; same weights, its own tensors and
  // statistics rows): in_b non-null doubles the grid
  const void* in_b; void* out_b; float* stat_partial_b;
  const void* add_g;        // optional: out += add_g (masked where add_mask <= 0), same layout as out
  const void* add_mask;
  int N, IH, IW, IC, OH, OW, OC;
  int R, stride, pad;
  int log2cp;               // log2 of the padded contraction channels per tap
  int ntaps, ksteps;
  int M;                    // N*OH*OW
  int dgrad;
  int dtype;
  int grid_x;               // filled by conv_plan
  int mb, nb;               // tile shape chosen by conv_plan
};
void conv_plan(ConvArgs& a);                       // chooses tile shape and grid
hipError_t conv_launch(const ConvArgs& a, hipStream_t s);
size_t conv_wpack_elems(int kchannels, int nchannels, int R, int dtype, int* log2cp, int* ksteps);
// Packs fp32 master weights W[Cout][Cin][R][R] into the operand layout of conv_launch.
// dgrad: 0 forward operand, 1 input-gradient operand (taps as stored), 2 input-gradient operand
// with mirrored taps (for kernels that run the input-gradient as a plain 3x3 correlation).
hipError_t pack_weights_launch(const float* W, void* wpack, int Cout, int Cin, int R, int dgrad,
                               int dtype, hipStream_t s);

// Gradient w.r.t. the weights: dW[co][ci][r][s] = sum_{n,p,q} dz[n,p,q,co] * x[n,p*st+r-pad,q*st+s-pad,ci].
// Two launches: per-split partial tiles, then a fixed-order sum into dW (deterministic).
struct WgradArgs {
  const void* x; const void* dz; float* partial; float* dW;
  int N, H, W, Cin, P, Q, Cout, R, stride, pad;
  int log2cp, J, JB;        // J = ntaps*CP columns, JB = ceil(J/16)
  int M;                    // N*P*Q
  int msplit, steps;        // splits over M, 4-pixel steps per wave
  int jgroups;              // column-block groups of up to 9 (vec: groups of 192 columns)
  int dtype;
  int vec;                  // 1: input channels a multiple of 4, the kernel with 4-channel gathers
};
void wgrad_plan(WgradArgs& a);
size_t wgrad_partial_elems(const WgradArgs& a);
hipError_t wgrad_launch(const WgradArgs& a, hipStream_t s);
hipError_t wgrad_reduce_launch(const WgradArgs& a, hipStream_t s);

// Whole-module variants driven by a device-side table (one launch per module instead of one
// per layer): repack every conv operand after an update; add up every layer's weight-gradient
// partials in a fixed order.
struct PackDesc { const float* W; void* wpack; int Cout, Cin, R, mode, log2cp, ksteps, OCB; unsigned total; };
struct WredDesc { const float* partial; float* dW; int rows, Cout, Cin, R, log2cp, Jp; };
// max_total: the largest `total` among the n operands (sizes the grid)
hipError_t pack_all_launch(const PackDesc* dev_descs, int n, int dtype, hipStream_t s, unsigned max_total = 0);
// max_outputs: the largest Cout*Jp among the n layers (sizes the grid)
hipError_t wgrad_reduce_all_launch(const WredDesc* dev_descs, int n, int max_outputs, hipStream_t s);

// LDS-tiled bf16 weight gradient for 3x3/stride-1 layers with 16/32/64 channels. Returns 0 rows
// when the shape is not covered. x may be the saved conv output the activation derives from:
// then scale/shift give relu(x*scale+shift) on the fly (nullptr: use x as stored).
// fuse (optional): the kernel forms dz itself, dz = A*g + B*z + C0 with g = dy where
// mask*mscale+mshift > 0 (mask null: g = dy), coefficients from `coef` or derived from `rows`,
// and writes it to dz_out for the input-gradient kernel: the BN-backward apply pass is absorbed.
struct WgradFuse {
  const void* dy; const void* mask; const float* mscale; const float* mshift;
  const void* z; const float* coef; const BnBwdRows* rows; void* dz_out;
};
struct WgradPair {
  const void* x; const float* scale; const float* shift; const void* dz; float* partial; int rows;
};
int wgrad_tiled_rows(int N, int H, int W, int Cin, int Cout, int R, int stride, int dtype);
// H, W, C: height, width, channels of the conv INPUT. Cout (0: = C), R, stride select the
// stride-2 variants (3x3 and 1x1, Cout = 2*C) that wgrad_tiled_rows also covers.
hipError_t wgrad_tiled_launch(const void* x, const float* scale, const float* shift, const void* dz,
                              const WgradFuse* fuse, float* partial, int N, int H, int W, int C, int rows,
                              hipStream_t s, int Cout = 0, int R = 3, int stride = 1);


// LDS-tiled 3x3/stride-1 convolution for 16/32/64 channels (bf16). Returns the grid (= number of
// statistics rows), 0 if the shape is not covered. scale/shift: optional relu(in*scale+shift)
// applied while staging. The same kernel computes the input gradient from an operand packed
// with mirrored taps.
// Statistics the epilogue accumulates into partial rows [grid][2][C]:
//   mode 1: sum / sum of squares of the stored outputs (batch-norm forward of this conv)
//   mode 2: the outputs are an error gradient v; with the ReLU mask of the layer below applied,
//           g = (mask*mscale+mshift > 0) ? v : 0, the rows hold sum g and sum g*xhat of that
//           layer's BN (xhat = (z - zmean)*zinvstd): its bn_bwd_reduce pass comes for free.
//           The stored output is g, not v: the mask is applied once, where the gradient is
//           produced, and its readers (BN backward of that layer, the shortcut term of the
//           block below) take it as already masked.
struct ConvStat {
  int mode;
  float* partial;
  const void* mask; const float* mscale; const float* mshift;
  const void* z; const float* zmean; const float* zinvstd;
};
int conv_tiled_max_grid();   // no launch uses more workgroups (= partial statistics rows) than this
int conv_tiled_grid(int N, int H, int W, int Cin, int Cout, int R, int stride, int dtype);
// in_rows (optional): scale/shift are not final yet; the kernel derives them from these rows.
// res (optional, forward with statistics only): the conv input is relu(in*scale+shift + res),
// the output of the residual block before; y_out (optional) receives that input tensor.
// groups > 1 (forward only): N counts the images of `groups` minibatches laid end to end, each
// with its own batch-norm statistics; grid workgroups are split evenly over the groups, the
// statistics rows (st.partial, in_rows->partial) are [group][grid/groups][2][C], and the
// per-channel vectors of group g lie g*vec_stride floats after those of group 0.
// apply (optional, input gradient only): `in` is apply->dy, the gradient after a batch norm's
// ReLU; the kernel forms dz = BN-backward(dy) from apply->rows while staging (as the fused
// weight-gradient kernel does), convolves dz, and stores it to apply->dz_out.
// pair (optional, with apply): the launch also carries the plain weight gradient of another
// layer of the same shape (input x, or relu(x*scale+shift); error gradient dz; `rows` partial
// tiles as wgrad_tiled_rows() says), on workgroups of its own.
hipError_t conv_tiled_launch(const void* in, const float* scale, const float* shift, const BnRows* in_rows,
                             const void* wpack, void* out, const ConvStat& st, const void* add_g,
                             const void* add_mask, int N, int H, int W, int C, int grid, hipStream_t s,
                             const void* res = nullptr, void* y_out = nullptr, int groups = 1,
                             int vec_stride = 0, const WgradFuse* apply = nullptr, const WgradPair* pair = nullptr);


// The same kernels with fp32 operands (kernels_conv_tiled_f32.hip): same arguments and rules;
// conv_tiled_grid / wgrad_tiled_rows answer for both operand types.
hipError_t conv_tiled_f32_launch(const void* in, const float* scale, const float* shift, const BnRows* in_rows,
                                 const void* wpack, void* out, const ConvStat& st, const void* add_g,
                                 const void* add_mask, int N, int H, int W, int C, int grid, hipStream_t s,
                                 const void* res = nullptr, void* y_out = nullptr, int groups = 1,
                                 int vec_stride = 0, const WgradFuse* apply = nullptr, const WgradPair* pair = nullptr);
hipError_t wgrad_tiled_f32_launch(const void* x, const float* scale, const float* shift, const void* dz,
                                  const WgradFuse* fuse, float* partial, int N, int H, int W, int C, int rows,
                                  hipStream_t s);
int conv_tiled_f32_grid(int N, int H, int W, int Cin, int Cout, int R, int stride);
int wgrad_tiled_f32_rows(int N, int H, int W, int Cin, int Cout, int R, int stride);

// GEMM-class kernel for wide bf16 layers (1x1 / 3x3, stride 1, contraction channels a power of
// two >= 64, output channels a multiple of 128): forward, or input gradient with an operand
// packed with mirrored taps. in [N*H*W][IC], out [N*H*W][OC], wpack as for conv_launch;
// stat_partial (optional): [conv_wide_rows(M)][2][OC] sums / sums of squares of the stored
// values; add_g / add_mask as in ConvArgs.
bool conv_wide_ok(int IC, int OC, int R, int stride, int dtype);
int conv_wide_rows(int M);
// scale/shift (optional, forward only): the conv input is relu(in*scale + shift) per input
// channel, applied while staging.
// second (optional, forward only): a second minibatch in the same launch, same weights.
// below (optional, input gradient only; mode 2): the epilogue forms the BN-backward sums of the
// layer below into below->partial, conv_wide_rows(M) rows (see ConvStat).
struct ConvWideSecond { const void* in; void* out; float* stat_partial; const float* scale; const float* shift; };
hipError_t conv_wide_launch(const void* in, const void* wpack, void* out, float* stat_partial, const void* add_g,
                            const void* add_mask, int N, int H, int W, int IC, int OC, int R, hipStream_t s,
                            const float* scale = nullptr, const float* shift = nullptr,
                            const ConvWideSecond* second = nullptr, const ConvStat* below = nullptr);

// Weight gradient of the same wide layers (Cin a power of two >= 128, Cout a multiple of 128):
// partial tiles [splits][Cout][R*R*Cin] over `splits` slices of the pixels, to be added by
// wgrad_reduce_all_launch. x [N*H*W][Cin], dz [N*H*W][Cout].
bool wgrad_wide_ok(int Cin, int Cout, int R, int stride, int dtype);
int wgrad_wide_splits(int M, int Cin, int Cout, int R);
// scale/shift (optional): x is relu(x*scale + shift) per input channel, applied while staging.
hipError_t wgrad_wide_launch(const void* x, const void* dz, float* partial, int N, int H, int W, int Cin, int Cout,
                             int R, int splits, hipStream_t s, const float* scale = nullptr, const float* shift = nullptr);

// Batch-norm statistics from per-workgroup partial sums -> mean, invstd, scale=gamma*invstd,
// shift=beta-mean*scale.
// partial_b (optional): a second set of rows finalised by the same launch into mean_b[0..C),
// invstd = mean_b + C, scale = mean_b + 2C, shift = mean_b + 3C.
hipError_t bn_finalize_launch(const float* partial, int rows, int C, const float* gamma,
                              const float* beta, float count, float eps, float* mean, float* invstd,
                              float* scale, float* shift, hipStream_t s, const float* partial_b = nullptr,
                              float* mean_b = nullptr);
// y = [relu](z*scale+shift [+ res*rscale+rshift | + res]); zrows / rrows (optional, C <= 64):
// derive scale/shift (rscale/rshift) from partial rows instead of reading final vectors.
hipError_t bn_apply_launch(const void* z, const float* scale, const float* shift, const BnRows* zrows,
                           const void* res, const float* rscale, const float* rshift, const BnRows* rrows,
                           void* y, size_t elems, int C, int relu, int dtype, hipStream_t s);
// The same for two minibatches of the same layer in one launch (same shapes; every pointer of
// its own). Needs 256*V % C == 0 (V = 8 for bf16, 4 for fp32); false: not covered, nothing launched.
struct BnApplySet {
  const void* z; const float* scale; const float* shift; BnRows zrows;
  const void* res; const float* rscale; const float* rshift; BnRows rrows; void* y;
};
bool bn_apply_pair_launch(const BnApplySet& a, const BnApplySet& b, size_t elems, int C, int relu, int dtype,
                          hipStream_t s, hipError_t* err);
// g = dy where the ReLU that follows was active, else 0: active means mask > 0, or
// mask*mscale+mshift > 0 when mscale is given (the mask tensor is then the conv output the
// activation derives from); mask == nullptr: g = dy. partial[grid][2][C] = (sum g, sum g*xhat)
int bn_bwd_grid(size_t elems, int C, int dtype);
hipError_t bn_bwd_reduce_launch(const void* dy, const void* mask, const float* mscale, const float* mshift,
                                const void* z, const float* mean, const float* invstd, float* partial,
                                size_t elems, int C, int dtype, hipStream_t s);
// dgamma, dbeta and the coefficients of dz = A*g + B*z + C0 (per channel; coef = [3][C])
hipError_t bn_bwd_finalize_launch(const float* partial, int rows, int C, const float* gamma,
                                  const float* mean, const float* invstd, float count, float* dgamma,
                                  float* dbeta, float* coef, hipStream_t s);
// coef: final coefficients [3][C], or rows (optional, C <= 64) to derive them from.
hipError_t bn_bwd_apply_launch(const void* dy, const void* mask, const float* mscale, const float* mshift,
                               const void* z, const float* coef, const BnBwdRows* rows, void* dz, size_t elems,
                               int C, int dtype, hipStream_t s);

// Head: global average pool, linear, softmax cross-entropy (mean over the batch) and its gradients.
struct HeadArgs {
  const void* h; const float* fcw; const float* fcb; const int32_t* labels;
  float* pooled; float* dlogits; float* loss_n; float* loss_out;
  float* dfcw; float* dfcb; void* dh;
  int N, HW, C, classes, dtype;
  float* logits_out;     // optional [N][classes]
};
// dfcw == nullptr: evaluation (no gradients; dh must be null too).
hipError_t head_launch(const HeadArgs& a, hipStream_t s);

// Running batch-norm estimates and evaluation vectors, all layers of a module per launch.
struct RunDesc {
  const float* mean; const float* invstd;      // batch statistics of the forward pass that just ran
  const float* gamma; const float* beta;
  float* rmean; float* rvar;                   // running estimates
  float* escale; float* eshift;                // what the evaluation forward normalises with
  int C; float count, eps;
};
hipError_t running_update_launch(const RunDesc* dev_descs, int n, int max_c, float rho, hipStream_t s);
hipError_t eval_vectors_launch(const RunDesc* dev_descs, int n, int max_c, hipStream_t s);

// lr_dev != nullptr: the step size is read from device memory (lets a captured graph be replayed
// with a different step size).
hipError_t sgd_launch(float* w, float* v, const float* g, size_t n, float lr, const float* lr_dev,
                      float mu, float wd, hipStream_t s);
hipError_t set_scalar_launch(float* dst, float v, hipStream_t s);
// Adam (Algorithm 2). pw[0], pw[1] hold beta1^n, beta2^n in device memory: adam_advance_launch
// multiplies them by beta1, beta2 (one more executed update), adam_launch then applies
// m <- b1 m + (1-b1) g', v <- b2 v + (1-b2) g'^2, w <- w - lr (m/(1-pw0)) / (sqrt(v/(1-pw1)) + eps)
// with g' = g + wd*w. Device-resident so that a captured graph replays correctly.
hipError_t adam_advance_launch(double* pw, float b1, float b2, hipStream_t s);
hipError_t adam_launch(float* w, float* m1, float* m2, const float* g, size_t n, float lr, const float* lr_dev,
                       float b1, float b2, float eps, float wd, const double* pw, hipStream_t s);
hipError_t copy_launch(const void* src, void* dst, size_t bytes, hipStream_t s);
hipError_t to_f32_launch(const void* src, float* dst, size_t elems, int dtype, hipStream_t s);

// Static device scratch (ddg_scratch.hip): a file-scope __device__ array of this many bytes per
// GPU. static_scratch returns its device address on the current device (looked up once per
// device) and its size. Every caller on a GPU shares the one array.
#define DDG_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
hipError_t static_scratch(void** ptr, size_t* bytes);

}  // namespace ddg
