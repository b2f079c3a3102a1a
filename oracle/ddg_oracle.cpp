// CPU oracle for Decoupled Parallel Backpropagation with delayed gradients (DDG).
//
// TEST INFRASTRUCTURE ONLY. This file is the slow, plain reference that the
// HIP library is checked against. Only tests, the smoke check and the bench's
// cpu_baseline leg may load it; the product path never does. It shares no code
// with the HIP sources.
//
// What it follows (arXiv 1804.10574):
//   * Section 2, Eq. 3: layer-by-layer forward h_l = F_l(h_{l-1}; w_l).
//   * Section 2, Eq. 4-5 and Section 3.1, Eq. 6-7: chain-rule backward; under
//     DDG module k back-propagates the error gradient of iteration t-K+k.
//   * Section 3.3, Eq. 8-9 and Algorithm 1: g_k^t is zero while t-K+k < 0,
//     otherwise the gradient w.r.t. the weights of G(k); every module then
//     updates its own weights with step size gamma_t.
//   * Section 5.2: SGD with momentum (0.9) and optional weight decay.
//   * Table 2: basic residual units; layer internals follow the original
//     ResNet (conv, batch normalisation with batch statistics, ReLU, identity or
//     projected shortcut). The paper leaves these to its citation.
//
// Reading taken where the paper is silent (module-internal activations of the
// delayed iteration): a module keeps only its INPUT of iteration s = t-K+k and
// re-runs its forward on it with its CURRENT weights before back-propagating.
// `stale_jacobian` mode instead snapshots the module's weights with every queued
// input and back-propagates through that snapshot: this realises Eq. 6-7/8-9
// literally and exists to pin the delay bookkeeping against plain backprop.
//
// Evaluation. The paper reports test error (Section 5) and leaves batch normalisation at test
// time to its citations. Reading taken: every BN layer keeps running estimates of mean and
// variance, r <- (1-rho)*r + rho*(batch statistic) with rho = 0.1, the variance estimate
// unbiased (batch variance * m/(m-1)), starting from mean 0 and variance 1; they are updated by
// the forward pass on the current minibatch (ddg_forward, and the forward of plain
// backpropagation), never by the re-forward of a stored input, which would count that
// minibatch twice. The evaluation forward normalises with the running estimates and leaves
// all training state (tape, queue, estimates) untouched.
//
// Storage precision. The paper does not state a number format. The benchmark this oracle
// serves fixes bf16 convolution operands with fp32 accumulation for some workloads; with
// `store_bf16` every tensor that such an implementation keeps in memory between layers
// (conv outputs, activations, error gradients, conv weights as operands) is rounded to
// bf16 (round-to-nearest-even) at the point where it is produced, while all arithmetic
// stays in the oracle's scalar type. This puts the sign decisions of ReLU on the same
// values on both sides; without it a sign flip of a near-zero pre-activation changes the
// masked gradient by O(1) for that element. Parameters, statistics, weight gradients and
// the update are never rounded. Where exactly the mode rounds (module input, conv weights as
// operands, conv outputs, stored activations and block outputs; on the way back the gradient
// of a conv output, of a stored activation before its ReLU mask, of the projection branch, of
// a block input, the gradient received from the module above, the head's input gradient) is
// pinned by tests/test_oracle_bf16_placement.py against a PyTorch float64 autograd network
// with explicit casts at those points: identical to 1e-15, and leaving out any one point
// moves the result by 3e-4 or more.
//
// Layouts: activations NCHW, conv weights [Cout][Cin][R][S], all row-major.
// Parameter order per block: conv.W, bn.gamma, bn.beta for each conv unit in
// order (conv1, conv2, [conv3], [projection]); head: fc.W[classes][C], fc.b.
//
// Every function is a template on the scalar type; float64 instances serve as
// the parity reference and for finite differences, float32 instances are timed
// as the CPU baseline.

#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstring>
#include <deque>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

enum { KIND_STEM = 0, KIND_BASIC = 1, KIND_BOTTLENECK = 2, KIND_HEAD = 3 };

inline int out_dim(int h, int R, int stride, int pad) { return (h + 2 * pad - R) / stride + 1; }

// Round to bfloat16 (8 bits of significand), nearest-even, through float32.
template <class T>
inline T round_bf16(T v) {
  float f = (float)v;
  unsigned int u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return v;  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  u &= 0xffff0000u;
  std::memcpy(&f, &u, 4);
  return (T)f;
}
template <class T>
inline void round_store(std::vector<T>& v, bool on) {
  if (on) for (auto& e : v) e = round_bf16(e);
}

// ---------------------------------------------------------------------------
// Convolution: y[n,co,p,q] = sum_{ci,r,s} x[n,ci,p*st+r-pad,q*st+s-pad] * w[co,ci,r,s]
// (zero padding, no bias). One instance of F_l in Eq. 3.
// ---------------------------------------------------------------------------
// Range of output columns q whose input column q*st + s - pad lies inside [0, W).
inline void q_range(int Q, int W, int st, int s, int pad, int& qlo, int& qhi) {
  qlo = 0;
  while (qlo < Q && qlo * st + s - pad < 0) ++qlo;
  qhi = Q;
  while (qhi > qlo && (qhi - 1) * st + s - pad >= W) --qhi;
}

template <class T>
void conv_fwd(const T* x, const T* w, T* y, int N, int Ci, int H, int W, int Co, int R,
              int st, int pad) {
  const int P = out_dim(H, R, st, pad), Q = out_dim(W, R, st, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int co = 0; co < Co; ++co) {
      T* yp = y + ((size_t)n * Co + co) * P * Q;
      for (int i = 0; i < P * Q; ++i) yp[i] = T(0);
      for (int ci = 0; ci < Ci; ++ci) {
        const T* xp = x + ((size_t)n * Ci + ci) * H * W;
        for (int r = 0; r < R; ++r)
          for (int s = 0; s < R; ++s) {
            const T wv = w[(((size_t)co * Ci + ci) * R + r) * R + s];
            int qlo, qhi;
            q_range(Q, W, st, s, pad, qlo, qhi);
            for (int p = 0; p < P; ++p) {
              const int ih = p * st + r - pad;
              if (ih < 0 || ih >= H) continue;
              const T* xr = xp + ih * W + (s - pad);
              T* yr = yp + p * Q;
              if (st == 1) for (int q = qlo; q < qhi; ++q) yr[q] += wv * xr[q];
              else for (int q = qlo; q < qhi; ++q) yr[q] += wv * xr[q * st];
            }
          }
      }
    }
}

// Adjoint w.r.t. the input (Eq. 5 / Eq. 7 for a conv layer), written as the
// scatter that mirrors the forward loop: every (output, tap) pair adds
// w * dy into the input position it read.
template <class T>
void conv_bwd_data(const T* dy, const T* w, T* dx, int N, int Ci, int H, int W, int Co, int R,
                   int st, int pad) {
  const int P = out_dim(H, R, st, pad), Q = out_dim(W, R, st, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int ci = 0; ci < Ci; ++ci) {
      T* dxp = dx + ((size_t)n * Ci + ci) * H * W;
      for (int i = 0; i < H * W; ++i) dxp[i] = T(0);
      for (int co = 0; co < Co; ++co) {
        const T* dyp = dy + ((size_t)n * Co + co) * P * Q;
        for (int r = 0; r < R; ++r)
          for (int s = 0; s < R; ++s) {
            const T wv = w[(((size_t)co * Ci + ci) * R + r) * R + s];
            int qlo, qhi;
            q_range(Q, W, st, s, pad, qlo, qhi);
            for (int p = 0; p < P; ++p) {
              const int ih = p * st + r - pad;
              if (ih < 0 || ih >= H) continue;
              T* dxr = dxp + ih * W + (s - pad);
              const T* dyr = dyp + p * Q;
              if (st == 1) for (int q = qlo; q < qhi; ++q) dxr[q] += wv * dyr[q];
              else for (int q = qlo; q < qhi; ++q) dxr[q * st] += wv * dyr[q];
            }
          }
      }
    }
}

// Adjoint w.r.t. the weights (Eq. 4 / Eq. 6 for a conv layer): for every tap, the sum
// over images and output positions of (input read by that tap) * dy.
template <class T>
void conv_bwd_weight(const T* x, const T* dy, T* dw, int N, int Ci, int H, int W, int Co, int R,
                     int st, int pad) {
  const int P = out_dim(H, R, st, pad), Q = out_dim(W, R, st, pad);
#pragma omp parallel for collapse(2) schedule(static)
  for (int co = 0; co < Co; ++co)
    for (int ci = 0; ci < Ci; ++ci) {
      T acc[9];
      for (int i = 0; i < R * R; ++i) acc[i] = T(0);
      for (int n = 0; n < N; ++n) {
        const T* xp = x + ((size_t)n * Ci + ci) * H * W;
        const T* dyp = dy + ((size_t)n * Co + co) * P * Q;
        for (int p = 0; p < P; ++p)
          for (int q = 0; q < Q; ++q) {
            const T d = dyp[p * Q + q];
            for (int r = 0; r < R; ++r) {
              const int ih = p * st + r - pad;
              if (ih < 0 || ih >= H) continue;
              for (int s = 0; s < R; ++s) {
                const int iw = q * st + s - pad;
                if (iw < 0 || iw >= W) continue;
                acc[r * R + s] += xp[ih * W + iw] * d;
              }
            }
          }
      }
      for (int i = 0; i < R * R; ++i) dw[((size_t)co * Ci + ci) * R * R + i] = acc[i];
    }
}

// ---------------------------------------------------------------------------
// Batch normalisation with batch statistics (training mode), per channel over
// m = N*H*W: mean, biased variance, xhat = (x-mean)*invstd, y = gamma*xhat+beta.
// ---------------------------------------------------------------------------
template <class T>
void bn_fwd(const T* x, const T* gamma, const T* beta, T eps, T* y, T* mean, T* invstd, int N,
            int C, int HW, T* var = nullptr) {
  const T m = T(N) * T(HW);
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    T s = T(0);
    for (int n = 0; n < N; ++n) {
      const T* xp = x + ((size_t)n * C + c) * HW;
      for (int i = 0; i < HW; ++i) s += xp[i];
    }
    const T mu = s / m;
    T v = T(0);
    for (int n = 0; n < N; ++n) {
      const T* xp = x + ((size_t)n * C + c) * HW;
      for (int i = 0; i < HW; ++i) v += (xp[i] - mu) * (xp[i] - mu);
    }
    const T is = T(1) / std::sqrt(v / m + eps);
    mean[c] = mu;
    invstd[c] = is;
    if (var) var[c] = v / m;   // biased batch variance
    for (int n = 0; n < N; ++n) {
      const T* xp = x + ((size_t)n * C + c) * HW;
      T* yp = y + ((size_t)n * C + c) * HW;
      for (int i = 0; i < HW; ++i) yp[i] = gamma[c] * ((xp[i] - mu) * is) + beta[c];
    }
  }
}

// Batch normalisation at evaluation time: fixed per-channel estimates instead of batch
// statistics, y = gamma*(x - rmean)/sqrt(rvar + eps) + beta.
template <class T>
void bn_eval(const T* x, const T* gamma, const T* beta, const T* rmean, const T* rvar, T eps, T* y,
             int N, int C, int HW) {
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    const T is = T(1) / std::sqrt(rvar[c] + eps);
    for (int n = 0; n < N; ++n) {
      const T* xp = x + ((size_t)n * C + c) * HW;
      T* yp = y + ((size_t)n * C + c) * HW;
      for (int i = 0; i < HW; ++i) yp[i] = gamma[c] * ((xp[i] - rmean[c]) * is) + beta[c];
    }
  }
}

// dbeta = sum dy; dgamma = sum dy*xhat; dx = gamma*invstd*(dy - dbeta/m - xhat*dgamma/m).
template <class T>
void bn_bwd(const T* dy, const T* x, const T* mean, const T* invstd, const T* gamma, T* dx,
            T* dgamma, T* dbeta, int N, int C, int HW) {
  const T m = T(N) * T(HW);
#pragma omp parallel for schedule(static)
  for (int c = 0; c < C; ++c) {
    T db = T(0), dg = T(0);
    for (int n = 0; n < N; ++n) {
      const T* xp = x + ((size_t)n * C + c) * HW;
      const T* dyp = dy + ((size_t)n * C + c) * HW;
      for (int i = 0; i < HW; ++i) {
        db += dyp[i];
        dg += dyp[i] * ((xp[i] - mean[c]) * invstd[c]);
      }
    }
    dbeta[c] = db;
    dgamma[c] = dg;
    for (int n = 0; n < N; ++n) {
      const T* xp = x + ((size_t)n * C + c) * HW;
      const T* dyp = dy + ((size_t)n * C + c) * HW;
      T* dxp = dx + ((size_t)n * C + c) * HW;
      for (int i = 0; i < HW; ++i) {
        const T xh = (xp[i] - mean[c]) * invstd[c];
        dxp[i] = gamma[c] * invstd[c] * (dyp[i] - db / m - xh * dg / m);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Head: global average pool, linear layer, softmax cross-entropy averaged over
// the minibatch. Returns the loss; fills the gradients when asked.
// ---------------------------------------------------------------------------
template <class T>
T head_fwd_bwd(const T* h, const T* fcw, const T* fcb, const int* labels, int N, int C, int HW,
               int classes, T* dh, T* dfcw, T* dfcb, T* logits_out) {
  std::vector<T> pooled((size_t)N * C), logits((size_t)N * classes), dlog((size_t)N * classes);
  for (int n = 0; n < N; ++n)
    for (int c = 0; c < C; ++c) {
      T s = T(0);
      const T* hp = h + ((size_t)n * C + c) * HW;
      for (int i = 0; i < HW; ++i) s += hp[i];
      pooled[(size_t)n * C + c] = s / T(HW);
    }
  T loss = T(0);
  for (int n = 0; n < N; ++n) {
    T mx = T(0);
    for (int j = 0; j < classes; ++j) {
      T a = fcb[j];
      for (int c = 0; c < C; ++c) a += fcw[(size_t)j * C + c] * pooled[(size_t)n * C + c];
      logits[(size_t)n * classes + j] = a;
      if (j == 0 || a > mx) mx = a;
    }
    T den = T(0);
    for (int j = 0; j < classes; ++j) den += std::exp(logits[(size_t)n * classes + j] - mx);
    const T logden = std::log(den);
    loss += -(logits[(size_t)n * classes + labels[n]] - mx - logden);
    for (int j = 0; j < classes; ++j) {
      const T p = std::exp(logits[(size_t)n * classes + j] - mx) / den;
      dlog[(size_t)n * classes + j] = (p - (j == labels[n] ? T(1) : T(0))) / T(N);
    }
  }
  loss /= T(N);
  if (logits_out) std::copy(logits.begin(), logits.end(), logits_out);
  if (dfcw) {
    for (int j = 0; j < classes; ++j) {
      T sb = T(0);
      for (int n = 0; n < N; ++n) sb += dlog[(size_t)n * classes + j];
      dfcb[j] = sb;
      for (int c = 0; c < C; ++c) {
        T s = T(0);
        for (int n = 0; n < N; ++n) s += dlog[(size_t)n * classes + j] * pooled[(size_t)n * C + c];
        dfcw[(size_t)j * C + c] = s;
      }
    }
  }
  if (dh) {
    for (int n = 0; n < N; ++n)
      for (int c = 0; c < C; ++c) {
        T s = T(0);
        for (int j = 0; j < classes; ++j) s += dlog[(size_t)n * classes + j] * fcw[(size_t)j * C + c];
        T* dp = dh + ((size_t)n * C + c) * HW;
        for (int i = 0; i < HW; ++i) dp[i] = s / T(HW);
      }
  }
  return loss;
}

// ---------------------------------------------------------------------------
// Network pieces with a tape of what the backward pass needs.
// ---------------------------------------------------------------------------
template <class T>
struct Unit {  // convolution followed by batch normalisation
  int ci = 0, co = 0, R = 0, st = 1, pad = 0;
  size_t ow = 0, og = 0, ob = 0;  // offsets of W, gamma, beta in the module's parameter vector
  int N = 0, H = 0, W = 0, P = 0, Q = 0;
  std::vector<T> x, z, mean, invstd;  // tape: conv input, conv output, batch statistics
  std::vector<T> rmean, rvar;         // running estimates for evaluation (start: 0 and 1)

  std::vector<T> wop;  // conv weights as the convolution sees them (rounded if store_bf16)
  // rho > 0: this pass is on the current minibatch and moves the running estimates
  std::vector<T> forward(const T* th, const std::vector<T>& in, int N_, int H_, int W_, T eps, bool rb,
                         T rho = T(0)) {
    N = N_; H = H_; W = W_;
    P = out_dim(H, R, st, pad); Q = out_dim(W, R, st, pad);
    x = in;
    wop.assign(th + ow, th + ow + (size_t)co * ci * R * R);
    round_store(wop, rb);
    z.assign((size_t)N * co * P * Q, T(0));
    conv_fwd(x.data(), wop.data(), z.data(), N, ci, H, W, co, R, st, pad);
    round_store(z, rb);
    mean.assign(co, T(0)); invstd.assign(co, T(0));
    std::vector<T> y(z.size()), var(co);
    bn_fwd(z.data(), th + og, th + ob, eps, y.data(), mean.data(), invstd.data(), N, co, P * Q, var.data());
    if (rho > T(0)) {
      const T m = T(N) * T(P * Q);
      for (int c = 0; c < co; ++c) {
        rmean[c] = (T(1) - rho) * rmean[c] + rho * mean[c];
        rvar[c] = (T(1) - rho) * rvar[c] + rho * (var[c] * m / (m - T(1)));
      }
    }
    return y;
  }
  // Evaluation: same conv, normalisation by the running estimates; nothing is taped.
  std::vector<T> forward_eval(const T* th, const std::vector<T>& in, int N_, int H_, int W_, T eps, bool rb,
                              int* P_out, int* Q_out) const {
    const int Pe = out_dim(H_, R, st, pad), Qe = out_dim(W_, R, st, pad);
    std::vector<T> w(th + ow, th + ow + (size_t)co * ci * R * R);
    round_store(w, rb);
    std::vector<T> ze((size_t)N_ * co * Pe * Qe, T(0));
    conv_fwd(in.data(), w.data(), ze.data(), N_, ci, H_, W_, co, R, st, pad);
    round_store(ze, rb);
    std::vector<T> y(ze.size());
    bn_eval(ze.data(), th + og, th + ob, rmean.data(), rvar.data(), eps, y.data(), N_, co, Pe * Qe);
    *P_out = Pe; *Q_out = Qe;
    return y;
  }
  // dy: gradient w.r.t. the BN output. Fills this unit's parameter gradients. The returned
  // input gradient is not yet rounded: the caller may add a shortcut term first.
  std::vector<T> backward(const T* th, T* g, const std::vector<T>& dy, bool need_dx, bool rb) {
    std::vector<T> dz(z.size());
    bn_bwd(dy.data(), z.data(), mean.data(), invstd.data(), th + og, dz.data(), g + og, g + ob, N,
           co, P * Q);
    round_store(dz, rb);
    conv_bwd_weight(x.data(), dz.data(), g + ow, N, ci, H, W, co, R, st, pad);
    std::vector<T> dx;
    if (need_dx) {
      dx.assign(x.size(), T(0));
      conv_bwd_data(dz.data(), wop.data(), dx.data(), N, ci, H, W, co, R, st, pad);
    }
    return dx;
  }
};

template <class T>
void relu_inplace(std::vector<T>& v) {
  for (auto& e : v) e = e > T(0) ? e : T(0);
}
template <class T>
void relu_mask(std::vector<T>& d, const std::vector<T>& out) {  // derivative at 0 is 0
  for (size_t i = 0; i < d.size(); ++i)
    if (!(out[i] > T(0))) d[i] = T(0);
}

template <class T>
struct Block {
  int kind = 0, cin = 0, cmid = 0, cout = 0, stride = 1, projection = 0;
  std::vector<Unit<T>> u;  // main-path units, then the projection unit if any
  int nmain = 0;
  size_t ofcw = 0, ofcb = 0;  // head only
  int N = 0, H = 0, W = 0;    // input geometry of the last forward
  std::vector<std::vector<T>> act;  // post-ReLU outputs of main units except the last
  std::vector<T> y;                 // block output (after the final ReLU)
  std::vector<T> xin;               // block input (head keeps it for its backward)
};

template <class T>
struct Module {
  int K = 1, k = 1;
  int N = 0, in_c = 0, in_h = 0, in_w = 0, out_c = 0, out_h = 0, out_w = 0;
  int classes = 0;
  bool has_head = false;
  std::vector<Block<T>> blocks;
  std::vector<T> theta, vel, grad;
  std::vector<T> mom2;             // Adam-DDG: second moment (vel holds the first moment)
  long nupd = 0;                   // Adam-DDG: updates executed so far
  bool has_grad = false;
  struct Entry { std::vector<T> u; std::vector<T> theta; long t; };
  std::deque<Entry> fifo;          // module inputs waiting for their delayed gradient
  std::vector<T> inbox; long inbox_t = -1;   // error gradient at this module's output
  std::vector<T> h_out;            // output of the last forward on the current minibatch
  T last_loss = T(0);
  std::vector<T> last_logits;

  size_t in_size() const { return (size_t)N * in_c * in_h * in_w; }
  size_t out_size() const { return (size_t)N * out_c * out_h * out_w; }
};

template <class T>
struct Net {
  int K = 1, k_first = 1;
  T momentum = T(0), wd = T(0), eps = T(1e-5);
  int adam = 0;                    // 0: momentum SGD (Algorithm 1), 1: Adam (Algorithm 2)
  T beta1 = T(0.9), beta2 = T(0.999), adam_eps = T(1e-8);
  int stale_jacobian = 0;
  int store_bf16 = 0;
  T bn_rho = T(0.1);               // weight of the newest batch statistic in the running estimates
  long t = 0;
  std::vector<Module<T>> mods;
  Module<T>& mod(int k) { return mods[k - k_first]; }
};

template <class T>
void add_unit(Block<T>& b, size_t& off, int ci, int co, int R, int st) {
  Unit<T> u;
  u.ci = ci; u.co = co; u.R = R; u.st = st; u.pad = (R == 3) ? 1 : 0;
  u.ow = off; off += (size_t)co * ci * R * R;
  u.og = off; off += co;
  u.ob = off; off += co;
  u.rmean.assign(co, T(0)); u.rvar.assign(co, T(1));
  b.u.push_back(u);
}

template <class T>
void build_module(Module<T>& m, const int* desc, int nblocks) {
  size_t off = 0;
  int c = m.in_c, h = m.in_h, w = m.in_w;
  for (int i = 0; i < nblocks; ++i) {
    Block<T> b;
    b.kind = desc[6 * i + 0]; b.cin = desc[6 * i + 1]; b.cmid = desc[6 * i + 2];
    b.cout = desc[6 * i + 3]; b.stride = desc[6 * i + 4]; b.projection = desc[6 * i + 5];
    if (b.kind == KIND_STEM) {
      add_unit(b, off, b.cin, b.cout, 3, b.stride); b.nmain = 1;
    } else if (b.kind == KIND_BASIC) {
      add_unit(b, off, b.cin, b.cout, 3, b.stride);
      add_unit(b, off, b.cout, b.cout, 3, 1); b.nmain = 2;
      if (b.projection) add_unit(b, off, b.cin, b.cout, 1, b.stride);
    } else if (b.kind == KIND_BOTTLENECK) {
      add_unit(b, off, b.cin, b.cmid, 1, 1);
      add_unit(b, off, b.cmid, b.cmid, 3, b.stride);
      add_unit(b, off, b.cmid, b.cout, 1, 1); b.nmain = 3;
      if (b.projection) add_unit(b, off, b.cin, b.cout, 1, b.stride);
    } else {  // head
      b.ofcw = off; off += (size_t)m.classes * b.cin;
      b.ofcb = off; off += m.classes;
      m.has_head = true;
    }
    if (b.kind != KIND_HEAD) {
      c = b.cout; h = (h - 1) / b.stride + 1; w = (w - 1) / b.stride + 1;
    }
    m.blocks.push_back(b);
  }
  m.out_c = c; m.out_h = h; m.out_w = w;
  m.theta.assign(off, T(0)); m.vel.assign(off, T(0)); m.grad.assign(off, T(0)); m.mom2.assign(off, T(0));
}

// Forward of one module (Eq. 3 for every layer of G(k)), taping intermediates.
template <class T>
std::vector<T> module_forward(Module<T>& m, const T* th, const std::vector<T>& in, T eps, bool rb,
                              T rho = T(0)) {
  std::vector<T> cur = in;
  int h = m.in_h, w = m.in_w;
  for (auto& b : m.blocks) {
    b.N = m.N; b.H = h; b.W = w;
    if (b.kind == KIND_HEAD) { b.xin = cur; continue; }  // evaluated in the backward call
    b.act.clear();
    std::vector<T> a = cur;
    for (int i = 0; i < b.nmain; ++i) {
      const int hh = (i == 0) ? h : b.u[i - 1].P, ww = (i == 0) ? w : b.u[i - 1].Q;
      a = b.u[i].forward(th, a, m.N, hh, ww, eps, rb, rho);
      if (i + 1 < b.nmain || b.kind == KIND_STEM) {
        relu_inplace(a);
        round_store(a, rb);
        if (i + 1 < b.nmain) b.act.push_back(a);
      }
    }
    if (b.kind != KIND_STEM) {
      std::vector<T> sc = (b.projection) ? b.u[b.nmain].forward(th, cur, m.N, h, w, eps, rb, rho) : cur;
      for (size_t i = 0; i < a.size(); ++i) a[i] = a[i] + sc[i];
      relu_inplace(a);
      round_store(a, rb);
    }
    b.y = a;
    h = b.u[b.nmain - 1].P; w = b.u[b.nmain - 1].Q;
    cur = a;
  }
  return cur;
}

// Evaluation forward of one module: the same layers with every BN normalising by its running
// estimates. Touches no training state. With a head: the mean loss is returned through
// loss_out (labels given) and the logits through logits_out; the returned tensor is the input
// of the head.
template <class T>
std::vector<T> module_forward_eval(const Module<T>& m, const std::vector<T>& in, T eps, bool rb,
                                   const int* labels, T* loss_out, T* logits_out) {
  const T* th = m.theta.data();
  std::vector<T> cur = in;
  int h = m.in_h, w = m.in_w;
  for (const auto& b : m.blocks) {
    if (b.kind == KIND_HEAD) {
      std::vector<int> zero_labels;
      if (!labels) { zero_labels.assign(m.N, 0); labels = zero_labels.data(); }
      const T loss = head_fwd_bwd<T>(cur.data(), th + b.ofcw, th + b.ofcb, labels, m.N, b.cin, h * w, m.classes,
                                     nullptr, nullptr, nullptr, logits_out);
      if (loss_out) *loss_out = loss;
      continue;
    }
    std::vector<T> a = cur;
    int hh = h, ww = w, P = h, Q = w;
    for (int i = 0; i < b.nmain; ++i) {
      a = b.u[i].forward_eval(th, a, m.N, hh, ww, eps, rb, &P, &Q);
      hh = P; ww = Q;
      if (i + 1 < b.nmain || b.kind == KIND_STEM) {
        relu_inplace(a);
        round_store(a, rb);
      }
    }
    if (b.kind != KIND_STEM) {
      int Ps, Qs;
      std::vector<T> sc = (b.projection) ? b.u[b.nmain].forward_eval(th, cur, m.N, h, w, eps, rb, &Ps, &Qs) : cur;
      for (size_t i = 0; i < a.size(); ++i) a[i] = a[i] + sc[i];
      relu_inplace(a);
      round_store(a, rb);
    }
    h = P; w = Q;
    cur = a;
  }
  return cur;
}

// Backward of one module through its tape (Eq. 4-5 / Eq. 6-7). `dtop` is the error
// gradient at the module output (ignored when the module ends in the head, whose
// loss gradient starts the chain). Writes all parameter gradients into g; returns the
// error gradient at the module input when need_dx.
template <class T>
std::vector<T> module_backward(Module<T>& m, const T* th, T* g, const std::vector<T>& dtop,
                               const int* labels, bool need_dx, bool rb) {
  std::vector<T> d = dtop;
  for (int bi = (int)m.blocks.size() - 1; bi >= 0; --bi) {
    auto& b = m.blocks[bi];
    const bool first = (bi == 0);
    if (b.kind == KIND_HEAD) {
      d.assign(b.xin.size(), T(0));
      m.last_logits.assign((size_t)m.N * m.classes, T(0));
      m.last_loss = head_fwd_bwd(b.xin.data(), th + b.ofcw, th + b.ofcb, labels, b.N, b.cin,
                                 b.H * b.W, m.classes, d.data(), g + b.ofcw, g + b.ofcb,
                                 m.last_logits.data());
      round_store(d, rb);
      continue;
    }
    relu_mask(d, b.y);  // the block ends in a ReLU
    const bool want_dx = need_dx || !first;
    std::vector<T> dsum = d, dx;
    for (int i = b.nmain - 1; i >= 0; --i) {
      const bool unit_dx = (i > 0) || want_dx;
      d = b.u[i].backward(th, g, d, unit_dx, rb);
      if (i > 0) { round_store(d, rb); relu_mask(d, b.act[i - 1]); }
    }
    if (b.kind != KIND_STEM && want_dx) {
      if (b.projection) {
        std::vector<T> dp = b.u[b.nmain].backward(th, g, dsum, true, rb);
        round_store(dp, rb);
        for (size_t i = 0; i < d.size(); ++i) d[i] = d[i] + dp[i];
      } else {
        for (size_t i = 0; i < d.size(); ++i) d[i] = d[i] + dsum[i];
      }
    } else if (b.kind != KIND_STEM && b.projection) {
      b.u[b.nmain].backward(th, g, dsum, false, rb);
    }
    round_store(d, rb);
  }
  return d;
}

// --- the three calls of one module's step -------------------------------------------

template <class T>
void ddg_forward(Net<T>& net, int k, long t, const T* h_in, T* h_out) {
  auto& m = net.mod(k);
  typename Module<T>::Entry e;
  e.u.assign(h_in, h_in + m.in_size());
  e.t = t;
  if (net.stale_jacobian) e.theta = m.theta;
  round_store(e.u, net.store_bf16 != 0);
  m.fifo.push_back(e);
  m.h_out = module_forward(m, m.theta.data(), m.fifo.back().u, net.eps, net.store_bf16 != 0, net.bn_rho);
  if (h_out) std::copy(m.h_out.begin(), m.h_out.end(), h_out);
}

// Evaluation forward of module k on h_in (running estimates, no training state touched).
template <class T>
void ddg_forward_eval(const Net<T>& net, int k, const T* h_in, T* h_out, const int* labels, T* loss_out,
                      T* logits_out) {
  const auto& m = net.mods[k - net.k_first];
  std::vector<T> in(h_in, h_in + m.in_size());
  round_store(in, net.store_bf16 != 0);
  const std::vector<T> out = module_forward_eval(m, in, net.eps, net.store_bf16 != 0, labels, loss_out, logits_out);
  if (h_out && !m.has_head) std::copy(out.begin(), out.end(), h_out);
}

// Returns 1 if a gradient was computed (s = t-K+k >= 0), else 0 (Eq. 8: zero gradient).
template <class T>
int ddg_backward_delayed(Net<T>& net, int k, long t, const T* delta_in, const int* labels,
                         T* delta_out, T* loss_out) {
  auto& m = net.mod(k);
  const long s = t - net.K + k;
  m.has_grad = false;
  if (s < 0) return 0;
  typename Module<T>::Entry e = m.fifo.front();
  m.fifo.pop_front();
  if (e.t != s) return -1;  // delay bookkeeping broken
  const T* th = net.stale_jacobian ? e.theta.data() : m.theta.data();
  // Re-forward the stored input. With no delay (last module) the tape left by ddg_forward
  // of this same iteration already is that forward: same input, same weights.
  const bool rb = net.store_bf16 != 0;
  if (net.K - k > 0) module_forward(m, th, e.u, net.eps, rb);
  std::vector<T> dtop;
  if (!m.has_head) { dtop.assign(delta_in, delta_in + m.out_size()); round_store(dtop, rb); }
  const bool need_dx = (k > 1);
  std::vector<T> dbelow = module_backward(m, th, m.grad.data(), dtop, labels, need_dx, rb);
  m.has_grad = true;
  if (need_dx && delta_out) std::copy(dbelow.begin(), dbelow.end(), delta_out);
  if (m.has_head && loss_out) *loss_out = m.last_loss;
  return 1;
}

// Adam with delayed gradients on module k (Algorithm 2), steps in the paper's order: first
// moment, second moment, both bias corrections, weight update. The exponent of the bias
// corrections is the number of updates this module has executed (its warm-up iterations
// execute none, so its moments are untouched until then). wd adds wd*w to the gradient.
template <class T>
void ddg_update_adam(Net<T>& net, int k, T lr) {
  auto& m = net.mod(k);
  if (!m.has_grad) return;
  m.nupd += 1;
  const T b1 = net.beta1, b2 = net.beta2;
  const T c1 = T(1) - std::pow(b1, (T)m.nupd), c2 = T(1) - std::pow(b2, (T)m.nupd);
  for (size_t i = 0; i < m.theta.size(); ++i) {
    const T g = m.grad[i] + net.wd * m.theta[i];
    m.vel[i] = b1 * m.vel[i] + (T(1) - b1) * g;
    m.mom2[i] = b2 * m.mom2[i] + (T(1) - b2) * g * g;
    const T mhat = m.vel[i] / c1;
    const T vhat = m.mom2[i] / c2;
    m.theta[i] = m.theta[i] - lr * mhat / (std::sqrt(vhat) + net.adam_eps);
  }
}

// Momentum SGD on module k: v <- mu*v + (g + wd*w); w <- w - lr*v. Skipped while the
// module has no gradient yet. (With net.adam set, the Adam update above instead.)
template <class T>
void ddg_update(Net<T>& net, int k, T lr) {
  if (net.adam) { ddg_update_adam(net, k, lr); return; }
  auto& m = net.mod(k);
  if (!m.has_grad) return;
  for (size_t i = 0; i < m.theta.size(); ++i) {
    m.vel[i] = net.momentum * m.vel[i] + (m.grad[i] + net.wd * m.theta[i]);
    m.theta[i] = m.theta[i] - lr * m.vel[i];
  }
}

// One DDG iteration over all K modules (Algorithm 1). Forward runs k = 1..K in order.
// In the backward phase every module reads only error gradients produced in the previous
// iteration; what it produces is staged and committed after all modules are done.
template <class T>
T ddg_step(Net<T>& net, const T* x, const int* labels, T lr) {
  const long t = net.t;
  const int K = net.K;
  std::vector<T> h(x, x + net.mod(1).in_size());
  for (int k = 1; k <= K; ++k) {
    std::vector<T> o(net.mod(k).out_size());
    ddg_forward(net, k, t, h.data(), o.data());
    h.swap(o);
  }
  std::vector<std::vector<T>> staged(K + 1);
  std::vector<long> staged_t(K + 1, -1);
  T loss = T(0);
  for (int k = 1; k <= K; ++k) {
    auto& m = net.mod(k);
    const long s = t - K + k;
    if (s < 0) { m.has_grad = false; continue; }
    const T* din = nullptr;
    if (k < K) {
      if (m.inbox_t != s) return T(-1e30);  // wrong delay
      din = m.inbox.data();
    }
    std::vector<T> dout(k > 1 ? m.in_size() : 0);
    T l = T(0);
    ddg_backward_delayed(net, k, t, din, labels, dout.data(), &l);
    if (k == K) loss = l;
    if (k > 1) { staged[k - 1].swap(dout); staged_t[k - 1] = s; }
  }
  for (int k = 1; k < K; ++k)
    if (staged_t[k] >= 0) { net.mod(k).inbox.swap(staged[k]); net.mod(k).inbox_t = staged_t[k]; }
  for (int k = 1; k <= K; ++k) ddg_update(net, k, lr);
  net.t = t + 1;
  return loss;
}

// Plain backpropagation over the chain of all modules (Section 2): forward, backward with
// the up-to-date error gradient handed down immediately, optional momentum-SGD update.
// Gradients stay in each module's grad; the error gradient at each module's output is
// left in its inbox (timestamp = net.t).
template <class T>
T bp_step(Net<T>& net, const T* x, const int* labels, T lr, int do_update) {
  const int K = net.K;
  std::vector<T> h(x, x + net.mod(1).in_size());
  round_store(h, net.store_bf16 != 0);  // the network input is a stored tensor too
  for (int k = 1; k <= K; ++k) {
    auto& m = net.mod(k);
    m.h_out = module_forward(m, m.theta.data(), h, net.eps, net.store_bf16 != 0, net.bn_rho);
    h = m.h_out;
  }
  std::vector<T> d;
  for (int k = K; k >= 1; --k) {
    auto& m = net.mod(k);
    if (k < K) { m.inbox = d; m.inbox_t = net.t; }
    d = module_backward(m, m.theta.data(), m.grad.data(), d, labels, k > 1, net.store_bf16 != 0);
    m.has_grad = true;
  }
  const T loss = net.mod(K).last_loss;
  if (do_update) {
    for (int k = 1; k <= K; ++k) ddg_update(net, k, lr);
    net.t += 1;
  }
  return loss;
}

template <class T>
Net<T>* net_create(int K, int k_first, int nmods, const int* nblocks, const int* desc, int batch,
                   int in_c, int in_h, int in_w, int classes, double momentum, double wd,
                   double eps, int stale_jacobian, int store_bf16) {
  auto* net = new Net<T>();
  net->store_bf16 = store_bf16;
  net->K = K; net->k_first = k_first;
  net->momentum = T(momentum); net->wd = T(wd); net->eps = T(eps);
  net->stale_jacobian = stale_jacobian;
  int c = in_c, h = in_h, w = in_w;
  const int* d = desc;
  for (int i = 0; i < nmods; ++i) {
    Module<T> m;
    m.K = K; m.k = k_first + i; m.N = batch; m.in_c = c; m.in_h = h; m.in_w = w;
    m.classes = classes;
    build_module(m, d, nblocks[i]);
    d += 6 * nblocks[i];
    c = m.out_c; h = m.out_h; w = m.out_w;
    net->mods.push_back(m);
  }
  return net;
}

}  // namespace

// ---------------------------------------------------------------------------
// C interface (ctypes). One set of symbols per scalar type.
// ---------------------------------------------------------------------------
#define ORC_API(SFX, T)                                                                          \
  extern "C" {                                                                                   \
  void orc_conv_fwd_##SFX(const T* x, const T* w, T* y, int N, int Ci, int H, int W, int Co,     \
                          int R, int st, int pad) { conv_fwd<T>(x, w, y, N, Ci, H, W, Co, R, st, pad); } \
  void orc_conv_bwd_data_##SFX(const T* dy, const T* w, T* dx, int N, int Ci, int H, int W,      \
                               int Co, int R, int st, int pad) {                                 \
    conv_bwd_data<T>(dy, w, dx, N, Ci, H, W, Co, R, st, pad); }                                  \
  void orc_conv_bwd_weight_##SFX(const T* x, const T* dy, T* dw, int N, int Ci, int H, int W,    \
                                 int Co, int R, int st, int pad) {                               \
    conv_bwd_weight<T>(x, dy, dw, N, Ci, H, W, Co, R, st, pad); }                                \
  void orc_bn_fwd_##SFX(const T* x, const T* gamma, const T* beta, double eps, T* y, T* mean,    \
                        T* invstd, int N, int C, int HW) {                                       \
    bn_fwd<T>(x, gamma, beta, T(eps), y, mean, invstd, N, C, HW); }                              \
  void orc_bn_bwd_##SFX(const T* dy, const T* x, const T* mean, const T* invstd, const T* gamma, \
                        T* dx, T* dgamma, T* dbeta, int N, int C, int HW) {                      \
    bn_bwd<T>(dy, x, mean, invstd, gamma, dx, dgamma, dbeta, N, C, HW); }                        \
  double orc_head_##SFX(const T* h, const T* fcw, const T* fcb, const int* labels, int N, int C, \
                        int HW, int classes, T* dh, T* dfcw, T* dfcb, T* logits) {               \
    return (double)head_fwd_bwd<T>(h, fcw, fcb, labels, N, C, HW, classes, dh, dfcw, dfcb, logits); } \
  void* orc_create_##SFX(int K, int k_first, int nmods, const int* nblocks, const int* desc,     \
                         int batch, int in_c, int in_h, int in_w, int classes, double momentum,  \
                         double wd, double eps, int stale_jacobian, int store_bf16) {            \
    return net_create<T>(K, k_first, nmods, nblocks, desc, batch, in_c, in_h, in_w, classes,     \
                         momentum, wd, eps, stale_jacobian, store_bf16); }                       \
  void orc_round_bf16_##SFX(T* v, long n) { for (long i = 0; i < n; ++i) v[i] = round_bf16<T>(v[i]); } \
  void orc_destroy_##SFX(void* p) { delete (Net<T>*)p; }                                         \
  long orc_param_count_##SFX(void* p, int k) { return (long)((Net<T>*)p)->mod(k).theta.size(); } \
  long orc_in_size_##SFX(void* p, int k) { return (long)((Net<T>*)p)->mod(k).in_size(); }        \
  long orc_out_size_##SFX(void* p, int k) { return (long)((Net<T>*)p)->mod(k).out_size(); }      \
  void orc_out_shape_##SFX(void* p, int k, int* chw) {                                           \
    auto& m = ((Net<T>*)p)->mod(k); chw[0] = m.out_c; chw[1] = m.out_h; chw[2] = m.out_w; }      \
  void orc_set_params_##SFX(void* p, int k, const T* v) {                                        \
    auto& m = ((Net<T>*)p)->mod(k); std::copy(v, v + m.theta.size(), m.theta.begin()); }         \
  void orc_set_velocity_##SFX(void* p, int k, const T* v) {                                      \
    auto& m = ((Net<T>*)p)->mod(k); std::copy(v, v + m.vel.size(), m.vel.begin()); }             \
  void orc_get_params_##SFX(void* p, int k, T* v) {                                              \
    auto& m = ((Net<T>*)p)->mod(k); std::copy(m.theta.begin(), m.theta.end(), v); }              \
  void orc_get_velocity_##SFX(void* p, int k, T* v) {                                            \
    auto& m = ((Net<T>*)p)->mod(k); std::copy(m.vel.begin(), m.vel.end(), v); }                  \
  int orc_get_grad_##SFX(void* p, int k, T* v) {                                                 \
    auto& m = ((Net<T>*)p)->mod(k); std::copy(m.grad.begin(), m.grad.end(), v);                  \
    return m.has_grad ? 1 : 0; }                                                                 \
  void orc_get_h_##SFX(void* p, int k, T* v) {                                                   \
    auto& m = ((Net<T>*)p)->mod(k); std::copy(m.h_out.begin(), m.h_out.end(), v); }              \
  long orc_get_delta_##SFX(void* p, int k, T* v) {                                               \
    auto& m = ((Net<T>*)p)->mod(k);                                                              \
    if (m.inbox_t >= 0 && v) std::copy(m.inbox.begin(), m.inbox.end(), v);                       \
    return m.inbox_t; }                                                                          \
  int orc_get_logits_##SFX(void* p, int k, T* v) {                                               \
    auto& m = ((Net<T>*)p)->mod(k); std::copy(m.last_logits.begin(), m.last_logits.end(), v);    \
    return (int)m.last_logits.size(); }                                                          \
  long orc_fifo_depth_##SFX(void* p, int k) { return (long)((Net<T>*)p)->mod(k).fifo.size(); }   \
  long orc_time_##SFX(void* p) { return ((Net<T>*)p)->t; }                                       \
  void orc_forward_##SFX(void* p, int k, long t, const T* h_in, T* h_out) {                      \
    ddg_forward<T>(*(Net<T>*)p, k, t, h_in, h_out); }                                            \
  int orc_backward_delayed_##SFX(void* p, int k, long t, const T* delta_in, const int* labels,   \
                                 T* delta_out, T* loss_out) {                                    \
    return ddg_backward_delayed<T>(*(Net<T>*)p, k, t, delta_in, labels, delta_out, loss_out); }  \
  void orc_update_##SFX(void* p, int k, double lr) { ddg_update<T>(*(Net<T>*)p, k, T(lr)); }     \
  void orc_set_adam_##SFX(void* p, int on, double b1, double b2, double eps) {                    \
    auto& n = *(Net<T>*)p; n.adam = on; n.beta1 = T(b1); n.beta2 = T(b2); n.adam_eps = T(eps); }  \
  void orc_set_moment2_##SFX(void* p, int k, const T* v) {                                       \
    auto& m = ((Net<T>*)p)->mod(k); std::copy(v, v + m.mom2.size(), m.mom2.begin()); }           \
  void orc_get_moment2_##SFX(void* p, int k, T* v) {                                             \
    auto& m = ((Net<T>*)p)->mod(k); std::copy(m.mom2.begin(), m.mom2.end(), v); }                \
  void orc_forward_eval_##SFX(void* p, int k, const T* h_in, T* h_out, const int* labels,        \
                              T* loss_out, T* logits_out) {                                      \
    ddg_forward_eval<T>(*(Net<T>*)p, k, h_in, h_out, labels, loss_out, logits_out); }            \
  void orc_set_bn_momentum_##SFX(void* p, double rho) { ((Net<T>*)p)->bn_rho = T(rho); }         \
  long orc_running_count_##SFX(void* p, int k) {                                                 \
    long n = 0;                                                                                  \
    for (auto& b : ((Net<T>*)p)->mod(k).blocks) for (auto& u : b.u) n += 2 * u.co;               \
    return n; }                                                                                  \
  /* per conv unit in parameter order: running mean[C], then running variance[C] */             \
  void orc_get_running_##SFX(void* p, int k, T* v) {                                             \
    for (auto& b : ((Net<T>*)p)->mod(k).blocks) for (auto& u : b.u) {                            \
      v = std::copy(u.rmean.begin(), u.rmean.end(), v); v = std::copy(u.rvar.begin(), u.rvar.end(), v); } } \
  void orc_set_running_##SFX(void* p, int k, const T* v) {                                       \
    for (auto& b : ((Net<T>*)p)->mod(k).blocks) for (auto& u : b.u) {                            \
      std::copy(v, v + u.co, u.rmean.begin()); v += u.co;                                        \
      std::copy(v, v + u.co, u.rvar.begin()); v += u.co; } }                                     \
  long orc_get_updates_##SFX(void* p, int k) { return ((Net<T>*)p)->mod(k).nupd; }               \
  void orc_set_updates_##SFX(void* p, int k, long n) { ((Net<T>*)p)->mod(k).nupd = n; }          \
  double orc_ddg_step_##SFX(void* p, const T* x, const int* labels, double lr) {                 \
    return (double)ddg_step<T>(*(Net<T>*)p, x, labels, T(lr)); }                                 \
  double orc_bp_step_##SFX(void* p, const T* x, const int* labels, double lr, int do_update) {   \
    return (double)bp_step<T>(*(Net<T>*)p, x, labels, T(lr), do_update); }                       \
  }

ORC_API(f64, double)
ORC_API(f32, float)

extern "C" int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
