// Implicit-GEMM convolution (forward and input-gradient) on CDNA4 matrix cores.
//
// GEMM view: rows = output channels (weights operand), columns = output pixels
// (activation operand), contraction = (tap, input channel). Each wave owns
// MB pixel-blocks x NB channel-blocks of 16x16 accumulators; a lane's accumulator
// registers are 4 consecutive channels of one pixel, so the result is stored NHWC
// with one 8/16-byte store per lane. Activation fragments are gathered straight
// from the NHWC tensor (one 16-byte load of 8 bf16 or 4 fp32 channels of one tap),
// which makes the im2col matrix implicit; zero padding, stride and the
// divisibility test of the input-gradient are folded into the gather predicate.
//
// The forward variant also accumulates per-channel sum and sum of squares of the
// stored outputs (batch-norm statistics) and writes one partial row per workgroup
// in a fixed order, so the statistics are deterministic.
#include "ddg_device.h"
#include "ddg_kernels.h"
#include <cstdlib>

namespace ddg {

// Keeps a loaded fragment alive at the point of its use whatever the predicate says: without it
// the compiler moves the load back under the predicate, which makes it a branch, and every
// branch around a load ends in a wait for all loads in flight.
__device__ __forceinline__ void keep_frag(uint4& f) { asm volatile("" : "+v"(f.x), "+v"(f.y), "+v"(f.z), "+v"(f.w)); }
__device__ __forceinline__ void keep_frag(float4& f) { asm volatile("" : "+v"(f.x), "+v"(f.y), "+v"(f.z), "+v"(f.w)); }

// VEC: the contraction channel count is a multiple of the fragment width (every layer but a
// 3-channel stem): gathers are whole fragments and none of them is conditional.
template <typename T, int MB, int NB, bool DGRAD, bool VEC>
__global__ __launch_bounds__(256) void conv_mfma_kernel(ConvArgs a) {
  using M_ = Mma<T>;
  using S_ = Store<T>;
  constexpr int KV = M_::KV;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int cb0 = blockIdx.y * NB;
  const int OCB = a.OC >> 4;
  // blockIdx.z = 1: the second minibatch of a two-group launch (same weights, own tensors)
  const T* __restrict__ in = reinterpret_cast<const T*>(blockIdx.z ? a.in_b : a.in);
  const T* __restrict__ wp = reinterpret_cast<const T*>(a.wpack);
  T* __restrict__ out = reinterpret_cast<T*>(blockIdx.z ? a.out_b : a.out);
  float* __restrict__ stat_partial = blockIdx.z ? a.stat_partial_b : a.stat_partial;
  const T* __restrict__ addg = reinterpret_cast<const T*>(a.add_g);
  const T* __restrict__ addm = reinterpret_cast<const T*>(a.add_mask);
  const int tiles = (a.M + 16 * MB - 1) / (16 * MB);
  const int ohow = a.OH * a.OW;
  const int cpmask = (1 << a.log2cp) - 1;
  const int sshift = a.stride - 1;  // stride is 1 or 2

  float ssum[NB][4], ssq[NB][4];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int j = 0; j < 4; ++j) { ssum[nb][j] = 0.f; ssq[nb][j] = 0.f; }

  for (int tile = blockIdx.x * 4 + wave; tile < tiles; tile += gridDim.x * 4) {
    int pn[MB], ph[MB], pw[MB];
    bool pv[MB];
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const int m = (tile * MB + i) * 16 + l16;
      pv[i] = m < a.M;
      const int mm = pv[i] ? m : 0;
      const int n = mm / ohow;
      const int rem = mm - n * ohow;
      const int oh = rem / a.OW;
      const int ow = rem - oh * a.OW;
      pn[i] = n;
      if (DGRAD) { ph[i] = oh + a.pad; pw[i] = ow + a.pad; }
      else { ph[i] = oh * a.stride - a.pad; pw[i] = ow * a.stride - a.pad; }
    }
    f32x4_t acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) acc[i][nb] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    for (int ks = 0; ks < a.ksteps; ++ks) {
      const int kidx = (ks * 4 + lg) * KV;
      const int tap = kidx >> a.log2cp;
      const int c0 = kidx & cpmask;
      const int r = (a.R == 3) ? tap / 3 : 0;
      const int s = (a.R == 3) ? tap - r * 3 : tap;
      const bool tap_ok = (tap < a.ntaps) && (c0 < a.IC);
      typename M_::frag_t wf[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        wf[nb] = M_::load(wp + ((size_t)(ks * OCB + cb0 + nb) * 64 + lane) * KV);
      typename M_::frag_t ld[MB];
      bool okv[MB];
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        int ih, iw;
        bool ok = tap_ok && pv[i];
        if (DGRAD) {
          const int th = ph[i] - r, tw = pw[i] - s;
          ok = ok && th >= 0 && tw >= 0 && ((th | tw) & sshift) == 0;
          ih = th >> sshift; iw = tw >> sshift;
          ok = ok && ih < a.IH && iw < a.IW;
        } else {
          ih = ph[i] + r; iw = pw[i] + s;
          ok = ok && ih >= 0 && ih < a.IH && iw >= 0 && iw < a.IW;
        }
        okv[i] = ok;
        if (VEC) {
          // a padded or masked position reads the tensor's first elements instead (dropped below)
          const unsigned off = ok ? (unsigned)((pn[i] * a.IH + ih) * a.IW + iw) * (unsigned)a.IC + (unsigned)c0 : 0u;   // (32 bits: the host checks)
          ld[i] = M_::load(in + off);
        } else {
          ld[i] = M_::zero();
          if (ok) {
            const T* p = in + ((size_t)(pn[i] * a.IH + ih) * a.IW + iw) * a.IC + c0;
            if constexpr (KV == 8) {
              // contraction channels not a multiple of 8 (3-channel images): element gather
              uint32_t e[8];
#pragma unroll
              for (int j = 0; j < 8; ++j) e[j] = (c0 + j < a.IC) ? (uint32_t)reinterpret_cast<const uint16_t*>(p)[j] : 0u;
              ld[i] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
            } else {
              const float* pf = reinterpret_cast<const float*>(p);
              ld[i] = make_float4(pf[0], c0 + 1 < a.IC ? pf[1] : 0.f, c0 + 2 < a.IC ? pf[2] : 0.f, c0 + 3 < a.IC ? pf[3] : 0.f);
            }
          }
        }
      }
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        typename M_::frag_t af = ld[i];
        if (VEC) {
          keep_frag(af);
          if (!okv[i]) af = M_::zero();
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[i][nb] = M_::mma(wf[nb], af, acc[i][nb]);
      }
    }

    // epilogue: lane = pixel l16 of block i, channels (cb0+nb)*16 + lg*4 .. +3
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const int m = (tile * MB + i) * 16 + l16;
      if (!pv[i]) continue;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const size_t idx = (size_t)m * a.OC + (cb0 + nb) * 16 + lg * 4;
        float v[4] = {acc[i][nb][0], acc[i][nb][1], acc[i][nb][2], acc[i][nb][3]};
        if (addg) {
          float g[4];
          S_::load4(addg + idx, g);
          if (addm) {
            float mk[4];
            S_::load4(addm + idx, mk);
#pragma unroll
            for (int j = 0; j < 4; ++j) g[j] = (mk[j] > 0.f) ? g[j] : 0.f;
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] += g[j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          v[j] = S_::round(v[j]);
          ssum[nb][j] += v[j];
          ssq[nb][j] += v[j] * v[j];
        }
        S_::store4(out + idx, v[0], v[1], v[2], v[3]);
      }
    }
  }

  if (stat_partial) {
    __shared__ float red[4][2][NB * 16];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float s1 = ssum[nb][j], s2 = ssq[nb][j];
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
          s1 += __shfl_xor(s1, o, 64);
          s2 += __shfl_xor(s2, o, 64);
        }
        if (l16 == 0) {
          red[wave][0][nb * 16 + lg * 4 + j] = s1;
          red[wave][1][nb * 16 + lg * 4 + j] = s2;
        }
      }
    __syncthreads();
    if (threadIdx.x < 2 * NB * 16) {
      const int which = threadIdx.x / (NB * 16), c = threadIdx.x % (NB * 16);
      const float t = ((red[0][which][c] + red[1][which][c]) + red[2][which][c]) + red[3][which][c];
      stat_partial[((size_t)blockIdx.x * 2 + which) * a.OC + cb0 * 16 + c] = t;
    }
  }
}

static int ceil_log2(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}

size_t conv_wpack_elems(int kchannels, int nchannels, int R, int dtype, int* log2cp, int* ksteps) {
  const int kv = mma_kv(dtype);
  int l2 = ceil_log2(kchannels);
  while ((1 << l2) < kv) ++l2;
  const int K = R * R * (1 << l2);
  const int kstep = 4 * kv;
  const int ks = (K + kstep - 1) / kstep;
  if (log2cp) *log2cp = l2;
  if (ksteps) *ksteps = ks;
  return (size_t)ks * (nchannels / 16) * 64 * kv;
}

void conv_plan(ConvArgs& a) {
  const int ocb = a.OC / 16;
  if (ocb % 4 == 0) { a.nb = 4; a.mb = 2; }
  else if (ocb % 2 == 0) { a.nb = 2; a.mb = 2; }
  else { a.nb = 1; a.mb = 4; }
  if (a.dtype != BF16) {
    // fp32 matrix instructions are 16 times slower per flop than bf16 ones: a wave's tile is
    // what bounds the launch, so tiles shrink until there are about two per SIMD
    a.nb = 1; a.mb = 4;
    while (a.mb > 1 && (long)((a.M + 16 * a.mb - 1) / (16 * a.mb)) * ocb < 2048) a.mb /= 2;
  }
  const int gy = ocb / a.nb;
  const int tiles = (a.M + 16 * a.mb - 1) / (16 * a.mb);
  int gx = (tiles + 3) / 4;
  const int cap = 512 / gy > 1 ? 512 / gy : 1;   // also the number of statistics rows
  if (gx > cap) gx = cap;
  if (gx < 1) gx = 1;
  a.grid_x = gx;
}

template <typename T>
static hipError_t conv_dispatch(const ConvArgs& a, hipStream_t s) {
  dim3 grid(a.grid_x, (a.OC / 16) / a.nb, a.in_b ? 2 : 1), block(256);
  const bool vec = a.IC % Mma<T>::KV == 0;
#define DDG_CONV_CASE(MB_, NB_)                                                                   \
  if (a.mb == MB_ && a.nb == NB_) {                                                               \
    if (vec) {                                                                                    \
      if (a.dgrad) DDG_LAUNCH((conv_mfma_kernel<T, MB_, NB_, true, true>), grid, block, 0, s, a);   \
      else DDG_LAUNCH((conv_mfma_kernel<T, MB_, NB_, false, true>), grid, block, 0, s, a);          \
    } else {                                                                                      \
      if (a.dgrad) DDG_LAUNCH((conv_mfma_kernel<T, MB_, NB_, true, false>), grid, block, 0, s, a);  \
      else DDG_LAUNCH((conv_mfma_kernel<T, MB_, NB_, false, false>), grid, block, 0, s, a);         \
    }                                                                                             \
    return hipGetLastError();                                                                     \
  }
  DDG_CONV_CASE(4, 1)
  DDG_CONV_CASE(2, 1)
  DDG_CONV_CASE(1, 1)
  DDG_CONV_CASE(2, 2)
  DDG_CONV_CASE(2, 4)
#undef DDG_CONV_CASE
  return hipErrorInvalidValue;
}

hipError_t conv_launch(const ConvArgs& a, hipStream_t s) {
  // the gathers form 32-bit element offsets
  if ((size_t)a.N * a.IH * a.IW * a.IC >= ((size_t)1 << 32)) return hipErrorInvalidValue;
  return a.dtype == BF16 ? conv_dispatch<bf16_t>(a, s) : conv_dispatch<float>(a, s);
}

// wpack[((ks*OCB + cb)*64 + lane)*KV + j] = W-element for row cb*16+lane%16 and
// contraction index k = (ks*4 + lane/16)*KV + j -> (tap = k >> log2cp, channel = k & (CP-1)).
template <typename T>
__global__ void pack_weights_kernel(const float* __restrict__ W, T* __restrict__ wpack, int Cout,
                                    int Cin, int R, int dgrad, int log2cp, int ksteps, int OCB) {
  constexpr int KV = Mma<T>::KV;
  const size_t total = (size_t)ksteps * OCB * 64 * KV;
  const int kc = dgrad ? Cout : Cin;   // contraction channels
  const int nc = dgrad ? Cin : Cout;   // output channels
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int j = (int)(i % KV);
    const int lane = (int)((i / KV) % 64);
    const int cb = (int)((i / (KV * 64)) % OCB);
    const int ks = (int)(i / ((size_t)KV * 64 * OCB));
    const int k = (ks * 4 + lane / 16) * KV + j;
    const int tap = k >> log2cp, c = k & ((1 << log2cp) - 1);
    const int n = cb * 16 + (lane & 15);
    float v = 0.f;
    if (tap < R * R && c < kc && n < nc) {
      int r = tap / R, s = tap % R;
      if (dgrad == 2) { r = R - 1 - r; s = R - 1 - s; }   // taps mirrored: the input-gradient as a plain correlation
      const int co = dgrad ? c : n, ci = dgrad ? n : c;
      v = W[(((size_t)co * Cin + ci) * R + r) * R + s];
    }
    Store<T>::store1(wpack + i, v);
  }
}

template <typename T>
__global__ void pack_all_kernel(const PackDesc* __restrict__ descs) {
  constexpr int KV = Mma<T>::KV;
  const PackDesc d = descs[blockIdx.y];
  const int kc = d.mode ? d.Cout : d.Cin, nc = d.mode ? d.Cin : d.Cout;
  T* wpack = reinterpret_cast<T*>(d.wpack);
  for (unsigned i = blockIdx.x * blockDim.x + threadIdx.x; i < d.total; i += gridDim.x * blockDim.x) {
    const int j = (int)(i % KV);
    const int lane = (int)((i / KV) % 64);
    const int cb = (int)((i / (KV * 64)) % d.OCB);
    const int ks = (int)(i / ((unsigned)KV * 64 * d.OCB));
    const int k = (ks * 4 + lane / 16) * KV + j;
    const int tap = k >> d.log2cp, c = k & ((1 << d.log2cp) - 1);
    const int n = cb * 16 + (lane & 15);
    float v = 0.f;
    if (tap < d.R * d.R && c < kc && n < nc) {
      int r = tap / d.R, s = tap % d.R;
      if (d.mode == 2) { r = d.R - 1 - r; s = d.R - 1 - s; }
      const int co = d.mode ? c : n, ci = d.mode ? n : c;
      v = d.W[(((size_t)co * d.Cin + ci) * d.R + r) * d.R + s];
    }
    Store<T>::store1(wpack + i, v);
  }
}

hipError_t pack_all_launch(const PackDesc* dev_descs, int n, int dtype, hipStream_t s, unsigned max_total) {
  if (n <= 0) return hipSuccess;
  // workgroups per operand: about 16 elements per thread of the largest one, between 16 and 128
  unsigned bx = max_total / 4096;
  bx = bx < 16 ? 16 : (bx > 128 ? 128 : bx);
  if (dtype == BF16) DDG_LAUNCH(pack_all_kernel<bf16_t>, dim3(bx, n), dim3(256), 0, s, dev_descs);
  else DDG_LAUNCH(pack_all_kernel<float>, dim3(bx, n), dim3(256), 0, s, dev_descs);
  return hipGetLastError();
}

hipError_t pack_weights_launch(const float* W, void* wpack, int Cout, int Cin, int R, int dgrad,
                               int dtype, hipStream_t s) {
  int log2cp, ksteps;
  const int kc = dgrad ? Cout : Cin, nc = dgrad ? Cin : Cout;
  const size_t total = conv_wpack_elems(kc, nc, R, dtype, &log2cp, &ksteps);
  int grid = (int)((total + 255) / 256);
  if (grid > 1024) grid = 1024;
  if (dtype == BF16)
    DDG_LAUNCH(pack_weights_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, W,
                       reinterpret_cast<bf16_t*>(wpack), Cout, Cin, R, dgrad, log2cp, ksteps, nc / 16);
  else
    DDG_LAUNCH(pack_weights_kernel<float>, dim3(grid), dim3(256), 0, s, W,
                       reinterpret_cast<float*>(wpack), Cout, Cin, R, dgrad, log2cp, ksteps, nc / 16);
  return hipGetLastError();
}

}  // namespace ddg
