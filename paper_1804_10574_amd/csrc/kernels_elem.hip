// Bandwidth-bound kernels: batch-norm finalise / apply / backward, the head
// (global average pool, linear, softmax cross-entropy), momentum SGD, copies.
//
// Tensors are NHWC, so a thread that walks the tensor with a stride that is a
// multiple of the channel count always sees the same channels: per-channel
// coefficients live in registers and every access is a 16-byte vector.
// Reductions write per-workgroup partial rows that a finalise kernel adds in a
// fixed order in double precision (deterministic, no atomics).
#include "ddg_device.h"
#include "ddg_kernels.h"
#include "ddg_stats.h"

namespace ddg {

// ---------------------------------------------------------------------------------
// Finalise per-channel statistics. partial is [rows][2][C] (sum, sum of squares).
// One workgroup per 16 channels; 16 row-slices per channel are combined in order.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void bn_finalize_kernel(const float* __restrict__ partial, int rows,
                                                          int C, const float* __restrict__ gamma,
                                                          const float* __restrict__ beta, float count,
                                                          float eps, float* mean, float* invstd,
                                                          float* scale, float* shift,
                                                          const float* __restrict__ partial_b, float* mean_b) {
  if (blockIdx.y) {   // the second set of rows and vectors
    partial = partial_b; mean = mean_b; invstd = mean_b + C; scale = mean_b + 2 * C; shift = mean_b + 3 * C;
  }
  __shared__ double r1[64][17], r2[64][17];
  const int cl = threadIdx.x & 15, slice = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cl;
  double s1 = 0.0, s2 = 0.0;
  if (c < C)
    for (int r = slice; r < rows; r += 64) {
      s1 += (double)partial[((size_t)r * 2 + 0) * C + c];
      s2 += (double)partial[((size_t)r * 2 + 1) * C + c];
    }
  r1[slice][cl] = s1; r2[slice][cl] = s2;
  __syncthreads();
  // the 64 slices in two short steps (8 x 8, each in a fixed order) instead of one chain of 64
  double p1 = 0.0, p2 = 0.0;
  if (slice < 8) {
#pragma unroll
    for (int i = 0; i < 8; ++i) { p1 += r1[slice * 8 + i][cl]; p2 += r2[slice * 8 + i][cl]; }
  }
  __syncthreads();
  if (slice < 8) { r1[slice][cl] = p1; r2[slice][cl] = p2; }
  __syncthreads();
  if (slice == 0 && c < C) {
    double t1 = 0.0, t2 = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { t1 += r1[i][cl]; t2 += r2[i][cl]; }
    const double mu = t1 / (double)count;
    double var = t2 / (double)count - mu * mu;
    if (var < 0.0) var = 0.0;
    const float is = (float)(1.0 / sqrt(var + (double)eps));
    const float sc = gamma[c] * is;
    mean[c] = (float)mu;
    invstd[c] = is;
    scale[c] = sc;
    shift[c] = beta[c] - (float)mu * sc;
  }
}

hipError_t bn_finalize_launch(const float* partial, int rows, int C, const float* gamma,
                              const float* beta, float count, float eps, float* mean, float* invstd,
                              float* scale, float* shift, hipStream_t s, const float* partial_b, float* mean_b) {
  DDG_LAUNCH(bn_finalize_kernel, dim3((C + 15) / 16, partial_b ? 2 : 1), dim3(1024), 0, s, partial, rows, C, gamma,
                     beta, count, eps, mean, invstd, scale, shift, partial_b, mean_b);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// y = [relu](z*scale + shift + shortcut), shortcut = res*rscale+rshift, res, or nothing
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void bn_apply_kernel(const T* __restrict__ z, const float* __restrict__ scale,
                                                       const float* __restrict__ shift, BnRows zrows,
                                                       const T* __restrict__ res,
                                                       const float* __restrict__ rscale,
                                                       const float* __restrict__ rshift, BnRows rrows,
                                                       T* __restrict__ y, size_t nvec, int C, int relu) {
  constexpr int V = Store<T>::VEC;
  const size_t stride = (size_t)gridDim.x * blockDim.x;  // host makes stride*V a multiple of C
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int c0 = (int)((i * V) % C);
  __shared__ float s_sc[STATS_CMAX], s_sh[STATS_CMAX], s_rs[STATS_CMAX], s_rh[STATS_CMAX];
  if (zrows.partial) { bn_fwd_from_rows_rt(zrows, C, s_sc, s_sh, blockIdx.x == 0); scale = s_sc; shift = s_sh; }
  if (rrows.partial) { bn_fwd_from_rows_rt(rrows, C, s_rs, s_rh, blockIdx.x == 0); rscale = s_rs; rshift = s_rh; }
  float sc[V], sh[V], rs[V], rh[V];
#pragma unroll
  for (int j = 0; j < V; ++j) {
    sc[j] = scale[c0 + j]; sh[j] = shift[c0 + j];
    rs[j] = rscale ? rscale[c0 + j] : 1.f;
    rh[j] = rshift ? rshift[c0 + j] : 0.f;
  }
  for (; i < nvec; i += stride) {
    float v[V];
    Store<T>::load_vec(z + i * V, v);
#pragma unroll
    for (int j = 0; j < V; ++j) v[j] = v[j] * sc[j] + sh[j];
    if (res) {
      float r[V];
      Store<T>::load_vec(res + i * V, r);
#pragma unroll
      for (int j = 0; j < V; ++j) v[j] += r[j] * rs[j] + rh[j];
    }
    if (relu) {
#pragma unroll
      for (int j = 0; j < V; ++j) v[j] = v[j] > 0.f ? v[j] : 0.f;
    }
    Store<T>::store_vec(y + i * V, v);
  }
}

// grid such that (grid*256*V) % C == 0 and the tensor is covered a few times over
static int elem_grid(size_t nvec, int C, int V, int max_blocks) {
  size_t blocks = (nvec + 255) / 256;
  if (blocks > (size_t)max_blocks) blocks = max_blocks;
  // 256*V elements per block; need blocks*256*V % C == 0
  int per = 256 * V;
  int need = 1;
  while ((size_t)need * per % C != 0) ++need;  // C <= 256*V*need, small loop
  blocks = ((blocks + need - 1) / need) * need;
  return (int)blocks;
}

// Same operation for the common case 256*V % C == 0 (a thread's channels are the same for all
// its vectors). A workgroup owns 256*U consecutive vectors; every thread issues all its loads
// first, the per-channel vectors are derived from the partial rows while those are in flight,
// and nothing loops: with U = 4 a thread keeps 128 bytes in flight, which is what it takes to
// approach the memory system's bandwidth with two workgroups per compute unit.
template <typename T, int U>
__global__ __launch_bounds__(256) void bn_apply_chunk_kernel(const T* __restrict__ z, const float* __restrict__ scale,
                                                             const float* __restrict__ shift, BnRows zrows,
                                                             const T* __restrict__ res,
                                                             const float* __restrict__ rscale,
                                                             const float* __restrict__ rshift, BnRows rrows,
                                                             T* __restrict__ y, size_t nvec, int C, int relu) {
  constexpr int V = Store<T>::VEC;
  typedef typename Store<T>::vec_t vec_t;
  const size_t base = (size_t)blockIdx.x * (256 * U) + threadIdx.x;
  const int c0 = (int)((threadIdx.x * V) % C);
  vec_t zq[U], rq[U];
#pragma unroll
  for (int j = 0; j < U; ++j) {
    const size_t i = base + (size_t)j * 256;
    if (i < nvec) {
      zq[j] = *reinterpret_cast<const vec_t*>(z + i * V);
      if (res) rq[j] = *reinterpret_cast<const vec_t*>(res + i * V);
    }
  }
  __shared__ float s_sc[STATS_CMAX], s_sh[STATS_CMAX], s_rs[STATS_CMAX], s_rh[STATS_CMAX];
  if (zrows.partial) { bn_fwd_from_rows_rt(zrows, C, s_sc, s_sh, blockIdx.x == 0); scale = s_sc; shift = s_sh; }
  if (rrows.partial) { bn_fwd_from_rows_rt(rrows, C, s_rs, s_rh, blockIdx.x == 0); rscale = s_rs; rshift = s_rh; }
  float sc[V], sh[V], rs[V], rh[V];
#pragma unroll
  for (int j = 0; j < V; ++j) {
    sc[j] = scale[c0 + j]; sh[j] = shift[c0 + j];
    rs[j] = rscale ? rscale[c0 + j] : 1.f;
    rh[j] = rshift ? rshift[c0 + j] : 0.f;
  }
#pragma unroll
  for (int j = 0; j < U; ++j) {
    const size_t i = base + (size_t)j * 256;
    if (i >= nvec) continue;
    float v[V];
    Store<T>::unpack_vec(zq[j], v);
#pragma unroll
    for (int e = 0; e < V; ++e) v[e] = v[e] * sc[e] + sh[e];
    if (res) {
      float r[V];
      Store<T>::unpack_vec(rq[j], r);
#pragma unroll
      for (int e = 0; e < V; ++e) v[e] += r[e] * rs[e] + rh[e];
    }
    if (relu) {
#pragma unroll
      for (int e = 0; e < V; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
    }
    Store<T>::store_vec(y + i * V, v);
  }
}

// Two minibatches of one layer per launch: blockIdx.y selects the set of pointers.
template <typename T, int U>
__global__ __launch_bounds__(256) void bn_apply_pair_kernel(BnApplySet s0, BnApplySet s1, size_t nvec, int C, int relu) {
  constexpr int V = Store<T>::VEC;
  typedef typename Store<T>::vec_t vec_t;
  const BnApplySet& q = blockIdx.y ? s1 : s0;
  const T* z = reinterpret_cast<const T*>(q.z);
  const T* res = reinterpret_cast<const T*>(q.res);
  T* y = reinterpret_cast<T*>(q.y);
  const float *scale = q.scale, *shift = q.shift, *rscale = q.rscale, *rshift = q.rshift;
  const size_t base = (size_t)blockIdx.x * (256 * U) + threadIdx.x;
  const int c0 = (int)((threadIdx.x * V) % C);
  vec_t zq[U], rq[U];
#pragma unroll
  for (int j = 0; j < U; ++j) {
    const size_t i = base + (size_t)j * 256;
    if (i < nvec) {
      zq[j] = *reinterpret_cast<const vec_t*>(z + i * V);
      if (res) rq[j] = *reinterpret_cast<const vec_t*>(res + i * V);
    }
  }
  __shared__ float s_sc[STATS_CMAX], s_sh[STATS_CMAX], s_rs[STATS_CMAX], s_rh[STATS_CMAX];
  if (q.zrows.partial) { bn_fwd_from_rows_rt(q.zrows, C, s_sc, s_sh, blockIdx.x == 0); scale = s_sc; shift = s_sh; }
  if (q.rrows.partial) { bn_fwd_from_rows_rt(q.rrows, C, s_rs, s_rh, blockIdx.x == 0); rscale = s_rs; rshift = s_rh; }
  float sc[V], sh[V], rs[V], rh[V];
#pragma unroll
  for (int j = 0; j < V; ++j) {
    sc[j] = scale[c0 + j]; sh[j] = shift[c0 + j];
    rs[j] = rscale ? rscale[c0 + j] : 1.f;
    rh[j] = rshift ? rshift[c0 + j] : 0.f;
  }
#pragma unroll
  for (int j = 0; j < U; ++j) {
    const size_t i = base + (size_t)j * 256;
    if (i >= nvec) continue;
    float v[V];
    Store<T>::unpack_vec(zq[j], v);
#pragma unroll
    for (int e = 0; e < V; ++e) v[e] = v[e] * sc[e] + sh[e];
    if (res) {
      float r[V];
      Store<T>::unpack_vec(rq[j], r);
#pragma unroll
      for (int e = 0; e < V; ++e) v[e] += r[e] * rs[e] + rh[e];
    }
    if (relu) {
#pragma unroll
      for (int e = 0; e < V; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
    }
    Store<T>::store_vec(y + i * V, v);
  }
}

template <typename T>
static void bn_apply_pair_dispatch(const BnApplySet& a, const BnApplySet& b, size_t nvec, int C, int relu, hipStream_t s) {
  if (nvec >= (size_t)512 * 1024)
    DDG_LAUNCH((bn_apply_pair_kernel<T, 4>), dim3((unsigned)((nvec + 1023) / 1024), 2), dim3(256), 0, s, a, b, nvec, C, relu);
  else if (nvec >= (size_t)512 * 512)
    DDG_LAUNCH((bn_apply_pair_kernel<T, 2>), dim3((unsigned)((nvec + 511) / 512), 2), dim3(256), 0, s, a, b, nvec, C, relu);
  else
    DDG_LAUNCH((bn_apply_pair_kernel<T, 1>), dim3((unsigned)((nvec + 255) / 256), 2), dim3(256), 0, s, a, b, nvec, C, relu);
}

bool bn_apply_pair_launch(const BnApplySet& a, const BnApplySet& b, size_t elems, int C, int relu, int dtype,
                          hipStream_t s, hipError_t* err) {
  const int V = dtype == BF16 ? 8 : 4;
  if ((256 * V) % C != 0) return false;
  // the same kind of work in both sets (the kernel decides per set, the shapes must agree)
  if (dtype == BF16) bn_apply_pair_dispatch<bf16_t>(a, b, elems / 8, C, relu, s);
  else bn_apply_pair_dispatch<float>(a, b, elems / 4, C, relu, s);
  *err = hipGetLastError();
  return true;
}

template <typename T>
static void bn_apply_dispatch(const T* z, const float* scale, const float* shift, const BnRows& zr, const T* res,
                              const float* rscale, const float* rshift, const BnRows& rr, T* y, size_t nvec, int C,
                              int relu, bool rows, hipStream_t s) {
  constexpr int V = Store<T>::VEC;
  if ((256 * V) % C != 0) {
    // a thread's channels change from vector to vector: grid-stride kernel
    const int maxb = rows ? 512 : 2048;
    DDG_LAUNCH(bn_apply_kernel<T>, dim3(elem_grid(nvec, C, V, maxb)), dim3(256), 0, s, z, scale, shift, zr, res, rscale,
               rshift, rr, y, nvec, C, relu);
    return;
  }
  // 4 vectors per thread once that still leaves two workgroups per compute unit
  if (nvec >= (size_t)512 * 1024) {
    DDG_LAUNCH((bn_apply_chunk_kernel<T, 4>), dim3((unsigned)((nvec + 1023) / 1024)), dim3(256), 0, s, z, scale, shift, zr,
               res, rscale, rshift, rr, y, nvec, C, relu);
  } else if (nvec >= (size_t)512 * 512) {
    DDG_LAUNCH((bn_apply_chunk_kernel<T, 2>), dim3((unsigned)((nvec + 511) / 512)), dim3(256), 0, s, z, scale, shift, zr,
               res, rscale, rshift, rr, y, nvec, C, relu);
  } else {
    DDG_LAUNCH((bn_apply_chunk_kernel<T, 1>), dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s, z, scale, shift, zr,
               res, rscale, rshift, rr, y, nvec, C, relu);
  }
}

hipError_t bn_apply_launch(const void* z, const float* scale, const float* shift, const BnRows* zrows,
                           const void* res, const float* rscale, const float* rshift, const BnRows* rrows,
                           void* y, size_t elems, int C, int relu, int dtype, hipStream_t s) {
  const BnRows zr = zrows ? *zrows : BnRows{}, rr = rrows ? *rrows : BnRows{};
  const bool rows = zrows || rrows;
  if (dtype == BF16)
    bn_apply_dispatch<bf16_t>((const bf16_t*)z, scale, shift, zr, (const bf16_t*)res, rscale, rshift, rr, (bf16_t*)y,
                              elems / 8, C, relu, rows, s);
  else
    bn_apply_dispatch<float>((const float*)z, scale, shift, zr, (const float*)res, rscale, rshift, rr, (float*)y,
                             elems / 4, C, relu, rows, s);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// BN backward, pass 1: g = dy masked by (mask > 0); partial sums of g and g*xhat.
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void bn_bwd_reduce_kernel(const T* __restrict__ dy, const T* __restrict__ mask,
                                                            const float* __restrict__ mscale,
                                                            const float* __restrict__ mshift,
                                                            const T* __restrict__ z, const float* __restrict__ mean,
                                                            const float* __restrict__ invstd,
                                                            float* __restrict__ partial, size_t nvec, int C) {
  constexpr int V = Store<T>::VEC;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int c0 = (int)((i * V) % C);
  float mu[V], is[V], s1[V], s2[V], ms[V], mh[V];
#pragma unroll
  for (int j = 0; j < V; ++j) {
    mu[j] = mean[c0 + j]; is[j] = invstd[c0 + j]; s1[j] = 0.f; s2[j] = 0.f;
    ms[j] = mscale ? mscale[c0 + j] : 1.f; mh[j] = mscale ? mshift[c0 + j] : 0.f;
  }
  // four vectors per trip, all requested before any is used (the sums keep their order)
  typedef typename Store<T>::vec_t vec_t;
  constexpr int U = 4;
  const bool own_mask = mask && mask != z;
  for (; i < nvec; i += U * stride) {
    vec_t gq[U], zq[U], mq[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t iu = i + u * stride;
      if (iu < nvec) {
        gq[u] = *reinterpret_cast<const vec_t*>(dy + iu * V);
        zq[u] = *reinterpret_cast<const vec_t*>(z + iu * V);
        if (own_mask) mq[u] = *reinterpret_cast<const vec_t*>(mask + iu * V);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (i + u * stride >= nvec) continue;
      float g[V], zz[V];
      Store<T>::unpack_vec(gq[u], g);
      Store<T>::unpack_vec(zq[u], zz);
      if (mask) {
        float mk[V];
        Store<T>::unpack_vec(own_mask ? mq[u] : zq[u], mk);
#pragma unroll
        for (int j = 0; j < V; ++j) g[j] = (mk[j] * ms[j] + mh[j]) > 0.f ? g[j] : 0.f;
      }
#pragma unroll
      for (int j = 0; j < V; ++j) {
        s1[j] += g[j];
        s2[j] += g[j] * ((zz[j] - mu[j]) * is[j]);
      }
    }
  }
  // threads with equal (threadIdx.x*V) % C hold the same channels; combine in thread order
  __shared__ float red[2][256][V + 1];
#pragma unroll
  for (int j = 0; j < V; ++j) { red[0][threadIdx.x][j] = s1[j]; red[1][threadIdx.x][j] = s2[j]; }
  __syncthreads();
  const int per = C / V < 256 ? C / V : 256;  // distinct channel vectors among the block's threads
  if ((int)threadIdx.x < per) {
    float t1[V], t2[V];
#pragma unroll
    for (int j = 0; j < V; ++j) { t1[j] = 0.f; t2[j] = 0.f; }
    for (int t = threadIdx.x; t < 256; t += per) {
#pragma unroll
      for (int j = 0; j < V; ++j) { t1[j] += red[0][t][j]; t2[j] += red[1][t][j]; }
    }
    // block b, thread t covers channels ((b*256+t)*V) % C
    const int cb = (int)((((size_t)blockIdx.x * 256 + threadIdx.x) * V) % C);
#pragma unroll
    for (int j = 0; j < V; ++j) {
      partial[((size_t)blockIdx.x * 2 + 0) * C + cb + j] = t1[j];
      partial[((size_t)blockIdx.x * 2 + 1) * C + cb + j] = t2[j];
    }
  }
}

// When C > 256*V a block covers only part of the channels; the other entries of its
// partial row must read as zero, so the row buffer is cleared by the finalise contract:
// rows are written completely only if 256*V % C == 0 or C % (256*V) == 0 handled below.
int bn_bwd_grid(size_t elems, int C, int dtype) {
  const int V = dtype == BF16 ? 8 : 4;
  return elem_grid(elems / V, C, V, 256);
}

template <typename T>
__global__ void zero_f32_kernel(float* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0.f;
}

hipError_t bn_bwd_reduce_launch(const void* dy, const void* mask, const float* mscale, const float* mshift,
                                const void* z, const float* mean, const float* invstd, float* partial,
                                size_t elems, int C, int dtype, hipStream_t s) {
  const int V = dtype == BF16 ? 8 : 4;
  const int grid = bn_bwd_grid(elems, C, dtype);
  if (C > 256 * V) {  // a block's row is only partly written: clear the rows first
    const size_t n = (size_t)grid * 2 * C;
    DDG_LAUNCH(zero_f32_kernel<float>, dim3(256), dim3(256), 0, s, partial, n);
  }
  if (dtype == BF16)
    DDG_LAUNCH(bn_bwd_reduce_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, (const bf16_t*)dy,
                       (const bf16_t*)mask, mscale, mshift, (const bf16_t*)z, mean, invstd, partial, elems / 8, C);
  else
    DDG_LAUNCH(bn_bwd_reduce_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)dy,
                       (const float*)mask, mscale, mshift, (const float*)z, mean, invstd, partial, elems / 4, C);
  return hipGetLastError();
}

// dbeta = sum g, dgamma = sum g*xhat; dz = A*g + B*z + C0 with
//   A = gamma*invstd, B = -gamma*invstd^2*dgamma/m, C0 = -gamma*invstd*dbeta/m - B*mean
__global__ __launch_bounds__(1024) void bn_bwd_finalize_kernel(const float* __restrict__ partial, int rows, int C,
                                                              const float* __restrict__ gamma,
                                                              const float* __restrict__ mean,
                                                              const float* __restrict__ invstd, float count,
                                                              float* dgamma, float* dbeta, float* coef) {
  __shared__ double r1[64][17], r2[64][17];
  const int cl = threadIdx.x & 15, slice = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cl;
  double s1 = 0.0, s2 = 0.0;
  if (c < C)
    for (int r = slice; r < rows; r += 64) {
      s1 += (double)partial[((size_t)r * 2 + 0) * C + c];
      s2 += (double)partial[((size_t)r * 2 + 1) * C + c];
    }
  r1[slice][cl] = s1; r2[slice][cl] = s2;
  __syncthreads();
  double p1 = 0.0, p2 = 0.0;   // two short steps, as in bn_finalize_kernel
  if (slice < 8) {
#pragma unroll
    for (int i = 0; i < 8; ++i) { p1 += r1[slice * 8 + i][cl]; p2 += r2[slice * 8 + i][cl]; }
  }
  __syncthreads();
  if (slice < 8) { r1[slice][cl] = p1; r2[slice][cl] = p2; }
  __syncthreads();
  if (slice == 0 && c < C) {
    double db = 0.0, dg = 0.0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { db += r1[i][cl]; dg += r2[i][cl]; }
    dbeta[c] = (float)db;
    dgamma[c] = (float)dg;
    const double g = gamma[c], is = invstd[c], mu = mean[c], m = count;
    const double A = g * is;
    const double B = -g * is * is * dg / m;
    const double C0 = -g * is * db / m - B * mu;
    coef[c] = (float)A;
    coef[C + c] = (float)B;
    coef[2 * C + c] = (float)C0;
  }
}

hipError_t bn_bwd_finalize_launch(const float* partial, int rows, int C, const float* gamma,
                                  const float* mean, const float* invstd, float count, float* dgamma,
                                  float* dbeta, float* coef, hipStream_t s) {
  DDG_LAUNCH(bn_bwd_finalize_kernel, dim3((C + 15) / 16), dim3(1024), 0, s, partial, rows, C, gamma,
                     mean, invstd, count, dgamma, dbeta, coef);
  return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(const T* __restrict__ dy, const T* __restrict__ mask,
                                                           const float* __restrict__ mscale,
                                                           const float* __restrict__ mshift,
                                                           const T* __restrict__ z, const float* __restrict__ coef,
                                                           BnBwdRows rows, T* __restrict__ dz, size_t nvec, int C) {
  constexpr int V = Store<T>::VEC;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int c0 = (int)((i * V) % C);
  __shared__ float s_coef[3 * STATS_CMAX];
  if (rows.partial) { bn_bwd_from_rows_rt(rows, C, s_coef, blockIdx.x == 0); coef = s_coef; }
  float A[V], B[V], C0[V], ms[V], mh[V];
#pragma unroll
  for (int j = 0; j < V; ++j) {
    A[j] = coef[c0 + j]; B[j] = coef[C + c0 + j]; C0[j] = coef[2 * C + c0 + j];
    ms[j] = mscale ? mscale[c0 + j] : 1.f; mh[j] = mscale ? mshift[c0 + j] : 0.f;
  }
  for (; i < nvec; i += stride) {
    float g[V], zz[V];
    Store<T>::load_vec(dy + i * V, g);
    Store<T>::load_vec(z + i * V, zz);
    if (mask) {
      float mk[V];
      Store<T>::load_vec(mask + i * V, mk);
#pragma unroll
      for (int j = 0; j < V; ++j) g[j] = (mk[j] * ms[j] + mh[j]) > 0.f ? g[j] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < V; ++j) g[j] = A[j] * g[j] + (B[j] * zz[j] + C0[j]);
    Store<T>::store_vec(dz + i * V, g);
  }
}

// The same operation without a loop, for final coefficients and 256*V % C == 0 (a thread's
// channels are the same for all its vectors): a workgroup owns 256*U consecutive vectors, a
// thread requests all its tensor data first and its per-channel constants (16-byte loads) while
// that is in flight.
template <typename T, int U>
__global__ __launch_bounds__(256) void bn_bwd_apply_chunk_kernel(const T* __restrict__ dy, const T* __restrict__ mask,
                                                                 const float* __restrict__ mscale,
                                                                 const float* __restrict__ mshift,
                                                                 const T* __restrict__ z, const float* __restrict__ coef,
                                                                 T* __restrict__ dz, size_t nvec, int C) {
  constexpr int V = Store<T>::VEC;
  typedef typename Store<T>::vec_t vec_t;
  const size_t base = (size_t)blockIdx.x * (256 * U) + threadIdx.x;
  const int c0 = (int)((threadIdx.x * V) % C);
  vec_t gq[U], zq[U], mq[U];
#pragma unroll
  for (int j = 0; j < U; ++j) {
    const size_t i = base + (size_t)j * 256;
    if (i < nvec) {
      gq[j] = *reinterpret_cast<const vec_t*>(dy + i * V);
      zq[j] = *reinterpret_cast<const vec_t*>(z + i * V);
      if (mask && mask != z) mq[j] = *reinterpret_cast<const vec_t*>(mask + i * V);
    }
  }
  float A[V], B[V], C0[V], ms[V], mh[V];
#pragma unroll
  for (int j = 0; j < V; j += 4) {
    *reinterpret_cast<float4*>(&A[j]) = *reinterpret_cast<const float4*>(coef + c0 + j);
    *reinterpret_cast<float4*>(&B[j]) = *reinterpret_cast<const float4*>(coef + C + c0 + j);
    *reinterpret_cast<float4*>(&C0[j]) = *reinterpret_cast<const float4*>(coef + 2 * C + c0 + j);
    if (mscale) {
      *reinterpret_cast<float4*>(&ms[j]) = *reinterpret_cast<const float4*>(mscale + c0 + j);
      *reinterpret_cast<float4*>(&mh[j]) = *reinterpret_cast<const float4*>(mshift + c0 + j);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) { ms[j + e] = 1.f; mh[j + e] = 0.f; }
    }
  }
#pragma unroll
  for (int j = 0; j < U; ++j) {
    const size_t i = base + (size_t)j * 256;
    if (i >= nvec) continue;
    float g[V], zz[V];
    Store<T>::unpack_vec(gq[j], g);
    Store<T>::unpack_vec(zq[j], zz);
    if (mask) {
      float mk[V];
      Store<T>::unpack_vec(mask != z ? mq[j] : zq[j], mk);
#pragma unroll
      for (int e = 0; e < V; ++e) g[e] = (mk[e] * ms[e] + mh[e]) > 0.f ? g[e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < V; ++e) g[e] = A[e] * g[e] + (B[e] * zz[e] + C0[e]);
    Store<T>::store_vec(dz + i * V, g);
  }
}

template <typename T>
static bool bn_bwd_apply_chunked(const T* dy, const T* mask, const float* mscale, const float* mshift, const T* z,
                                 const float* coef, T* dz, size_t nvec, int C, hipStream_t s) {
  constexpr int V = Store<T>::VEC;
  // final coefficients, a thread's channels fixed, 16-byte aligned per-channel vectors
  if (!coef || (256 * V) % C != 0 || C % 4 != 0) return false;
  if (((uintptr_t)coef | (uintptr_t)mscale | (uintptr_t)mshift) & 15u) return false;
  if (nvec >= (size_t)512 * 1024)
    DDG_LAUNCH((bn_bwd_apply_chunk_kernel<T, 2>), dim3((unsigned)((nvec + 511) / 512)), dim3(256), 0, s, dy, mask, mscale,
               mshift, z, coef, dz, nvec, C);
  else
    DDG_LAUNCH((bn_bwd_apply_chunk_kernel<T, 1>), dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, s, dy, mask, mscale,
               mshift, z, coef, dz, nvec, C);
  return true;
}

hipError_t bn_bwd_apply_launch(const void* dy, const void* mask, const float* mscale, const float* mshift,
                               const void* z, const float* coef, const BnBwdRows* rows, void* dz, size_t elems,
                               int C, int dtype, hipStream_t s) {
  const BnBwdRows br = rows ? *rows : BnBwdRows{};
  const int maxb = rows ? 512 : 2048;
  if (!rows) {
    const bool done = dtype == BF16
        ? bn_bwd_apply_chunked<bf16_t>((const bf16_t*)dy, (const bf16_t*)mask, mscale, mshift, (const bf16_t*)z, coef,
                                       (bf16_t*)dz, elems / 8, C, s)
        : bn_bwd_apply_chunked<float>((const float*)dy, (const float*)mask, mscale, mshift, (const float*)z, coef,
                                      (float*)dz, elems / 4, C, s);
    if (done) return hipGetLastError();
  }
  if (dtype == BF16) {
    const size_t nvec = elems / 8;
    DDG_LAUNCH(bn_bwd_apply_kernel<bf16_t>, dim3(elem_grid(nvec, C, 8, maxb)), dim3(256), 0, s,
                       (const bf16_t*)dy, (const bf16_t*)mask, mscale, mshift, (const bf16_t*)z, coef, br, (bf16_t*)dz, nvec, C);
  } else {
    const size_t nvec = elems / 4;
    DDG_LAUNCH(bn_bwd_apply_kernel<float>, dim3(elem_grid(nvec, C, 4, maxb)), dim3(256), 0, s,
                       (const float*)dy, (const float*)mask, mscale, mshift, (const float*)z, coef, br, (float*)dz, nvec, C);
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Running batch-norm estimates (for evaluation) of all layers of a module in one launch:
//   rmean <- (1-rho)*rmean + rho*mean,  rvar <- (1-rho)*rvar + rho*var*m/(m-1)
// with the batch statistics of the forward pass that just ran (var = 1/invstd^2 - eps), and
// the per-channel vectors the evaluation forward normalises with:
//   escale = gamma/sqrt(rvar + eps),  eshift = beta - rmean*escale.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void running_update_kernel(const RunDesc* __restrict__ descs, float rho) {
  const RunDesc d = descs[blockIdx.y];
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d.C) return;
  const float is = d.invstd[c];
  const float var = 1.f / (is * is) - d.eps;
  d.rmean[c] = (1.f - rho) * d.rmean[c] + rho * d.mean[c];
  d.rvar[c] = (1.f - rho) * d.rvar[c] + rho * (var * d.count / (d.count - 1.f));
}

__global__ __launch_bounds__(256) void eval_vectors_kernel(const RunDesc* __restrict__ descs) {
  const RunDesc d = descs[blockIdx.y];
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d.C) return;
  const float sc = d.gamma[c] / sqrtf(d.rvar[c] + d.eps);
  d.escale[c] = sc;
  d.eshift[c] = d.beta[c] - d.rmean[c] * sc;
}

hipError_t running_update_launch(const RunDesc* dev_descs, int n, int max_c, float rho, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  DDG_LAUNCH(running_update_kernel, dim3((max_c + 255) / 256, n), dim3(256), 0, s, dev_descs, rho);
  return hipGetLastError();
}

hipError_t eval_vectors_launch(const RunDesc* dev_descs, int n, int max_c, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  DDG_LAUNCH(eval_vectors_kernel, dim3((max_c + 255) / 256, n), dim3(256), 0, s, dev_descs);
  return hipGetLastError();
}

// mean of the per-sample losses, added in order (evaluation; training gets it from head_wgrad_kernel)
__global__ void loss_mean_kernel(const float* __restrict__ loss_n, int N, float* __restrict__ out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    float l = 0.f;
    for (int n = 0; n < N; ++n) l += loss_n[n];
    *out = l / (float)N;
  }
}

// ---------------------------------------------------------------------------------
// Head. Small: N x C x classes is a few hundred thousand operations.
// ---------------------------------------------------------------------------------
// Per sample (one workgroup of 256 threads): global average pool, logits, stable softmax, loss,
// dlogits = (p - onehot)/N, and dh = dlogits * fcw / HW broadcast over the pixels. Every sum
// runs in a fixed order. Dynamic LDS: 2*C + 2*classes + 256 floats.
template <typename T>
__global__ __launch_bounds__(256) void head_sample_kernel(const T* __restrict__ h, const float* __restrict__ fcw,
                                                          const float* __restrict__ fcb,
                                                          const int32_t* __restrict__ labels,
                                                          float* __restrict__ pooled, float* __restrict__ dlogits,
                                                          float* __restrict__ loss_n, T* __restrict__ dh, int N,
                                                          int HW, int C, int classes, float* __restrict__ logits_out) {
  extern __shared__ float sm[];
  float* s_pool = sm;               // [C]
  float* s_dh = sm + C;             // [C]
  float* s_lg = sm + 2 * C;         // [classes]
  float* s_dl = s_lg + classes;     // [classes]
  float* s_red = s_dl + classes;    // [256]
  const int n = blockIdx.x, tid = threadIdx.x;
  // pool: thread (channel lane cl, pixel class g); pixel classes are added in order afterwards
  const int cpt = C < 256 ? C : 256, groups = 256 / cpt;
  const int cl = tid % cpt, g = tid / cpt;
  for (int c0 = 0; c0 < C; c0 += cpt) {
    const int c = c0 + cl;
    float a = 0.f;
    if (g < groups && c < C) {
      const T* p = h + (size_t)n * HW * C + c;
#pragma unroll 8
      for (int i = g; i < HW; i += groups) a += Store<T>::load1(p + (size_t)i * C);
    }
    s_red[tid] = a;
    __syncthreads();
    if (g == 0 && c < C) {
      float t = 0.f;
      for (int q = 0; q < groups; ++q) t += s_red[q * cpt + cl];
      t /= (float)HW;
      s_pool[c] = t;
      pooled[(size_t)n * C + c] = t;
    }
    __syncthreads();
  }
  // logits
  for (int j = tid; j < classes; j += 256) {
    float a = fcb[j];
    const float* w = fcw + (size_t)j * C;
#pragma unroll 8
    for (int c = 0; c < C; ++c) a += w[c] * s_pool[c];
    s_lg[j] = a;
    if (logits_out) logits_out[(size_t)n * classes + j] = a;
  }
  __syncthreads();
  float mx = s_lg[0];
  for (int j = 1; j < classes; ++j) mx = s_lg[j] > mx ? s_lg[j] : mx;
  for (int j = tid; j < classes; j += 256) s_dl[j] = expf(s_lg[j] - mx);
  __syncthreads();
  float den = 0.f;
  for (int j = 0; j < classes; ++j) den += s_dl[j];
  // a label outside [0, classes) has no class to point at: that sample's loss (and with it the
  // mean loss) is NaN, so the caller sees it, and nothing outside the logits is read
  const int y = labels[n];
  const bool y_ok = (unsigned)y < (unsigned)classes;
  __syncthreads();
  for (int j = tid; j < classes; j += 256) {
    const float d = (s_dl[j] / den - (j == y ? 1.f : 0.f)) / (float)N;
    s_dl[j] = d;
    dlogits[(size_t)n * classes + j] = d;
  }
  if (tid == 0) loss_n[n] = y_ok ? -(s_lg[y] - mx - logf(den)) : __builtin_nanf("");
  if (!dh) return;
  __syncthreads();
  for (int c = tid; c < C; c += 256) {
    float a = 0.f;
#pragma unroll 4
    for (int j = 0; j < classes; ++j) a += s_dl[j] * fcw[(size_t)j * C + c];
    s_dh[c] = Store<T>::round(a / (float)HW);
  }
  __syncthreads();
  // broadcast over the pixels, 4 channels per store
  const int c4n = C / 4;
  for (int e = tid; e < HW * c4n; e += 256) {
    const int i = e / c4n, c = (e - i * c4n) * 4;
    Store<T>::store4(dh + ((size_t)n * HW + i) * C + c, s_dh[c], s_dh[c + 1], s_dh[c + 2], s_dh[c + 3]);
  }
}

// One workgroup per class j: dfcw[j][:] = sum_n dlogits[n][j] * pooled[n][:], dfcb[j]; thread
// (channel lane, sample class g) adds samples g, g+groups, ... in order, then the classes are
// added in order. Workgroup 0 also writes the mean loss.
__global__ __launch_bounds__(256) void head_wgrad_kernel(const float* __restrict__ pooled,
                                                         const float* __restrict__ dlogits,
                                                         const float* __restrict__ loss_n, float* __restrict__ dfcw,
                                                         float* __restrict__ dfcb, float* loss_out, int N, int C,
                                                         int classes) {
  __shared__ float s_red[256];
  const int j = blockIdx.x, tid = threadIdx.x;
  const int cpt = C < 256 ? C : 256, groups = 256 / cpt;
  const int cl = tid % cpt, g = tid / cpt;
  for (int c0 = 0; c0 < C; c0 += cpt) {
    const int c = c0 + cl;
    float a = 0.f;
    if (g < groups && c < C) {
#pragma unroll 8
      for (int n = g; n < N; n += groups) a += dlogits[(size_t)n * classes + j] * pooled[(size_t)n * C + c];
    }
    s_red[tid] = a;
    __syncthreads();
    if (g == 0 && c < C) {
      float t = 0.f;
      for (int q = 0; q < groups; ++q) t += s_red[q * cpt + cl];
      dfcw[(size_t)j * C + c] = t;
    }
    __syncthreads();
  }
  // bias gradient (and the mean loss): 256 partial sums over samples, added in order
  float a = 0.f, l = 0.f;
  for (int n = tid; n < N; n += 256) {
    a += dlogits[(size_t)n * classes + j];
    if (j == 0) l += loss_n[n];
  }
  s_red[tid] = a;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
    for (int q = 0; q < 256; ++q) t += s_red[q];
    dfcb[j] = t;
  }
  if (j == 0 && loss_out) {
    __syncthreads();
    s_red[tid] = l;
    __syncthreads();
    if (tid == 0) {
      float t = 0.f;
      for (int q = 0; q < 256; ++q) t += s_red[q];
      *loss_out = t / (float)N;
    }
  }
}

hipError_t head_launch(const HeadArgs& a, hipStream_t s) {
  if (a.C % 4 != 0) return hipErrorInvalidValue;
  const size_t lds = (size_t)(2 * a.C + 2 * a.classes + 256) * sizeof(float);
  if (a.dtype == BF16)
    DDG_LAUNCH(head_sample_kernel<bf16_t>, dim3(a.N), dim3(256), lds, s, (const bf16_t*)a.h, a.fcw, a.fcb, a.labels,
               a.pooled, a.dlogits, a.loss_n, (bf16_t*)a.dh, a.N, a.HW, a.C, a.classes, a.logits_out);
  else
    DDG_LAUNCH(head_sample_kernel<float>, dim3(a.N), dim3(256), lds, s, (const float*)a.h, a.fcw, a.fcb, a.labels,
               a.pooled, a.dlogits, a.loss_n, (float*)a.dh, a.N, a.HW, a.C, a.classes, a.logits_out);
  if (!a.dfcw) {   // evaluation: no gradients; the mean loss if asked for
    if (a.loss_out) DDG_LAUNCH(loss_mean_kernel, dim3(1), dim3(64), 0, s, a.loss_n, a.N, a.loss_out);
    return hipGetLastError();
  }
  DDG_LAUNCH(head_wgrad_kernel, dim3(a.classes), dim3(256), 0, s, a.pooled, a.dlogits, a.loss_n, a.dfcw, a.dfcb,
             a.loss_out, a.N, a.C, a.classes);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Momentum SGD over the module's flat parameter vector.
// ---------------------------------------------------------------------------------
__global__ void sgd_kernel(float* __restrict__ w, float* __restrict__ v, const float* __restrict__ g, size_t n,
                           float lr, const float* __restrict__ lr_dev, float mu, float wd) {
  if (lr_dev) lr = *lr_dev;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const float wi = w[i];
    const float vi = mu * v[i] + (g[i] + wd * wi);
    v[i] = vi;
    w[i] = wi - lr * vi;
  }
}

__global__ void adam_advance_kernel(double* pw, double b1, double b2) { pw[0] *= b1; pw[1] *= b2; }

hipError_t adam_advance_launch(double* pw, float b1, float b2, hipStream_t s) {
  DDG_LAUNCH(adam_advance_kernel, dim3(1), dim3(1), 0, s, pw, (double)b1, (double)b2);
  return hipGetLastError();
}

__global__ void adam_kernel(float* __restrict__ w, float* __restrict__ m1, float* __restrict__ m2,
                            const float* __restrict__ g, size_t n, float lr, const float* __restrict__ lr_dev,
                            float b1, float b2, float eps, float wd, const double* __restrict__ pw) {
  if (lr_dev) lr = *lr_dev;
  const float c1 = (float)(1.0 - pw[0]), c2 = (float)(1.0 - pw[1]);
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const float wi = w[i];
    const float gi = g[i] + wd * wi;
    const float mi = b1 * m1[i] + (1.f - b1) * gi;
    const float vi = b2 * m2[i] + (1.f - b2) * gi * gi;
    m1[i] = mi; m2[i] = vi;
    w[i] = wi - lr * (mi / c1) / (sqrtf(vi / c2) + eps);
  }
}

hipError_t adam_launch(float* w, float* m1, float* m2, const float* g, size_t n, float lr, const float* lr_dev,
                       float b1, float b2, float eps, float wd, const double* pw, hipStream_t s) {
  int grid = (int)((n + 255) / 256);
  if (grid > 2048) grid = 2048;
  if (grid < 1) grid = 1;
  DDG_LAUNCH(adam_kernel, dim3(grid), dim3(256), 0, s, w, m1, m2, g, n, lr, lr_dev, b1, b2, eps, wd, pw);
  return hipGetLastError();
}

__global__ void set_scalar_kernel(float* dst, float v) { *dst = v; }

hipError_t set_scalar_launch(float* dst, float v, hipStream_t s) {
  DDG_LAUNCH(set_scalar_kernel, dim3(1), dim3(1), 0, s, dst, v);
  return hipGetLastError();
}

hipError_t sgd_launch(float* w, float* v, const float* g, size_t n, float lr, const float* lr_dev, float mu,
                      float wd, hipStream_t s) {
  int grid = (int)((n + 255) / 256);
  if (grid > 2048) grid = 2048;
  if (grid < 1) grid = 1;
  DDG_LAUNCH(sgd_kernel, dim3(grid), dim3(256), 0, s, w, v, g, n, lr, lr_dev, mu, wd);
  return hipGetLastError();
}

__global__ void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t nvec,
                            const unsigned char* __restrict__ srcb, unsigned char* __restrict__ dstb, size_t tail0,
                            size_t bytes) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
  if (blockIdx.x == 0)
    for (size_t b = tail0 + threadIdx.x; b < bytes; b += blockDim.x) dstb[b] = srcb[b];
}

hipError_t copy_launch(const void* src, void* dst, size_t bytes, hipStream_t s) {
  const size_t nvec = bytes / 16;
  int grid = (int)((nvec + 255) / 256);
  if (grid > 2048) grid = 2048;
  if (grid < 1) grid = 1;
  DDG_LAUNCH(copy_kernel, dim3(grid), dim3(256), 0, s, (const uint4*)src, (uint4*)dst, nvec,
                     (const unsigned char*)src, (unsigned char*)dst, nvec * 16, bytes);
  return hipGetLastError();
}

template <typename T>
__global__ void to_f32_kernel(const T* __restrict__ src, float* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = Store<T>::load1(src + i);
}

hipError_t to_f32_launch(const void* src, float* dst, size_t elems, int dtype, hipStream_t s) {
  int grid = (int)((elems + 255) / 256);
  if (grid > 2048) grid = 2048;
  if (grid < 1) grid = 1;
  if (dtype == BF16) DDG_LAUNCH(to_f32_kernel<bf16_t>, dim3(grid), dim3(256), 0, s, (const bf16_t*)src, dst, elems);
  else DDG_LAUNCH(to_f32_kernel<float>, dim3(grid), dim3(256), 0, s, (const float*)src, dst, elems);
  return hipGetLastError();
}

}  // namespace ddg
