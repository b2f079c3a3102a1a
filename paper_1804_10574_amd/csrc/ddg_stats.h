// Per-channel batch-norm quantities computed from per-workgroup partial rows by the kernel
// that CONSUMES them: every workgroup adds the rows [rows][2][C] in the same fixed order
// (so all get bit-identical values), keeps the result in LDS, and workgroup 0 also writes
// it to memory for later kernels. This removes a tiny, latency-bound finalise launch from
// the dependency chain between a producer and its consumer. Used for C <= 64, where the
// rows are a few tens of KB and stay in L2; wider layers use the finalise kernels.
#pragma once
#include "ddg_device.h"
#include "ddg_kernels.h"

namespace ddg {

constexpr int STATS_CMAX = 64;

// 256 threads. f(c, t1, t2) runs once per channel (in one thread) with the two column sums.
// A row is 2*C floats; a thread owns one 16-byte column group and every nsl-th row, keeps 16
// loads in flight, and adds its rows in order; the row slices are then combined in order.
template <typename F>
__device__ __forceinline__ void reduce_stat_rows(const float* __restrict__ partial, int rows, int C, F f) {
  __shared__ float4 sh[256];
  const int tid = threadIdx.x;
  const int ncol4 = C / 2;               // float4 groups per row (2*C/4)
  const int nsl = 256 / ncol4;           // row slices
  const int c4 = tid % ncol4, slice = tid / ncol4;
  const float4* __restrict__ p4 = reinterpret_cast<const float4*>(partial);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int r0 = slice; r0 < rows; r0 += nsl * 16) {
    float4 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int rr = r0 + u * nsl;
      v[u] = rr < rows ? p4[(size_t)rr * ncol4 + c4] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
  }
  sh[tid] = acc;
  __syncthreads();
  if (tid < C) {
    const float* shf = reinterpret_cast<const float*>(sh);
    double t1 = 0.0, t2 = 0.0;
    for (int k = 0; k < nsl; ++k) {
      t1 += (double)shf[(k * ncol4) * 4 + tid];        // columns 0..C-1: first sum
      t2 += (double)shf[(k * ncol4) * 4 + C + tid];    // columns C..2C-1: second sum
    }
    f(tid, t1, t2);
  }
  __syncthreads();
}

// Forward statistics -> scale = gamma*invstd, shift = beta - mean*scale in LDS (s_scale, s_shift);
// workgroup 0 (write != 0) also stores mean, invstd, scale, shift.
__device__ __forceinline__ void bn_fwd_from_rows(const BnRows& p, int C, float* s_scale, float* s_shift, bool write) {
  reduce_stat_rows(p.partial, p.rows, C, [&](int c, double t1, double t2) {
    const double mu = t1 / (double)p.count;
    double var = t2 / (double)p.count - mu * mu;
    if (var < 0.0) var = 0.0;
    const float is = (float)(1.0 / sqrt(var + (double)p.eps));
    const float sc = p.gamma[c] * is;
    const float sh = p.beta[c] - (float)mu * sc;
    s_scale[c] = sc; s_shift[c] = sh;
    if (write) { p.mean[c] = (float)mu; p.invstd[c] = is; p.scale[c] = sc; p.shift[c] = sh; }
  });
}

// Backward sums (sum g, sum g*xhat) -> coefficients of dz = A*g + B*z + C0 in LDS (s_coef[3][C]);
// workgroup 0 also stores dgamma, dbeta.
__device__ __forceinline__ void bn_bwd_from_rows(const BnBwdRows& p, int C, float* s_coef, bool write) {
  reduce_stat_rows(p.partial, p.rows, C, [&](int c, double db, double dg) {
    const double g = p.gamma[c], is = p.invstd[c], mu = p.mean[c], m = p.count;
    const double A = g * is, B = -g * is * is * dg / m, C0 = -g * is * db / m - B * mu;
    s_coef[c] = (float)A; s_coef[C + c] = (float)B; s_coef[2 * C + c] = (float)C0;
    if (write) { p.dgamma[c] = (float)dg; p.dbeta[c] = (float)db; }
  });
}

}  // namespace ddg
