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

// 256 threads, C a compile-time constant in {16, 32, 64}. f(c, t1, t2) runs once per channel (in
// one thread) with the two column sums. A row is 2*C floats; a thread owns one 16-byte column
// group and every NSL-th row, keeps 16 loads in flight and adds its rows in order (fp32, like
// the rows themselves). The NSL row slices of a column are then combined in a fixed order in
// fp64 in two short steps (four values per thread, then 256/(2C) per column), all unrolled.
template <int C, typename F>
__device__ __forceinline__ void reduce_stat_rows(const float* __restrict__ partial, int rows, F f) {
  static_assert(C == 16 || C == 32 || C == 64, "channel count");
  constexpr int NCOL4 = C / 2;            // float4 groups per row (2*C/4)
  constexpr int NSL = 256 / NCOL4;        // row slices: 32, 16, 8
  constexpr int G = 256 / (2 * C);        // second-step groups per column: 8, 4, 2 (NSL == 4*G)
  __shared__ float4 sh[256];
  __shared__ double sh2[256];
  const int tid = threadIdx.x;
  const int c4 = tid % NCOL4, slice = tid / NCOL4;
  const float4* __restrict__ p4 = reinterpret_cast<const float4*>(partial);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int r0 = slice; r0 < rows; r0 += NSL * 16) {
    float4 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int rr = r0 + u * NSL;
      v[u] = rr < rows ? p4[(size_t)rr * NCOL4 + c4] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
  }
  sh[tid] = acc;
  __syncthreads();
  {
    // thread (column col of 2C, group g): slices g*4 .. g*4+3
    const float* shf = reinterpret_cast<const float*>(sh);
    const int col = tid % (2 * C), g = tid / (2 * C);
    double t = 0.0;
#pragma unroll
    for (int k = 0; k < 4; ++k) t += (double)shf[((g * 4 + k) * NCOL4) * 4 + col];
    sh2[g * (2 * C) + col] = t;
  }
  __syncthreads();
  if (tid < C) {
    double t1 = 0.0, t2 = 0.0;
#pragma unroll
    for (int g = 0; g < G; ++g) { t1 += sh2[g * (2 * C) + tid]; t2 += sh2[g * (2 * C) + C + tid]; }
    f(tid, t1, t2);
  }
  __syncthreads();
}

// Forward statistics -> scale = gamma*invstd, shift = beta - mean*scale in LDS (s_scale, s_shift);
// workgroup 0 (write != 0) also stores mean, invstd, scale, shift.
template <int C>
__device__ __forceinline__ void bn_fwd_from_rows(const BnRows& p, float* s_scale, float* s_shift, bool write) {
  reduce_stat_rows<C>(p.partial, p.rows, [&](int c, double t1, double t2) {
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
template <int C>
__device__ __forceinline__ void bn_bwd_from_rows(const BnBwdRows& p, float* s_coef, bool write) {
  reduce_stat_rows<C>(p.partial, p.rows, [&](int c, double db, double dg) {
    const double g = p.gamma[c], is = p.invstd[c], mu = p.mean[c], m = p.count;
    const double A = g * is, B = -g * is * is * dg / m, C0 = -g * is * db / m - B * mu;
    s_coef[c] = (float)A; s_coef[C + c] = (float)B; s_coef[2 * C + c] = (float)C0;
    if (write) { p.dgamma[c] = (float)dg; p.dbeta[c] = (float)db; }
  });
}

// Run-time channel count (16, 32 or 64; the host checks): one of the three instances.
__device__ __forceinline__ void bn_fwd_from_rows_rt(const BnRows& p, int C, float* s_scale, float* s_shift, bool write) {
  if (C == 16) bn_fwd_from_rows<16>(p, s_scale, s_shift, write);
  else if (C == 32) bn_fwd_from_rows<32>(p, s_scale, s_shift, write);
  else bn_fwd_from_rows<64>(p, s_scale, s_shift, write);
}
__device__ __forceinline__ void bn_bwd_from_rows_rt(const BnBwdRows& p, int C, float* s_coef, bool write) {
  if (C == 16) bn_bwd_from_rows<16>(p, s_coef, write);
  else if (C == 32) bn_bwd_from_rows<32>(p, s_coef, write);
  else bn_bwd_from_rows<64>(p, s_coef, write);
}

}  // namespace ddg
