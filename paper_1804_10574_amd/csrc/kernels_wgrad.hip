// Weight-gradient convolution: dW[co][tap][ci] = sum over pixels m of dz[m][co] * x[pix(m,tap)][ci].
//
// The contraction runs over pixels, which are the slow index of both NHWC operands, so
// this version feeds the fp32 matrix-core atom (one element per lane, no transposition
// needed): rows = output channels, columns = (tap, input channel), k = 4 pixels per
// instruction. bf16 tensors are widened on load; products of bf16 values are exact in fp32.
// Work is split over pixel ranges; each workgroup writes one partial tile and a second
// kernel adds the partials in a fixed order (no atomics: results are reproducible).
#include "ddg_device.h"
#include "ddg_kernels.h"
#include <cstdlib>

namespace ddg {

constexpr int WG_NJ = 9;  // column blocks (16 wide) per wave

template <typename T>
__global__ __launch_bounds__(256) void wgrad_mfma_kernel(WgradArgs a) {
  using S_ = Store<T>;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int cob = blockIdx.y;
  const int jb0 = blockIdx.z * WG_NJ;
  const T* __restrict__ x = reinterpret_cast<const T*>(a.x);
  const T* __restrict__ dz = reinterpret_cast<const T*>(a.dz);
  const int cpmask = (1 << a.log2cp) - 1;
  const int ntaps = a.R * a.R;

  // per-lane column descriptors: column j -> (tap, ci)
  int jr[WG_NJ], js[WG_NJ], jc[WG_NJ];
  bool jv[WG_NJ];
#pragma unroll
  for (int b = 0; b < WG_NJ; ++b) {
    const int j = (jb0 + b) * 16 + l16;
    const int tap = j >> a.log2cp;
    jc[b] = j & cpmask;
    jr[b] = tap / a.R - a.pad;
    js[b] = tap % a.R - a.pad;
    jv[b] = (jb0 + b) < a.JB && tap < ntaps && jc[b] < a.Cin;
  }
  f32x4_t acc[WG_NJ];
#pragma unroll
  for (int b = 0; b < WG_NJ; ++b) acc[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int pq = a.P * a.Q;
  const bool fdiv = a.M < (1 << 22);
  const float inv_pq = 1.0f / (float)pq, inv_q = 1.0f / (float)a.Q;
  long m0 = ((long)blockIdx.x * 4 + wave) * (long)a.steps * 4;
  for (int st = 0; st < a.steps; ++st) {
    const long m = m0 + (long)st * 4 + lg;
    const bool mv = m < a.M;
    const int mm = mv ? (int)m : 0;
    // (small non-negative integers divide exactly through fp32; an integer division costs as
    // much as the step's matrix instructions)
    const int n = fdiv ? (int)(((float)mm + 0.5f) * inv_pq) : mm / pq;
    const int rem = mm - n * pq;
    const int p = fdiv ? (int)(((float)rem + 0.5f) * inv_q) : rem / a.Q;
    const int q = rem - p * a.Q;
    const float dv = mv ? S_::load1(dz + (size_t)mm * a.Cout + cob * 16 + l16) : 0.f;
    const int ihb = p * a.stride, iwb = q * a.stride;
#pragma unroll
    for (int b = 0; b < WG_NJ; ++b) {
      const int ih = ihb + jr[b], iw = iwb + js[b];
      const bool ok = mv && jv[b] && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
      const float xv = ok ? S_::load1(x + ((size_t)(n * a.H + ih) * a.W + iw) * a.Cin + jc[b]) : 0.f;
      acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv, acc[b], 0, 0, 0);
    }
  }

  // sum the four waves in a fixed order, then write the partial tile
  __shared__ float red[4][WG_NJ][16][17];
#pragma unroll
  for (int b = 0; b < WG_NJ; ++b)
#pragma unroll
    for (int i = 0; i < 4; ++i) red[wave][b][lg * 4 + i][l16] = acc[b][i];
  __syncthreads();
  const int Jp = a.JB * 16;
  for (int e = threadIdx.x; e < WG_NJ * 256; e += 256) {
    const int b = e >> 8, row = (e >> 4) & 15, col = e & 15;
    if (jb0 + b >= a.JB) continue;
    const float t = ((red[0][b][row][col] + red[1][b][row][col]) + red[2][b][row][col]) + red[3][b][row][col];
    a.partial[((size_t)blockIdx.x * a.Cout + cob * 16 + row) * Jp + (jb0 + b) * 16 + col] = t;
  }
}

// The same contraction with 16-byte (fp32) / 8-byte (bf16) gathers of x, for layers whose input
// channel count is a multiple of 4: a lane loads 4 consecutive channels of one (pixel, tap) and
// feeds them to 4 instructions, so the 16 columns of instruction e of group G are the columns
// ((G*16 + lane%16)*4 + e) of the (tap, channel) index: a permutation of the columns that only
// the write-out has to know. One load per 4 instructions instead of one per instruction.
constexpr int WGV_NG = 3;  // groups of 64 columns per wave

template <typename T>
__global__ __launch_bounds__(256) void wgrad_mfma_vec_kernel(WgradArgs a) {
  using S_ = Store<T>;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int cob = blockIdx.y;
  const int g0 = blockIdx.z * WGV_NG;
  const T* __restrict__ x = reinterpret_cast<const T*>(a.x);
  const T* __restrict__ dz = reinterpret_cast<const T*>(a.dz);
  const int cpmask = (1 << a.log2cp) - 1;
  const int ntaps = a.R * a.R;
  const int Jp = a.JB * 16;

  int jr[WGV_NG], js[WGV_NG], jc[WGV_NG];
  bool jv[WGV_NG];
#pragma unroll
  for (int g = 0; g < WGV_NG; ++g) {
    const int j = ((g0 + g) * 16 + l16) * 4;      // first of the lane's 4 columns (same tap: 4 divides the padded channel count)
    const int tap = j >> a.log2cp;
    jc[g] = j & cpmask;
    jr[g] = tap / a.R - a.pad;
    js[g] = tap % a.R - a.pad;
    jv[g] = j < Jp && tap < ntaps && jc[g] < a.Cin;
  }
  f32x4_t acc[WGV_NG][4];
#pragma unroll
  for (int g = 0; g < WGV_NG; ++g)
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[g][e] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int pq = a.P * a.Q;
  const bool fdiv = a.M < (1 << 22);
  const float inv_pq = 1.0f / (float)pq, inv_q = 1.0f / (float)a.Q;
  long m0 = ((long)blockIdx.x * 4 + wave) * (long)a.steps * 4;
  // Nothing in the loop is conditional (a masked position loads element 0 and contributes a
  // zero), and the loads of step st+1 are requested before the matrix instructions of step st.
  struct StepRegs { float dv; float xq[WGV_NG][4]; unsigned ok; };   // ok bit g: group g valid, bit 31: pixel valid
  auto issue = [&](StepRegs& r, int st) __attribute__((always_inline)) {
    const long m = m0 + (long)st * 4 + lg;
    const bool mv = st < a.steps && m < a.M;
    const int mm = mv ? (int)m : 0;
    // (small non-negative integers divide exactly through fp32; an integer division costs as
    // much as the step's matrix instructions)
    const int n = fdiv ? (int)(((float)mm + 0.5f) * inv_pq) : mm / pq;
    const int rem = mm - n * pq;
    const int p = fdiv ? (int)(((float)rem + 0.5f) * inv_q) : rem / a.Q;
    const int q = rem - p * a.Q;
    r.dv = S_::load1(dz + ((unsigned)mm * (unsigned)a.Cout + (unsigned)(cob * 16 + l16)));
    const int ihb = p * a.stride, iwb = q * a.stride;
    unsigned okb = mv ? 0x80000000u : 0u;
#pragma unroll
    for (int g = 0; g < WGV_NG; ++g) {
      const int ih = ihb + jr[g], iw = iwb + js[g];
      const bool ok = mv && jv[g] && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
      const unsigned off = ok ? (unsigned)((n * a.H + ih) * a.W + iw) * (unsigned)a.Cin + (unsigned)jc[g] : 0u;   // (32 bits: the host checks)
      S_::load4(x + off, r.xq[g]);
      okb |= (ok ? 1u : 0u) << g;
    }
    r.ok = okb;
  };
  auto contract = [&](StepRegs& r) __attribute__((always_inline)) {
    // (the empty statements keep the loads where they are: left to itself the compiler moves a
    // load under its predicate, and a branch around a load ends in a wait for every load in flight)
    asm volatile("" : "+v"(r.dv));
    const float dv = (r.ok >> 31) ? r.dv : 0.f;
#pragma unroll
    for (int g = 0; g < WGV_NG; ++g) {
      asm volatile("" : "+v"(r.xq[g][0]), "+v"(r.xq[g][1]), "+v"(r.xq[g][2]), "+v"(r.xq[g][3]));
      const bool ok = (r.ok >> g) & 1u;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        acc[g][e] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, ok ? r.xq[g][e] : 0.f, acc[g][e], 0, 0, 0);
    }
  };
  StepRegs ra, rb;     // two sets, used in turn (a step past the end is masked: it adds zeros)
  issue(ra, 0);
  for (int st = 0; st < a.steps; st += 2) {
    issue(rb, st + 1);
    contract(ra);
    issue(ra, st + 2);
    contract(rb);
  }

  // sum the four waves in a fixed order, then write the partial tile (columns back in order)
  __shared__ float red[4][WGV_NG * 4][16][17];
#pragma unroll
  for (int g = 0; g < WGV_NG; ++g)
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int i = 0; i < 4; ++i) red[wave][g * 4 + e][lg * 4 + i][l16] = acc[g][e][i];
  __syncthreads();
  for (int t = threadIdx.x; t < WGV_NG * 16 * 64; t += 256) {
    const int jj = t & 63, row = (t >> 6) & 15, g = t >> 10;
    const int col = jj >> 2, e = jj & 3, b = g * 4 + e;
    const int j = (g0 + g) * 64 + jj;
    if (j >= Jp) continue;
    const float v = ((red[0][b][row][col] + red[1][b][row][col]) + red[2][b][row][col]) + red[3][b][row][col];
    a.partial[((size_t)blockIdx.x * a.Cout + cob * 16 + row) * Jp + j] = v;
  }
}

// dW[co][ci][r][s] = sum over splits (in order) of partial[split][co][tap*CP + ci]
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(WgradArgs a) {
  const int Jp = a.JB * 16;
  const int total = a.Cout * Jp;
  // 16 threads share one output: each sums a strided subset, then a fixed-order tree
  __shared__ float red[16][17];
  const int sub = threadIdx.x & 15, loc = threadIdx.x >> 4;
  const int e = blockIdx.x * 16 + loc;
  float s = 0.f;
  if (e < total)
    for (int sp = sub; sp < a.msplit; sp += 16) s += a.partial[(size_t)sp * total + e];
  red[loc][sub] = s;
  __syncthreads();
  if (sub == 0 && e < total) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += red[loc][i];
    const int co = e / Jp, j = e - co * Jp;
    const int tap = j >> a.log2cp, ci = j & ((1 << a.log2cp) - 1);
    if (tap < a.R * a.R && ci < a.Cin) {
      const int r = tap / a.R, sx = tap % a.R;
      a.dW[(((size_t)co * a.Cin + ci) * a.R + r) * a.R + sx] = t;
    }
  }
}

// All layers of a module in one launch: blockIdx.y picks the layer, a workgroup covers 64 groups
// of 4 consecutive outputs. Thread (column group, row class rc) adds the rows rc, rc+4, ... in
// increasing order with 8 independent 16-byte loads in flight (a wave reads 1 KiB of one row);
// the four row classes are then added in a fixed order.
__global__ __launch_bounds__(256) void wgrad_reduce_all_kernel(const WredDesc* __restrict__ descs) {
  const WredDesc d = descs[blockIdx.y];
  const int total4 = d.Cout * d.Jp / 4;
  if ((int)blockIdx.x * 64 >= total4) return;
  const int cl = threadIdx.x & 63, rc = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + cl;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (col < total4) {
    const float4* __restrict__ p = reinterpret_cast<const float4*>(d.partial) + col;
    for (int r0 = rc; r0 < d.rows; r0 += 32) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int r = r0 + 4 * u;
        v[u] = r < d.rows ? p[(size_t)r * total4] : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
  }
  __shared__ float4 red[4][64];
  red[rc][cl] = s;
  __syncthreads();
  if (rc == 0 && col < total4) {
    const float4 a0 = red[0][cl], a1 = red[1][cl], a2 = red[2][cl], a3 = red[3][cl];
    const float t[4] = {((a0.x + a1.x) + a2.x) + a3.x, ((a0.y + a1.y) + a2.y) + a3.y,
                        ((a0.z + a1.z) + a2.z) + a3.z, ((a0.w + a1.w) + a2.w) + a3.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = col * 4 + i;
      const int co = e / d.Jp, j = e - co * d.Jp;
      const int tap = j >> d.log2cp, ci = j & ((1 << d.log2cp) - 1);
      if (tap < d.R * d.R && ci < d.Cin) {
        const int r = tap / d.R, sx = tap % d.R;
        d.dW[(((size_t)co * d.Cin + ci) * d.R + r) * d.R + sx] = t[i];
      }
    }
  }
}

hipError_t wgrad_reduce_all_launch(const WredDesc* dev_descs, int n, int max_outputs, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int gx = (max_outputs / 4 + 63) / 64;
  DDG_LAUNCH(wgrad_reduce_all_kernel, dim3(gx > 0 ? gx : 1, n), dim3(256), 0, s, dev_descs);
  return hipGetLastError();
}

void wgrad_plan(WgradArgs& a) {
  int l2 = 0;
  while ((1 << l2) < a.Cin) ++l2;
  a.log2cp = l2;
  a.J = a.R * a.R * (1 << l2);
  a.JB = (a.J + 15) / 16;
  a.vec = (a.Cin % 4 == 0) ? 1 : 0;       // the kernel with 4-channel gathers
  a.jgroups = a.vec ? (a.JB * 16 + 64 * WGV_NG - 1) / (64 * WGV_NG) : (a.JB + WG_NJ - 1) / WG_NJ;
  const int tiles = (a.Cout / 16) * a.jgroups;
  int want = 512 / tiles;                // workgroups over the pixel range (two per compute unit; more only add partial tiles)
  if (const char* e = getenv("DDG_TUNE_WGRAD_GENERIC_WGS")) {   // timing experiments, within [64, 4096]
    const int v = atoi(e);
    if (v >= 64 && v <= 4096) want = v / tiles;
  }
  if (want < 1) want = 1;
  const long quads = ((long)a.M + 3) / 4;  // 4-pixel steps in total
  long steps = (quads + (long)want * 4 - 1) / ((long)want * 4);
  if (steps < 8) steps = 8;
  a.steps = (int)steps;
  a.msplit = (int)((quads + steps * 4 - 1) / (steps * 4));
  if (a.msplit < 1) a.msplit = 1;
}

size_t wgrad_partial_elems(const WgradArgs& a) { return (size_t)a.msplit * a.Cout * a.JB * 16; }

hipError_t wgrad_launch(const WgradArgs& a, hipStream_t s) {
  dim3 grid(a.msplit, a.Cout / 16, a.jgroups), block(256);
  if (a.vec) {
    if (a.Cin % 4 != 0) return hipErrorInvalidValue;
    // 32-bit element offsets inside
    if ((size_t)a.N * a.H * a.W * a.Cin >= ((size_t)1 << 32) || (size_t)a.M * a.Cout >= ((size_t)1 << 32)) return hipErrorInvalidValue;
    if (a.dtype == BF16) DDG_LAUNCH(wgrad_mfma_vec_kernel<bf16_t>, grid, block, 0, s, a);
    else DDG_LAUNCH(wgrad_mfma_vec_kernel<float>, grid, block, 0, s, a);
    return hipGetLastError();
  }
  if (a.dtype == BF16) DDG_LAUNCH(wgrad_mfma_kernel<bf16_t>, grid, block, 0, s, a);
  else DDG_LAUNCH(wgrad_mfma_kernel<float>, grid, block, 0, s, a);
  return hipGetLastError();
}

hipError_t wgrad_reduce_launch(const WgradArgs& a, hipStream_t s) {
  const int total = a.Cout * a.JB * 16;
  DDG_LAUNCH(wgrad_reduce_kernel, dim3((total + 15) / 16), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ddg
