// Weight gradient of wide bf16 layers (1x1 and 3x3, stride 1; input and output channels
// multiples of 128): the companion of conv_wide_kernel.
//
//   dW[co][tap][ci] = sum over pixels p of dz[p][co] * x[pix(p, tap)][ci]
//
// A GEMM whose contraction index, the pixel, is the slow index of both NHWC operands. A
// workgroup owns a 128 (co) x 128 (ci) tile of one tap and a slice of the pixels; it stages
// 64 pixels of both operands per step exactly as they lie in memory ([pixel][128 channels],
// row stride 288 bytes) and takes MFMA fragments out of LDS with the transposing read of
// gfx950 (ds_read_b64_tr_b16: a lane ends up with 8 consecutive pixels of one channel). A tap
// is a shifted pixel row with zeros outside the image. Global loads of the next 64 pixels are
// in flight while the current ones are contracted (double-buffered through registers).
//
// Eight waves as 2 (pixel halves of a step) x 2 (co) x 2 (ci), 64 x 64 each = 16 accumulator
// tiles of mfma_f32_16x16x32_bf16; the two pixel halves meet in LDS at the end, so a workgroup
// writes one tile for twice the matrix work in flight. The pixel slices (split-K) give the
// launch enough workgroups; each writes an fp32 partial tile [split][co][tap*Cin + ci], which
// wgrad_reduce_all_kernel adds in a fixed order (deterministic). The partial tiles are what
// this kernel costs in memory traffic (64 KB per workgroup, written here and read by the
// reduction), hence one workgroup of eight waves per compute unit rather than two of four.
#include "ddg_device.h"
#include "ddg_kernels.h"
#include <cstdlib>

namespace ddg {

struct WgradWideArgs {
  const bf16_t* x;       // [M][Cin]
  const bf16_t* dz;      // [M][Cout]
  const float* scale;    // optional per-channel transform of x: relu(x*scale+shift)
  const float* shift;
  float* partial;        // [splits][Cout][J], J = taps*Cin
  int M, H, W, HW, Cin, Cout, R, J;
  int nsplits;           // pixel slices: slice i covers 64-pixel steps [i*nsteps/nsplits, (i+1)*nsteps/nsplits)
  int nsteps;            // ceil(M/64)
  int cit, taps;         // Cin/128, R*R: tile index = (cot*taps + tap)*cit + ci tile
  int by_xcd;            // 1: workgroups are renumbered so that a pixel slice stays on one XCD
};

namespace wgw {
constexpr int BP = 64;                     // pixels per step
constexpr int ROW = 256 + 32;              // bytes per staged pixel (128 channels), 32 modulo 128
constexpr int OPB = BP * ROW;              // one operand, one buffer: 18432
constexpr int BUF = 2 * OPB;
constexpr int LDS = 2 * BUF;               // 73728
}

typedef short wtr4_t __attribute__((ext_vector_type(4)));
// 8-pixel fragment of one channel per lane: two transposing reads 4 pixels apart
__device__ __forceinline__ uint4 wide_frag_tr(const unsigned char* p) {
  typedef wtr4_t __attribute__((address_space(3))) * lds_ptr_t;
  const wtr4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
  const wtr4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * wgw::ROW));
  const uint2 l = __builtin_bit_cast(uint2, lo), h = __builtin_bit_cast(uint2, hi);
  return make_uint4(l.x, l.y, h.x, h.y);
}

__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2))) void wgrad_wide_kernel(WgradWideArgs a) {
  using namespace wgw;
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, lg = lane >> 4;
  const int wa = wave & 1, wb = (wave >> 1) & 1;     // co half, ci half
  const int kg = wave >> 2;                          // pixels 32*kg .. 32*kg + 31 of every step
  // Workgroups go to the 8 XCDs round-robin in launch order. All tiles of one pixel slice read
  // the same rows of x and dz, so the (slice, tile) pairs are numbered slice-major and XCD j is
  // given the j-th eighth of that sequence: the rows of a slice then come from memory once into
  // one XCD's L2 (two at a boundary) and every other tile finds them there.
  int tile = blockIdx.x, split = blockIdx.y;
  if (a.by_xcd) {
    const int T = gridDim.x * gridDim.y, L = blockIdx.x + gridDim.x * blockIdx.y;
    const int xcd = L & 7, q = T >> 3, r = T & 7;
    const int V = xcd * q + (xcd < r ? xcd : r) + (L >> 3);   // XCD j holds q (+1 if j < r) workgroups
    split = V / (int)gridDim.x;
    tile = V - split * (int)gridDim.x;
  }
  const int cit = tile % a.cit;
  const int tap = (tile / a.cit) % a.taps;
  const int cot = tile / (a.cit * a.taps);
  const int co0 = cot * 128, ci0 = cit * 128;
  int dr = 0, ds = 0;
  if (a.R == 3) { dr = tap / 3 - 1; ds = tap - (tap / 3) * 3 - 1; }
  const int s0 = split * a.nsteps / a.nsplits;
  const int s1 = (split + 1) * a.nsteps / a.nsplits;

  // staging map: 16-byte unit tid + q*512 of a 64 x 128 tile = pixel (tid>>4) + 32*q, chunk tid&15
  const int ch = tid & 15, prow = tid >> 4;
  const int xshift = (dr * a.W + ds) * a.Cin;
  uint4 z0, z1, x0, x1;   // (named: arrays here are not promoted to registers)
  auto ldz = [&](int m) __attribute__((always_inline)) {
    return m < a.M ? *reinterpret_cast<const uint4*>(a.dz + (size_t)m * a.Cout + co0 + ch * 8) : make_uint4(0, 0, 0, 0);
  };
  // small non-negative integers divide exactly through fp32 (the host checks M < 2^22)
  const float inv_hw = 1.0f / (float)a.HW, inv_w = 1.0f / (float)a.W;
  unsigned xin = 0;      // bit q: row q of the step in the registers lies inside the image for this tap
  auto ldx = [&](int m, int q) __attribute__((always_inline)) {
    const int n = (int)(((float)m + 0.5f) * inv_hw);
    const int rem = m - n * a.HW;
    const int hh = (int)(((float)rem + 0.5f) * inv_w);
    const int h = hh + dr, w = rem - hh * a.W + ds;
    const bool in = m < a.M && h >= 0 && h < a.H && w >= 0 && w < a.W;
    xin |= (in ? 1u : 0u) << q;
    return in ? *reinterpret_cast<const uint4*>(a.x + (size_t)m * a.Cin + xshift + ci0 + ch * 8) : make_uint4(0, 0, 0, 0);
  };
  auto issue = [&](int step) __attribute__((always_inline)) {
    const int m = step * BP + prow;
    z0 = ldz(m); z1 = ldz(m + 32);
    xin = 0;
    x0 = ldx(m, 0); x1 = ldx(m + 32, 1);
  };
  // per-channel constants of this thread's 8 input channels (the same in every step)
  float tsc[8], tsh[8];
  const bool xform = a.scale != nullptr;
  if (xform) {
#pragma unroll
    for (int e = 0; e < 8; ++e) { tsc[e] = a.scale[ci0 + ch * 8 + e]; tsh[e] = a.shift[ci0 + ch * 8 + e]; }
  }
  // a pixel outside the image or past the end stays zero: the transform applies to loaded rows only
  auto act = [&](uint4 q, bool in) __attribute__((always_inline)) {
    float f[8];
    Store<bf16_t>::unpack_vec(q, f);
#pragma unroll
    for (int e = 0; e < 8; ++e) { const float t = f[e] * tsc[e] + tsh[e]; f[e] = (in && t > 0.f) ? t : 0.f; }
    uint4 o;
    o.x = Store<bf16_t>::pack2(f[0], f[1]); o.y = Store<bf16_t>::pack2(f[2], f[3]);
    o.z = Store<bf16_t>::pack2(f[4], f[5]); o.w = Store<bf16_t>::pack2(f[6], f[7]);
    return o;
  };
  auto stash = [&](int buf) __attribute__((always_inline)) {
    unsigned char* Z = smem + buf * BUF + prow * ROW + ch * 16;
    unsigned char* X = Z + OPB;
    if (xform) { x0 = act(x0, xin & 1u); x1 = act(x1, xin & 2u); }
    *reinterpret_cast<uint4*>(Z) = z0; *reinterpret_cast<uint4*>(Z + 32 * ROW) = z1;
    *reinterpret_cast<uint4*>(X) = x0; *reinterpret_cast<uint4*>(X + 32 * ROW) = x1;
  };

  f32x4_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // fragment address of (k-step 0, channel block 0): lane s of a 16-lane block points at
  // channels 4*(s%4).. of pixel lg*8 + s/4; the second read is 4 pixels further
  const int frag = (lg * 8 + (l16 >> 2)) * ROW + (l16 & 3) * 8;
  const int zoff = frag + wa * 128 + kg * 32 * ROW;   // + i*32 (channel block)
  const int xoff = OPB + frag + wb * 128 + kg * 32 * ROW;

  issue(s0);          // (the host gives every slice at least one step)
  stash(0);
  __syncthreads();
  for (int s = s0; s < s1; ++s) {
    const bool more = s + 1 < s1;
    if (more) issue(s + 1);
    const unsigned char* B = smem + ((s - s0) & 1) * BUF;
    uint4 zf[4], xf[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) zf[i] = wide_frag_tr(B + zoff + i * 32);
#pragma unroll
    for (int j = 0; j < 4; ++j) xf[j] = wide_frag_tr(B + xoff + j * 32);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = Mma<bf16_t>::mma(zf[i], xf[j], acc[i][j]);
    if (more) stash((s + 1 - s0) & 1);
    __syncthreads();
  }

  // the two pixel halves meet: waves 4-7 hand their accumulators over through LDS (the staging
  // buffers are free after the loop's last barrier), [wave & 3][register][lane], 64 KB
  float* ex = reinterpret_cast<float*>(smem) + (wave & 3) * 64 * 64 + lane;
  if (kg == 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) ex[((i * 4 + j) * 4 + e) * 64] = acc[i][j][e];
  }
  __syncthreads();
  if (kg == 0) {
    // lane (l16, lg) of tile (i, j) holds co = co0 + (wa*4 + i)*16 + lg*4 + e, ci = ci0 + (wb*4 + j)*16 + l16
    float* dst = a.partial + ((size_t)split * a.Cout + co0 + wa * 64 + lg * 4) * a.J + (size_t)tap * a.Cin + ci0 + wb * 64 + l16;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          dst[(size_t)(i * 16 + e) * a.J + j * 16] = acc[i][j][e] + ex[((i * 4 + j) * 4 + e) * 64];
  }
}

bool wgrad_wide_ok(int Cin, int Cout, int R, int stride, int dtype) {
  if (dtype != BF16 || stride != 1 || (R != 1 && R != 3)) return false;
  if (Cin < 128 || (Cin & (Cin - 1)) != 0) return false;   // power of two: the partial tile's column is tap*Cin + ci
  return Cout % 128 == 0;
}

// Number of pixel slices (= partial tiles per output element) for a layer: enough workgroups to
// fill the GPU (one of eight waves per compute unit), at least 2 steps of 64 pixels each.
// DDG_TUNE_WGRAD_WIDE_WGS overrides the target workgroup count within [64, 2048].
int wgrad_wide_splits(int M, int Cin, int Cout, int R) {
  int target = 256;
  if (const char* e = getenv("DDG_TUNE_WGRAD_WIDE_WGS")) {
    const int v = atoi(e);
    if (v >= 64 && v <= 2048) target = v;
  }
  const int tiles = (Cout / 128) * (Cin / 128) * R * R;
  const int nsteps = (M + wgw::BP - 1) / wgw::BP;
  int splits = target / tiles;      // never more workgroups than the target: one past what fits at once costs a whole extra round
  if (splits > nsteps / 2) splits = nsteps / 2;
  return splits < 1 ? 1 : splits;
}

hipError_t wgrad_wide_launch(const void* x, const void* dz, float* partial, int N, int H, int W, int Cin, int Cout,
                             int R, int splits, hipStream_t s, const float* scale, const float* shift) {
  if (!wgrad_wide_ok(Cin, Cout, R, 1, BF16) || splits < 1) return hipErrorInvalidValue;
  if ((size_t)N * H * W >= ((size_t)1 << 22)) return hipErrorInvalidValue;   // pixel indices divide through fp32 inside
  WgradWideArgs a{};
  a.x = (const bf16_t*)x; a.dz = (const bf16_t*)dz; a.partial = partial; a.scale = scale; a.shift = shift;
  a.M = N * H * W; a.H = H; a.W = W; a.HW = H * W; a.Cin = Cin; a.Cout = Cout; a.R = R; a.J = R * R * Cin;
  a.nsteps = (a.M + wgw::BP - 1) / wgw::BP;
  if (splits > a.nsteps) return hipErrorInvalidValue;   // an empty slice
  a.nsplits = splits;
  a.by_xcd = getenv("DDG_NO_WGRAD_XCD") ? 0 : 1;
  a.cit = Cin / 128; a.taps = R * R;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_wide_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, wgw::LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const dim3 grid((Cout / 128) * a.taps * a.cit, splits);
  DDG_LAUNCH(wgrad_wide_kernel, grid, dim3(512), wgw::LDS, s, a);
  return hipGetLastError();
}

}  // namespace ddg
