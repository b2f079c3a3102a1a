// Weight gradient of a 3x3, stride-1, pad-1 convolution on the bf16 matrix cores,
// for the CIFAR-shaped layers (16/32/64 channels, feature maps 32/16/8 wide).
//
//   dW[co][tap][ci] = sum over pixels m of dz[m][co] * a[pix(m,tap)][ci]
//
// The contraction index is the pixel, which is the slow index of both NHWC operands, while
// an MFMA lane wants 8 consecutive contraction values. So both operands are transposed once
// on their way into LDS ([channel][row][column] planes, written with 2-byte stores); after
// that every fragment is one aligned 16-byte LDS read. The three horizontal taps of a row
// are made from the aligned 8-column chunk plus its two neighbour columns with register
// shifts, so each staged element is read from LDS three times (once per vertical tap) and
// not nine. The activation a can be produced on the fly from the saved conv output:
// a = relu(z*scale + shift) is applied while staging (scale == nullptr: use x as stored).
//
// The error gradient dz can likewise be formed while staging: with dy given, the kernel applies
// the ReLU mask and the batch-norm backward formula dz = A*g + B*z + C0 (coefficients final, or
// derived from the partial rows of the BN-backward sums), uses dz for the contraction and
// writes it out once for the input-gradient kernel that follows: no separate apply pass.
//
// A workgroup walks over tiles of 8 image rows, keeps its accumulators in registers across
// tiles, and writes one partial tile at the end; wgrad_reduce_kernel adds the partials in a
// fixed order (deterministic).
#include "ddg_device.h"
#include "ddg_kernels.h"
#include "ddg_stats.h"
#include <cstdlib>

namespace ddg {

struct WgradTiledArgs {
  const bf16_t* x;       // [N,H,W,CIN] conv input, or the conv output it is derived from
  const float* scale;    // optional per-channel transform of x: relu(x*scale+shift)
  const float* shift;
  const bf16_t* dz;      // [N,H,W,COUT] (ignored when dy is given)
  // optional: form dz = A*g + B*zc + C0 with g = dy where mask*mscale+mshift > 0 (mask null: g = dy)
  const bf16_t* dy; const bf16_t* mask; const float* mscale; const float* mshift;
  const bf16_t* zc; const float* coef; BnBwdRows rows; bf16_t* dz_out;
  float* partial;        // [grid.x][COUT][9*CIN]
  int N, H, W;
  int tiles;             // N * H/8
};

template <int CIN, int COUT, int W>
struct WgradTiledCfg {
  static constexpr int TH = 8;
  static constexpr int ROWS = TH + 2;
  static constexpr int WP = W + 16;                       // 8 pad columns left and right
  static constexpr int CIB_ALL = CIN / 16;
  static constexpr int CIB = (CIN == 64) ? 1 : CIB_ALL;   // ci-blocks per workgroup
  static constexpr int OT = CIB_ALL / CIB;                // grid.y
  static constexpr int CINW = CIB * 16;                   // input channels staged per workgroup
  static constexpr int COB = COUT / 16;
  static constexpr int KSPLIT = 4 / COB;                  // waves sharing one co-block
  static constexpr int KSTEPS = TH * W / 32;
  static constexpr int round8odd(int v) { return ((v + 7) / 8) % 2 == 1 ? ((v + 7) / 8) * 8 : ((v + 7) / 8 + 1) * 8; }
  static constexpr int PSX = round8odd(ROWS * WP);        // plane stride of x^T (elements)
  static constexpr int PSZ = round8odd(TH * W);           // plane stride of dz^T
  static constexpr int LDS_X = CINW * PSX;
  static constexpr int LDS_Z = COUT * PSZ;
};

template <int CIN, int COUT, int W>
__global__ __launch_bounds__(256) void wgrad_tiled_kernel(WgradTiledArgs a) {
  using Cfg = WgradTiledCfg<CIN, COUT, W>;
  constexpr int TH = Cfg::TH, ROWS = Cfg::ROWS, WP = Cfg::WP, CIB = Cfg::CIB, CINW = Cfg::CINW;
  constexpr int COB = Cfg::COB, KSPLIT = Cfg::KSPLIT, KSTEPS = Cfg::KSTEPS, PSX = Cfg::PSX, PSZ = Cfg::PSZ;
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* xT = reinterpret_cast<uint16_t*>(smem);
  uint16_t* zT = xT + Cfg::LDS_X;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int cb = wave % COB, kpart = wave / COB;
  const int ci0 = blockIdx.y * CINW;   // first staged input channel

  // pad columns (image columns -1 and W) stay zero for the whole kernel
  for (int i = tid; i < CINW * ROWS; i += 256) {
    const int c = i / ROWS, rr = i - c * ROWS;
    xT[c * PSX + rr * WP + 7] = 0;
    xT[c * PSX + rr * WP + W + 8] = 0;
  }

  f32x4_t acc[9][CIB];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int b = 0; b < CIB; ++b) acc[t][b] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int tiles_per_img = a.H / TH;
  constexpr int XCH = CINW / 8;                 // 16-byte chunks per staged pixel of x
  constexpr int XVEC = ROWS * W * XCH;
  constexpr int XPT = (XVEC + 255) / 256;
  constexpr int ZCH = COUT / 8;
  constexpr int ZVEC = TH * W * ZCH;            // 512 for all three shapes
  constexpr int ZPT = ZVEC / 256;
  static_assert(ZVEC % 256 == 0 && 256 % XCH == 0 && 256 % ZCH == 0, "staging layout");
  const int xch = tid % XCH, zch = tid % ZCH;   // this thread's channel chunks (fixed)
  const bool fuse = a.dy != nullptr;
  const bool two_masks = fuse && a.mask && a.mask != a.zc;

  // registers that hold the next tile while the current one is contracted
  uint4 xs[XPT], ds[ZPT], zs[ZPT], ms[ZPT];
  bool xin[XPT];
  auto issue = [&](int tile) {
    const int n = tile / tiles_per_img, r0 = (tile - n * tiles_per_img) * TH;
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
      const int v = tid + i * 256;
      xs[i] = make_uint4(0, 0, 0, 0);
      xin[i] = false;
      if (v < XVEC) {
        const int px = v / XCH;
        const int col = px % W, rr = px / W;
        const int ih = r0 - 1 + rr;
        if (ih >= 0 && ih < a.H) {
          xin[i] = true;
          xs[i] = *reinterpret_cast<const uint4*>(a.x + ((size_t)(n * a.H + ih) * W + col) * CIN + ci0 + xch * 8);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < ZPT; ++i) {
      const int px = (tid + i * 256) / ZCH;
      const size_t gi = ((size_t)(n * a.H + r0) * W + px) * COUT + zch * 8;
      if (fuse) {
        ds[i] = *reinterpret_cast<const uint4*>(a.dy + gi);
        zs[i] = *reinterpret_cast<const uint4*>(a.zc + gi);
        if (two_masks) ms[i] = *reinterpret_cast<const uint4*>(a.mask + gi);
      } else {
        ds[i] = *reinterpret_cast<const uint4*>(a.dz + gi);
      }
    }
  };

  int tile = blockIdx.x;
  if (tile < a.tiles) issue(tile);

  // per-channel constants of this thread's chunks (derived while the first loads are in flight)
  float tsc[8], tsh[8];
  if (a.scale) {
#pragma unroll
    for (int j = 0; j < 8; ++j) { tsc[j] = a.scale[ci0 + xch * 8 + j]; tsh[j] = a.shift[ci0 + xch * 8 + j]; }
  }
  float cA[8], cB[8], cC[8], cms[8], cmh[8];
  if (fuse) {
    __shared__ float s_coef[3 * COUT];
    const float* coef = a.coef;
    if (a.rows.partial) {
      bn_bwd_from_rows<COUT>(a.rows, s_coef, blockIdx.x == 0 && blockIdx.y == 0);
      coef = s_coef;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int c = zch * 8 + j;
      cA[j] = coef[c]; cB[j] = coef[COUT + c]; cC[j] = coef[2 * COUT + c];
      cms[j] = a.mscale ? a.mscale[c] : 1.f; cmh[j] = a.mscale ? a.mshift[c] : 0.f;
    }
  }

  auto unpack = [](const uint4& q, float (&f)[8]) {
    f[0] = __uint_as_float(q.x << 16); f[1] = __uint_as_float(q.x & 0xffff0000u);
    f[2] = __uint_as_float(q.y << 16); f[3] = __uint_as_float(q.y & 0xffff0000u);
    f[4] = __uint_as_float(q.z << 16); f[5] = __uint_as_float(q.z & 0xffff0000u);
    f[6] = __uint_as_float(q.w << 16); f[7] = __uint_as_float(q.w & 0xffff0000u);
  };
  auto pack = [](const float (&f)[8]) {
    uint4 q;
    q.x = Store<bf16_t>::pack2(f[0], f[1]); q.y = Store<bf16_t>::pack2(f[2], f[3]);
    q.z = Store<bf16_t>::pack2(f[4], f[5]); q.w = Store<bf16_t>::pack2(f[6], f[7]);
    return q;
  };
  auto scatter = [](uint16_t* d, int stride, const uint4& q) {   // 8 channels -> 8 planes
    d[0 * stride] = (uint16_t)(q.x & 0xffff); d[1 * stride] = (uint16_t)(q.x >> 16);
    d[2 * stride] = (uint16_t)(q.y & 0xffff); d[3 * stride] = (uint16_t)(q.y >> 16);
    d[4 * stride] = (uint16_t)(q.z & 0xffff); d[5 * stride] = (uint16_t)(q.z >> 16);
    d[6 * stride] = (uint16_t)(q.w & 0xffff); d[7 * stride] = (uint16_t)(q.w >> 16);
  };
  // transform the held registers and write them transposed into LDS
  auto stage = [&](int tile) {
    const int n = tile / tiles_per_img, r0 = (tile - n * tiles_per_img) * TH;
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
      const int v = tid + i * 256;
      if (v < XVEC) {
        uint4 q = xs[i];
        if (a.scale && xin[i]) {
          float f[8];
          unpack(q, f);
#pragma unroll
          for (int j = 0; j < 8; ++j) { const float t = f[j] * tsc[j] + tsh[j]; f[j] = t > 0.f ? t : 0.f; }
          q = pack(f);
        }
        const int px = v / XCH;
        scatter(xT + (xch * 8) * PSX + (px / W) * WP + (px % W) + 8, PSX, q);
      }
    }
#pragma unroll
    for (int i = 0; i < ZPT; ++i) {
      const int px = (tid + i * 256) / ZCH;
      uint4 q = ds[i];
      if (fuse) {
        float g[8], zz[8];
        unpack(ds[i], g);
        unpack(zs[i], zz);
        if (a.mask) {
          float mk[8];
          unpack(two_masks ? ms[i] : zs[i], mk);
#pragma unroll
          for (int j = 0; j < 8; ++j) g[j] = (mk[j] * cms[j] + cmh[j]) > 0.f ? g[j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) g[j] = cA[j] * g[j] + (cB[j] * zz[j] + cC[j]);
        q = pack(g);
        if (blockIdx.y == 0)
          *reinterpret_cast<uint4*>(a.dz_out + ((size_t)(n * a.H + r0) * W + px) * COUT + zch * 8) = q;
      }
      scatter(zT + (zch * 8) * PSZ + px, PSZ, q);
    }
  };

  for (; tile < a.tiles; tile += gridDim.x) {
    __syncthreads();          // the previous tile has been contracted
    stage(tile);
    __syncthreads();
    if (tile + (int)gridDim.x < a.tiles) issue(tile + gridDim.x);   // in flight during the MFMA phase
    // ---- contraction over the tile's pixels ----
    for (int ks = kpart; ks < KSTEPS; ks += KSPLIT) {
      const int px = ks * 32 + lg * 8;           // first of this lane's 8 pixels
      const int row = px / W, col = px % W;
      const uint4 zf = *reinterpret_cast<const uint4*>(zT + (cb * 16 + l16) * PSZ + px);
#pragma unroll
      for (int b = 0; b < CIB; ++b) {
        const uint16_t* plane = xT + (b * 16 + l16) * PSX;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
          const uint16_t* rowp = plane + (row + r) * WP + col + 8;
          const uint4 m = *reinterpret_cast<const uint4*>(rowp);
          const uint32_t left = rowp[-1], right = rowp[8];
          uint4 s0, s2;
          s0.x = (m.x << 16) | left;
          s0.y = __builtin_amdgcn_alignbit(m.y, m.x, 16);
          s0.z = __builtin_amdgcn_alignbit(m.z, m.y, 16);
          s0.w = __builtin_amdgcn_alignbit(m.w, m.z, 16);
          s2.x = __builtin_amdgcn_alignbit(m.y, m.x, 16);
          s2.y = __builtin_amdgcn_alignbit(m.z, m.y, 16);
          s2.z = __builtin_amdgcn_alignbit(m.w, m.z, 16);
          s2.w = (m.w >> 16) | (right << 16);
          acc[r * 3 + 0][b] = Mma<bf16_t>::mma(zf, s0, acc[r * 3 + 0][b]);
          acc[r * 3 + 1][b] = Mma<bf16_t>::mma(zf, m, acc[r * 3 + 1][b]);
          acc[r * 3 + 2][b] = Mma<bf16_t>::mma(zf, s2, acc[r * 3 + 2][b]);
        }
      }
    }
  }

  // ---- combine the waves that share a co-block (fixed order), write the partial tile ----
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem);   // [KSPLIT][COB][9*CIB][16 co][17]
  constexpr int FR = 9 * CIB;
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int b = 0; b < CIB; ++b)
#pragma unroll
      for (int i = 0; i < 4; ++i)
        red[(((kpart * COB + cb) * FR + t * CIB + b) * 16 + lg * 4 + i) * 17 + l16] = acc[t][b][i];
  __syncthreads();
  constexpr int J = 9 * CIN;
  for (int e = tid; e < COB * FR * 256; e += 256) {
    const int ci_l = e & 15, co_l = (e >> 4) & 15, f = (e >> 8) % FR, cbb = (e >> 8) / FR;
    float s = 0.f;
#pragma unroll
    for (int kp = 0; kp < KSPLIT; ++kp) s += red[(((kp * COB + cbb) * FR + f) * 16 + co_l) * 17 + ci_l];
    const int t = f / CIB, b = f % CIB;
    a.partial[((size_t)blockIdx.x * COUT + cbb * 16 + co_l) * J + t * CIN + ci0 + b * 16 + ci_l] = s;
  }
}

template <int CIN, int COUT, int W>
static hipError_t wgrad_tiled_launch_t(const WgradTiledArgs& a, int grid_x, hipStream_t s) {
  using Cfg = WgradTiledCfg<CIN, COUT, W>;
  size_t lds = (size_t)(Cfg::LDS_X + Cfg::LDS_Z) * 2;
  const size_t red = (size_t)Cfg::KSPLIT * Cfg::COB * 9 * Cfg::CIB * 16 * 17 * 4;
  if (red > lds) lds = red;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_tiled_kernel<CIN, COUT, W>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  DDG_LAUNCH((wgrad_tiled_kernel<CIN, COUT, W>), dim3(grid_x, Cfg::OT), dim3(256), lds, s, a);
  return hipGetLastError();
}

// Returns the number of partial rows (grid.x) the tiled kernel will use for this shape, or 0
// if the shape is not covered (then the generic kernel is used).
int wgrad_tiled_rows(int N, int H, int W, int Cin, int Cout, int R, int stride, int dtype) {
  if (dtype != BF16 || R != 3 || stride != 1 || Cin != Cout) return 0;
  if (!((Cin == 16 && W == 32) || (Cin == 32 && W == 16) || (Cin == 64 && W == 8))) return 0;
  if (H % 8 != 0) return 0;
  const int tiles = N * (H / 8);
  int want = (Cin == 16) ? 256 : (Cin == 32 ? 128 : 32);
  if (const char* e = getenv("DDG_TUNE_WGRAD_ROWS")) want = atoi(e) > 0 ? atoi(e) : want;
  if (want > tiles) want = tiles;
  return want;
}

hipError_t wgrad_tiled_launch(const void* x, const float* scale, const float* shift, const void* dz,
                              const WgradFuse* fuse, float* partial, int N, int H, int W, int C, int rows,
                              hipStream_t s) {
  WgradTiledArgs a{};
  a.x = (const bf16_t*)x; a.scale = scale; a.shift = shift; a.dz = (const bf16_t*)dz; a.partial = partial;
  if (fuse) {
    a.dy = (const bf16_t*)fuse->dy; a.mask = (const bf16_t*)fuse->mask; a.mscale = fuse->mscale; a.mshift = fuse->mshift;
    a.zc = (const bf16_t*)fuse->z; a.coef = fuse->coef; a.dz_out = (bf16_t*)fuse->dz_out;
    if (fuse->rows) a.rows = *fuse->rows;
  }
  a.N = N; a.H = H; a.W = W; a.tiles = N * (H / 8);
  if (C == 16 && W == 32) return wgrad_tiled_launch_t<16, 16, 32>(a, rows, s);
  if (C == 32 && W == 16) return wgrad_tiled_launch_t<32, 32, 16>(a, rows, s);
  if (C == 64 && W == 8) return wgrad_tiled_launch_t<64, 64, 8>(a, rows, s);
  return hipErrorInvalidValue;
}

}  // namespace ddg
