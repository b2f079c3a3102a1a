// Weight-gradient kernel body for the CIFAR-shaped 3x3 layers (see kernels_wgrad_tiled.hip for
// the method); a header so that a launch that carries two kinds of work can include it.
#pragma once
#include "ddg_device.h"
#include "ddg_kernels.h"
#include "ddg_stats.h"

namespace ddg {

// W, a.H: width and height of the conv OUTPUT (= of the input for stride 1; the input of a
// stride-2 layer is 2H x 2W).
struct WgradTiledArgs {
  const bf16_t* x;       // [N,H*S,W*S,CIN] conv input, or the conv output it is derived from
  const float* scale;    // optional per-channel transform of x: relu(x*scale+shift)
  const float* shift;
  const bf16_t* dz;      // [N,H,W,COUT] (ignored when dy is given)
  // optional: form dz = A*g + B*zc + C0 with g = dy where mask*mscale+mshift > 0 (mask null: g = dy)
  const bf16_t* dy; const bf16_t* mask; const float* mscale; const float* mshift;
  const bf16_t* zc; const float* coef; BnBwdRows rows; bf16_t* dz_out;
  float* partial;        // [grid.x][COUT][R*R*CIN]
  int N, H, W;
  int tiles;             // N * H/8
};

// S: stride (1 or 2), R: kernel size (3 with pad 1, or 1 with pad 0)
template <int CIN, int COUT, int W, int S = 1, int R = 3>
struct WgradTiledCfg {
  static constexpr int TH = 8;
  static constexpr int PAD = R / 2;
  static constexpr int ROWS = (TH - 1) * S + R;           // input rows a tile of TH output rows reads
  static constexpr int WC = (W - 1) * S + R;              // input columns (pad columns included)
  static constexpr int WI = W * S;                        // input width
  static constexpr int TAPS = R * R;
  static constexpr int CIB_ALL = CIN / 16;
  static constexpr int CIB = (CIN == 64) ? 1 : CIB_ALL;   // ci-blocks per workgroup
  static constexpr int OT = CIB_ALL / CIB;                // grid.y
  static constexpr int CINW = CIB * 16;                   // input channels staged per workgroup
  static constexpr int COB = COUT / 16;
  static constexpr int KSPLIT = 4 / COB;                  // waves sharing one co-block
  static constexpr int KSTEPS = TH * W / 32;
  static constexpr int KPW = KSTEPS / KSPLIT;             // k-steps per wave and tile
  // bytes per staged pixel: at least 2*channels, and 32 or 96 modulo 128
  static constexpr int lds_pix(int ch) { return ch == 16 ? 32 : (ch == 32 ? 96 : 160); }
  static constexpr int PIXX = lds_pix(CINW);
  static constexpr int PIXZ = lds_pix(COUT);
  static constexpr int LDS_X = ROWS * WC * PIXX;          // bytes
  static constexpr int LDS_Z = TH * W * PIXZ;
  static constexpr int RED = (KSPLIT - 1) * COB * TAPS * CIB * 4 * 64 * 4;   // bytes, cross-wave sum
  static constexpr int LDS = (LDS_X + LDS_Z) > RED ? (LDS_X + LDS_Z) : RED;
};

typedef short tr4_t __attribute__((ext_vector_type(4)));
// 8-pixel fragment of one channel per lane: two transposing reads 4 pixels apart
__device__ __forceinline__ uint4 lds_frag_tr(const unsigned char* p, int half_stride) {
  typedef tr4_t __attribute__((address_space(3))) * lds_ptr_t;
  const tr4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
  const tr4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + half_stride));
  const uint2 l = __builtin_bit_cast(uint2, lo), h = __builtin_bit_cast(uint2, hi);
  return make_uint4(l.x, l.y, h.x, h.y);
}

// The kernel body. bx of gx: this workgroup's index among those that walk over the tiles (one
// partial tile each); by: which slice of the input channels it stages (0 .. Cfg::OT-1).
// FUSE = false leaves the path that forms dz out of the code (a.dy is ignored).
template <int CIN, int COUT, int W, bool FUSE = true, int S = 1, int R = 3>
__device__ __forceinline__ void wgrad_tiled_body(const WgradTiledArgs& a, unsigned char* smem, int bx, int by, int gx) {
  using Cfg = WgradTiledCfg<CIN, COUT, W, S, R>;
  constexpr int TH = Cfg::TH, ROWS = Cfg::ROWS, WC = Cfg::WC, CIB = Cfg::CIB, CINW = Cfg::CINW;
  constexpr int PAD = Cfg::PAD, WI = Cfg::WI, TAPS = Cfg::TAPS;
  constexpr int COB = Cfg::COB, KSPLIT = Cfg::KSPLIT, KPW = Cfg::KPW, PIXX = Cfg::PIXX, PIXZ = Cfg::PIXZ;
  unsigned char* xt = smem;                 // [ROWS][WC] pixels x CINW channels
  unsigned char* zt = smem + Cfg::LDS_X;    // [TH*W] pixels x COUT channels

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int cb = wave % COB, kpart = wave / COB;
  const int ci0 = by * CINW;   // first staged input channel
  const int tiles_per_img = a.H / TH;

  // ---- staging maps (the same for every tile)
  constexpr int XCH = CINW / 8;                 // 16-byte chunks per staged pixel of x
  constexpr int XVEC = ROWS * WC * XCH;
  constexpr int XPT = (XVEC + 255) / 256;
  constexpr int ZCH = COUT / 8;
  constexpr int ZVEC = TH * W * ZCH;            // 512 for all three shapes
  constexpr int ZPT = ZVEC / 256;
  static_assert(ZVEC % 256 == 0 && 256 % XCH == 0 && 256 % ZCH == 0, "staging layout");
  const int xch = tid % XCH, zch = tid % ZCH;   // this thread's channel chunks (fixed)
  int xgoff[XPT], xrow[XPT], xloff[XPT];
#pragma unroll
  for (int i = 0; i < XPT; ++i) {
    const int v = tid + i * 256;
    const int px = v / XCH;
    const int rr = px / WC, cc = px - rr * WC;
    const bool col_ok = v < XVEC && cc >= PAD && cc - PAD < WI;
    xrow[i] = col_ok ? rr : -1;                                   // -1: nothing to load (pad column: zero)
    xgoff[i] = ((rr - PAD) * WI + (cc - PAD)) * CIN + ci0 + xch * 8;   // relative to the tile's first input pixel
    xloff[i] = v < XVEC ? px * PIXX + xch * 16 : -1;
  }
  const bool fuse = FUSE && a.dy != nullptr;
  const bool two_masks = fuse && a.mask && a.mask != a.zc;

  // registers that hold the next tile while the current one is contracted
  uint4 xs[XPT], ds[ZPT], zs[FUSE ? ZPT : 1], ms[FUSE ? ZPT : 1];
  unsigned xin = 0;
  auto issue = [&](int tile) {
    const int n = tile / tiles_per_img, r0 = (tile - n * tiles_per_img) * TH;
    const bf16_t* xb = a.x + ((size_t)(n * a.H * S + r0 * S) * WI) * CIN;
    xin = 0;
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
      xs[i] = make_uint4(0, 0, 0, 0);
      const int ih = r0 * S - PAD + xrow[i];
      if (xrow[i] >= 0 && ih >= 0 && ih < a.H * S) {
        xin |= 1u << i;
        xs[i] = *reinterpret_cast<const uint4*>(xb + xgoff[i]);
      }
    }
    const size_t zb = ((size_t)(n * a.H + r0) * W) * COUT + (size_t)tid * 8;   // chunk v at zb + i*2048
#pragma unroll
    for (int i = 0; i < ZPT; ++i) {
      const size_t gi = zb + (size_t)i * 2048;
      if (FUSE && fuse) {
        ds[i] = *reinterpret_cast<const uint4*>(a.dy + gi);
        zs[i] = *reinterpret_cast<const uint4*>(a.zc + gi);
        if (two_masks) ms[i] = *reinterpret_cast<const uint4*>(a.mask + gi);
      } else {
        ds[i] = *reinterpret_cast<const uint4*>(a.dz + gi);
      }
    }
  };

  int tile = bx;
  if (tile < a.tiles) issue(tile);

  // ---- fragment addresses: lane and k-step part in a register, tap / ci-block / half as immediates
  // k-step q of this wave covers pixels p = (kpart + q*KSPLIT)*32 + lg*8 .. +7 of the tile
  const int sub = l16 >> 2, chq = (l16 & 3) * 8;     // pixel within a group of 4; byte offset of 4 channels
  int zaddr[KPW], xaddr[KPW];
#pragma unroll
  for (int q = 0; q < KPW; ++q) {
    const int p = (kpart + q * KSPLIT) * 32 + lg * 8;
    const int row = p / W, col = p % W;
    zaddr[q] = Cfg::LDS_X + (p + sub) * PIXZ + cb * 32 + chq;
    xaddr[q] = (row * S * WC + (col + sub) * S) * PIXX + chq;
  }

  // per-channel constants of this thread's chunks (derived while the first loads are in flight)
  float tsc[8], tsh[8];
  if (a.scale) {
#pragma unroll
    for (int j = 0; j < 8; ++j) { tsc[j] = a.scale[ci0 + xch * 8 + j]; tsh[j] = a.shift[ci0 + xch * 8 + j]; }
  }
  float cA[8], cB[8], cC[8], cms[8], cmh[8];
  if (FUSE && fuse) {
    __shared__ float s_coef[3 * COUT];
    const float* coef = a.coef;
    if (a.rows.partial) {
      bn_bwd_from_rows<COUT>(a.rows, s_coef, bx == 0 && by == 0);
      coef = s_coef;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int c = zch * 8 + j;
      cA[j] = coef[c]; cB[j] = coef[COUT + c]; cC[j] = coef[2 * COUT + c];
      cms[j] = a.mscale ? a.mscale[c] : 1.f; cmh[j] = a.mscale ? a.mshift[c] : 0.f;
    }
  }

  auto pack = [](const float (&f)[8]) {
    uint4 q;
    q.x = Store<bf16_t>::pack2(f[0], f[1]); q.y = Store<bf16_t>::pack2(f[2], f[3]);
    q.z = Store<bf16_t>::pack2(f[4], f[5]); q.w = Store<bf16_t>::pack2(f[6], f[7]);
    return q;
  };
  // transform the held registers and write them into LDS as they lie in memory
  auto stage = [&](int tile) {
    const int n = tile / tiles_per_img, r0 = (tile - n * tiles_per_img) * TH;
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
      if (xloff[i] >= 0) {
        uint4 q = xs[i];
        if (a.scale && ((xin >> i) & 1u)) {
          float f[8];
          Store<bf16_t>::unpack_vec(q, f);
#pragma unroll
          for (int j = 0; j < 8; ++j) { const float t = f[j] * tsc[j] + tsh[j]; f[j] = t > 0.f ? t : 0.f; }
          q = pack(f);
        }
        *reinterpret_cast<uint4*>(xt + xloff[i]) = q;
      }
    }
    const size_t zb = ((size_t)(n * a.H + r0) * W) * COUT + (size_t)tid * 8;
#pragma unroll
    for (int i = 0; i < ZPT; ++i) {
      uint4 q = ds[i];
      if (FUSE && fuse) {
        float g[8], zz[8];
        Store<bf16_t>::unpack_vec(ds[i], g);
        Store<bf16_t>::unpack_vec(zs[i], zz);
        if (a.mask) {
          float mk[8];
          Store<bf16_t>::unpack_vec(two_masks ? ms[i] : zs[i], mk);
#pragma unroll
          for (int j = 0; j < 8; ++j) g[j] = (mk[j] * cms[j] + cmh[j]) > 0.f ? g[j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) g[j] = cA[j] * g[j] + (cB[j] * zz[j] + cC[j]);
        q = pack(g);
        if (by == 0) *reinterpret_cast<uint4*>(a.dz_out + zb + (size_t)i * 2048) = q;
      }
      const int px = (tid + i * 256) / ZCH;
      *reinterpret_cast<uint4*>(zt + px * PIXZ + zch * 16) = q;
    }
  };

  f32x4_t acc[TAPS][CIB];
#pragma unroll
  for (int t = 0; t < TAPS; ++t)
#pragma unroll
    for (int b = 0; b < CIB; ++b) acc[t][b] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  for (; tile < a.tiles; tile += gx) {
    __syncthreads();          // the previous tile has been contracted
    stage(tile);
    __syncthreads();
    if (tile + gx < a.tiles) issue(tile + gx);   // in flight during the MFMA phase
    // ---- contraction over this wave's pixels of the tile ----
#pragma unroll
    for (int q = 0; q < KPW; ++q) {
      const uint4 zf = lds_frag_tr(smem + zaddr[q], 4 * PIXZ);
      const unsigned char* xp = xt + xaddr[q];
#pragma unroll
      for (int b = 0; b < CIB; ++b)
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
          for (int sx = 0; sx < R; ++sx) {
            const uint4 xf = lds_frag_tr(xp + (r * WC + sx) * PIXX + b * 32, 4 * S * PIXX);
            acc[r * R + sx][b] = Mma<bf16_t>::mma(zf, xf, acc[r * R + sx][b]);
          }
    }
  }

  // ---- add the waves that share a co-block in a fixed order; the first of them writes the
  // partial tile: lane (l16, lg) holds ci = b*16 + l16, co = cb*16 + lg*4 + i of tap t ----
  constexpr int J = TAPS * CIN;
  if (KSPLIT > 1) {
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem);   // [KSPLIT-1][COB][9*CIB*4][64 lanes]
    constexpr int SLOTS = TAPS * CIB * 4;
    if (kpart > 0) {
      float* w = red + (size_t)((kpart - 1) * COB + cb) * SLOTS * 64 + lane;
#pragma unroll
      for (int t = 0; t < TAPS; ++t)
#pragma unroll
        for (int b = 0; b < CIB; ++b)
#pragma unroll
          for (int i = 0; i < 4; ++i) w[((t * CIB + b) * 4 + i) * 64] = acc[t][b][i];
    }
    __syncthreads();
    if (kpart == 0) {
#pragma unroll
      for (int kp = 1; kp < KSPLIT; ++kp) {
        const float* w = red + (size_t)((kp - 1) * COB + cb) * SLOTS * 64 + lane;
#pragma unroll
        for (int t = 0; t < TAPS; ++t)
#pragma unroll
          for (int b = 0; b < CIB; ++b)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[t][b][i] += w[((t * CIB + b) * 4 + i) * 64];
      }
    }
  }
  if (kpart == 0) {
    float* dst = a.partial + ((size_t)bx * COUT + cb * 16 + lg * 4) * J + ci0 + l16;
#pragma unroll
    for (int t = 0; t < TAPS; ++t)
#pragma unroll
      for (int b = 0; b < CIB; ++b)
#pragma unroll
        for (int i = 0; i < 4; ++i) dst[(size_t)i * J + t * CIN + b * 16] = acc[t][b][i];
  }
}

}  // namespace ddg
