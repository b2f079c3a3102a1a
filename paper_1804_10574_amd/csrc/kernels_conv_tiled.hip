// 3x3, stride-1, pad-1 convolution (forward and input-gradient) for the CIFAR layer shapes:
// C = Cin = Cout in {16, 32, 64} on feature maps W = 32, 16, 8 wide, bf16 operands.
//
// A workgroup stages the (8+2) x (W+2) halo tile of the input once in LDS (NHWC, each pixel
// padded by 16 bytes so that 16 pixels read 16 distinct LDS bank groups); the nine taps are
// then shifted LDS addresses: the im2col matrix never exists. While staging, the input can be
// turned into the activation it stands for, a = relu(x*scale + shift) (batch-norm + ReLU of
// the previous layer), so that activation is never written to memory. Zero padding is
// applied after that transform.
//
// Each wave owns 4 pixel-blocks x 1 output-channel block (16x16 MFMA tiles) and keeps its
// slice of the weights in registers for the whole kernel; a workgroup walks over several
// tiles, prefetching the next tile's global loads during the MFMA phase. The epilogue stores
// NHWC, optionally adds a (masked) shortcut gradient, and accumulates batch-norm statistics
// (sum, sum of squares of the stored values) in registers; one partial row per workgroup.
#include "ddg_device.h"
#include "ddg_kernels.h"
#include "ddg_stats.h"
#include <cstdlib>

namespace ddg {

struct ConvTiledArgs {
  const bf16_t* in;        // [N,H,W,C]
  const float* scale;      // optional input transform relu(in*scale+shift)
  const float* shift;
  BnRows in_rows;          // in_rows.partial != null: scale/shift come from these partial rows
  const bf16_t* wpack;     // packed operand [ks][C/16][64][8]
  bf16_t* out;             // [N,H,W,C]
  ConvStat st;             // epilogue statistics: partial rows [grid][2][C]
  const bf16_t* add_g;     // optional epilogue term, same layout as out
  const bf16_t* add_mask;  // add_g counts only where add_mask > 0
  int N, H;
  int tiles;               // N * H/8
};

template <int C, int W>
struct ConvTiledCfg {
  static constexpr int TH = 8, ROWS = TH + 2, WC = W + 2;
  static constexpr int PIX = C * 2 + 16;                 // bytes per staged pixel
  static constexpr int TILE_BYTES = ROWS * WC * PIX;
  static constexpr int CH = C / 8;                       // 16-byte chunks per pixel
  static constexpr int NCHUNK = ROWS * WC * CH;          // chunks per tile (halo columns included)
  static constexpr int PER_THREAD = (NCHUNK + 255) / 256;
  static constexpr int KSTEPS = (9 * C + 31) / 32;
  static constexpr int PG = W / 8;                       // waves along the pixel dimension
  static constexpr int COB = C / 16;
};

// MODE is the epilogue's statistics mode, fixed at compile time: 0 none, 1 sum / sum of squares
// of the stored output (forward), 2 the BN-backward sums of the layer below (input gradient).
template <int C, int W, int MODE>
__global__ __launch_bounds__(256) void conv3x3_tiled_kernel(ConvTiledArgs a) {
  using Cfg = ConvTiledCfg<C, W>;
  constexpr int TH = Cfg::TH, WC = Cfg::WC, PIX = Cfg::PIX, CH = Cfg::CH, NCHUNK = Cfg::NCHUNK;
  constexpr int PT = Cfg::PER_THREAD, KSTEPS = Cfg::KSTEPS, PG = Cfg::PG, COB = Cfg::COB;
  extern __shared__ __align__(16) unsigned char tile[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int pgrp = wave % PG, cb = wave / PG;

  // this wave's weights: KSTEPS fragments of its output-channel block
  uint4 wf[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks)
    wf[ks] = *reinterpret_cast<const uint4*>(a.wpack + ((size_t)(ks * COB + cb) * 64 + lane) * 8);

  // staging: chunk v -> (pixel of the halo tile, 8-channel chunk); a thread's channel chunk is
  // the same for all its chunks because 256 % CH == 0
  const int my_ch = tid % CH;
  const bool xform = a.scale != nullptr || a.in_rows.partial != nullptr;
  float tsc[8], tsh[8];

  // per-lane LDS byte offsets of the 4 pixel-blocks (tap 0,0; channel 0)
  int pbase[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int pt = (pgrp * 4 + i) * 16 + l16;     // pixel inside the 8 x W tile
    pbase[i] = ((pt / W) * WC + (pt % W)) * PIX;
  }
  // per-k-step tap offset of this lane's 8-channel chunk
  int koff[KSTEPS];
  bool kval[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) {
    const int kidx = (ks * 4 + lg) * 8;
    const int tap = kidx / C, c0 = kidx % C;
    kval[ks] = tap < 9;
    const int t = kval[ks] ? tap : 0;
    koff[ks] = ((t / 3) * WC + (t % 3)) * PIX + c0 * 2;
  }

  float ssum[4] = {0.f, 0.f, 0.f, 0.f}, ssq[4] = {0.f, 0.f, 0.f, 0.f};
  // mode 2: per-channel constants of the BN below, for this lane's 4 channels
  float bmu[4], bis[4], bms[4], bmh[4];
  const bf16_t* st_mask = reinterpret_cast<const bf16_t*>(a.st.mask);
  const bf16_t* st_z = reinterpret_cast<const bf16_t*>(a.st.z);
  if (MODE == 2) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int c = cb * 16 + lg * 4 + j;
      bmu[j] = a.st.zmean[c]; bis[j] = a.st.zinvstd[c];
      bms[j] = a.st.mscale ? a.st.mscale[c] : 1.f; bmh[j] = a.st.mscale ? a.st.mshift[c] : 0.f;
    }
  }
  const int tiles_per_img = a.H / TH;

  uint4 stage[PT];
  bool inimg[PT];
  auto issue_loads = [&](int t) {
    const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int v = tid + i * 256;
      stage[i] = make_uint4(0, 0, 0, 0);
      inimg[i] = false;
      if (v < NCHUNK) {
        const int px = v / CH;
        const int rr = px / WC, cc = px % WC;
        const int ih = r0 - 1 + rr, iw = cc - 1;
        if (ih >= 0 && ih < a.H && iw >= 0 && iw < W) {
          inimg[i] = true;
          stage[i] = *reinterpret_cast<const uint4*>(a.in + ((size_t)(n * a.H + ih) * W + iw) * C + my_ch * 8);
        }
      }
    }
  };
  auto write_stage = [&]() {
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      const int v = tid + i * 256;
      if (v < NCHUNK) {
        uint4 q = stage[i];
        if (xform && inimg[i]) {
          float f[8];
          f[0] = __uint_as_float(q.x << 16); f[1] = __uint_as_float(q.x & 0xffff0000u);
          f[2] = __uint_as_float(q.y << 16); f[3] = __uint_as_float(q.y & 0xffff0000u);
          f[4] = __uint_as_float(q.z << 16); f[5] = __uint_as_float(q.z & 0xffff0000u);
          f[6] = __uint_as_float(q.w << 16); f[7] = __uint_as_float(q.w & 0xffff0000u);
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float t = f[j] * tsc[j] + tsh[j];
            f[j] = t > 0.f ? t : 0.f;
          }
          q.x = Store<bf16_t>::pack2(f[0], f[1]); q.y = Store<bf16_t>::pack2(f[2], f[3]);
          q.z = Store<bf16_t>::pack2(f[4], f[5]); q.w = Store<bf16_t>::pack2(f[6], f[7]);
        }
        const int px = v / CH;
        *reinterpret_cast<uint4*>(tile + px * PIX + my_ch * 16) = q;
      }
    }
  };

  int t = blockIdx.x;
  if (t < a.tiles) issue_loads(t);
  // per-channel transform of the input; while the first tile's loads are in flight
  if (a.in_rows.partial) {
    __shared__ float s_sc[C], s_sh[C];
    bn_fwd_from_rows(a.in_rows, C, s_sc, s_sh, blockIdx.x == 0);
#pragma unroll
    for (int j = 0; j < 8; ++j) { tsc[j] = s_sc[my_ch * 8 + j]; tsh[j] = s_sh[my_ch * 8 + j]; }
  } else if (a.scale) {
#pragma unroll
    for (int j = 0; j < 8; ++j) { tsc[j] = a.scale[my_ch * 8 + j]; tsh[j] = a.shift[my_ch * 8 + j]; }
  }
  for (; t < a.tiles; t += gridDim.x) {
    __syncthreads();            // the previous tile has been consumed
    write_stage();
    __syncthreads();
    const int tn = t + gridDim.x;
    if (tn < a.tiles) issue_loads(tn);   // in flight during the MFMA phase

    f32x4_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint4 af = make_uint4(0, 0, 0, 0);
        if (kval[ks]) af = *reinterpret_cast<const uint4*>(tile + pbase[i] + koff[ks]);
        acc[i] = Mma<bf16_t>::mma(wf[ks], af, acc[i]);
      }
    }

    // epilogue: lane = pixel l16 of block i, channels cb*16 + lg*4 .. +3
    const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int pt = (pgrp * 4 + i) * 16 + l16;
      const size_t idx = ((size_t)(n * a.H + r0) * W + pt) * C + cb * 16 + lg * 4;
      float v[4] = {acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
      if (a.add_g) {
        float g[4];
        Store<bf16_t>::load4(a.add_g + idx, g);
        if (a.add_mask) {
          float mk[4];
          Store<bf16_t>::load4(a.add_mask + idx, mk);
#pragma unroll
          for (int j = 0; j < 4; ++j) g[j] = (mk[j] > 0.f) ? g[j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] += g[j];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = Store<bf16_t>::round(v[j]);
      Store<bf16_t>::store4(a.out + idx, v[0], v[1], v[2], v[3]);
      if (MODE == 1) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { ssum[j] += v[j]; ssq[j] += v[j] * v[j]; }
      } else if (MODE == 2) {
        float mk[4], zz[4];
        Store<bf16_t>::load4(st_mask + idx, mk);
        if (st_z == st_mask) {
#pragma unroll
          for (int j = 0; j < 4; ++j) zz[j] = mk[j];
        } else {
          Store<bf16_t>::load4(st_z + idx, zz);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float g = (mk[j] * bms[j] + bmh[j]) > 0.f ? v[j] : 0.f;
          ssum[j] += g;
          ssq[j] += g * ((zz[j] - bmu[j]) * bis[j]);
        }
      }
    }
  }

  if (MODE != 0) {
    // channel cb*16 + lg*4 + j: sum over the 16 pixel lanes, then over the PG waves of this cb
    __shared__ float red[4][2][16];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float s1 = ssum[j], s2 = ssq[j];
#pragma unroll
      for (int o = 1; o < 16; o <<= 1) {
        s1 += __shfl_xor(s1, o, 64);
        s2 += __shfl_xor(s2, o, 64);
      }
      if (l16 == 0) { red[wave][0][lg * 4 + j] = s1; red[wave][1][lg * 4 + j] = s2; }
    }
    __syncthreads();
    if (tid < 2 * C) {
      const int which = tid / C, c = tid % C;
      const int cbb = c / 16, cl = c % 16;
      float s = 0.f;
#pragma unroll
      for (int g = 0; g < PG; ++g) s += red[cbb * PG + g][which][cl];
      a.st.partial[((size_t)blockIdx.x * 2 + which) * C + c] = s;
    }
  }
}

int conv_tiled_grid(int N, int H, int W, int Cin, int Cout, int R, int stride, int dtype) {
  if (dtype != BF16 || R != 3 || stride != 1 || Cin != Cout) return 0;
  if (!((Cin == 16 && W == 32) || (Cin == 32 && W == 16) || (Cin == 64 && W == 8))) return 0;
  if (H % 8 != 0) return 0;
  const int tiles = N * (H / 8);
  int cap = 512;
  if (const char* e = getenv("DDG_TUNE_CONV_GRID")) cap = atoi(e) > 0 ? atoi(e) : cap;
  return tiles < cap ? tiles : cap;
}

template <int C, int W>
static hipError_t conv_tiled_launch_t(const ConvTiledArgs& a, int grid, hipStream_t s) {
  using Cfg = ConvTiledCfg<C, W>;
  if (a.st.mode == 1) DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 1>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  else if (a.st.mode == 2) DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 2>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  else DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 0>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  return hipGetLastError();
}

hipError_t conv_tiled_launch(const void* in, const float* scale, const float* shift, const BnRows* in_rows,
                             const void* wpack, void* out, const ConvStat& st, const void* add_g,
                             const void* add_mask, int N, int H, int W, int C, int grid, hipStream_t s) {
  ConvTiledArgs a;
  a.in = (const bf16_t*)in; a.scale = scale; a.shift = shift; a.wpack = (const bf16_t*)wpack;
  if (in_rows) a.in_rows = *in_rows; else a.in_rows = BnRows{};
  a.out = (bf16_t*)out; a.st = st; a.add_g = (const bf16_t*)add_g;
  a.add_mask = (const bf16_t*)add_mask; a.N = N; a.H = H; a.tiles = N * (H / 8);
  if (C == 16 && W == 32) return conv_tiled_launch_t<16, 32>(a, grid, s);
  if (C == 32 && W == 16) return conv_tiled_launch_t<32, 16>(a, grid, s);
  if (C == 64 && W == 8) return conv_tiled_launch_t<64, 8>(a, grid, s);
  return hipErrorInvalidValue;
}

}  // namespace ddg
