// 3x3, stride-1, pad-1 convolution (forward and input-gradient) with fp32 operands for the CIFAR
// layer shapes: C = Cin = Cout in {16, 32, 64} on feature maps W = 32, 16, 8 wide (and any
// height that is a multiple of 8), on the fp32 matrix instruction mfma_f32_16x16x4_f32.
//
// A workgroup stages the (8+2) x (W+2) halo tile of the input once in LDS, as it lies in memory
// (NHWC, each pixel padded by 16 bytes so that the 16 pixels of a fragment read fall into
// distinct bank groups); the nine taps are then shifted LDS addresses: the im2col matrix never
// exists, and every input element is read from memory once per tile instead of once per tap.
// Zero padding is written into the halo. The fp32 matrix instruction does 2 Kflop in the time
// the bf16 one does 32, so these layers are matrix-core bound: what the staging buys is that
// the fragment reads (one 16-byte LDS read per four matrix instructions) no longer compete
// with anything.
//
// Each wave owns 4 pixel-blocks x 1 output-channel block (16x16 accumulators) of the tile;
// its slice of the weights stays in registers for 16 and 32 channels (36 / 72 registers) and
// is re-read per tile from the packed operand (L1/L2 resident) for 64 channels. A workgroup
// walks over several tiles, prefetching the next tile's global loads into registers during the
// matrix phase. The epilogue stores NHWC, optionally adds a (masked) shortcut gradient, and
// accumulates batch-norm statistics (sum, sum of squares of the stored values); one partial
// row per workgroup, added in a fixed order.
#include "ddg_device.h"
#include "ddg_kernels.h"
#include <cstdlib>

namespace ddg {

struct ConvLds32Args {
  const float* in;         // [N,H,W,C]
  const float* wpack;      // [k-step][C/16][64][4]; the input gradient takes the operand with mirrored taps
  float* out;              // [N,H,W,C]
  float* stat_partial;     // [gridDim.x][2][C] or null
  // optional second minibatch (blockIdx.z = 1; forward only): same weights, its own tensors
  const float* in_b; float* out_b; float* stat_partial_b;
  const float* add_g;      // optional epilogue term, same layout as out
  const float* add_mask;   // add_g counts only where add_mask > 0
  int N, H;
  int tiles;               // N * H/8
};

template <int C, int W>
struct ConvLds32Cfg {
  static constexpr int TH = 8, ROWS = TH + 2, WC = W + 2;
  static constexpr int PIX = C * 4 + 16;                 // bytes per staged pixel
  static constexpr int TILE_BYTES = ROWS * WC * PIX;
  static constexpr int CH = C / 4;                       // 16-byte chunks per pixel
  static constexpr int NCHUNK = ROWS * WC * CH;          // chunks per tile (halo columns included)
  static constexpr int PER_THREAD = (NCHUNK + 255) / 256;
  static constexpr int KSTEPS = 9 * C / 16;              // fragments of 16 k-values
  static constexpr int PG = W / 8;                       // waves along the pixel dimension
  static constexpr int COB = C / 16;
  static constexpr bool WREG = C <= 32;                  // the wave's weights stay in registers
};

template <int C, int W>
__global__ __launch_bounds__(256) void conv3x3_lds_f32_kernel(ConvLds32Args a) {
  using Cfg = ConvLds32Cfg<C, W>;
  constexpr int TH = Cfg::TH, WC = Cfg::WC, PIX = Cfg::PIX, CH = Cfg::CH, NCHUNK = Cfg::NCHUNK;
  constexpr int PT = Cfg::PER_THREAD, KSTEPS = Cfg::KSTEPS, PG = Cfg::PG, COB = Cfg::COB;
  extern __shared__ __align__(16) unsigned char tile[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int pgrp = wave % PG, cb = wave / PG;
  const int tiles_per_img = a.H / TH;
  const bool second = blockIdx.z != 0;
  const float* __restrict__ g_in = second ? a.in_b : a.in;
  float* __restrict__ g_out = second ? a.out_b : a.out;
  float* __restrict__ g_stat = second ? a.stat_partial_b : a.stat_partial;

  // ---- staging map (the same for every tile): chunk v = tid + i*256 -> halo pixel, 4 channels
  const int my_ch = tid % CH;
  int goff[PT];        // element offset of the chunk relative to the tile's first pixel (row r0, column 0)
  int loff[PT];        // LDS byte offset, -1: no chunk
  int srow[PT];        // halo row of the chunk, -1: no chunk or a pad column (stays zero)
#pragma unroll
  for (int i = 0; i < PT; ++i) {
    const int v = tid + i * 256;
    const int px = v / CH;
    const int rr = px / WC, cc = px - rr * WC;
    const bool col_ok = v < NCHUNK && cc >= 1 && cc <= W;
    srow[i] = col_ok ? rr : -1;
    goff[i] = ((rr - 1) * W + (cc - 1)) * C + my_ch * 4;
    loff[i] = v < NCHUNK ? px * PIX + my_ch * 16 : -1;
  }
  float4 stage[PT];
  auto issue_loads = [&](int t) {
    const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
    const unsigned tb = (unsigned)((n * a.H + r0) * W) * C;   // (32 bits: the host checks)
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      stage[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      const int ih = r0 - 1 + srow[i];
      if (srow[i] >= 0 && ih >= 0 && ih < a.H) stage[i] = *reinterpret_cast<const float4*>(g_in + tb + goff[i]);
    }
  };
  int t = blockIdx.x;
  if (t < a.tiles) issue_loads(t);

  // ---- this wave's weights: KSTEPS fragments of its output-channel block
  const float* wsrc = a.wpack + ((size_t)cb * 64 + lane) * 4;     // + ks * COB*64*4
  float4 wf[Cfg::WREG ? KSTEPS : 1];
  if (Cfg::WREG) {
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) wf[ks] = *reinterpret_cast<const float4*>(wsrc + (size_t)ks * COB * 64 * 4);
  }

  // ---- LDS fragment address of (pixel block 0, this lane): pixel pt = pgrp*64 + l16 (+ i*16)
  const int ptl = pgrp * 64 + l16;
  const int lane_base = ((ptl / W) * WC + (ptl % W)) * PIX + lg * 16;
  // output element offset of (block 0, this lane) inside a tile; block i adds i*16*C
  const int out_lane = ptl * C + cb * 16 + lg * 4;

  float ssum[4] = {0.f, 0.f, 0.f, 0.f}, ssq[4] = {0.f, 0.f, 0.f, 0.f};

  for (; t < a.tiles; t += gridDim.x) {
    __syncthreads();            // the previous tile has been consumed
#pragma unroll
    for (int i = 0; i < PT; ++i)
      if (loff[i] >= 0) *reinterpret_cast<float4*>(tile + loff[i]) = stage[i];
    __syncthreads();
    const int tn = t + gridDim.x;
    if (tn < a.tiles) issue_loads(tn);   // in flight during the matrix phase

    const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
    const unsigned obase = (unsigned)((n * a.H + r0) * W) * C + out_lane;
    // what the epilogue reads, requested now
    float4 eg[4], em[4];
    if (a.add_g) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        eg[i] = *reinterpret_cast<const float4*>(a.add_g + obase + i * 16 * C);
        if (a.add_mask) em[i] = *reinterpret_cast<const float4*>(a.add_mask + obase + i * 16 * C);
      }
    }

    f32x4_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      // k-values (ks*4 + lg)*4 .. +3: tap k/C, channels k%C (a fragment never straddles taps)
      const int kidx = ks * 16;
      const int tap = kidx / C, c0 = kidx % C;
      const unsigned char* kp = tile + lane_base + ((tap / 3) * WC + (tap % 3)) * PIX + c0 * 4;
      float4 w4;
      if (Cfg::WREG) w4 = wf[ks];
      else w4 = *reinterpret_cast<const float4*>(wsrc + (size_t)ks * COB * 64 * 4);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int blk = (((i * 16) / W) * WC + (i * 16) % W) * PIX;   // constant after unrolling
        const float4 af = *reinterpret_cast<const float4*>(kp + blk);
        acc[i] = Mma<float>::mma(w4, af, acc[i]);
      }
      // keep the fragment reads of later k-steps from being hoisted above this point: every
      // fragment the scheduler moves up front costs four registers for the whole loop
      if ((ks & 1) == 1) __builtin_amdgcn_sched_barrier(0);
    }

    // epilogue: lane = pixel l16 of block i, channels cb*16 + lg*4 .. +3
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v[4] = {acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
      if (a.add_g) {
        float g[4] = {eg[i].x, eg[i].y, eg[i].z, eg[i].w};
        if (a.add_mask) {
          const float mk[4] = {em[i].x, em[i].y, em[i].z, em[i].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) g[j] = (mk[j] > 0.f) ? g[j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] += g[j];
      }
      *reinterpret_cast<float4*>(g_out + obase + i * 16 * C) = make_float4(v[0], v[1], v[2], v[3]);
#pragma unroll
      for (int j = 0; j < 4; ++j) { ssum[j] += v[j]; ssq[j] += v[j] * v[j]; }
    }
  }

  if (g_stat) {
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
      g_stat[((size_t)blockIdx.x * 2 + which) * C + c] = s;
    }
  }
}

// Workgroups per launch (= partial statistics rows): every tile its own workgroup up to two per
// compute unit; beyond that workgroups walk over several tiles.
int conv_lds32_grid(int N, int H, int W, int Cin, int Cout, int R, int stride, int dtype) {
  if (dtype != F32 || R != 3 || stride != 1 || Cin != Cout) return 0;
  if (!((Cin == 16 && W == 32) || (Cin == 32 && W == 16) || (Cin == 64 && W == 8))) return 0;
  if (H % 8 != 0) return 0;
  if ((size_t)N * H * W * Cin >= ((size_t)1 << 31)) return 0;   // 32-bit element offsets inside
  const int tiles = N * (H / 8);
  return tiles < 512 ? tiles : 512;
}

template <int C, int W>
static hipError_t conv_lds32_launch_t(const ConvLds32Args& a, int grid, hipStream_t s) {
  using Cfg = ConvLds32Cfg<C, W>;
  static_assert(Cfg::TILE_BYTES <= 48 * 1024, "dynamic LDS within the default limit");
  DDG_LAUNCH((conv3x3_lds_f32_kernel<C, W>), dim3(grid, 1, a.in_b ? 2 : 1), dim3(256), Cfg::TILE_BYTES, s, a);
  return hipGetLastError();
}

hipError_t conv_lds32_launch(const void* in, const void* wpack, void* out, float* stat_partial, const void* in_b,
                             void* out_b, float* stat_partial_b, const void* add_g, const void* add_mask, int N,
                             int H, int W, int C, int grid, hipStream_t s) {
  if (grid < 1 || grid != conv_lds32_grid(N, H, W, C, C, 3, 1, F32)) return hipErrorInvalidValue;
  if (in_b && (!out_b || add_g || (stat_partial != nullptr) != (stat_partial_b != nullptr))) return hipErrorInvalidValue;
  ConvLds32Args a{};
  a.in = (const float*)in; a.wpack = (const float*)wpack; a.out = (float*)out; a.stat_partial = stat_partial;
  a.in_b = (const float*)in_b; a.out_b = (float*)out_b; a.stat_partial_b = stat_partial_b;
  a.add_g = (const float*)add_g; a.add_mask = (const float*)add_mask;
  a.N = N; a.H = H; a.tiles = N * (H / 8);
  if (C == 16 && W == 32) return conv_lds32_launch_t<16, 32>(a, grid, s);
  if (C == 32 && W == 16) return conv_lds32_launch_t<32, 16>(a, grid, s);
  if (C == 64 && W == 8) return conv_lds32_launch_t<64, 8>(a, grid, s);
  return hipErrorInvalidValue;
}


// ---------------------------------------------------------------------------------------------
// Weight gradient of the same layers: dW[co][tap][ci] = sum over pixels p of dz[p][co] * x[p + tap][ci].
// The contraction runs over pixels, so with the fp32 matrix instruction (k = 4 pixels per
// instruction, one element per lane and operand) no transposition is needed: a lane reads
// dz[pixel lg][channel l16] and x[pixel lg + tap][channel l16] as they lie in the staged tiles.
// A workgroup stages the halo tile of x and the tile of dz in LDS (every element is read from
// memory once per tile instead of once per tap), keeps its share of the 16x16 accumulator blocks
// of dW in registers across all its tiles, and writes one partial tile; the partial tiles are
// added in a fixed order by the module's reduction launch (no atomics).
//   16 channels:  9 blocks, every wave holds all of them and takes a quarter of the pixels (the
//                 four waves' sums are added through LDS in a fixed order at the end);
//   32 channels: 36 blocks, wave = (output-channel block, input-channel block), all 9 taps;
//   64 channels: 144 blocks, wave = output-channel block, all input-channel blocks and taps;
//                its tiles are 4 rows high so that a 128-image minibatch has 256 of them.
// ---------------------------------------------------------------------------------------------
struct WgradLds32Args {
  const float* x;          // [N,H,W,C] conv input
  const float* dz;         // [N,H,W,C] gradient w.r.t. the conv output
  float* partial;          // [gridDim.x][C][9*C]
  int N, H;
  int tiles;               // N * H/TH
};

template <int C, int W>
struct WgradLds32Cfg {
  static constexpr int TH = C == 64 ? 4 : 8, ROWS = TH + 2, WC = W + 2;
  static constexpr int PIX = C * 4 + 16;
  static constexpr int X_BYTES = ROWS * WC * PIX, Z_BYTES = TH * W * PIX;
  static constexpr int CH = C / 4;
  static constexpr int NX = ROWS * WC * CH, NZ = TH * W * CH;           // 16-byte chunks per tile
  static constexpr int PTX = (NX + 255) / 256, PTZ = (NZ + 255) / 256;
  static constexpr int NCB = C / 16;                                    // channel blocks
  static constexpr int NACC = C == 64 ? 36 : 9;                         // accumulator blocks per wave
  static constexpr int KS = TH * W / 4;                                 // 4-pixel steps per tile
  static constexpr int RED_BYTES = C == 16 ? 4 * 9 * 256 * 4 : 0;       // 16 channels: the four waves' blocks
  static constexpr int LDS = (X_BYTES + Z_BYTES) > RED_BYTES ? (X_BYTES + Z_BYTES) : RED_BYTES;
};

template <int C, int W>
__global__ __launch_bounds__(256) void wgrad3x3_lds_f32_kernel(WgradLds32Args a) {
  using Cfg = WgradLds32Cfg<C, W>;
  constexpr int TH = Cfg::TH, WC = Cfg::WC, PIX = Cfg::PIX, CH = Cfg::CH;
  constexpr int PTX = Cfg::PTX, PTZ = Cfg::PTZ, NACC = Cfg::NACC, KS = Cfg::KS;
  extern __shared__ __align__(16) unsigned char lds[];
  unsigned char* xs = lds;
  unsigned char* zs = lds + Cfg::X_BYTES;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int tiles_per_img = a.H / TH;
  // this wave's blocks: output-channel block cob; input-channel blocks cib0 .. cib0 + NCI - 1
  constexpr int NCI = C == 64 ? 4 : 1;
  const int cob = C == 16 ? 0 : (C == 32 ? wave >> 1 : wave);
  const int cib0 = C == 32 ? (wave & 1) : 0;

  // ---- staging maps (the same for every tile)
  const int my_ch = tid % CH;
  int xg[PTX], xl[PTX], xr[PTX];     // element offset from the tile's first pixel; LDS offset (-1: none); halo row (-1: stays zero)
#pragma unroll
  for (int i = 0; i < PTX; ++i) {
    const int v = tid + i * 256;
    const int px = v / CH;
    const int rr = px / WC, cc = px - rr * WC;
    const bool col_ok = v < Cfg::NX && cc >= 1 && cc <= W;
    xr[i] = col_ok ? rr : -1;
    xg[i] = ((rr - 1) * W + (cc - 1)) * C + my_ch * 4;
    xl[i] = v < Cfg::NX ? px * PIX + my_ch * 16 : -1;
  }
  int zg[PTZ], zl[PTZ];
#pragma unroll
  for (int i = 0; i < PTZ; ++i) {
    const int v = tid + i * 256;
    const int px = v / CH;
    zg[i] = px * C + my_ch * 4;
    zl[i] = v < Cfg::NZ ? px * PIX + my_ch * 16 : -1;
  }
  float4 sx[PTX], sz[PTZ];
  auto issue_loads = [&](int t) {
    const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
    const unsigned tb = (unsigned)((n * a.H + r0) * W) * C;   // (32 bits: the host checks)
#pragma unroll
    for (int i = 0; i < PTX; ++i) {
      sx[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      const int ih = r0 - 1 + xr[i];
      if (xr[i] >= 0 && ih >= 0 && ih < a.H) sx[i] = *reinterpret_cast<const float4*>(a.x + tb + xg[i]);
    }
#pragma unroll
    for (int i = 0; i < PTZ; ++i) {
      sz[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (zl[i] >= 0) sz[i] = *reinterpret_cast<const float4*>(a.dz + tb + zg[i]);
    }
  };
  int t = blockIdx.x;
  if (t < a.tiles) issue_loads(t);

  f32x4_t acc[NACC];
#pragma unroll
  for (int b = 0; b < NACC; ++b) acc[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  for (; t < a.tiles; t += gridDim.x) {
    __syncthreads();            // the previous tile has been consumed
#pragma unroll
    for (int i = 0; i < PTX; ++i)
      if (xl[i] >= 0) *reinterpret_cast<float4*>(xs + xl[i]) = sx[i];
#pragma unroll
    for (int i = 0; i < PTZ; ++i)
      if (zl[i] >= 0) *reinterpret_cast<float4*>(zs + zl[i]) = sz[i];
    __syncthreads();
    const int tn = t + gridDim.x;
    if (tn < a.tiles) issue_loads(tn);   // in flight during the matrix phase

    // 4-pixel steps: 16 channels: wave w takes steps w, w+4, ...; else every wave takes all
    constexpr int S0 = C == 16 ? 4 : 1;
    for (int s = (C == 16 ? wave : 0); s < KS; s += S0) {
      const int p = s * 4 + lg;                      // this lane's pixel of the step
      const int r = p / W, c = p % W;
      const float dv = *reinterpret_cast<const float*>(zs + p * PIX + (cob * 16 + l16) * 4);
      const unsigned char* xb = xs + (r * WC + c) * PIX + (cib0 * 16 + l16) * 4;
#pragma unroll
      for (int ci = 0; ci < NCI; ++ci)
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
          const float xv = *reinterpret_cast<const float*>(xb + ((tap / 3) * WC + tap % 3) * PIX + ci * 64);
          acc[ci * 9 + tap] = __builtin_amdgcn_mfma_f32_16x16x4f32(dv, xv, acc[ci * 9 + tap], 0, 0, 0);
        }
    }
  }

  // ---- write the partial tile: block (cob, tap, cib): rows co = cob*16 + lg*4 + v, column
  // tap*C + cib*16 + l16
  constexpr int J = 9 * C;
  float* dst = a.partial + (size_t)blockIdx.x * C * J;
  if (C == 16) {
    // the four waves hold sums over different pixels of the same 9 blocks: add them in order
    __syncthreads();            // the tiles are no longer read
    float* red = reinterpret_cast<float*>(lds);      // [wave][block][row][col]
#pragma unroll
    for (int b = 0; b < 9; ++b)
#pragma unroll
      for (int v = 0; v < 4; ++v) red[((wave * 9 + b) * 16 + lg * 4 + v) * 16 + l16] = acc[b][v];
    __syncthreads();
    for (int e = tid; e < 9 * 256; e += 256) {
      const int b = e >> 8, row = (e >> 4) & 15, col = e & 15;
      const float s4 = ((red[((0 * 9 + b) * 16 + row) * 16 + col] + red[((1 * 9 + b) * 16 + row) * 16 + col]) +
                        red[((2 * 9 + b) * 16 + row) * 16 + col]) + red[((3 * 9 + b) * 16 + row) * 16 + col];
      dst[(size_t)row * J + b * 16 + col] = s4;
    }
  } else {
#pragma unroll
    for (int ci = 0; ci < NCI; ++ci)
#pragma unroll
      for (int tap = 0; tap < 9; ++tap)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          dst[(size_t)(cob * 16 + lg * 4 + v) * J + tap * C + (cib0 + ci) * 16 + l16] = acc[ci * 9 + tap][v];
  }
}

// Partial tiles (= workgroups) of the LDS-staged fp32 weight gradient, 0 if the shape is not covered.
int wgrad_lds32_rows(int N, int H, int W, int Cin, int Cout, int R, int stride, int dtype) {
  if (conv_lds32_grid(N, H, W, Cin, Cout, R, stride, dtype) == 0) return 0;
  const int tiles = N * (H / (Cin == 64 ? 4 : 8));
  int cap = 128;     // (measured on ResNet-20: 128 and 256 give the same iteration time; fewer partial tiles to add)
  if (const char* e = getenv("DDG_TUNE_WGRAD_LDS32_ROWS")) { const int v = atoi(e); if (v >= 16 && v <= 1024) cap = v; }
  return tiles < cap ? tiles : cap;
}

template <int C, int W>
static hipError_t wgrad_lds32_launch_t(const WgradLds32Args& a, int rows, hipStream_t s) {
  using Cfg = WgradLds32Cfg<C, W>;
  static_assert(Cfg::LDS <= 48 * 1024, "dynamic LDS within the default limit");
  DDG_LAUNCH((wgrad3x3_lds_f32_kernel<C, W>), dim3(rows), dim3(256), Cfg::LDS, s, a);
  return hipGetLastError();
}

hipError_t wgrad_lds32_launch(const void* x, const void* dz, float* partial, int N, int H, int W, int C, int rows,
                              hipStream_t s) {
  if (rows < 1 || rows != wgrad_lds32_rows(N, H, W, C, C, 3, 1, F32)) return hipErrorInvalidValue;
  WgradLds32Args a{};
  a.x = (const float*)x; a.dz = (const float*)dz; a.partial = partial; a.N = N; a.H = H;
  a.tiles = N * (H / (C == 64 ? 4 : 8));
  if (C == 16 && W == 32) return wgrad_lds32_launch_t<16, 32>(a, rows, s);
  if (C == 32 && W == 16) return wgrad_lds32_launch_t<32, 16>(a, rows, s);
  if (C == 64 && W == 8) return wgrad_lds32_launch_t<64, 8>(a, rows, s);
  return hipErrorInvalidValue;
}

}  // namespace ddg
