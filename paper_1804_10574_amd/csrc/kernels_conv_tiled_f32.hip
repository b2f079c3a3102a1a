// The LDS-tiled 3x3 stride-1 kernels of the CIFAR layer shapes (16/32/64 channels on maps 32/16/8
// wide) with fp32 operands: the same tiles, staging maps, on-load transforms, epilogues and
// launch interface as the bf16 kernels of kernels_conv_tiled.hip and ddg_wgrad_tiled.h, on the
// fp32 matrix instruction mfma_f32_16x16x4_f32 (one element per lane and operand, k = 4).
//
// Forward / input gradient: a workgroup stages the (8+2) x (W+2) halo tile of its input once in
// LDS (NHWC, each pixel padded by 16 bytes); while staging the input can be turned into the
// tensor it stands for: relu(x*scale+shift) (batch norm + ReLU of the layer before, the vectors
// final or derived from that layer's partial statistics rows), relu(x*scale+shift + res) (the
// output of the residual block before, which the kernel also stores), or the batch-norm backward
// dz = A*g + B*z + C0 of the gradient it is given (stored for the weight gradient). Each wave
// owns 4 pixel blocks x 1 output-channel block; a lane's fragment is four consecutive k-values
// read with one 16-byte LDS read and fed to four matrix instructions. The epilogue adds a
// (masked) shortcut gradient, and accumulates either the batch statistics of the output or the
// batch-norm backward sums of the layer below (whose ReLU mask it applies to what it stores).
//
// Weight gradient: the contraction runs over pixels, k = 4 pixels per instruction, so both
// operands are read from the staged tiles as they lie there (no transposition). x can be
// relu(z*scale+shift) formed while staging; dz can be formed from (dy, mask, z) in the same way
// and is then also stored. Accumulator blocks live in registers across a workgroup's tiles; one
// partial tile per workgroup, added by the module's reduction launch in a fixed order.
#include "ddg_device.h"
#include "ddg_kernels.h"
#include "ddg_stats.h"
#include <cstdlib>

namespace ddg {

// (the field meanings are those of the bf16 kernels' argument structs)
struct ConvTiledF32Args {
  const float* in; const float* res; float* y_out;
  const float* scale; const float* shift; BnRows in_rows;
  const float* wpack; float* out; ConvStat st;
  const float* add_g; const float* add_mask;
  const float* bz; const float* bmask; const float* bmscale; const float* bmshift; BnBwdRows brows; float* dz_out;
  int N, H, tiles, groups, vec_stride;
};

struct WgradTiledF32Args {
  const float* x; const float* scale; const float* shift;   // conv input, or what it derives from by relu(x*scale+shift)
  const float* dz;                                           // ignored when dy is given
  const float* dy; const float* mask; const float* mscale; const float* mshift;
  const float* zc; const float* coef; BnBwdRows rows; float* dz_out;
  float* partial;                                            // [rows][C][9*C]
  int N, H, tiles;                                           // tiles = N * H/TH
};

template <int C, int W>
struct ConvTiledF32Cfg {
  // 64 channels: tiles of 4 rows, so that a minibatch of 128 8x8 maps has a tile for every
  // compute unit (the fp32 matrix instruction makes these layers compute-bound)
  static constexpr int TH = C == 64 ? 4 : 8, ROWS = TH + 2, WC = W + 2;
  static constexpr int PIX = C * 4 + 16;                 // bytes per staged pixel
  static constexpr int TILE_BYTES = ROWS * WC * PIX;
  static constexpr int CH = C / 4;                       // 16-byte chunks per pixel
  static constexpr int NCHUNK = ROWS * WC * CH;
  static constexpr int PER_THREAD = (NCHUNK + 255) / 256;
  static constexpr int KSTEPS = 9 * C / 16;              // fragments of 16 k-values (4 per lane)
  static constexpr int PG = W / 8;
  static constexpr int COB = C / 16;
  static constexpr int NB = TH * W / (16 * PG);          // pixel blocks per wave: 4, 4, 2
  static constexpr bool WREG = C <= 32;                  // the wave's weights stay in registers
};

enum { XF32_PLAIN = 0, XF32_RES = 1, XF32_APPLY = 2, XF32_APPLY_MASK = 3 };

// MODE: 0 no statistics, 1 sum / sum of squares of the output, 2 batch-norm backward sums of the
// layer below. bidx of gdim: this workgroup's index among those of this work.
template <int C, int W, int MODE, int XF>
__device__ __forceinline__ void conv3x3_tiled_f32_body(const ConvTiledF32Args& a, unsigned char* tile, int bidx, int gdim) {
  using Cfg = ConvTiledF32Cfg<C, W>;
  constexpr bool RES = XF == XF32_RES, APPLY = XF == XF32_APPLY || XF == XF32_APPLY_MASK;
  constexpr int TH = Cfg::TH, WC = Cfg::WC, PIX = Cfg::PIX, CH = Cfg::CH, NCHUNK = Cfg::NCHUNK;
  constexpr int PT = Cfg::PER_THREAD, KSTEPS = Cfg::KSTEPS, PG = Cfg::PG, COB = Cfg::COB, NB = Cfg::NB;
  static_assert(PT <= 8, "four bits per chunk in one word");

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int pgrp = wave % PG, cb = wave / PG;
  const int tiles_per_img = a.H / TH;
  const int g1 = gdim / a.groups;
  const int grp = bidx / g1, bl = bidx - grp * g1;
  const int tiles_g = a.tiles / a.groups, t_end = (grp + 1) * tiles_g;

  // ---- staging map (the same for every tile): chunk v = tid + i*256 -> halo pixel, 4 channels
  const int my_ch = tid % CH;
  int goff[PT], loff[PT];
  unsigned srows = 0;    // 4 bits per chunk: halo row + 1; 0: no chunk, or a pad column (stays zero)
#pragma unroll
  for (int i = 0; i < PT; ++i) {
    const int v = tid + i * 256;
    const int px = v / CH;
    const int rr = px / WC, cc = px - rr * WC;
    const bool col_ok = v < NCHUNK && cc >= 1 && cc <= W;
    srows |= (col_ok ? (unsigned)(rr + 1) : 0u) << (4 * i);
    goff[i] = ((rr - 1) * W + (cc - 1)) * C + my_ch * 4;
    loff[i] = v < NCHUNK ? px * PIX + my_ch * 16 : -1;
  }
  float4 stage[PT], stage2[(RES || APPLY) ? PT : 1], stage3[XF == XF32_APPLY_MASK ? PT : 1];
  unsigned inimg = 0;       // bit i: chunk i of the tile in flight lies inside the image
  unsigned tile_base = 0;   // element offset of the staged tile's first pixel (32 bits: the host checks)
  auto issue_loads = [&](int t) {
    const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
    const unsigned tb = (unsigned)((n * a.H + r0) * W) * C;
    tile_base = tb;
    inimg = 0;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      stage[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      const int sr = (int)((srows >> (4 * i)) & 15u) - 1;
      const int ih = r0 - 1 + sr;
      if (sr >= 0 && ih >= 0 && ih < a.H) {
        inimg |= 1u << i;
        stage[i] = *reinterpret_cast<const float4*>(a.in + tb + goff[i]);
        if (RES) stage2[i] = *reinterpret_cast<const float4*>(a.res + tb + goff[i]);
        if (APPLY) stage2[i] = *reinterpret_cast<const float4*>(a.bz + tb + goff[i]);
        if (XF == XF32_APPLY_MASK) stage3[i] = *reinterpret_cast<const float4*>(a.bmask + tb + goff[i]);
      }
    }
  };
  int t = grp * tiles_g + bl;
  if (t < t_end) issue_loads(t);

  // ---- this wave's weights: KSTEPS fragments of its output-channel block
  const float* wsrc = a.wpack + ((size_t)cb * 64 + lane) * 4;     // + ks * COB*64*4
  float4 wf[Cfg::WREG ? KSTEPS : 1];
  if (Cfg::WREG) {
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) wf[ks] = *reinterpret_cast<const float4*>(wsrc + (size_t)ks * COB * 64 * 4);
  }

  const int ptl = pgrp * (NB * 16) + l16;
  const int lane_base = ((ptl / W) * WC + (ptl % W)) * PIX + lg * 16;
  const int out_lane = ptl * C + cb * 16 + lg * 4;

  // ---- per-channel vectors of the on-load transform, in LDS (derived while the first loads fly)
  const bool xform = !APPLY && (a.scale != nullptr || a.in_rows.partial != nullptr);
  __shared__ __align__(16) float s_sc[APPLY ? 4 : C], s_sh[APPLY ? 4 : C];
  __shared__ __align__(16) float s_coef[APPLY ? 5 * C : 4];   // A, B, C0, mask scale, mask shift
  if (APPLY) {
    if (tid < C) {
      s_coef[3 * C + tid] = a.bmscale ? a.bmscale[tid] : 1.f;
      s_coef[4 * C + tid] = a.bmscale ? a.bmshift[tid] : 0.f;
    }
    bn_bwd_from_rows<C>(a.brows, s_coef, bidx == 0);   // ends with a barrier
  } else if (a.in_rows.partial) {
    BnRows r = a.in_rows;
    r.partial += (size_t)grp * r.rows * 2 * C;
    const int vo = grp * a.vec_stride;
    r.mean += vo; r.invstd += vo; r.scale += vo; r.shift += vo;
    bn_fwd_from_rows<C>(r, s_sc, s_sh, bl == 0);
  } else if (a.scale) {
    const int vo = grp * a.vec_stride;
    if (tid < C) { s_sc[tid] = a.scale[vo + tid]; s_sh[tid] = a.shift[vo + tid]; }
    __syncthreads();
  }
  auto write_stage = [&]() {
    const unsigned stage_base = tile_base;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      if (loff[i] >= 0) {
        float4 q = stage[i];
        const unsigned sr1 = (srows >> (4 * i)) & 15u;   // halo row + 1
        const bool own_row = sr1 >= 2 && sr1 <= TH + 1;  // the tile's own rows are this workgroup's to store
        if (APPLY && ((inimg >> i) & 1u)) {
          const float4 zz = stage2[i];
          if (a.bmask) {
            const float4 mk = XF == XF32_APPLY_MASK ? stage3[i] : stage2[i];
            const float4 ms = *reinterpret_cast<const float4*>(&s_coef[3 * C + my_ch * 4]);
            const float4 mh = *reinterpret_cast<const float4*>(&s_coef[4 * C + my_ch * 4]);
            q.x = (mk.x * ms.x + mh.x) > 0.f ? q.x : 0.f; q.y = (mk.y * ms.y + mh.y) > 0.f ? q.y : 0.f;
            q.z = (mk.z * ms.z + mh.z) > 0.f ? q.z : 0.f; q.w = (mk.w * ms.w + mh.w) > 0.f ? q.w : 0.f;
          }
          const float4 cA = *reinterpret_cast<const float4*>(&s_coef[my_ch * 4]);
          const float4 cB = *reinterpret_cast<const float4*>(&s_coef[C + my_ch * 4]);
          const float4 cC = *reinterpret_cast<const float4*>(&s_coef[2 * C + my_ch * 4]);
          q.x = cA.x * q.x + (cB.x * zz.x + cC.x); q.y = cA.y * q.y + (cB.y * zz.y + cC.y);
          q.z = cA.z * q.z + (cB.z * zz.z + cC.z); q.w = cA.w * q.w + (cB.w * zz.w + cC.w);
          if (own_row) *reinterpret_cast<float4*>(a.dz_out + stage_base + goff[i]) = q;
        }
        if (xform && ((inimg >> i) & 1u)) {
          const float4 sc = *reinterpret_cast<const float4*>(&s_sc[my_ch * 4]);
          const float4 sh = *reinterpret_cast<const float4*>(&s_sh[my_ch * 4]);
          q.x = q.x * sc.x + sh.x; q.y = q.y * sc.y + sh.y; q.z = q.z * sc.z + sh.z; q.w = q.w * sc.w + sh.w;
          if (RES) {
            const float4 r = stage2[i];
            q.x += r.x; q.y += r.y; q.z += r.z; q.w += r.w;
          }
          q.x = q.x > 0.f ? q.x : 0.f; q.y = q.y > 0.f ? q.y : 0.f; q.z = q.z > 0.f ? q.z : 0.f; q.w = q.w > 0.f ? q.w : 0.f;
          if (RES && a.y_out && own_row) *reinterpret_cast<float4*>(a.y_out + stage_base + goff[i]) = q;
        }
        *reinterpret_cast<float4*>(tile + loff[i]) = q;
      }
    }
  };

  float ssum[4] = {0.f, 0.f, 0.f, 0.f}, ssq[4] = {0.f, 0.f, 0.f, 0.f};
  // mode 2: per-channel constants of the BN below (mean, invstd, mask scale, mask shift) in LDS
  __shared__ __align__(16) float s_below[MODE == 2 ? 4 * C : 4];
  const float* st_mask = reinterpret_cast<const float*>(a.st.mask);
  const float* st_z = reinterpret_cast<const float*>(a.st.z);
  const bool two_tensors = MODE == 2 && st_z != st_mask;
  if (MODE == 2) {
    if (tid < C) {
      s_below[tid] = a.st.zmean[tid]; s_below[C + tid] = a.st.zinvstd[tid];
      s_below[2 * C + tid] = a.st.mscale ? a.st.mscale[tid] : 1.f;
      s_below[3 * C + tid] = a.st.mscale ? a.st.mshift[tid] : 0.f;
    }
    // (made visible by the barriers of the tile loop before any epilogue runs)
  }

  for (; t < t_end; t += g1) {
    __syncthreads();            // the previous tile has been consumed
    write_stage();
    __syncthreads();
    const int tn = t + g1;
    if (tn < t_end) issue_loads(tn);   // in flight during the matrix phase

    const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
    const unsigned obase = (unsigned)((n * a.H + r0) * W) * C + out_lane;
    // what the epilogue reads, requested now
    float4 eg[NB], em[NB], ek[NB], ez[NB];
    if (a.add_g) {
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        eg[i] = *reinterpret_cast<const float4*>(a.add_g + obase + i * 16 * C);
        if (a.add_mask) em[i] = *reinterpret_cast<const float4*>(a.add_mask + obase + i * 16 * C);
      }
    }
    if (MODE == 2) {
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        ek[i] = *reinterpret_cast<const float4*>(st_mask + obase + i * 16 * C);
        if (two_tensors) ez[i] = *reinterpret_cast<const float4*>(st_z + obase + i * 16 * C);
      }
    }

    f32x4_t acc[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // 64 channels: the weight fragments do not fit the registers; they come from the packed
    // operand (L1/L2 resident) through a ring of four, requested three to four k-steps ahead
    float4 wq[Cfg::WREG ? 1 : 4];
    if (!Cfg::WREG) {
#pragma unroll
      for (int j = 0; j < 4; ++j) wq[j] = *reinterpret_cast<const float4*>(wsrc + (size_t)j * COB * 64 * 4);
    }
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      // k-values ks*16 + lg*4 .. +3: tap k/C, channels k%C (a fragment never straddles taps)
      const int kidx = ks * 16;
      const int tap = kidx / C, c0 = kidx % C;
      const unsigned char* kp = tile + lane_base + ((tap / 3) * WC + (tap % 3)) * PIX + c0 * 4;
      const float4 w4 = Cfg::WREG ? wf[Cfg::WREG ? ks : 0] : wq[Cfg::WREG ? 0 : (ks & 3)];
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int blk = (((i * 16) / W) * WC + (i * 16) % W) * PIX;   // constant after unrolling
        const float4 af = *reinterpret_cast<const float4*>(kp + blk);
        acc[i] = Mma<float>::mma(w4, af, acc[i]);
      }
      if ((ks & 1) == 1) {
        if (!Cfg::WREG) {   // the two slots just used take the fragments of k-steps ks+3 and ks+4
          if (ks + 3 < KSTEPS) wq[(ks + 3) & 3] = *reinterpret_cast<const float4*>(wsrc + (size_t)(ks + 3) * COB * 64 * 4);
          if (ks + 4 < KSTEPS) wq[(ks + 4) & 3] = *reinterpret_cast<const float4*>(wsrc + (size_t)(ks + 4) * COB * 64 * 4);
        }
        // keep the fragment reads of later k-steps from being hoisted above this point
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // epilogue: lane = pixel l16 of block i, channels cb*16 + lg*4 .. +3
#pragma unroll
    for (int i = 0; i < NB; ++i) {
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
      float xh[4];
      if (MODE == 2) {
        // the gradient leaves this kernel already multiplied by the ReLU mask of the layer below
        const float mk[4] = {ek[i].x, ek[i].y, ek[i].z, ek[i].w};
        const int cq = cb * 16 + lg * 4;
        const float4 bmu = *reinterpret_cast<const float4*>(&s_below[cq]);
        const float4 bis = *reinterpret_cast<const float4*>(&s_below[C + cq]);
        const float4 bms = *reinterpret_cast<const float4*>(&s_below[2 * C + cq]);
        const float4 bmh = *reinterpret_cast<const float4*>(&s_below[3 * C + cq]);
        const float zz[4] = {two_tensors ? ez[i].x : mk[0], two_tensors ? ez[i].y : mk[1],
                             two_tensors ? ez[i].z : mk[2], two_tensors ? ez[i].w : mk[3]};
        const float mu4[4] = {bmu.x, bmu.y, bmu.z, bmu.w}, is4[4] = {bis.x, bis.y, bis.z, bis.w};
        const float ms4[4] = {bms.x, bms.y, bms.z, bms.w}, mh4[4] = {bmh.x, bmh.y, bmh.z, bmh.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          v[j] = (mk[j] * ms4[j] + mh4[j]) > 0.f ? v[j] : 0.f;
          xh[j] = (zz[j] - mu4[j]) * is4[j];
        }
      }
      *reinterpret_cast<float4*>(a.out + obase + i * 16 * C) = make_float4(v[0], v[1], v[2], v[3]);
      if (MODE == 1) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { ssum[j] += v[j]; ssq[j] += v[j] * v[j]; }
      } else if (MODE == 2) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { ssum[j] += v[j]; ssq[j] += v[j] * xh[j]; }
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
      a.st.partial[((size_t)bidx * 2 + which) * C + c] = s;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Weight gradient: dW[co][tap][ci] = sum over pixels p of dz[p][co] * x[p + tap][ci].
//   16 channels:  9 accumulator blocks, every wave holds all of them and takes a quarter of the
//                 pixels (the four waves' sums are added through LDS in a fixed order at the end);
//   32 channels: 36 blocks, wave = (output-channel block, input-channel block), all 9 taps;
//   64 channels: 144 blocks, wave = output-channel block, all input-channel blocks and taps;
//                its tiles are 4 rows high.
// ---------------------------------------------------------------------------------------------
template <int C, int W>
struct WgradTiledF32Cfg {
  static constexpr int TH = C == 64 ? 4 : 8, ROWS = TH + 2, WC = W + 2;
  static constexpr int PIX = C * 4 + 16;
  static constexpr int X_BYTES = ROWS * WC * PIX, Z_BYTES = TH * W * PIX;
  static constexpr int CH = C / 4;
  static constexpr int NX = ROWS * WC * CH, NZ = TH * W * CH;           // 16-byte chunks per tile
  static constexpr int PTX = (NX + 255) / 256, PTZ = (NZ + 255) / 256;
  static constexpr int NACC = C == 64 ? 36 : 9;                         // accumulator blocks per wave
  static constexpr int KS = TH * W / 4;                                 // 4-pixel steps per tile
  static constexpr int RED_BYTES = C == 16 ? 4 * 9 * 256 * 4 : 0;
  static constexpr int LDS = (X_BYTES + Z_BYTES) > RED_BYTES ? (X_BYTES + Z_BYTES) : RED_BYTES;
};

// bx of gx: this workgroup's index among those that walk over the tiles (one partial tile each).
// FUSE = false leaves the path that forms dz out of the code.
template <int C, int W, bool FUSE>
__device__ __forceinline__ void wgrad_tiled_f32_body(const WgradTiledF32Args& a, unsigned char* lds, int bx, int gx) {
  using Cfg = WgradTiledF32Cfg<C, W>;
  constexpr int TH = Cfg::TH, WC = Cfg::WC, PIX = Cfg::PIX, CH = Cfg::CH;
  constexpr int PTX = Cfg::PTX, PTZ = Cfg::PTZ, NACC = Cfg::NACC, KS = Cfg::KS;
  static_assert(Cfg::NZ % 256 == 0, "every thread stages the same number of dz chunks");
  unsigned char* xs = lds;
  unsigned char* zs = lds + Cfg::X_BYTES;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int tiles_per_img = a.H / TH;
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
  const bool fuse = FUSE && a.dy != nullptr;
  const bool two_masks = fuse && a.mask && a.mask != a.zc;
  float4 sx[PTX], sz[PTZ], szz[FUSE ? PTZ : 1], szm[FUSE ? PTZ : 1];
  unsigned xin = 0;
  auto issue_loads = [&](int t) {
    const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
    const unsigned tb = (unsigned)((n * a.H + r0) * W) * C;   // (32 bits: the host checks)
    xin = 0;
#pragma unroll
    for (int i = 0; i < PTX; ++i) {
      sx[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      const int ih = r0 - 1 + xr[i];
      if (xr[i] >= 0 && ih >= 0 && ih < a.H) { xin |= 1u << i; sx[i] = *reinterpret_cast<const float4*>(a.x + tb + xg[i]); }
    }
#pragma unroll
    for (int i = 0; i < PTZ; ++i) {
      const unsigned gi = tb + (unsigned)(tid + i * 256) * 4;     // dz chunks lie as in memory
      if (FUSE && fuse) {
        sz[i] = *reinterpret_cast<const float4*>(a.dy + gi);
        szz[i] = *reinterpret_cast<const float4*>(a.zc + gi);
        if (two_masks) szm[i] = *reinterpret_cast<const float4*>(a.mask + gi);
      } else {
        sz[i] = *reinterpret_cast<const float4*>(a.dz + gi);
      }
    }
  };
  int t = bx;
  if (t < a.tiles) issue_loads(t);

  // per-channel constants of this thread's chunks
  float4 tsc = make_float4(1.f, 1.f, 1.f, 1.f), tsh = make_float4(0.f, 0.f, 0.f, 0.f);
  if (a.scale) {
    tsc = *reinterpret_cast<const float4*>(a.scale + my_ch * 4);
    tsh = *reinterpret_cast<const float4*>(a.shift + my_ch * 4);
  }
  float4 cA, cB, cC, cms, cmh;
  if (FUSE && fuse) {
    __shared__ __align__(16) float s_coef[3 * C];
    const float* coef = a.coef;
    if (a.rows.partial) {
      bn_bwd_from_rows<C>(a.rows, s_coef, bx == 0);
      coef = s_coef;
    }
    cA = *reinterpret_cast<const float4*>(coef + my_ch * 4);
    cB = *reinterpret_cast<const float4*>(coef + C + my_ch * 4);
    cC = *reinterpret_cast<const float4*>(coef + 2 * C + my_ch * 4);
    cms = a.mscale ? *reinterpret_cast<const float4*>(a.mscale + my_ch * 4) : make_float4(1.f, 1.f, 1.f, 1.f);
    cmh = a.mscale ? *reinterpret_cast<const float4*>(a.mshift + my_ch * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
  }

  f32x4_t acc[NACC];
#pragma unroll
  for (int b = 0; b < NACC; ++b) acc[b] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  for (; t < a.tiles; t += gx) {
    __syncthreads();            // the previous tile has been consumed
#pragma unroll
    for (int i = 0; i < PTX; ++i) {
      if (xl[i] >= 0) {
        float4 q = sx[i];
        if (a.scale && ((xin >> i) & 1u)) {
          q.x = q.x * tsc.x + tsh.x; q.y = q.y * tsc.y + tsh.y; q.z = q.z * tsc.z + tsh.z; q.w = q.w * tsc.w + tsh.w;
          q.x = q.x > 0.f ? q.x : 0.f; q.y = q.y > 0.f ? q.y : 0.f; q.z = q.z > 0.f ? q.z : 0.f; q.w = q.w > 0.f ? q.w : 0.f;
        }
        *reinterpret_cast<float4*>(xs + xl[i]) = q;
      }
    }
    {
      const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
      const unsigned tb = (unsigned)((n * a.H + r0) * W) * C;
#pragma unroll
      for (int i = 0; i < PTZ; ++i) {
        float4 q = sz[i];
        if (FUSE && fuse) {
          const float4 zz = szz[i];
          if (a.mask) {
            const float4 mk = two_masks ? szm[i] : szz[i];
            q.x = (mk.x * cms.x + cmh.x) > 0.f ? q.x : 0.f; q.y = (mk.y * cms.y + cmh.y) > 0.f ? q.y : 0.f;
            q.z = (mk.z * cms.z + cmh.z) > 0.f ? q.z : 0.f; q.w = (mk.w * cms.w + cmh.w) > 0.f ? q.w : 0.f;
          }
          q.x = cA.x * q.x + (cB.x * zz.x + cC.x); q.y = cA.y * q.y + (cB.y * zz.y + cC.y);
          q.z = cA.z * q.z + (cB.z * zz.z + cC.z); q.w = cA.w * q.w + (cB.w * zz.w + cC.w);
          *reinterpret_cast<float4*>(a.dz_out + tb + (unsigned)(tid + i * 256) * 4) = q;
        }
        const int px = (tid + i * 256) / CH;
        *reinterpret_cast<float4*>(zs + px * PIX + my_ch * 16) = q;
      }
    }
    __syncthreads();
    const int tn = t + gx;
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

  // ---- the partial tile: block (cob, tap, cib): rows co = cob*16 + lg*4 + v, column tap*C + cib*16 + l16
  constexpr int J = 9 * C;
  float* dst = a.partial + (size_t)bx * C * J;
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

// ---------------------------------------------------------------------------------------------
template <int C, int W, int MODE, int XF>
__global__ __launch_bounds__(256) void conv3x3_tiled_f32_kernel(ConvTiledF32Args a) {
  extern __shared__ __align__(16) unsigned char smem[];
  conv3x3_tiled_f32_body<C, W, MODE, XF>(a, smem, blockIdx.x, gridDim.x);
}

// The input-gradient kernel of a unit (which forms its dz while staging) and the plain weight
// gradient of the unit above it in one launch, as in the bf16 path.
template <int C, int W, int MODE, int XF>
__global__ __launch_bounds__(256) void bwd_pair_f32_kernel(ConvTiledF32Args ca, WgradTiledF32Args wa, int conv_grid, int wg_rows) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int b = blockIdx.x;
  if (b < conv_grid) conv3x3_tiled_f32_body<C, W, MODE, XF>(ca, smem, b, conv_grid);
  else wgrad_tiled_f32_body<C, W, false>(wa, smem, b - conv_grid, wg_rows);
}

template <int C, int W>
__global__ __launch_bounds__(256) void wgrad_tiled_f32_kernel(WgradTiledF32Args a) {
  extern __shared__ __align__(16) unsigned char smem[];
  wgrad_tiled_f32_body<C, W, true>(a, smem, blockIdx.x, gridDim.x);
}

// Workgroups per launch (= partial statistics rows) and partial weight-gradient tiles, 0 if the
// shape is not covered (never more than conv_tiled_max_grid()).
// DDG_TUNE_CONV_GRID_F32 / DDG_TUNE_WGRAD_ROWS_F32 override within [32, max] / [16, 1024].
static bool tiled_f32_shape(int N, int H, int W, int Cin, int Cout, int R, int stride) {
  if (R != 3 || stride != 1 || Cin != Cout) return false;
  if (!((Cin == 16 && W == 32) || (Cin == 32 && W == 16) || (Cin == 64 && W == 8))) return false;
  if (H % 8 != 0) return false;
  return (size_t)N * H * W * Cin < ((size_t)1 << 31);   // 32-bit element offsets inside
}
int conv_tiled_f32_grid(int N, int H, int W, int Cin, int Cout, int R, int stride) {
  if (!tiled_f32_shape(N, H, W, Cin, Cout, R, stride)) return 0;
  int cap = 128;   // (measured on ResNet-20 at batch 128: 64 / 96 / 128 / 160 / 192 / 256 -> 110 / 116 / 135 / 129 / 130 / 131 K images/sec)
  if (const char* e = getenv("DDG_TUNE_CONV_GRID_F32")) { const int v = atoi(e); if (v >= 32 && v <= conv_tiled_max_grid()) cap = v; }
  if (cap > conv_tiled_max_grid()) cap = conv_tiled_max_grid();
  if (Cin == 64 && !getenv("DDG_TUNE_CONV_GRID_F32")) cap = 256;   // (4-row tiles: one per compute unit)
  if (cap > conv_tiled_max_grid()) cap = conv_tiled_max_grid();
  const int tiles = N * (H / (Cin == 64 ? 4 : 8));
  return tiles < cap ? tiles : cap;
}
int wgrad_tiled_f32_rows(int N, int H, int W, int Cin, int Cout, int R, int stride) {
  if (!tiled_f32_shape(N, H, W, Cin, Cout, R, stride)) return 0;
  const int tiles = N * (H / (Cin == 64 ? 4 : 8));
  int cap = 128;     // (measured on ResNet-20: 128 and 256 give the same iteration time; fewer partial tiles to add)
  if (const char* e = getenv("DDG_TUNE_WGRAD_ROWS_F32")) { const int v = atoi(e); if (v >= 16 && v <= 1024) cap = v; }
  return tiles < cap ? tiles : cap;
}

template <int C, int W>
static hipError_t conv_tiled_f32_launch_t(const ConvTiledF32Args& a, int grid, hipStream_t s, const WgradTiledF32Args* wa, int wg_rows) {
  using Cfg = ConvTiledF32Cfg<C, W>;
  static_assert(Cfg::TILE_BYTES <= 48 * 1024, "dynamic LDS within the default limit");
  if (wa) {
    using WCfg = WgradTiledF32Cfg<C, W>;
    if (!a.bz || a.st.mode == 1 || a.scale || a.in_rows.partial || !a.brows.partial || !a.dz_out || wg_rows < 1)
      return hipErrorInvalidValue;
    constexpr int lds = Cfg::TILE_BYTES > WCfg::LDS ? Cfg::TILE_BYTES : WCfg::LDS;
    static_assert(lds <= 48 * 1024, "dynamic LDS within the default limit");
    const bool own_mask = a.bmask && a.bmask != a.bz;
    const dim3 g(grid + wg_rows);
    if (a.st.mode == 2) {
      if (own_mask) DDG_LAUNCH((bwd_pair_f32_kernel<C, W, 2, XF32_APPLY_MASK>), g, dim3(256), lds, s, a, *wa, grid, wg_rows);
      else DDG_LAUNCH((bwd_pair_f32_kernel<C, W, 2, XF32_APPLY>), g, dim3(256), lds, s, a, *wa, grid, wg_rows);
    } else {
      if (own_mask) DDG_LAUNCH((bwd_pair_f32_kernel<C, W, 0, XF32_APPLY_MASK>), g, dim3(256), lds, s, a, *wa, grid, wg_rows);
      else DDG_LAUNCH((bwd_pair_f32_kernel<C, W, 0, XF32_APPLY>), g, dim3(256), lds, s, a, *wa, grid, wg_rows);
    }
    return hipGetLastError();
  }
  if (a.res) {
    if (a.st.mode != 1 || !(a.scale || a.in_rows.partial)) return hipErrorInvalidValue;
    DDG_LAUNCH((conv3x3_tiled_f32_kernel<C, W, 1, XF32_RES>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  } else if (a.bz) {
    if (a.st.mode == 1 || a.scale || a.in_rows.partial || !a.brows.partial || !a.dz_out) return hipErrorInvalidValue;
    const bool own_mask = a.bmask && a.bmask != a.bz;
    if (a.st.mode == 2) {
      if (own_mask) DDG_LAUNCH((conv3x3_tiled_f32_kernel<C, W, 2, XF32_APPLY_MASK>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
      else DDG_LAUNCH((conv3x3_tiled_f32_kernel<C, W, 2, XF32_APPLY>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
    } else {
      if (own_mask) DDG_LAUNCH((conv3x3_tiled_f32_kernel<C, W, 0, XF32_APPLY_MASK>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
      else DDG_LAUNCH((conv3x3_tiled_f32_kernel<C, W, 0, XF32_APPLY>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
    }
  } else if (a.st.mode == 1) DDG_LAUNCH((conv3x3_tiled_f32_kernel<C, W, 1, XF32_PLAIN>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  else if (a.st.mode == 2) DDG_LAUNCH((conv3x3_tiled_f32_kernel<C, W, 2, XF32_PLAIN>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  else DDG_LAUNCH((conv3x3_tiled_f32_kernel<C, W, 0, XF32_PLAIN>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  return hipGetLastError();
}

// Same arguments and rules as conv_tiled_launch (which forwards here for fp32 tensors).
hipError_t conv_tiled_f32_launch(const void* in, const float* scale, const float* shift, const BnRows* in_rows,
                                 const void* wpack, void* out, const ConvStat& st, const void* add_g,
                                 const void* add_mask, int N, int H, int W, int C, int grid, hipStream_t s,
                                 const void* res, void* y_out, int groups, int vec_stride, const WgradFuse* apply,
                                 const WgradPair* pair) {
  if (groups < 1 || N % groups != 0 || grid % groups != 0) return hipErrorInvalidValue;
  if (groups > 1 && (st.mode != 1 || add_g)) return hipErrorInvalidValue;   // forward only
  if ((size_t)N * H * W * C >= ((size_t)1 << 31)) return hipErrorInvalidValue;   // 32-bit element offsets inside
  ConvTiledF32Args a{};
  if (apply) {
    if (groups != 1 || res || !apply->rows) return hipErrorInvalidValue;
    if (apply->dy != in) return hipErrorInvalidValue;   // the gradient is the conv input
    a.bz = (const float*)apply->z; a.bmask = (const float*)apply->mask; a.bmscale = apply->mscale;
    a.bmshift = apply->mshift; a.brows = *apply->rows; a.dz_out = (float*)apply->dz_out;
  }
  a.groups = groups; a.vec_stride = vec_stride;
  a.in = (const float*)in; a.scale = scale; a.shift = shift; a.wpack = (const float*)wpack;
  a.res = (const float*)res; a.y_out = (float*)y_out;
  if (in_rows) a.in_rows = *in_rows; else a.in_rows = BnRows{};
  a.out = (float*)out; a.st = st; a.add_g = (const float*)add_g; a.add_mask = (const float*)add_mask;
  a.N = N; a.H = H; a.tiles = N * (H / (C == 64 ? 4 : 8));
  WgradTiledF32Args wa{};
  if (pair) {
    const int wtiles = N * (H / (C == 64 ? 4 : 8));
    if (!apply || pair->rows < 1 || pair->rows > wtiles) return hipErrorInvalidValue;
    wa.x = (const float*)pair->x; wa.scale = pair->scale; wa.shift = pair->shift; wa.dz = (const float*)pair->dz;
    wa.partial = pair->partial; wa.N = N; wa.H = H; wa.tiles = wtiles;
  }
  const WgradTiledF32Args* wp = pair ? &wa : nullptr;
  const int wr = pair ? pair->rows : 0;
  if (C == 16 && W == 32) return conv_tiled_f32_launch_t<16, 32>(a, grid, s, wp, wr);
  if (C == 32 && W == 16) return conv_tiled_f32_launch_t<32, 16>(a, grid, s, wp, wr);
  if (C == 64 && W == 8) return conv_tiled_f32_launch_t<64, 8>(a, grid, s, wp, wr);
  return hipErrorInvalidValue;
}

template <int C, int W>
static hipError_t wgrad_tiled_f32_launch_t(const WgradTiledF32Args& a, int rows, hipStream_t s) {
  using Cfg = WgradTiledF32Cfg<C, W>;
  static_assert(Cfg::LDS <= 48 * 1024, "dynamic LDS within the default limit");
  DDG_LAUNCH((wgrad_tiled_f32_kernel<C, W>), dim3(rows), dim3(256), Cfg::LDS, s, a);
  return hipGetLastError();
}

// Same arguments and rules as wgrad_tiled_launch for the stride-1 shapes.
hipError_t wgrad_tiled_f32_launch(const void* x, const float* scale, const float* shift, const void* dz,
                                  const WgradFuse* fuse, float* partial, int N, int H, int W, int C, int rows,
                                  hipStream_t s) {
  WgradTiledF32Args a{};
  a.x = (const float*)x; a.scale = scale; a.shift = shift; a.dz = (const float*)dz; a.partial = partial;
  if (fuse) {
    a.dy = (const float*)fuse->dy; a.mask = (const float*)fuse->mask; a.mscale = fuse->mscale; a.mshift = fuse->mshift;
    a.zc = (const float*)fuse->z; a.coef = fuse->coef; a.dz_out = (float*)fuse->dz_out;
    if (fuse->rows) a.rows = *fuse->rows;
    if (!a.zc || !a.dz_out || (!a.coef && !a.rows.partial)) return hipErrorInvalidValue;
  } else if (!dz) return hipErrorInvalidValue;
  if ((size_t)N * H * W * C >= ((size_t)1 << 31)) return hipErrorInvalidValue;
  a.N = N; a.H = H; a.tiles = N * (H / (C == 64 ? 4 : 8));
  if (rows < 1 || rows > a.tiles) return hipErrorInvalidValue;
  if (C == 16 && W == 32) return wgrad_tiled_f32_launch_t<16, 32>(a, rows, s);
  if (C == 32 && W == 16) return wgrad_tiled_f32_launch_t<32, 16>(a, rows, s);
  if (C == 64 && W == 8) return wgrad_tiled_f32_launch_t<64, 8>(a, rows, s);
  return hipErrorInvalidValue;
}

}  // namespace ddg
