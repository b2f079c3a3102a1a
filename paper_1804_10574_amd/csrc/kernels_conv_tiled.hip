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
#include "ddg_wgrad_tiled.h"
#include <cstdlib>

namespace ddg {

struct ConvTiledArgs {
  const bf16_t* in;        // [N,H,W,C]
  const bf16_t* res;       // optional (RES kernels): input = relu(in*scale+shift + res), same layout
  bf16_t* y_out;           // optional (RES kernels): that input is also stored here (tile rows only)
  const float* scale;      // optional input transform relu(in*scale+shift)
  const float* shift;
  BnRows in_rows;          // in_rows.partial != null: scale/shift come from these partial rows
  const bf16_t* wpack;     // packed operand [ks][C/16][64][8]
  bf16_t* out;             // [N,H,W,C]
  ConvStat st;             // epilogue statistics: partial rows [grid][2][C]
  const bf16_t* add_g;     // optional epilogue term, same layout as out
  const bf16_t* add_mask;  // add_g counts only where add_mask > 0
  // XF_APPLY kernels: `in` is dy, the gradient w.r.t. the ReLU output after a batch norm, and the
  // convolved tensor is dz = A*g + B*bz + C0 with g = dy where bmask*bmscale+bmshift > 0 (bmask
  // null: g = dy); A, B, C0 derive from the partial rows `brows` of that BN's backward sums.
  // dz is formed while staging and also stored to dz_out (tile rows only).
  const bf16_t* bz; const bf16_t* bmask; const float* bmscale; const float* bmshift;
  BnBwdRows brows; bf16_t* dz_out;
  int N, H;                // N counts the images of all groups
  int tiles;               // N * H/8
  // groups > 1: the batch is `groups` independent minibatches laid end to end (batch-norm
  // statistics are per minibatch). A workgroup works on one group only: workgroups
  // [g*grid/groups, (g+1)*grid/groups) take group g, write that group's statistics rows
  // (rows are indexed by workgroup), and use that group's input transform: in_rows.partial and
  // st.partial advance by rows*2*C per group, the per-channel vectors by vec_stride floats.
  int groups;
  int vec_stride;
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

// Waves per SIMD the register allocation aims for (more co-resident workgroups when several
// streams run): the largest value each variant reaches without spilling.
// What staging does to the loaded input: nothing or relu(in*scale+shift) (decided at run time),
// the residual-block output relu(in*scale+shift + res), or the batch-norm backward formula
// (XF_APPLY: the ReLU mask is the BN's own conv output bz; XF_APPLY_MASK: a separate tensor).
enum { XF_PLAIN = 0, XF_RES = 1, XF_APPLY = 2, XF_APPLY_MASK = 3 };

constexpr int conv_tiled_waves(int C, int MODE, int XF) {
  return C == 64 ? (XF != XF_PLAIN ? 1 : 2)
                 : (((C == 32 && (XF != XF_PLAIN || MODE == 2)) || (C == 16 && XF >= XF_APPLY && MODE == 2)) ? 2 : 3);
}

// MODE is the epilogue's statistics mode, fixed at compile time: 0 none, 1 sum / sum of squares
// of the stored output (forward), 2 the BN-backward sums of the layer below (input gradient).
//
// Instruction count matters as much as bytes here (a wave64 VALU instruction occupies its SIMD
// for four cycles, and these kernels run a few microseconds): the staging map of a thread is
// computed once, LDS fragment addresses are one per-lane register per k-step plus an
// instruction immediate per pixel block, fragment reads are unconditional 16-byte reads, the
// tensors the epilogue needs are requested before the MFMA phase, and fp32 -> bf16 uses the
// packed hardware conversion.
// RES: the input is the output of the residual block before, y = relu(in*scale+shift + res),
// formed while staging and written to y_out by the workgroup that owns the rows.
// bidx of gdim: this workgroup's index in the launch (or in the part of a launch this work has).
template <int C, int W, int MODE, int XF>
__device__ __forceinline__ void conv3x3_tiled_body(const ConvTiledArgs& a, unsigned char* tile, int bidx, int gdim) {
  using Cfg = ConvTiledCfg<C, W>;
  constexpr bool RES = XF == XF_RES, APPLY = XF == XF_APPLY || XF == XF_APPLY_MASK;
  constexpr int TH = Cfg::TH, WC = Cfg::WC, PIX = Cfg::PIX, CH = Cfg::CH, NCHUNK = Cfg::NCHUNK;
  constexpr int PT = Cfg::PER_THREAD, KSTEPS = Cfg::KSTEPS, PG = Cfg::PG, COB = Cfg::COB;
  constexpr bool RAGGED_K = (9 * C) % 32 != 0;   // the last k-step runs past tap 8 for some lanes

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lg = lane >> 4;
  const int pgrp = wave % PG, cb = wave / PG;
  const int tiles_per_img = a.H / TH;
  // this workgroup's group, its index among the group's workgroups, the group's tile range
  const int g1 = gdim / a.groups;
  const int grp = bidx / g1, bl = bidx - grp * g1;
  const int tiles_g = a.tiles / a.groups, t_end = (grp + 1) * tiles_g;

  // ---- staging map (the same for every tile): chunk v = tid + i*256 -> halo pixel, 8 channels
  const int my_ch = tid % CH;
  int goff[PT];      // element offset of the chunk relative to the tile's first pixel (row r0, column 0)
  unsigned srows = 0;  // 4 bits per chunk: halo row 0..9 of the chunk + 1; 0: no chunk, or a pad column (stays zero)
  int loff[PT];      // LDS byte offset
#pragma unroll
  for (int i = 0; i < PT; ++i) {
    const int v = tid + i * 256;
    const int px = v / CH;
    const int rr = px / WC, cc = px - rr * WC;
    const bool col_ok = v < NCHUNK && cc >= 1 && cc <= W;
    srows |= (col_ok ? (unsigned)(rr + 1) : 0u) << (4 * i);
    goff[i] = ((rr - 1) * W + (cc - 1)) * C + my_ch * 8;
    loff[i] = v < NCHUNK ? px * PIX + my_ch * 16 : -1;
  }
  uint4 stage[PT], stage2[(RES || APPLY) ? PT : 1], stage3[XF == XF_APPLY_MASK ? PT : 1];
  unsigned inimg = 0;   // bit i: chunk i of the tile in flight lies inside the image
  unsigned tile_base = 0;   // element offset of the staged tile's first pixel (the host checks 32 bits suffice)
  auto issue_loads = [&](int t) {
    const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
    const unsigned tb = (unsigned)((n * a.H + r0) * W) * C;
    tile_base = tb;
    inimg = 0;
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      stage[i] = make_uint4(0, 0, 0, 0);
      const int sr = (int)((srows >> (4 * i)) & 15u) - 1;   // halo row, -1: nothing to load
      const int ih = r0 - 1 + sr;
      if (sr >= 0 && ih >= 0 && ih < a.H) {
        inimg |= 1u << i;
        stage[i] = *reinterpret_cast<const uint4*>(a.in + tb + goff[i]);
        if (RES) stage2[i] = *reinterpret_cast<const uint4*>(a.res + tb + goff[i]);
        if (APPLY) stage2[i] = *reinterpret_cast<const uint4*>(a.bz + tb + goff[i]);
        if (XF == XF_APPLY_MASK) stage3[i] = *reinterpret_cast<const uint4*>(a.bmask + tb + goff[i]);
      }
    }
  };
  int t = grp * tiles_g + bl;
  if (t < t_end) issue_loads(t);

  // ---- this wave's weights: KSTEPS fragments of its output-channel block
  uint4 wf[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks)
    wf[ks] = *reinterpret_cast<const uint4*>(a.wpack + ((size_t)(ks * COB + cb) * 64 + lane) * 8);

  // ---- LDS fragment addresses: lane part + k-step part in a register, pixel block as immediate
  // pixel of block i, lane l16: pt = (pgrp*4 + i)*16 + l16; its row/column split is additive in i
  const int ptl = pgrp * 64 + l16;
  const int lane_base = ((ptl / W) * WC + (ptl % W)) * PIX;
  int kaddr[KSTEPS];
  bool klast_ok = true;
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) {
    const int kidx = (ks * 4 + lg) * 8;
    const int tap = kidx / C, c0 = kidx % C;
    const bool ok = tap < 9;
    if (ks == KSTEPS - 1) klast_ok = ok;
    const int tp = ok ? tap : 0;
    kaddr[ks] = lane_base + ((tp / 3) * WC + (tp % 3)) * PIX + c0 * 2;
  }

  // ---- per-channel transform of the input (while the first tile's loads are in flight); the
  // vectors stay in LDS and a thread reads its 8 channels when it stages (registers are scarce)
  const bool xform = !APPLY && (a.scale != nullptr || a.in_rows.partial != nullptr);
  __shared__ __align__(16) float s_sc[APPLY ? 4 : C], s_sh[APPLY ? 4 : C];
  // XF_APPLY: A, B, C0 of the formula, then the mask's scale and shift
  __shared__ __align__(16) float s_coef[APPLY ? 5 * C : 4];
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
    const unsigned stage_base = tile_base;   // of the tile held in the registers
#pragma unroll
    for (int i = 0; i < PT; ++i) {
      if (loff[i] >= 0) {
        uint4 q = stage[i];
        if (APPLY && ((inimg >> i) & 1u)) {
          auto ld8 = [&](const float* p, float (&d)[8]) {
            *reinterpret_cast<float4*>(&d[0]) = *reinterpret_cast<const float4*>(p + my_ch * 8);
            *reinterpret_cast<float4*>(&d[4]) = *reinterpret_cast<const float4*>(p + my_ch * 8 + 4);
          };
          float g[8], zz[8], k0[8], k1[8];
          Store<bf16_t>::unpack_vec(q, g);
          Store<bf16_t>::unpack_vec(stage2[i], zz);
          if (a.bmask) {
            float mk[8];
            Store<bf16_t>::unpack_vec(XF == XF_APPLY_MASK ? stage3[i] : stage2[i], mk);
            ld8(&s_coef[3 * C], k0); ld8(&s_coef[4 * C], k1);
#pragma unroll
            for (int j = 0; j < 8; ++j) g[j] = (mk[j] * k0[j] + k1[j]) > 0.f ? g[j] : 0.f;
          }
          ld8(&s_coef[C], k0); ld8(&s_coef[2 * C], k1);
#pragma unroll
          for (int j = 0; j < 8; ++j) zz[j] = k0[j] * zz[j] + k1[j];
          ld8(&s_coef[0], k0);
#pragma unroll
          for (int j = 0; j < 8; ++j) g[j] = k0[j] * g[j] + zz[j];
          q.x = Store<bf16_t>::pack2(g[0], g[1]); q.y = Store<bf16_t>::pack2(g[2], g[3]);
          q.z = Store<bf16_t>::pack2(g[4], g[5]); q.w = Store<bf16_t>::pack2(g[6], g[7]);
          const unsigned sr1 = (srows >> (4 * i)) & 15u;   // halo row + 1
          if (sr1 >= 2 && sr1 <= TH + 1)
            *reinterpret_cast<uint4*>(a.dz_out + stage_base + goff[i]) = q;
        }
        if (xform && ((inimg >> i) & 1u)) {
          float f[8], tsc[8], tsh[8];
          *reinterpret_cast<float4*>(&tsc[0]) = *reinterpret_cast<const float4*>(&s_sc[my_ch * 8]);
          *reinterpret_cast<float4*>(&tsc[4]) = *reinterpret_cast<const float4*>(&s_sc[my_ch * 8 + 4]);
          *reinterpret_cast<float4*>(&tsh[0]) = *reinterpret_cast<const float4*>(&s_sh[my_ch * 8]);
          *reinterpret_cast<float4*>(&tsh[4]) = *reinterpret_cast<const float4*>(&s_sh[my_ch * 8 + 4]);
          Store<bf16_t>::unpack_vec(q, f);
          if (RES) {
            float r[8];
            Store<bf16_t>::unpack_vec(stage2[i], r);
#pragma unroll
            for (int j = 0; j < 8; ++j) f[j] = f[j] * tsc[j] + tsh[j] + r[j];
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) f[j] = f[j] * tsc[j] + tsh[j];
          }
#pragma unroll
          for (int j = 0; j < 8; ++j) f[j] = f[j] > 0.f ? f[j] : 0.f;
          q.x = Store<bf16_t>::pack2(f[0], f[1]); q.y = Store<bf16_t>::pack2(f[2], f[3]);
          q.z = Store<bf16_t>::pack2(f[4], f[5]); q.w = Store<bf16_t>::pack2(f[6], f[7]);
          // the tile's own rows (halo rows 1..8) are this workgroup's to store
          const unsigned sr1 = (srows >> (4 * i)) & 15u;   // halo row + 1
          if (RES && a.y_out && sr1 >= 2 && sr1 <= TH + 1)
            *reinterpret_cast<uint4*>(a.y_out + stage_base + goff[i]) = q;
        }
        *reinterpret_cast<uint4*>(tile + loff[i]) = q;
      }
    }
  };

  float ssum[4] = {0.f, 0.f, 0.f, 0.f}, ssq[4] = {0.f, 0.f, 0.f, 0.f};
  // mode 2: per-channel constants of the BN below (mean, invstd, mask scale, mask shift) in LDS;
  // a lane reads those of its 4 channels in the epilogue
  __shared__ __align__(16) float s_below[MODE == 2 ? 4 * C : 4];
  const bf16_t* st_mask = reinterpret_cast<const bf16_t*>(a.st.mask);
  const bf16_t* st_z = reinterpret_cast<const bf16_t*>(a.st.z);
  const bool two_tensors = MODE == 2 && st_z != st_mask;
  if (MODE == 2) {
    if (tid < C) {
      s_below[tid] = a.st.zmean[tid]; s_below[C + tid] = a.st.zinvstd[tid];
      s_below[2 * C + tid] = a.st.mscale ? a.st.mscale[tid] : 1.f;
      s_below[3 * C + tid] = a.st.mscale ? a.st.mshift[tid] : 0.f;
    }
    // (made visible by the barriers of the tile loop before any epilogue runs)
  }
  // output element offset of (block 0, this lane) inside a tile; block i adds i*16*C
  const int out_lane = ptl * C + cb * 16 + lg * 4;

  for (; t < t_end; t += g1) {
    __syncthreads();            // the previous tile has been consumed
    write_stage();
    __syncthreads();
    const int tn = t + g1;
    if (tn < t_end) issue_loads(tn);   // in flight during the MFMA phase

    // what the epilogue reads, requested now
    const int n = t / tiles_per_img, r0 = (t - n * tiles_per_img) * TH;
    const unsigned obase = (unsigned)((n * a.H + r0) * W) * C + out_lane;
    uint2 eg[4], em[4], ek[4], ez[4];
    if (a.add_g) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        eg[i] = *reinterpret_cast<const uint2*>(a.add_g + obase + i * 16 * C);
        if (a.add_mask) em[i] = *reinterpret_cast<const uint2*>(a.add_mask + obase + i * 16 * C);
      }
    }
    if (MODE == 2) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        ek[i] = *reinterpret_cast<const uint2*>(st_mask + obase + i * 16 * C);
        if (two_tensors) ez[i] = *reinterpret_cast<const uint2*>(st_z + obase + i * 16 * C);
      }
    }

    f32x4_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) {
      const unsigned char* kp = tile + kaddr[ks];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int blk = (((i * 16) / W) * WC + (i * 16) % W) * PIX;   // constant after unrolling
        uint4 af = *reinterpret_cast<const uint4*>(kp + blk);
        if (RAGGED_K && ks == KSTEPS - 1 && !klast_ok) af = make_uint4(0, 0, 0, 0);
        acc[i] = Mma<bf16_t>::mma(wf[ks], af, acc[i]);
      }
    }

    // epilogue: lane = pixel l16 of block i, channels cb*16 + lg*4 .. +3
    auto lo = [](uint32_t u) { return __uint_as_float(u << 16); };
    auto hi = [](uint32_t u) { return __uint_as_float(u & 0xffff0000u); };
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v[4] = {acc[i][0], acc[i][1], acc[i][2], acc[i][3]};
      if (a.add_g) {
        float g[4] = {lo(eg[i].x), hi(eg[i].x), lo(eg[i].y), hi(eg[i].y)};
        if (a.add_mask) {
          const float mk[4] = {lo(em[i].x), hi(em[i].x), lo(em[i].y), hi(em[i].y)};
#pragma unroll
          for (int j = 0; j < 4; ++j) g[j] = (mk[j] > 0.f) ? g[j] : 0.f;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] += g[j];
      }
      uint2 o;
      o.x = Store<bf16_t>::pack2(v[0], v[1]); o.y = Store<bf16_t>::pack2(v[2], v[3]);
      float bmu[4], bis[4], zz[4];
      if (MODE == 2) {
        // the gradient leaves this kernel already multiplied by the ReLU mask of the layer below
        // (every reader of it applies that mask first, so it is applied once, here)
        const float mk[4] = {lo(ek[i].x), hi(ek[i].x), lo(ek[i].y), hi(ek[i].y)};
        const int cq = cb * 16 + lg * 4;
        const float4 bmu4 = *reinterpret_cast<const float4*>(&s_below[cq]);
        const float4 bis4 = *reinterpret_cast<const float4*>(&s_below[C + cq]);
        const float4 bms4 = *reinterpret_cast<const float4*>(&s_below[2 * C + cq]);
        const float4 bmh4 = *reinterpret_cast<const float4*>(&s_below[3 * C + cq]);
        bmu[0] = bmu4.x; bmu[1] = bmu4.y; bmu[2] = bmu4.z; bmu[3] = bmu4.w;
        bis[0] = bis4.x; bis[1] = bis4.y; bis[2] = bis4.z; bis[3] = bis4.w;
        const float bms[4] = {bms4.x, bms4.y, bms4.z, bms4.w}, bmh[4] = {bmh4.x, bmh4.y, bmh4.z, bmh4.w};
        if (two_tensors) { zz[0] = lo(ez[i].x); zz[1] = hi(ez[i].x); zz[2] = lo(ez[i].y); zz[3] = hi(ez[i].y); }
        else { zz[0] = mk[0]; zz[1] = mk[1]; zz[2] = mk[2]; zz[3] = mk[3]; }
        const uint32_t k0 = (mk[0] * bms[0] + bmh[0]) > 0.f ? 0x0000ffffu : 0u;
        const uint32_t k1 = (mk[1] * bms[1] + bmh[1]) > 0.f ? 0xffff0000u : 0u;
        const uint32_t k2 = (mk[2] * bms[2] + bmh[2]) > 0.f ? 0x0000ffffu : 0u;
        const uint32_t k3 = (mk[3] * bms[3] + bmh[3]) > 0.f ? 0xffff0000u : 0u;
        o.x &= k0 | k1; o.y &= k2 | k3;
      }
      *reinterpret_cast<uint2*>(a.out + obase + i * 16 * C) = o;
      if (MODE != 0) {
        const float r[4] = {lo(o.x), hi(o.x), lo(o.y), hi(o.y)};   // the values as stored
        if (MODE == 1) {
#pragma unroll
          for (int j = 0; j < 4; ++j) { ssum[j] += r[j]; ssq[j] += r[j] * r[j]; }
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            ssum[j] += r[j];
            ssq[j] += r[j] * ((zz[j] - bmu[j]) * bis[j]);
          }
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
      a.st.partial[((size_t)bidx * 2 + which) * C + c] = s;
    }
  }
}

template <int C, int W, int MODE, int XF = XF_PLAIN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(conv_tiled_waves(C, MODE, XF)))) void conv3x3_tiled_kernel(ConvTiledArgs a) {
  extern __shared__ __align__(16) unsigned char tile[];
  conv3x3_tiled_body<C, W, MODE, XF>(a, tile, blockIdx.x, gridDim.x);
}

// Two independent pieces of backward work of one shape in one launch (a launch costs a few
// microseconds of dispatch whatever it carries): the first conv_grid workgroups run the
// input-gradient kernel of a unit (which forms its dz while staging), the others the plain weight
// gradient of the unit above it, whose dz the launch before has stored.
template <int C, int W, int MODE, int XF>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(conv_tiled_waves(C, MODE, XF)))) void bwd_pair_kernel(ConvTiledArgs ca, WgradTiledArgs wa, int conv_grid, int wg_rows) {
  extern __shared__ __align__(16) unsigned char tile[];
  const int b = blockIdx.x;
  if (b < conv_grid) {
    conv3x3_tiled_body<C, W, MODE, XF>(ca, tile, b, conv_grid);
  } else {
    const int v = b - conv_grid;
    wgrad_tiled_body<C, C, W, false>(wa, tile, v % wg_rows, v / wg_rows, wg_rows);
  }
}

// Workgroups per launch for a layer with C channels (and so the number of partial statistics
// rows the launch writes). Every workgroup loads its wave's weights and adds up the rows of the
// layer before, so on the small feature maps fewer, longer-running workgroups mean less L2
// traffic. DDG_TUNE_CONV_GRID_C16/_C32/_C64 override the defaults within [32, 2048].
static int conv_tiled_cap(int C) {
  int cap = C == 16 ? 256 : (C == 32 ? 128 : 96);   // (measured: c64 flat between 64 and 96, worse at 48 and at 128+)
  const char* name = C == 16 ? "DDG_TUNE_CONV_GRID_C16" : (C == 32 ? "DDG_TUNE_CONV_GRID_C32" : "DDG_TUNE_CONV_GRID_C64");
  if (const char* e = getenv(name)) {
    const int v = atoi(e);
    if (v >= 32 && v <= 2048) cap = v;
  }
  return cap;
}

// No launch uses more workgroups than this (sizes row buffers).
int conv_tiled_max_grid() {
  int m = conv_tiled_cap(16);
  if (conv_tiled_cap(32) > m) m = conv_tiled_cap(32);
  if (conv_tiled_cap(64) > m) m = conv_tiled_cap(64);
  return m;
}

int conv_tiled_grid(int N, int H, int W, int Cin, int Cout, int R, int stride, int dtype) {
  if (dtype == F32) return conv_tiled_f32_grid(N, H, W, Cin, Cout, R, stride);
  if (dtype != BF16 || R != 3 || stride != 1 || Cin != Cout) return 0;
  if (!((Cin == 16 && W == 32) || (Cin == 32 && W == 16) || (Cin == 64 && W == 8))) return 0;
  if (H % 8 != 0) return 0;
  const int tiles = N * (H / 8);
  const int cap = conv_tiled_cap(Cin);
  return tiles < cap ? tiles : cap;
}

template <int C, int W>
static hipError_t conv_tiled_launch_t(const ConvTiledArgs& a, int grid, hipStream_t s, const WgradTiledArgs* wa, int wg_rows) {
  using Cfg = ConvTiledCfg<C, W>;
  if (wa) {
    using WCfg = WgradTiledCfg<C, C, W>;
    if (!a.bz || a.st.mode == 1 || a.scale || a.in_rows.partial || !a.brows.partial || !a.dz_out || wg_rows < 1)
      return hipErrorInvalidValue;
    constexpr int lds = Cfg::TILE_BYTES > WCfg::LDS ? Cfg::TILE_BYTES : WCfg::LDS;
    static_assert(lds <= 48 * 1024, "dynamic LDS within the default limit");
    const bool own_mask = a.bmask && a.bmask != a.bz;
    const dim3 g(grid + wg_rows * WCfg::OT);
    if (a.st.mode == 2) {
      if (own_mask) DDG_LAUNCH((bwd_pair_kernel<C, W, 2, XF_APPLY_MASK>), g, dim3(256), lds, s, a, *wa, grid, wg_rows);
      else DDG_LAUNCH((bwd_pair_kernel<C, W, 2, XF_APPLY>), g, dim3(256), lds, s, a, *wa, grid, wg_rows);
    } else {
      if (own_mask) DDG_LAUNCH((bwd_pair_kernel<C, W, 0, XF_APPLY_MASK>), g, dim3(256), lds, s, a, *wa, grid, wg_rows);
      else DDG_LAUNCH((bwd_pair_kernel<C, W, 0, XF_APPLY>), g, dim3(256), lds, s, a, *wa, grid, wg_rows);
    }
    return hipGetLastError();
  }
  if (a.res) {
    if (a.st.mode != 1 || !(a.scale || a.in_rows.partial)) return hipErrorInvalidValue;
    DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 1, XF_RES>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  } else if (a.bz) {
    // input-gradient kernel that applies the batch-norm backward formula to its input
    if (a.st.mode == 1 || a.scale || a.in_rows.partial || !a.brows.partial || !a.dz_out) return hipErrorInvalidValue;
    const bool own_mask = a.bmask && a.bmask != a.bz;
    if (a.st.mode == 2) {
      if (own_mask) DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 2, XF_APPLY_MASK>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
      else DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 2, XF_APPLY>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
    } else {
      if (own_mask) DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 0, XF_APPLY_MASK>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
      else DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 0, XF_APPLY>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
    }
  } else if (a.st.mode == 1) DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 1>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  else if (a.st.mode == 2) DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 2>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  else DDG_LAUNCH((conv3x3_tiled_kernel<C, W, 0>), dim3(grid), dim3(256), Cfg::TILE_BYTES, s, a);
  return hipGetLastError();
}

hipError_t conv_tiled_launch(const void* in, const float* scale, const float* shift, const BnRows* in_rows,
                             const void* wpack, void* out, const ConvStat& st, const void* add_g,
                             const void* add_mask, int N, int H, int W, int C, int grid, hipStream_t s,
                             const void* res, void* y_out, int groups, int vec_stride, const WgradFuse* apply,
                             const WgradPair* pair) {
  if (groups < 1 || N % groups != 0 || grid % groups != 0) return hipErrorInvalidValue;
  if (groups > 1 && (st.mode != 1 || add_g)) return hipErrorInvalidValue;   // forward only
  ConvTiledArgs a{};
  if (apply) {
    if (groups != 1 || res || !apply->rows) return hipErrorInvalidValue;
    if (apply->dy != in) return hipErrorInvalidValue;   // the gradient is the conv input
    a.bz = (const bf16_t*)apply->z; a.bmask = (const bf16_t*)apply->mask; a.bmscale = apply->mscale;
    a.bmshift = apply->mshift; a.brows = *apply->rows; a.dz_out = (bf16_t*)apply->dz_out;
  }
  a.groups = groups; a.vec_stride = vec_stride;
  a.in = (const bf16_t*)in; a.scale = scale; a.shift = shift; a.wpack = (const bf16_t*)wpack;
  a.res = (const bf16_t*)res; a.y_out = (bf16_t*)y_out;
  if (in_rows) a.in_rows = *in_rows; else a.in_rows = BnRows{};
  a.out = (bf16_t*)out; a.st = st; a.add_g = (const bf16_t*)add_g;
  a.add_mask = (const bf16_t*)add_mask; a.N = N; a.H = H; a.tiles = N * (H / 8);
  if ((size_t)N * H * W * C >= ((size_t)1 << 31)) return hipErrorInvalidValue;   // 32-bit element offsets inside
  WgradTiledArgs wa{};
  if (pair) {
    if (!apply || pair->rows < 1 || pair->rows > N * (H / 8)) return hipErrorInvalidValue;
    wa.x = (const bf16_t*)pair->x; wa.scale = pair->scale; wa.shift = pair->shift; wa.dz = (const bf16_t*)pair->dz;
    wa.partial = pair->partial; wa.N = N; wa.H = H; wa.W = W; wa.tiles = N * (H / 8);
  }
  const WgradTiledArgs* wp = pair ? &wa : nullptr;
  const int wr = pair ? pair->rows : 0;
  if (C == 16 && W == 32) return conv_tiled_launch_t<16, 32>(a, grid, s, wp, wr);
  if (C == 32 && W == 16) return conv_tiled_launch_t<32, 16>(a, grid, s, wp, wr);
  if (C == 64 && W == 8) return conv_tiled_launch_t<64, 8>(a, grid, s, wp, wr);
  return hipErrorInvalidValue;
}

}  // namespace ddg
