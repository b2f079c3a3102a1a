// Convolution (forward and input-gradient) for wide bf16 layers: 1x1 and 3x3, stride 1,
// contraction channels a power of two >= 64, output channels a multiple of 128 (the bottleneck
// stage of an ImageNet-shaped ResNet: 1024 -> 256 -> 256 -> 1024 at 14x14). By arithmetic
// intensity these layers are matrix-core bound, so this is a GEMM-class kernel: a workgroup
// owns a 64-pixel x 128-channel output tile and walks over the contraction in chunks of 64 or
// 128 channels of one tap, one barrier per chunk.
//
//   pixel operand:  64 rows x one chunk of channels, through registers into one of two LDS
//                   buffers (rows padded by 16 bytes, so the 16 rows of a fragment read fall
//                   into distinct bank groups); a 3x3 tap is a shifted pixel row, out-of-image
//                   rows are zero: no im2col matrix.
//   weight operand: the packed operand of the generic kernel is already fragment-ordered
//                   ([k-step][16-channel block][lane][8]), so a wave loads the fragments it
//                   multiplies with straight from global memory into registers, 1 KiB
//                   contiguous per load; weights never touch LDS and no two waves of a
//                   workgroup load the same fragment.
//   Loads are requested two chunks ahead (named register sets, loop body written out twice)
//   and none of them is conditional, so the compiler's wait counts leave the newest in flight.
//
// Eight waves: 4 (32 channels each) x 2 (halves of a chunk's k-steps). A wave owns all 64
// pixels x 32 channels = 8 accumulator tiles of mfma_f32_16x16x32_bf16 (weights as rows, so a
// lane holds 4 consecutive channels of one pixel) for its half of the contraction; two waves
// per SIMD let one wave's LDS and global traffic run under the other's MFMAs. The two halves
// meet in an fp32 LDS tile, from which stores (and the optional masked shortcut-gradient term)
// are 16-byte accesses along the channels; the batch-norm statistics of the stored values go
// to one partial row per 64-pixel tile.
#include "ddg_device.h"
#include "ddg_kernels.h"
#include <cstdlib>

namespace ddg {

struct ConvWideArgs {
  const bf16_t* in;        // [M][IC]
  const bf16_t* wpack;     // [k-step][OC/16][64][8], k = tap*IC + channel
  bf16_t* out;             // [M][OC]
  float* stat_partial;     // [gridDim.x][2][OC] or null
  const bf16_t* add_g;     // optional: out += add_g (where add_mask > 0, if given)
  const bf16_t* add_mask;
  const float* scale;      // optional (XFORM kernels): the conv input is relu(in*scale + shift), per input channel
  const float* shift;
  // STATS = 2 (input gradient): the outputs are an error gradient v; with the ReLU mask of the
  // layer below applied, g = (bmask*bmscale + bmshift > 0) ? v : 0 (bmask null: g = v), the rows
  // hold sum g and sum g*xhat of that layer's BN (xhat = (bz - bmean)*binvstd): its
  // bn_bwd_reduce pass comes for free. stat_partial receives the rows, and the stored output is
  // g (the mask is applied here, once; readers take the gradient as already masked).
  const bf16_t* bmask; const float* bmscale; const float* bmshift;
  const bf16_t* bz; const float* bmean; const float* binvstd;
  // optional second minibatch (blockIdx.z = 1; forward only): same weights, its own tensors
  const bf16_t* in_b; bf16_t* out_b; float* stat_partial_b; const float* scale_b; const float* shift_b;
  int M, H, W, HW, IC, OC, R;
};

namespace wide {
constexpr int BM = 64, BN = 128;
constexpr int OROW = BN * 4 + 16;                 // bytes per pixel row of the epilogue's fp32 tile
constexpr int prow_bytes(int BK) { return BK * 2 + 16; }          // bytes per staged pixel row
constexpr int pix_bytes(int BK) { return BM * prow_bytes(BK); }   // one pixel buffer
// dynamic LDS: the two pixel buffers, later reused by the epilogue's fp32 tile and statistics scratch
constexpr int lds_bytes(int BK) { return 2 * pix_bytes(BK) > BM * OROW ? 2 * pix_bytes(BK) : BM * OROW; }
}

// Registers that carry a thread's share of a chunk's pixel operand to LDS, and a wave's weight
// fragments of a chunk (used from the registers).
struct WidePix { uint4 p, q; bool ok, okq; };       // q: second row of the thread (BK = 128)
struct WideWts { uint4 w0, w1, w2, w3; };           // w2, w3: second k-step of the wave (BK = 128)

// XFORM: the input is turned into the activation it stands for, relu(in*scale + shift) (batch
// norm + ReLU of the layer before), while it is written to LDS; zero padding comes after that.
// BK: contraction channels per chunk (one barrier each). 128 halves the number of barriers; 64
// keeps the kernel at 128 registers, two workgroups per compute unit (launches with many tiles).
// STATS: 0 none, 1 sum / sum of squares of the stored outputs (forward), 2 the BN-backward sums of
// the layer below (input gradient).
// R: kernel size (1 or 3), a template parameter because the loop is instruction-issue bound: a
// chunk is only 8-16 MFMAs per wave, so every address or predicate instruction per chunk counts
// (tap validity is a 9-bit mask computed once, wave-uniform values live in scalar registers,
// addresses are a uniform pointer plus a 32-bit lane offset).
template <int STATS, bool XFORM, int BK, int R>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(BK == 64 ? 4 : 2))) void conv_wide_kernel(ConvWideArgs a) {
  using namespace wide;
  constexpr int PROW = prow_bytes(BK), P_BYTES = pix_bytes(BK), LDS = lds_bytes(BK);
  constexpr int UPR = BK / 8;                     // 16-byte units per staged pixel row
  constexpr bool TWO = BK == 128;                 // two rows per thread, two k-steps per wave
  constexpr int KSW = BK / 64;                    // k-steps per wave and chunk
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: scalar registers
  const int l16 = lane & 15, lg = lane >> 4;
  const int wn = wave & 3, kg = wave >> 2;        // 32-channel group; k-step of a chunk
  const bool second = blockIdx.z != 0;
  const bf16_t* __restrict__ g_in = second ? a.in_b : a.in;
  bf16_t* __restrict__ g_out = second ? a.out_b : a.out;
  float* __restrict__ g_stat = second ? a.stat_partial_b : a.stat_partial;
  const float* __restrict__ g_scale = second ? a.scale_b : a.scale;
  const float* __restrict__ g_shift = second ? a.shift_b : a.shift;
  const int m0 = blockIdx.x * BM;
  const int OCB = a.OC >> 4;
  const int cb0 = blockIdx.y * (BN / 16);
  const int cpt = a.IC / BK;                      // chunks per tap (a power of two)
  const int l2cpt = 31 - __clz(cpt);
  const int nchunks = R * R * cpt;

  // ---- staging map of the pixel operand: row tid/UPR (and 32 rows further for BK = 128),
  // 16-byte unit tid%UPR
  const int pc = tid % UPR, prow = tid / UPR;
  const int mA = m0 + prow, mB = mA + 32;
  const bool vA = mA < a.M, vB = TWO && mB < a.M;
  const int remA = (vA ? mA : 0) % a.HW, remB = (vB ? mB : 0) % a.HW;
  const int hA = remA / a.W, wA = remA - hA * a.W, hB = remB / a.W, wB = remB - hB * a.W;
  const int baseA = (vA ? mA : 0) * a.IC + pc * 8, baseB = (vB ? mB : 0) * a.IC + pc * 8;
  // bit t: tap t of this thread's row lies inside the image (R = 1: the row itself is valid)
  unsigned tapsA = 0, tapsB = 0;
#pragma unroll
  for (int t = 0; t < R * R; ++t) {
    const int dr = R == 3 ? t / 3 - 1 : 0, ds = R == 3 ? t % 3 - 1 : 0;
    tapsA |= (vA && hA + dr >= 0 && hA + dr < a.H && wA + ds >= 0 && wA + ds < a.W ? 1u : 0u) << t;
    tapsB |= (vB && hB + dr >= 0 && hB + dr < a.H && wB + ds >= 0 && wB + ds < a.W ? 1u : 0u) << t;
  }
  // this wave's weight fragments of k-step 0: channel blocks cb0 + wn*2, +1 (uniform pointer, lane
  // offset); k-step ks adds ks*wstep
  const bf16_t* wsrc = a.wpack + (size_t)(cb0 + wn * 2) * 64 * 8;
  const int wlane = lane * 8;
  const size_t wstep = (size_t)OCB * 64 * 8;      // elements per k-step of the packed operand

  // Chunk kc: 64 channels of one tap. Loads are issued two to three chunks before they are needed (the
  // memory latency is several times the time a chunk takes to contract). Nothing here is
  // conditional, so that the compiler can count the loads in flight and wait only for the
  // oldest: a row outside the image loads its own pixel instead and is zeroed when it is written
  // to LDS; a chunk index past the end repeats the last chunk (never used).
  auto issue_pix = [&](WidePix& r, int kc_want) __attribute__((always_inline)) {
    const int kc = kc_want < nchunks ? kc_want : nchunks - 1;
    const int tap = R == 3 ? kc >> l2cpt : 0, c0 = (kc & (cpt - 1)) * BK;
    int sh = 0;
    if (R == 3) { const int dr = tap / 3 - 1, ds = tap - (tap / 3) * 3 - 1; sh = (dr * a.W + ds) * a.IC; }
    const bf16_t* src = g_in + c0;                 // uniform
    r.ok = (tapsA >> tap) & 1u;
    r.p = *reinterpret_cast<const uint4*>(src + (baseA + (r.ok ? sh : 0)));
    if (TWO) {
      r.okq = (tapsB >> tap) & 1u;
      r.q = *reinterpret_cast<const uint4*>(src + (baseB + (r.okq ? sh : 0)));
    }
  };
  auto issue_wts = [&](WideWts& r, int kc_want) __attribute__((always_inline)) {
    const int kc = kc_want < nchunks ? kc_want : nchunks - 1;
    const bf16_t* wa = wsrc + (size_t)((kc * 2 + kg) * KSW) * wstep;   // uniform
    r.w0 = *reinterpret_cast<const uint4*>(wa + wlane);
    r.w1 = *reinterpret_cast<const uint4*>(wa + 64 * 8 + wlane);
    if (TWO) {
      r.w2 = *reinterpret_cast<const uint4*>(wa + wstep + wlane);
      r.w3 = *reinterpret_cast<const uint4*>(wa + wstep + 64 * 8 + wlane);
    }
  };
  // XFORM: scale and shift of all input channels, after the pixel buffers
  float* tab = reinterpret_cast<float*>(smem + LDS);
  if (XFORM) {
    for (int c = tid; c < a.IC; c += 512) { tab[c] = g_scale[c]; tab[a.IC + c] = g_shift[c]; }
    __syncthreads();
  }
  auto stash = [&](const WidePix& r, int buf, int kc) __attribute__((always_inline)) {
    unsigned char* P = smem + buf * P_BYTES;
    uint4 q = r.p, q2 = r.q;
    if (XFORM) {
      const int c = (kc & (cpt - 1)) * BK + pc * 8;     // this thread's 8 input channels of chunk kc
      float sc[8], sh[8];
      *reinterpret_cast<float4*>(&sc[0]) = *reinterpret_cast<const float4*>(&tab[c]);
      *reinterpret_cast<float4*>(&sc[4]) = *reinterpret_cast<const float4*>(&tab[c + 4]);
      *reinterpret_cast<float4*>(&sh[0]) = *reinterpret_cast<const float4*>(&tab[a.IC + c]);
      *reinterpret_cast<float4*>(&sh[4]) = *reinterpret_cast<const float4*>(&tab[a.IC + c + 4]);
      auto act = [&](uint4 v) __attribute__((always_inline)) {
        float f[8];
        Store<bf16_t>::unpack_vec(v, f);
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float t = f[e] * sc[e] + sh[e]; f[e] = t > 0.f ? t : 0.f; }
        uint4 o;
        o.x = Store<bf16_t>::pack2(f[0], f[1]); o.y = Store<bf16_t>::pack2(f[2], f[3]);
        o.z = Store<bf16_t>::pack2(f[4], f[5]); o.w = Store<bf16_t>::pack2(f[6], f[7]);
        return o;
      };
      q = act(q);
      if (TWO) q2 = act(q2);
    }
    *reinterpret_cast<uint4*>(P + prow * PROW + pc * 16) = r.ok ? q : make_uint4(0, 0, 0, 0);
    if (TWO) *reinterpret_cast<uint4*>(P + (prow + 32) * PROW + pc * 16) = r.okq ? q2 : make_uint4(0, 0, 0, 0);
  };

  f32x4_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  // this wave's k-steps of every chunk: waves 0-3 take the first half of its channels, waves 4-7 the rest
  const int poff = l16 * PROW + lg * 16 + kg * BK;             // + i*16*PROW (+ 64 for the second k-step)
  auto contract = [&](int buf, const WideWts& w) __attribute__((always_inline)) {
    const unsigned char* B = smem + buf * P_BYTES;
    uint4 pf[4], pg[TWO ? 4 : 1];
#pragma unroll
    for (int i = 0; i < 4; ++i) pf[i] = *reinterpret_cast<const uint4*>(B + poff + i * 16 * PROW);
    if (TWO) {
#pragma unroll
      for (int i = 0; i < 4; ++i) pg[i] = *reinterpret_cast<const uint4*>(B + poff + i * 16 * PROW + 64);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[i][0] = Mma<bf16_t>::mma(w.w0, pf[i], acc[i][0]);
      acc[i][1] = Mma<bf16_t>::mma(w.w1, pf[i], acc[i][1]);
    }
    if (TWO) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[i][0] = Mma<bf16_t>::mma(w.w2, pg[i], acc[i][0]);
        acc[i][1] = Mma<bf16_t>::mma(w.w3, pg[i], acc[i][1]);
      }
    }
  };

  // Pixel set c % 2 and weight set c % 2 carry chunk c. At the top of iteration c: LDS buffer
  // c % 2 holds the pixels of chunk c, the pixel sets hold chunks c+1 and c+2, the weight sets
  // chunks c and c+1. The loop body is written out twice so that every set is a named variable.
  WidePix p0, p1;
  WideWts w0, w1;
  issue_pix(p0, 0);
  issue_wts(w0, 0);
  stash(p0, 0, 0);
  issue_pix(p1, 1); issue_wts(w1, 1);
  issue_pix(p0, 2);
  __syncthreads();
  // one iteration: move the pixels of chunk c+1 from their registers to the other LDS buffer
  // (free since the barrier that ended iteration c-1) and request chunk c+4 into those
  // registers; contract chunk c with its weights and request the weights of chunk c+2
#define DDG_WIDE_STEP(c, pnext, wcur)                               \
  {                                                                 \
    if ((c) + 1 < nchunks) stash(pnext, ((c) + 1) & 1, (c) + 1);    \
    issue_pix(pnext, (c) + 3);                                      \
    contract((c) & 1, wcur);                                        \
    issue_wts(wcur, (c) + 2);                                       \
    __syncthreads();                                                \
  }
  for (int kc = 0; kc < nchunks; kc += 2) {
    DDG_WIDE_STEP(kc, p1, w0)
    if (kc + 1 >= nchunks) break;
    DDG_WIDE_STEP(kc + 1, p0, w1)
  }
#undef DDG_WIDE_STEP

  // ---- epilogue. The accumulators (lane = pixel i*16 + l16, channels (wn*2 + j)*16 +
  // lg*4 .. +3) go through LDS as fp32 [64 pixels][128 channels]: the two wave groups add their
  // halves of the contraction there (first group, then second: a fixed order), and memory then
  // sees 16-byte accesses, 256 contiguous bytes per pixel: thread = pixels (tid>>4) + 32*q,
  // channels (tid&15)*8 .. +7
  static_assert(2 * P_BYTES <= LDS && BM * OROW <= LDS && 32 * 2 * BN * 4 <= LDS, "pixel buffers, fp32 tile and statistics scratch fit");
  if (kg == 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        *reinterpret_cast<f32x4_t*>(smem + (i * 16 + l16) * OROW + ((wn * 2 + j) * 16 + lg * 4) * 4) = acc[i][j];
  }
  __syncthreads();
  if (kg == 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        f32x4_t* p = reinterpret_cast<f32x4_t*>(smem + (i * 16 + l16) * OROW + ((wn * 2 + j) * 16 + lg * 4) * 4);
        *p = *p + acc[i][j];
      }
  }
  __syncthreads();
  const int oc = tid & 15, orow = tid >> 4;       // orow 0..31
  float ssum[8], ssq[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { ssum[e] = 0.f; ssq[e] = 0.f; }
  float bmu[8], bis[8], bms[8], bmh[8];           // STATS = 2: constants of the BN below, this thread's 8 channels
  if (STATS == 2) {
    const int c = cb0 * 16 + oc * 8;
    auto ld8 = [&](const float* p, float (&d)[8], float dflt) __attribute__((always_inline)) {
      float4 lo = make_float4(dflt, dflt, dflt, dflt), hi = lo;
      if (p) { lo = *reinterpret_cast<const float4*>(p + c); hi = *reinterpret_cast<const float4*>(p + c + 4); }
      d[0] = lo.x; d[1] = lo.y; d[2] = lo.z; d[3] = lo.w; d[4] = hi.x; d[5] = hi.y; d[6] = hi.z; d[7] = hi.w;
    };
    ld8(a.bmean, bmu, 0.f); ld8(a.binvstd, bis, 1.f);
    ld8(a.bmscale, bms, 1.f); ld8(a.bmscale ? a.bmshift : nullptr, bmh, 0.f);
  }
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int row = orow + 32 * q, m = m0 + row;
    if (m < a.M) {
      float v[8];
      *reinterpret_cast<float4*>(&v[0]) = *reinterpret_cast<const float4*>(smem + row * OROW + oc * 32);
      *reinterpret_cast<float4*>(&v[4]) = *reinterpret_cast<const float4*>(smem + row * OROW + oc * 32 + 16);
      const size_t idx = (size_t)m * a.OC + cb0 * 16 + oc * 8;
      if (a.add_g) {
        float g[8];
        Store<bf16_t>::unpack_vec(*reinterpret_cast<const uint4*>(a.add_g + idx), g);
        if (a.add_mask) {
          float mk[8];
          Store<bf16_t>::unpack_vec(*reinterpret_cast<const uint4*>(a.add_mask + idx), mk);
#pragma unroll
          for (int e = 0; e < 8; ++e) g[e] = mk[e] > 0.f ? g[e] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += g[e];
      }
      uint4 o;
      o.x = Store<bf16_t>::pack2(v[0], v[1]); o.y = Store<bf16_t>::pack2(v[2], v[3]);
      o.z = Store<bf16_t>::pack2(v[4], v[5]); o.w = Store<bf16_t>::pack2(v[6], v[7]);
      if (STATS != 2) *reinterpret_cast<uint4*>(g_out + idx) = o;
      if (STATS == 1) {
        float r[8];
        Store<bf16_t>::unpack_vec(o, r);            // the values as stored
#pragma unroll
        for (int e = 0; e < 8; ++e) { ssum[e] += r[e]; ssq[e] += r[e] * r[e]; }
      }
      if (STATS == 2) {
        // the gradient leaves this kernel already multiplied by the ReLU mask of the layer below
        // (every reader of it applies that mask first, so it is applied once, here)
        float r[8], zz[8], mk[8];
        Store<bf16_t>::unpack_vec(o, r);
        const uint4 zq = *reinterpret_cast<const uint4*>(a.bz + idx);
        Store<bf16_t>::unpack_vec(zq, zz);
        uint4 mq = zq;
        if (a.bmask && a.bmask != a.bz) mq = *reinterpret_cast<const uint4*>(a.bmask + idx);
        Store<bf16_t>::unpack_vec(mq, mk);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float g = (!a.bmask || mk[e] * bms[e] + bmh[e] > 0.f) ? r[e] : 0.f;
          r[e] = g;
          ssum[e] += g;
          ssq[e] += g * ((zz[e] - bmu[e]) * bis[e]);
        }
        o.x = Store<bf16_t>::pack2(r[0], r[1]); o.y = Store<bf16_t>::pack2(r[2], r[3]);   // (exact: bf16 values or zeros)
        o.z = Store<bf16_t>::pack2(r[4], r[5]); o.w = Store<bf16_t>::pack2(r[6], r[7]);
        *reinterpret_cast<uint4*>(g_out + idx) = o;
      }
    }
  }
  if (STATS) {
    // per channel: the 32 row classes in a fixed order
    __syncthreads();                               // the fp32 tile has been read
    float* red = reinterpret_cast<float*>(smem);   // [32 row classes][2][128]
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      red[(orow * 2 + 0) * BN + oc * 8 + e] = ssum[e];
      red[(orow * 2 + 1) * BN + oc * 8 + e] = ssq[e];
    }
    __syncthreads();
    if (tid < 2 * BN) {
      const int which = tid / BN, c = tid % BN;
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < 32; ++r) s += red[(r * 2 + which) * BN + c];
      g_stat[((size_t)blockIdx.x * 2 + which) * a.OC + cb0 * 16 + c] = s;
    }
  }
}

template <int BK, int R>
static hipError_t conv_wide_dispatch(const ConvWideArgs& a, dim3 grid, int stats, bool xf, int IC, hipStream_t s) {
  const int tab_max = 2 * 2048 * (int)sizeof(float);
  const int lds = wide::lds_bytes(BK) + (xf ? 2 * IC * (int)sizeof(float) : 0);
  static bool attr_set = false;
  if (!attr_set) {
    const void* fns[5] = {reinterpret_cast<const void*>(&conv_wide_kernel<1, false, BK, R>),
                          reinterpret_cast<const void*>(&conv_wide_kernel<0, false, BK, R>),
                          reinterpret_cast<const void*>(&conv_wide_kernel<1, true, BK, R>),
                          reinterpret_cast<const void*>(&conv_wide_kernel<0, true, BK, R>),
                          reinterpret_cast<const void*>(&conv_wide_kernel<2, false, BK, R>)};
    for (const void* f : fns) {
      hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, wide::lds_bytes(BK) + tab_max);
      if (e != hipSuccess) return e;
    }
    attr_set = true;
  }
  if (stats == 2) {
    if (xf) return hipErrorInvalidValue;
    DDG_LAUNCH((conv_wide_kernel<2, false, BK, R>), grid, dim3(512), lds, s, a);
  } else if (stats == 1) {
    if (xf) DDG_LAUNCH((conv_wide_kernel<1, true, BK, R>), grid, dim3(512), lds, s, a);
    else DDG_LAUNCH((conv_wide_kernel<1, false, BK, R>), grid, dim3(512), lds, s, a);
  } else {
    if (xf) DDG_LAUNCH((conv_wide_kernel<0, true, BK, R>), grid, dim3(512), lds, s, a);
    else DDG_LAUNCH((conv_wide_kernel<0, false, BK, R>), grid, dim3(512), lds, s, a);
  }
  return hipGetLastError();
}

// Shapes the kernel covers (the module code asks before it plans a layer).
bool conv_wide_ok(int IC, int OC, int R, int stride, int dtype) {
  if (dtype != BF16 || stride != 1 || (R != 1 && R != 3)) return false;
  if (IC < 64 || (IC & (IC - 1)) != 0) return false;      // power of two: k = tap*IC + channel in the packed operand
  return OC % wide::BN == 0;
}
int conv_wide_rows(int M) { return (M + wide::BM - 1) / wide::BM; }

hipError_t conv_wide_launch(const void* in, const void* wpack, void* out, float* stat_partial, const void* add_g,
                            const void* add_mask, int N, int H, int W, int IC, int OC, int R, hipStream_t s,
                            const float* scale, const float* shift, const ConvWideSecond* second, const ConvStat* below) {
  if (!conv_wide_ok(IC, OC, R, 1, BF16)) return hipErrorInvalidValue;
  const size_t M = (size_t)N * H * W;
  if (M * (size_t)(IC > OC ? IC : OC) >= ((size_t)1 << 31)) return hipErrorInvalidValue;   // 32-bit element offsets inside
  ConvWideArgs a{};
  a.in = (const bf16_t*)in; a.wpack = (const bf16_t*)wpack; a.out = (bf16_t*)out; a.stat_partial = stat_partial;
  a.add_g = (const bf16_t*)add_g; a.add_mask = (const bf16_t*)add_mask; a.scale = scale; a.shift = shift;
  if (second) {
    if (add_g || (scale != nullptr) != (second->scale != nullptr) || (stat_partial != nullptr) != (second->stat_partial != nullptr))
      return hipErrorInvalidValue;
    a.in_b = (const bf16_t*)second->in; a.out_b = (bf16_t*)second->out; a.stat_partial_b = second->stat_partial;
    a.scale_b = second->scale; a.shift_b = second->shift;
  }
  int stats = stat_partial ? 1 : 0;
  if (below) {   // the BN-backward sums of the layer below, from the gradient this launch produces
    if (below->mode != 2 || stat_partial || second || scale || !below->partial || !below->z || !below->zmean || !below->zinvstd)
      return hipErrorInvalidValue;
    a.stat_partial = below->partial; a.bmask = (const bf16_t*)below->mask; a.bmscale = below->mscale; a.bmshift = below->mshift;
    a.bz = (const bf16_t*)below->z; a.bmean = below->zmean; a.binvstd = below->zinvstd;
    stats = 2;
  }
  a.M = (int)M; a.H = H; a.W = W; a.HW = H * W; a.IC = IC; a.OC = OC; a.R = R;
  const dim3 grid(conv_wide_rows((int)M), OC / wide::BN, second ? 2 : 1);
  const bool xf = scale != nullptr;
  if (xf && (add_g || IC > 2048)) return hipErrorInvalidValue;   // forward only; the table lives in LDS
  // few tiles (one workgroup per compute unit at most): the long chunk; else two workgroups per unit
  const bool long_chunk = IC >= 128 && grid.x * grid.y * grid.z <= 256;
  if (R == 3)
    return long_chunk ? conv_wide_dispatch<128, 3>(a, grid, stats, xf, IC, s) : conv_wide_dispatch<64, 3>(a, grid, stats, xf, IC, s);
  return long_chunk ? conv_wide_dispatch<128, 1>(a, grid, stats, xf, IC, s) : conv_wide_dispatch<64, 1>(a, grid, stats, xf, IC, s);
}

}  // namespace ddg
