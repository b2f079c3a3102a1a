// Weight gradient of a 3x3, stride-1, pad-1 convolution on the bf16 matrix cores,
// for the CIFAR-shaped layers (16/32/64 channels, feature maps 32/16/8 wide).
//
//   dW[co][tap][ci] = sum over pixels m of dz[m][co] * a[pix(m,tap)][ci]
//
// The contraction index is the pixel, which is the slow index of both NHWC operands, while an
// MFMA lane wants 8 consecutive contraction values of one channel. gfx950 can transpose on the
// way out of LDS (ds_read_b64_tr_b16: in every block of 16 lanes, lane s supplies the address
// of 4 consecutive 16-bit values, and lane i receives value i%4 of lanes i/4, i/4+4, i/4+8,
// i/4+12). So both operands are staged exactly as they lie in memory, [pixel][channel] with
// 16-byte writes; lane s of a block points at channels 4*(s%4).. of pixel P + s/4, lane i gets
// channel i of pixels P..P+3, and two such reads make one 8-pixel fragment. A tap is a shifted
// pixel address into the halo tile: the im2col matrix never exists and nothing is shifted in
// registers. The pixel stride in LDS is 32 or 96 bytes modulo 128, which spreads the four
// pixels of a 16-lane block over all banks.
//
// The activation a can be produced on the fly from the saved conv output:
// a = relu(z*scale + shift) is applied while staging (scale == nullptr: use x as stored).
//
// The error gradient dz can likewise be formed while staging: with dy given, the kernel applies
// the ReLU mask and the batch-norm backward formula dz = A*g + B*z + C0 (coefficients final, or
// derived from the partial rows of the BN-backward sums), uses dz for the contraction and
// writes it out once for the input-gradient kernel that follows: no separate apply pass.
//
// A workgroup walks over tiles of 8 image rows, keeps its accumulators in registers across
// tiles (the next tile's global loads are in flight meanwhile), and writes one partial tile at
// the end; wgrad_reduce_all_kernel adds the partials in a fixed order (deterministic).
#include "ddg_wgrad_tiled.h"
#include <cstdlib>

namespace ddg {

template <int CIN, int COUT, int W, int S = 1, int R = 3>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((CIN == 32 || S == 2) ? 2 : 3))) void wgrad_tiled_kernel(WgradTiledArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  wgrad_tiled_body<CIN, COUT, W, true, S, R>(a, smem, blockIdx.x, blockIdx.y, gridDim.x);
}

template <int CIN, int COUT, int W, int S = 1, int R = 3>
static hipError_t wgrad_tiled_launch_t(const WgradTiledArgs& a, int grid_x, hipStream_t s) {
  using Cfg = WgradTiledCfg<CIN, COUT, W, S, R>;
  const size_t lds = (size_t)Cfg::LDS;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_tiled_kernel<CIN, COUT, W, S, R>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  DDG_LAUNCH((wgrad_tiled_kernel<CIN, COUT, W, S, R>), dim3(grid_x, Cfg::OT), dim3(256), lds, s, a);
  return hipGetLastError();
}

// The layers between two stages: 3x3 stride 2 and the 1x1 stride-2 projection, Cout = 2*Cin,
// from 32x32 (16 channels) or 16x16 (32 channels) inputs.
static bool wgrad_tiled_stride2(int H, int W, int Cin, int Cout, int R, int stride) {
  return stride == 2 && (R == 3 || R == 1) && Cout == 2 * Cin && ((Cin == 16 && W == 32) || (Cin == 32 && W == 16)) &&
         H % 16 == 0;
}

// Returns the number of partial rows (grid.x) the tiled kernel will use for this shape, or 0
// if the shape is not covered (then the generic kernel is used).
int wgrad_tiled_rows(int N, int H, int W, int Cin, int Cout, int R, int stride, int dtype) {
  if (dtype == F32) return wgrad_tiled_f32_rows(N, H, W, Cin, Cout, R, stride);
  if (dtype == BF16 && wgrad_tiled_stride2(H, W, Cin, Cout, R, stride)) {
    const int tiles = N * (H / 2 / 8);
    const int want = 64;
    return want < tiles ? want : tiles;
  }
  if (dtype != BF16 || R != 3 || stride != 1 || Cin != Cout) return 0;
  if (!((Cin == 16 && W == 32) || (Cin == 32 && W == 16) || (Cin == 64 && W == 8))) return 0;
  if (H % 8 != 0) return 0;
  const int tiles = N * (H / 8);
  int want = (Cin == 16) ? 128 : (Cin == 32 ? 64 : 16);
  if (const char* e = getenv("DDG_TUNE_WGRAD_ROWS")) {   // override within [8, 1024]
    const int v = atoi(e);
    if (v >= 8 && v <= 1024) want = v;
  }
  const char* name = Cin == 16 ? "DDG_TUNE_WGRAD_ROWS_C16" : (Cin == 32 ? "DDG_TUNE_WGRAD_ROWS_C32" : "DDG_TUNE_WGRAD_ROWS_C64");
  if (const char* e = getenv(name)) {                    // per-shape override within [8, 256]
    const int v = atoi(e);
    if (v >= 8 && v <= 256) want = v;
  }
  if (want > tiles) want = tiles;
  return want;
}

hipError_t wgrad_tiled_launch(const void* x, const float* scale, const float* shift, const void* dz,
                              const WgradFuse* fuse, float* partial, int N, int H, int W, int C, int rows,
                              hipStream_t s, int Cout, int R, int stride) {
  if (Cout == 0) Cout = C;
  WgradTiledArgs a{};
  a.x = (const bf16_t*)x; a.scale = scale; a.shift = shift; a.dz = (const bf16_t*)dz; a.partial = partial;
  if (fuse) {
    a.dy = (const bf16_t*)fuse->dy; a.mask = (const bf16_t*)fuse->mask; a.mscale = fuse->mscale; a.mshift = fuse->mshift;
    a.zc = (const bf16_t*)fuse->z; a.coef = fuse->coef; a.dz_out = (bf16_t*)fuse->dz_out;
    if (fuse->rows) a.rows = *fuse->rows;
  }
  if (wgrad_tiled_stride2(H, W, C, Cout, R, stride)) {
    a.N = N; a.H = H / 2; a.W = W / 2; a.tiles = N * (a.H / 8);     // output geometry
    if (rows < 1 || rows > a.tiles) return hipErrorInvalidValue;
    if (C == 16 && R == 3) return wgrad_tiled_launch_t<16, 32, 16, 2, 3>(a, rows, s);
    if (C == 16 && R == 1) return wgrad_tiled_launch_t<16, 32, 16, 2, 1>(a, rows, s);
    if (C == 32 && R == 3) return wgrad_tiled_launch_t<32, 64, 8, 2, 3>(a, rows, s);
    if (C == 32 && R == 1) return wgrad_tiled_launch_t<32, 64, 8, 2, 1>(a, rows, s);
    return hipErrorInvalidValue;
  }
  if (Cout != C || R != 3 || stride != 1) return hipErrorInvalidValue;
  a.N = N; a.H = H; a.W = W; a.tiles = N * (H / 8);
  if (C == 16 && W == 32) return wgrad_tiled_launch_t<16, 16, 32>(a, rows, s);
  if (C == 32 && W == 16) return wgrad_tiled_launch_t<32, 32, 16>(a, rows, s);
  if (C == 64 && W == 8) return wgrad_tiled_launch_t<64, 64, 8>(a, rows, s);
  return hipErrorInvalidValue;
}

}  // namespace ddg
