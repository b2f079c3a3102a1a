// What this GPU attains on the two resources the roofline figures are priced against: HBM
// bandwidth (a large copy and a large read) and the dense matrix-core rate (register-resident
// MFMA loops, bf16 and fp32). A measuring tool: it prints its figures and is no part of the
// library; the datasheet peaks (8 TB/s, 2.5 PFLOP/s bf16, 157.3 TFLOP/s fp32) stay the
// denominators of every reported fraction.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e_), __FILE__, __LINE__); exit(1); } } while (0)

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// 16 bytes per thread and trip; n16 = number of 16-byte units
__global__ __launch_bounds__(256) void copy16(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// Variants of the copy, to see whether the plain one undersells the memory system: four 16-byte
// loads in flight per thread before the stores; the same with non-temporal accesses.
template <bool NT>
__global__ __launch_bounds__(256) void copy16x4(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x * 4;
  for (size_t i = (size_t)blockIdx.x * blockDim.x * 4 + threadIdx.x; i < n16; i += stride) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t j = i + (size_t)u * blockDim.x;
      if (j < n16) {
        if (NT) { const unsigned* p = reinterpret_cast<const unsigned*>(src + j);
                  v[u] = make_uint4(__builtin_nontemporal_load(p), __builtin_nontemporal_load(p + 1), __builtin_nontemporal_load(p + 2), __builtin_nontemporal_load(p + 3)); }
        else v[u] = src[j];
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t j = i + (size_t)u * blockDim.x;
      if (j < n16) {
        if (NT) { unsigned* p = reinterpret_cast<unsigned*>(dst + j);
                  __builtin_nontemporal_store(v[u].x, p); __builtin_nontemporal_store(v[u].y, p + 1);
                  __builtin_nontemporal_store(v[u].z, p + 2); __builtin_nontemporal_store(v[u].w, p + 3); }
        else dst[j] = v[u];
      }
    }
  }
}

__global__ __launch_bounds__(256) void read16(const uint4* __restrict__ src, unsigned* __restrict__ sink, size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  unsigned acc = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) {
    const uint4 v = src[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9e3779b9u) sink[0] = acc;   // (keeps the loads alive; practically never true)
}

// 8 independent accumulators per wave, operands in registers: nothing but MFMA issue
__global__ __launch_bounds__(256) void mfma_bf16_loop(float* out, int iters) {
  bf16x8_t a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(threadIdx.x % 7); b[i] = (__bf16)(float)(threadIdx.x % 5); }
  f32x4_t acc[8];
  for (int j = 0; j < 8; ++j) acc[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
  for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

typedef float f32x16_t __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void mfma_bf16_32_loop(float* out, int iters) {
  bf16x8_t a, b;
  for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(threadIdx.x % 7); b[i] = (__bf16)(float)(threadIdx.x % 5); }
  f32x16_t acc[4];
  for (int j = 0; j < 4; ++j)
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
  for (int j = 0; j < 4; ++j)
    for (int e = 0; e < 16; ++e) s += acc[j][e];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void mfma_f32_loop(float* out, int iters) {
  const float a = (float)(threadIdx.x % 7), b = (float)(threadIdx.x % 5);
  f32x4_t acc[8];
  for (int j = 0; j < 8; ++j) acc[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
  for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <typename F>
static double best_ms(F launch, int reps) {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  launch();
  CK(hipDeviceSynchronize());
  double best = 1e30;
  for (int r = 0; r < reps; ++r) {
    CK(hipEventRecord(e0, 0));
    launch();
    CK(hipEventRecord(e1, 0));
    CK(hipEventSynchronize(e1));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    if (ms < best) best = ms;
  }
  CK(hipEventDestroy(e0)); CK(hipEventDestroy(e1));
  return best;
}

int main() {
  hipDeviceProp_t prop;
  CK(hipGetDeviceProperties(&prop, 0));
  printf("device: %s, %d compute units, %d MHz\n", prop.gcnArchName, prop.multiProcessorCount, prop.clockRate / 1000);
  const int cus = prop.multiProcessorCount;

  for (size_t mib : {64, 1024, 4096}) {
    const size_t bytes = mib << 20, n16 = bytes / 16;
    uint4 *src, *dst; unsigned* sink;
    CK(hipMalloc(&src, bytes)); CK(hipMalloc(&dst, bytes)); CK(hipMalloc(&sink, 256));
    CK(hipMemset(src, 1, bytes)); CK(hipMemset(dst, 0, bytes));
    const int grid = cus * 16;
    const double tc = best_ms([&] { hipLaunchKernelGGL(copy16, dim3(grid), dim3(256), 0, 0, src, dst, n16); }, 10);
    const double tr = best_ms([&] { hipLaunchKernelGGL(read16, dim3(grid), dim3(256), 0, 0, src, sink, n16); }, 10);
    printf("copy %5zu MiB: %.3f ms, %.0f GB/s read+written = %.3f of 8 TB/s;  read only: %.3f ms, %.0f GB/s = %.3f\n", mib, tc,
           2.0 * bytes / tc / 1e6, 2.0 * bytes / tc / 1e6 / 8000.0, tr, (double)bytes / tr / 1e6, (double)bytes / tr / 1e6 / 8000.0);
    // the same copy written three other ways (does the plain kernel undersell the memory system?)
    for (int wgs : {4, 16}) {
      const int g4 = cus * wgs;
      const double t4 = best_ms([&] { hipLaunchKernelGGL(copy16x4<false>, dim3(g4), dim3(256), 0, 0, src, dst, n16); }, 10);
      const double tn = best_ms([&] { hipLaunchKernelGGL(copy16x4<true>, dim3(g4), dim3(256), 0, 0, src, dst, n16); }, 10);
      printf("      variants, %2d workgroups per compute unit: 4 loads in flight %.0f GB/s; non-temporal %.0f GB/s\n", wgs,
             2.0 * bytes / t4 / 1e6, 2.0 * bytes / tn / 1e6);
    }
    const double tm = best_ms([&] { (void)hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, 0); }, 10);
    printf("      the runtime's own device-to-device copy: %.0f GB/s\n", 2.0 * bytes / tm / 1e6);
    CK(hipFree(src)); CK(hipFree(dst)); CK(hipFree(sink));
  }

  float* out;
  const int grid = cus * 8, iters = 20000;      // 8 workgroups of 4 waves per compute unit
  CK(hipMalloc(&out, (size_t)grid * 256 * sizeof(float)));
  const double waves = (double)grid * 4;
  const double tb = best_ms([&] { hipLaunchKernelGGL(mfma_bf16_loop, dim3(grid), dim3(256), 0, 0, out, iters); }, 5);
  const double fb = waves * iters * 8.0 * (2.0 * 16 * 16 * 32);
  printf("mfma_f32_16x16x32_bf16 loop: %.3f ms, %.1f TFLOP/s = %.3f of 2500\n", tb, fb / tb / 1e9, fb / tb / 1e9 / 2500.0);
  const double t32 = best_ms([&] { hipLaunchKernelGGL(mfma_bf16_32_loop, dim3(grid), dim3(256), 0, 0, out, iters); }, 5);
  const double f32 = waves * iters * 4.0 * (2.0 * 32 * 32 * 16);
  printf("mfma_f32_32x32x16_bf16 loop: %.3f ms, %.1f TFLOP/s = %.3f of 2500\n", t32, f32 / t32 / 1e9, f32 / t32 / 1e9 / 2500.0);
  const double tf = best_ms([&] { hipLaunchKernelGGL(mfma_f32_loop, dim3(grid), dim3(256), 0, 0, out, iters); }, 5);
  const double ff = waves * iters * 8.0 * (2.0 * 16 * 16 * 4);
  printf("mfma_f32_16x16x4_f32 loop:   %.3f ms, %.1f TFLOP/s = %.3f of 157.3\n", tf, ff / tf / 1e9, ff / tf / 1e9 / 157.3);
  CK(hipFree(out));
  return 0;
}
