// Device-side helpers shared by the HIP kernels: storage types, bf16 rounding,
// 16-byte vector access and the MFMA atoms for gfx950 (wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ddg {

struct bf16_t { uint16_t v; };

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round-to-nearest-even, NaN stays NaN: gfx950 converts a pair in one
// instruction (v_cvt_pk_bf16_f32), which the compiler selects for these vector conversions.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  return __builtin_bit_cast(uint16_t, (__bf16)f);
}

template <typename T> struct Store;

template <> struct Store<float> {
  static constexpr int VEC = 4;  // elements per 16 bytes
  typedef float4 vec_t;
  __device__ static __forceinline__ float load1(const float* p) { return *p; }
  __device__ static __forceinline__ void store1(float* p, float v) { *p = v; }
  __device__ static __forceinline__ float round(float v) { return v; }
  __device__ static __forceinline__ void load_vec(const float* p, float (&o)[4]) {
    float4 v = *reinterpret_cast<const float4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
  __device__ static __forceinline__ void unpack_vec(const float4& v, float (&o)[4]) {
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
  __device__ static __forceinline__ void store_vec(float* p, const float (&o)[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(o[0], o[1], o[2], o[3]);
  }
  __device__ static __forceinline__ void store4(float* p, float a, float b, float c, float d) {
    *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
  }
  __device__ static __forceinline__ void load4(const float* p, float (&o)[4]) { load_vec(p, o); }
};

template <> struct Store<bf16_t> {
  static constexpr int VEC = 8;
  typedef uint4 vec_t;
  __device__ static __forceinline__ float load1(const bf16_t* p) { return bf16_to_f32(p->v); }
  __device__ static __forceinline__ void store1(bf16_t* p, float v) { p->v = f32_to_bf16(v); }
  __device__ static __forceinline__ float round(float v) { return bf16_to_f32(f32_to_bf16(v)); }
  __device__ static __forceinline__ void unpack_vec(const uint4& v, float (&o)[8]) {
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
    o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
    o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
  }
  __device__ static __forceinline__ void load_vec(const bf16_t* p, float (&o)[8]) {
    uint4 v = *reinterpret_cast<const uint4*>(p);
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
    o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
    o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
  }
  __device__ static __forceinline__ uint32_t pack2(float lo, float hi) { return f32x2_to_bf16x2(lo, hi); }
  __device__ static __forceinline__ void store_vec(bf16_t* p, const float (&o)[8]) {
    uint4 v;
    v.x = pack2(o[0], o[1]); v.y = pack2(o[2], o[3]); v.z = pack2(o[4], o[5]); v.w = pack2(o[6], o[7]);
    *reinterpret_cast<uint4*>(p) = v;
  }
  __device__ static __forceinline__ void store4(bf16_t* p, float a, float b, float c, float d) {
    uint2 v; v.x = pack2(a, b); v.y = pack2(c, d);
    *reinterpret_cast<uint2*>(p) = v;
  }
  __device__ static __forceinline__ void load4(const bf16_t* p, float (&o)[4]) {
    uint2 v = *reinterpret_cast<const uint2*>(p);
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
  }
};

// MFMA atoms, 16x16 output tile per wave. Operand X (first) supplies rows, operand Y
// (second) supplies columns; lane l feeds row/column l%16 with the KV consecutive
// k-values starting at (l/16)*KV. The accumulator lane l holds column l%16, rows
// (l/16)*4 .. +3.
template <typename T> struct Mma;

template <> struct Mma<float> {
  // Four instructions of k = 4 per fragment: a lane holds 4 consecutive k-values (one 16-byte
  // load) and instruction j contracts element j of every lane, i.e. the k-values
  // {(l/16)*4 + j}. Any assignment of k-values to instructions is as good as another as long
  // as both operands use the same one, and this one makes every gather a 16-byte access.
  static constexpr int KV = 4;      // k-values per lane
  static constexpr int KSTEP = 16;  // k per fragment
  typedef float4 frag_t;
  __device__ static __forceinline__ frag_t zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
  __device__ static __forceinline__ frag_t load(const float* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static __forceinline__ f32x4_t mma(frag_t x, frag_t y, f32x4_t c) {
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(x.x, y.x, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(x.y, y.y, c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(x.z, y.z, c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x4f32(x.w, y.w, c, 0, 0, 0);
  }
};

template <> struct Mma<bf16_t> {
  static constexpr int KV = 8;
  static constexpr int KSTEP = 32;
  typedef uint4 frag_t;  // 8 bf16
  __device__ static __forceinline__ frag_t zero() { return make_uint4(0, 0, 0, 0); }
  __device__ static __forceinline__ frag_t load(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
  __device__ static __forceinline__ f32x4_t mma(frag_t x, frag_t y, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, x),
                                                   __builtin_bit_cast(bf16x8_t, y), c, 0, 0, 0);
  }
};

}  // namespace ddg
