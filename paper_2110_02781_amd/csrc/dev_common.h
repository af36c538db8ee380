// Device-side helpers shared by the HIP kernels: storage types, 8-wide vector
// loads/stores with fp32 conversion, and the "activation view" that lets a
// consumer apply the producer's BatchNorm scale/shift and activation on load.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ftp {

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// value as it reads back after being stored in T
template <typename T> __device__ __forceinline__ float round_to(float v) { return to_f32(from_f32<T>(v)); }

// ---- 8 consecutive elements <-> 8 floats (pointer must be 8-element aligned) ----
__device__ __forceinline__ void load8(const float* p, float v[8]) {
  float4 a = *reinterpret_cast<const float4*>(p);
  float4 b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, float v[8]) {
  uint4 r = *reinterpret_cast<const uint4*>(p);
  v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
  v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
  v[4] = __uint_as_float(r.z << 16); v[5] = __uint_as_float(r.z & 0xffff0000u);
  v[6] = __uint_as_float(r.w << 16); v[7] = __uint_as_float(r.w & 0xffff0000u);
}
__device__ __forceinline__ void store8(float* p, const float v[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16_t* p, const float v[8]) {
  uint4 r;
  r.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
  r.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
  r.z = (uint32_t)f32_to_bf16(v[4]) | ((uint32_t)f32_to_bf16(v[5]) << 16);
  r.w = (uint32_t)f32_to_bf16(v[6]) | ((uint32_t)f32_to_bf16(v[7]) << 16);
  *reinterpret_cast<uint4*>(p) = r;
}

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2 };

__device__ __forceinline__ float act_apply(float y, int act) {
  if (act == ACT_RELU) return fmaxf(y, 0.f);
  if (act == ACT_RELU6) return fminf(fmaxf(y, 0.f), 6.f);
  return y;
}
// derivative is 1 strictly inside the linear region
__device__ __forceinline__ float act_mask(float y, int act) {
  if (act == ACT_RELU) return y > 0.f ? 1.f : 0.f;
  if (act == ACT_RELU6) return (y > 0.f && y < 6.f) ? 1.f : 0.f;
  return 1.f;
}

// A tensor as its consumer sees it: value(m, c) = act(scale[c] * z[m][c] + shift[c]),
// rounded to the storage type (what a materialised BatchNorm+activation output
// would hold, and what the bfloat16 MFMA operands hold anyway);
// scale == nullptr means the tensor is stored already activated.
struct View {
  const void* z;
  const float* scale;
  const float* shift;
  int act;
};

template <typename T>
__device__ __forceinline__ float view_at(const View& v, size_t idx, int c) {
  float x = to_f32(reinterpret_cast<const T*>(v.z)[idx]);
  if (v.scale) x = round_to<T>(act_apply(fmaf(x, v.scale[c], v.shift[c]), v.act));
  return x;
}

// 8 consecutive channels starting at channel c (c % 8 == 0)
template <typename T>
__device__ __forceinline__ void view_load8(const View& v, size_t idx, int c, float out[8]) {
  load8(reinterpret_cast<const T*>(v.z) + idx, out);
  if (v.scale) {
    float s[8], b[8];
    load8(v.scale + c, s);
    load8(v.shift + c, b);
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = round_to<T>(act_apply(fmaf(out[e], s[e], b[e]), v.act));
  }
}

}  // namespace ftp
