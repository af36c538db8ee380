// Device-side helpers shared by the HIP kernels: storage types, 8-wide vector
// loads/stores with fp32 conversion, and the "activation view" that lets a
// consumer apply the producer's BatchNorm scale/shift and activation on load.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ftp {

typedef uint16_t bf16_t;  // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round to nearest even in hardware (v_cvt_pk_bf16_f32 converts two floats per instruction)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32x2_to_bf16x2(float lo, float hi) {
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }

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
  r.x = f32x2_to_bf16x2(v[0], v[1]);
  r.y = f32x2_to_bf16x2(v[2], v[3]);
  r.z = f32x2_to_bf16x2(v[4], v[5]);
  r.w = f32x2_to_bf16x2(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = r;
}

// raw 8-element vector as loaded from global memory
template <typename T> struct Raw;
template <> struct Raw<float> { float4 a, b; };
template <> struct Raw<bf16_t> { uint4 a; };

__device__ __forceinline__ void raw_load(Raw<float>& r, const float* p) {
  r.a = *reinterpret_cast<const float4*>(p);
  r.b = *reinterpret_cast<const float4*>(p + 4);
}
__device__ __forceinline__ void raw_load(Raw<bf16_t>& r, const bf16_t* p) { r.a = *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void raw_unpack(const Raw<float>& r, float v[8]) {
  v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w; v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
}
__device__ __forceinline__ void raw_unpack(const Raw<bf16_t>& r, float v[8]) {
  v[0] = __uint_as_float(r.a.x << 16); v[1] = __uint_as_float(r.a.x & 0xffff0000u);
  v[2] = __uint_as_float(r.a.y << 16); v[3] = __uint_as_float(r.a.y & 0xffff0000u);
  v[4] = __uint_as_float(r.a.z << 16); v[5] = __uint_as_float(r.a.z & 0xffff0000u);
  v[6] = __uint_as_float(r.a.w << 16); v[7] = __uint_as_float(r.a.w & 0xffff0000u);
}

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2 };

// Every activation here is a clamp to [lo, hi]: none = (-inf, inf), ReLU = [0, inf), ReLU6 = [0, 6].
// One v_med3_f32 applies it; the derivative is 1 strictly inside the interval.
__device__ __forceinline__ float act_lo(int act) { return act == ACT_NONE ? -INFINITY : 0.f; }
__device__ __forceinline__ float act_hi(int act) { return act == ACT_RELU6 ? 6.f : INFINITY; }
__device__ __forceinline__ float clamp_act(float y, float lo, float hi) { return __builtin_amdgcn_fmed3f(y, lo, hi); }
__device__ __forceinline__ float act_apply(float y, int act) { return clamp_act(y, act_lo(act), act_hi(act)); }
__device__ __forceinline__ float act_mask(float y, int act) { return (y > act_lo(act) && y < act_hi(act)) ? 1.f : 0.f; }

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
    const float lo = act_lo(v.act), hi = act_hi(v.act);
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = round_to<T>(clamp_act(fmaf(out[e], s[e], b[e]), lo, hi));
  }
}

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Renumbering them so that
// consecutive logical ids share an XCD keeps blocks that touch the same cache lines (column tiles of one row range,
// neighbouring spatial tiles, adjacent channel groups of one pixel row) behind one L2.
__device__ __forceinline__ int xcd_logical(const int b, const int nb) {    // b in [0, nb), block 0 of the range on XCD 0
  const int x = b & 7, idx = b >> 3, q = nb >> 3, rem = nb & 7;
  return x * q + (x < rem ? x : rem) + idx;
}
__device__ __forceinline__ int xcd_logical_block() { return xcd_logical(blockIdx.x, gridDim.x); }

// four consecutive channels as a float4
__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ float4 load4(const bf16_t* p) {
  const uint2 u = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                     __uint_as_float(u.y & 0xffff0000u));
}
__device__ __forceinline__ void store4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ void store4(bf16_t* p, float4 v) {
  uint2 u;
  u.x = f32x2_to_bf16x2(v.x, v.y);
  u.y = f32x2_to_bf16x2(v.z, v.w);
  *reinterpret_cast<uint2*>(p) = u;
}
__device__ __forceinline__ float4 fma4(float4 a, float4 b, float4 c) {
  return make_float4(fmaf(a.x, b.x, c.x), fmaf(a.y, b.y, c.y), fmaf(a.z, b.z, c.z), fmaf(a.w, b.w, c.w));
}

// Sum over the 64 lanes of a wavefront without touching LDS: butterflies inside each row of 16 lanes
// with data-parallel-primitive moves (VALU rate; cross-lane permutes through LDS cost ~20 cycles per
// instruction), then the four row totals in lane order.  Every lane returns the same value.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float x) {
  x += dpp_move<0xB1>(x);    // quad_perm [1,0,3,2]
  x += dpp_move<0x4E>(x);    // quad_perm [2,3,0,1]
  x += dpp_move<0x141>(x);   // row_half_mirror
  x += dpp_move<0x140>(x);   // row_mirror
  const int xi = __builtin_bit_cast(int, x);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 48));
  return ((r0 + r1) + r2) + r3;
}

}  // namespace ftp
