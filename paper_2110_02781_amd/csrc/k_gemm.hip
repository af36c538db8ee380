// Pointwise (1x1) convolution and fully connected layers as MFMA GEMMs.
//
// One kernel computes C[i][j] = sum_r X(i, r) * Y(j, r) for the three passes:
//   forward : i = pixel m, j = cout n, r = cin k   X = A'[m][k]   Y = W[n][k]
//   dgrad   : i = pixel m, j = cin k,  r = cout n  X = dZ[m][n]   Y = W[n][k]  (read transposed)
//   wgrad   : i = cout n,  j = cin k,  r = pixel m X = dZ[m][n]   Y = A'[m][k] (both transposed,
//             the pixel range split over blocks into fp32 partials summed in a fixed order)
// A' is read through a View (the producer's BatchNorm + activation applied on load).
//
// Block = 256 threads = 4 wavefronts, tile 128 (i) x 64 (j), reduction chunks of
// 32 staged through LDS in "r contiguous" layout; each wavefront owns a 32 x 64
// strip = two 32x32 MFMA accumulators.  bfloat16 uses v_mfma_f32_32x32x16_bf16
// (8 consecutive r per lane), float uses v_mfma_f32_32x32x2_f32 (true fp32).
#include "dev_common.h"
#include "kernels.h"

namespace ftp {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

enum { BI = 128, BJ = 64, BR = 32 };
enum { MODE_FWD = 0, MODE_DGRAD = 1, MODE_WGRAD = 2 };

template <typename T> struct Lds;
template <> struct Lds<float> { enum { LD = BR + 4 }; };
template <> struct Lds<bf16_t> { enum { LD = BR + 8 }; };

struct GemmArgs {
  const void* x;     // dZ (dgrad, wgrad) or A (fwd; through view)
  const void* y;     // W (fwd, dgrad) or A (wgrad; through view)
  View view;         // prologue of A' (fwd: on x, wgrad: on y)
  const float* bias; // fwd
  const void* res;   // dgrad: added to the result
  void* out;         // T (fwd, dgrad) or float partials (wgrad)
  size_t M;
  int K, N;
  int jtiles, itiles;
  size_t mchunk;     // wgrad: pixels per split
};

__device__ __forceinline__ void lds_put8(float* dst, const float v[8]) { store8(dst, v); }
__device__ __forceinline__ void lds_put8(bf16_t* dst, const float v[8]) { store8(dst, v); }

// ---- tile loaders ---------------------------------------------------------------
// "r contiguous" source: element (i, r) at src[i * ld + r]; rows valid < nrow, r valid < nr
template <typename T, int ROWS, bool USE_VIEW>
__device__ __forceinline__ void load_tile_rc(T* lds, const T* __restrict__ src, size_t ld, size_t row0,
                                             size_t nrow, size_t r0, size_t nr, const View& vw) {
  constexpr int LD = Lds<T>::LD;
  constexpr int NVEC = ROWS * (BR / 8);
  const bool vec_ok = (ld % 8) == 0;
  for (int v = threadIdx.x; v < NVEC; v += 256) {
    int i = v / (BR / 8), rv = v % (BR / 8);
    size_t row = row0 + i, r = r0 + (size_t)rv * 8;
    float val[8];
    if (row < nrow && r + 8 <= nr && vec_ok) {
      load8(src + row * ld + r, val);
      if (USE_VIEW && vw.scale) {
        float s[8], b[8];
        load8(vw.scale + r, s);
        load8(vw.shift + r, b);
#pragma unroll
        for (int e = 0; e < 8; ++e) val[e] = act_apply(fmaf(val[e], s[e], b[e]), vw.act);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float x = 0.f;
        if (row < nrow && r + e < nr) {
          x = to_f32(src[row * ld + r + e]);
          if (USE_VIEW && vw.scale) x = act_apply(fmaf(x, vw.scale[r + e], vw.shift[r + e]), vw.act);
        }
        val[e] = x;
      }
    }
    lds_put8(lds + i * LD + rv * 8, val);
  }
}

// "i contiguous" source: element (i, r) at src[r * ld + i]  (transposed on the way into LDS)
template <typename T, int ROWS, bool USE_VIEW>
__device__ __forceinline__ void load_tile_ic(T* lds, const T* __restrict__ src, size_t ld, size_t i0,
                                             size_t ni, size_t r0, size_t nr, const View& vw) {
  constexpr int LD = Lds<T>::LD;
  constexpr int NVEC = (ROWS / 8) * BR;
  const bool vec_ok = (ld % 8) == 0;
  for (int v = threadIdx.x; v < NVEC; v += 256) {
    int r = v / (ROWS / 8), iv = v % (ROWS / 8);
    size_t rr = r0 + r, ii = i0 + (size_t)iv * 8;
    float val[8];
    if (rr < nr && ii + 8 <= ni && vec_ok) {
      load8(src + rr * ld + ii, val);
      if (USE_VIEW && vw.scale) {
        float s[8], b[8];
        load8(vw.scale + ii, s);
        load8(vw.shift + ii, b);
#pragma unroll
        for (int e = 0; e < 8; ++e) val[e] = act_apply(fmaf(val[e], s[e], b[e]), vw.act);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float x = 0.f;
        if (rr < nr && ii + e < ni) {
          x = to_f32(src[rr * ld + ii + e]);
          if (USE_VIEW && vw.scale) x = act_apply(fmaf(x, vw.scale[ii + e], vw.shift[ii + e]), vw.act);
        }
        val[e] = x;
      }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) lds[(iv * 8 + e) * LD + r] = from_f32<T>(val[e]);
  }
}

// ---- MFMA over one staged chunk ----------------------------------------------------
__device__ __forceinline__ void mma_chunk(const bf16_t* xs, const bf16_t* ys, int wave, int lane, f16v acc[2]) {
  constexpr int LD = Lds<bf16_t>::LD;
  const int i = wave * 32 + (lane & 31), h = lane >> 5;
#pragma unroll
  for (int ks = 0; ks < BR / 16; ++ks) {
    uint4 a = *reinterpret_cast<const uint4*>(xs + i * LD + ks * 16 + h * 8);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      uint4 b = *reinterpret_cast<const uint4*>(ys + (t * 32 + (lane & 31)) * LD + ks * 16 + h * 8);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), acc[t], 0, 0, 0);
    }
  }
}

__device__ __forceinline__ void mma_chunk(const float* xs, const float* ys, int wave, int lane, f16v acc[2]) {
  constexpr int LD = Lds<float>::LD;
  const int i = wave * 32 + (lane & 31), h = lane >> 5;
#pragma unroll
  for (int q = 0; q < BR / 8; ++q) {
    // lane half h holds r = 8q+4h .. +3; instruction t multiplies r = 8q+t and 8q+4+t
    float4 a = *reinterpret_cast<const float4*>(xs + i * LD + q * 8 + h * 4);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      float4 b = *reinterpret_cast<const float4*>(ys + (t * 32 + (lane & 31)) * LD + q * 8 + h * 4);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc[t], 0, 0, 0);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc[t], 0, 0, 0);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc[t], 0, 0, 0);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc[t], 0, 0, 0);
    }
  }
}

template <typename T, int MODE>
__global__ __launch_bounds__(256) void pw_gemm_k(GemmArgs p) {
  constexpr int LD = Lds<T>::LD;
  __shared__ __attribute__((aligned(16))) T xs[BI * LD];
  __shared__ __attribute__((aligned(16))) T ys[BJ * LD];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int tile = blockIdx.x % (p.jtiles * p.itiles);
  const int split = blockIdx.x / (p.jtiles * p.itiles);
  const int jt = tile % p.jtiles, it = tile / p.jtiles;
  const size_t i0 = (size_t)it * BI, j0 = (size_t)jt * BJ;
  const T* X = reinterpret_cast<const T*>(p.x);
  const T* Y = reinterpret_cast<const T*>(p.y);

  size_t rbeg = 0, rend;
  if (MODE == MODE_FWD) rend = p.K;
  else if (MODE == MODE_DGRAD) rend = p.N;
  else { rbeg = (size_t)split * p.mchunk; rend = rbeg + p.mchunk < p.M ? rbeg + p.mchunk : p.M; }

  f16v acc[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  for (size_t r0 = rbeg; r0 < rend; r0 += BR) {
    __syncthreads();
    if (MODE == MODE_FWD) {
      load_tile_rc<T, BI, true>(xs, X, p.K, i0, p.M, r0, rend, p.view);     // A'[m][k]
      load_tile_rc<T, BJ, false>(ys, Y, p.K, j0, p.N, r0, rend, p.view);    // W[n][k]
    } else if (MODE == MODE_DGRAD) {
      load_tile_rc<T, BI, false>(xs, X, p.N, i0, p.M, r0, rend, p.view);    // dZ[m][n]
      load_tile_ic<T, BJ, false>(ys, Y, p.K, j0, p.K, r0, rend, p.view);    // W[n][k] as (j=k, r=n)
    } else {
      load_tile_ic<T, BI, false>(xs, X, p.N, i0, p.N, r0, rend, p.view);    // dZ[m][n] as (i=n, r=m)
      load_tile_ic<T, BJ, true>(ys, Y, p.K, j0, p.K, r0, rend, p.view);     // A'[m][k] as (j=k, r=m)
    }
    __syncthreads();
    mma_chunk(xs, ys, wave, lane, acc);
  }

  // accumulator layout: register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l%32]
  const int h = lane >> 5, jl = lane & 31;
  const size_t ni = (MODE == MODE_WGRAD) ? (size_t)p.N : p.M;
  const int nj = (MODE == MODE_FWD) ? p.N : p.K;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    size_t j = j0 + t * 32 + jl;
    if (j >= (size_t)nj) continue;
    float bj = (MODE == MODE_FWD && p.bias) ? p.bias[j] : 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      size_t i = i0 + wave * 32 + 8 * (r / 4) + 4 * h + (r % 4);
      if (i >= ni) continue;
      float v = acc[t][r];
      if (MODE == MODE_FWD) {
        reinterpret_cast<T*>(p.out)[i * p.N + j] = from_f32<T>(v + bj);
      } else if (MODE == MODE_DGRAD) {
        if (p.res) v += to_f32(reinterpret_cast<const T*>(p.res)[i * p.K + j]);
        reinterpret_cast<T*>(p.out)[i * p.K + j] = from_f32<T>(v);
      } else {
        reinterpret_cast<float*>(p.out)[((size_t)split * p.N + i) * p.K + j] = v;
      }
    }
  }
}

template <int MODE>
static void launch(int dt, hipStream_t st, const GemmArgs& a, int nsplit) {
  unsigned grid = (unsigned)((size_t)a.jtiles * a.itiles * nsplit);
  if (dt == 0) hipLaunchKernelGGL((pw_gemm_k<float, MODE>), dim3(grid), dim3(256), 0, st, a);
  else hipLaunchKernelGGL((pw_gemm_k<bf16_t, MODE>), dim3(grid), dim3(256), 0, st, a);
}

void pw_fwd(int dt, hipStream_t st, HView av, const void* w, const float* bias, size_t M, int K, int N,
            void* z) {
  GemmArgs a{};
  a.x = av.z; a.y = w; a.view = View{av.z, av.scale, av.shift, av.act};
  a.bias = bias; a.out = z; a.M = M; a.K = K; a.N = N;
  a.itiles = (int)((M + BI - 1) / BI); a.jtiles = (N + BJ - 1) / BJ;
  KScope ks(st, "pw_fwd", ((double)M * K + (double)M * N + (double)N * K) * (dt == 0 ? 4.0 : 2.0), 2.0 * M * K * N);
  launch<MODE_FWD>(dt, st, a, 1);
}

void pw_dgrad(int dt, hipStream_t st, const void* dz, const void* w, const void* res, size_t M, int K,
              int N, void* dA) {
  GemmArgs a{};
  a.x = dz; a.y = w; a.res = res; a.out = dA; a.M = M; a.K = K; a.N = N;
  a.itiles = (int)((M + BI - 1) / BI); a.jtiles = (K + BJ - 1) / BJ;
  KScope ks(st, "pw_dgrad", ((double)M * K * (res ? 2.0 : 1.0) + (double)M * N + (double)N * K) * (dt == 0 ? 4.0 : 2.0), 2.0 * M * K * N);
  launch<MODE_DGRAD>(dt, st, a, 1);
}

static void wgrad_shape(size_t M, int K, int N, int* S, size_t* mchunk) {
  size_t tiles = (size_t)((N + BI - 1) / BI) * ((K + BJ - 1) / BJ);
  size_t s = (1024 + tiles - 1) / tiles;
  size_t smax = (M + 255) / 256;
  if (s > smax) s = smax;
  if (s < 1) s = 1;
  size_t mc = (M + s - 1) / s;
  mc = ((mc + BR - 1) / BR) * BR;
  *mchunk = mc;
  *S = (int)((M + mc - 1) / mc);
}

size_t pw_wgrad_ws(size_t M, int K, int N) {
  int S; size_t mc;
  wgrad_shape(M, K, N, &S, &mc);
  return (size_t)S * N * K;
}

void reduce_partials(hipStream_t st, const float* ws, int P, size_t QC, int C, size_t stride_q,
                     size_t stride_c, float* g);

void pw_wgrad(int dt, hipStream_t st, const void* dz, HView av, size_t M, int K, int N, float* ws,
              float* g_w) {
  int S; size_t mc;
  wgrad_shape(M, K, N, &S, &mc);
  GemmArgs a{};
  a.x = dz; a.y = av.z; a.view = View{av.z, av.scale, av.shift, av.act};
  a.out = ws; a.M = M; a.K = K; a.N = N; a.mchunk = mc;
  a.itiles = (N + BI - 1) / BI; a.jtiles = (K + BJ - 1) / BJ;
  {
    KScope ks(st, "pw_wgrad", ((double)M * K + (double)M * N) * (dt == 0 ? 4.0 : 2.0) + (double)S * N * K * 4, 2.0 * M * K * N);
    launch<MODE_WGRAD>(dt, st, a, S);
  }
  reduce_partials(st, ws, S, (size_t)N * K, K, (size_t)K, 1, g_w);
}

}  // namespace ftp
