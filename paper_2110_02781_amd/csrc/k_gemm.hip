// Pointwise (1x1) convolution and fully connected layers as MFMA GEMMs.
//
// One kernel computes C[i][j] = sum_r X(i, r) * Y(j, r) for the three passes:
//   forward : i = pixel m, j = cout n, r = cin k   X = A'[m][k]   Y = W[n][k]
//   dgrad   : i = pixel m, j = cin k,  r = cout n  X = dZ[m][n]   Y = W[n][k]  (read transposed)
//   wgrad   : i = cout n,  j = cin k,  r = pixel m X = dZ[m][n]   Y = A'[m][k] (both transposed,
//             the pixel range split over blocks into fp32 partials summed in a fixed order)
// A' is read through a View (the producer's BatchNorm + activation applied on load).
//
// These GEMMs stream a tall activation matrix once against a small weight matrix,
// so they are HBM-bound; the kernel is built around that:
//   * a block owns one 64-wide column tile and walks a contiguous range of row
//     tiles, so weights stay in L2 and per-column BatchNorm sums accumulate in
//     registers over the whole range (one partial per block, fixed order);
//   * the next reduction chunk is fetched from HBM into registers while the
//     current one is multiplied out of LDS (software pipeline over a flat
//     (row tile, chunk) sequence);
//   * the weight tile is stored row-permuted so that a lane's two accumulators are adjacent
//     columns: results leave straight from the MFMA registers and every store instruction
//     writes whole 128/256-byte row segments.
// Three tile shapes: 128 x 64 with the four wavefronts splitting the rows (tall problems);
// 32 x 64 with the four wavefronts splitting a 128-long reduction chunk (few row tiles, long
// reductions); and 16 x 16 with fragments loaded straight from global memory (at most 2048
// rows: pure latency, see pw_gemm_tiny_body), where data gradient and weight gradient of a
// layer share one launch and the weight gradient needs no partial buffers.
// bfloat16 uses v_mfma_f32_32x32x16_bf16 (16x16x32 in the short kernels), float uses
// v_mfma_f32_32x32x2_f32 (16x16x4).
#include <type_traits>
#include "dev_common.h"
#include "kernels.h"

namespace ftp {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

enum { BJ = 64, CLD = BJ + 4 };
enum { MODE_FWD = 0, MODE_DGRAD = 1, MODE_WGRAD = 2 };

template <bool SMALL> struct Shape {
  enum { TI = SMALL ? 32 : 128, CH = SMALL ? 128 : 32 };
};
template <typename T> struct Pad;
template <> struct Pad<float> { enum { V = 4 }; };
template <> struct Pad<bf16_t> { enum { V = 8 }; };

struct GemmArgs {
  const void* x;     // dZ (dgrad, wgrad) or A (fwd; through view)
  const void* y;     // W (fwd, dgrad) or A (wgrad; through view)
  View view;         // prologue of A' (fwd: on x, wgrad: on y)
  const float* bias; // fwd
  const void* res;   // dgrad: added to the result
  void* out;         // T (fwd, dgrad) or float partials (wgrad)
  float* stats;      // fwd: partial[nranges][2][N] column sums of the stored output, or nullptr
  size_t M;
  int K, N;
  int jtiles, itiles;
  int nranges;       // fwd/dgrad: row-tile ranges; wgrad: splits of the pixel range
  int tiles_per_range;
  size_t mchunk;     // wgrad: pixels per split
};

// One operand tile: ROWS (i or j) x CH (r).  RC = source is r-contiguous (element (i,r) at
// src[i*ld + r]); otherwise i-contiguous (element (i,r) at src[r*ld + i]) and transposed on the
// way into LDS.  The view prologue indexes scale/shift by the channel, which is r for RC
// sources and i for the others.
// PERM stores tile row n at LDS row (n & 1) * 32 + (n >> 1) (64-row tiles only), so that the two
// MFMA column sub-tiles of a lane are the adjacent columns 2*lane and 2*lane+1.
__device__ __forceinline__ int perm64(int n) { return ((n & 1) << 5) | (n >> 1); }

template <typename T, int ROWS, int CH, bool RC, bool USE_VIEW, bool PERM = false>
struct TileLoader {
  enum { NVEC = ROWS * CH / 8, PER = (NVEC + 255) / 256, LD = CH + Pad<T>::V };
  Raw<T> raw[PER];
  unsigned ok;      // bit q: raw[q] holds a full in-bounds vector

  __device__ __forceinline__ void coords(int v, int& i, int& r) const {
    if (RC) { i = v / (CH / 8); r = (v % (CH / 8)) * 8; }
    else { r = v / (ROWS / 8); i = (v % (ROWS / 8)) * 8; }
  }

  __device__ __forceinline__ void fetch(const T* __restrict__ src, size_t ld, size_t i0, size_t ni, size_t r0,
                                        size_t nr) {
    ok = 0;
    const bool vec_ok = (ld % 8) == 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      int v = threadIdx.x + q * 256;
      if (v >= NVEC) break;
      int i, r;
      coords(v, i, r);
      size_t gi = i0 + i, gr = r0 + r;
      bool full = vec_ok && (RC ? (gi < ni && gr + 8 <= nr) : (gr < nr && gi + 8 <= ni));
      if (full) {
        raw_load(raw[q], RC ? src + gi * ld + gr : src + gr * ld + gi);
        ok |= 1u << q;
      }
    }
  }

  __device__ __forceinline__ void commit(T* lds, const T* __restrict__ src, size_t ld, size_t i0, size_t ni,
                                         size_t r0, size_t nr, const View& vw) const {
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      int v = threadIdx.x + q * 256;
      if (v >= NVEC) break;
      int i, r;
      coords(v, i, r);
      size_t gi = i0 + i, gr = r0 + r;
      float val[8];
      size_t ch = RC ? gr : gi;      // first channel of the vector
      if (ok & (1u << q)) {
        raw_unpack(raw[q], val);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          size_t ei = RC ? gi : gi + e, er = RC ? gr + e : gr;
          val[e] = (ei < ni && er < nr) ? to_f32(RC ? src[ei * ld + er] : src[er * ld + ei]) : 0.f;
        }
      }
      if (USE_VIEW && vw.scale) {
        if (ok & (1u << q)) {          // whole vector in range: channels ch .. ch+7 exist
          float sc[8], sh[8];
          load8(vw.scale + ch, sc);
          load8(vw.shift + ch, sh);
          const float lo = act_lo(vw.act), hi = act_hi(vw.act);
#pragma unroll
          for (int e = 0; e < 8; ++e) val[e] = clamp_act(fmaf(val[e], sc[e], sh[e]), lo, hi);
        } else {
          size_t nch = RC ? nr : ni;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            // out-of-range elements must stay exactly zero
            bool in = RC ? (gi < ni && gr + e < nr) : (gr < nr && gi + e < ni);
            if (in && ch + e < nch) val[e] = act_apply(fmaf(val[e], vw.scale[ch + e], vw.shift[ch + e]), vw.act);
          }
        }
      }
      if (RC) {
        store8(lds + (PERM ? perm64(i) : i) * LD + r, val);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) lds[(PERM ? perm64(i + e) : i + e) * LD + r] = from_f32<T>(val[e]);
      }
    }
  }
};

// Transposing loader for "i contiguous" sources (element (i, r) at src[r*ld + i]).  A thread takes
// two consecutive reduction rows r, r+1 of the same 8 columns and writes LDS in (r, r+1) pairs:
// one 32-bit (bfloat16) or 64-bit (float) store per column instead of two 16/32-bit ones, and for
// plain bfloat16 data the pair is assembled from the raw bits without a float round trip.
__device__ __forceinline__ void lds_put_pair(float* p, float a, float b) { *reinterpret_cast<float2*>(p) = make_float2(a, b); }
__device__ __forceinline__ void lds_put_pair(bf16_t* p, float a, float b) { *reinterpret_cast<uint32_t*>(p) = f32x2_to_bf16x2(a, b); }

template <typename T, int ROWS, int CH, bool USE_VIEW, bool PERM>
struct TransLoader {
  enum { NITEM = (ROWS / 8) * (CH / 2), PER = (NITEM + 255) / 256, LD = CH + Pad<T>::V };
  Raw<T> raw[PER][2];
  unsigned ok;      // bit 2q+u: raw[q][u] holds a full in-bounds vector

  // consecutive lanes take consecutive row pairs of the same 8 columns, so their LDS stores fall into
  // consecutive words of one LDS row (the other order would put 16 lanes on one bank)
  __device__ __forceinline__ void coords(int item, int& i, int& r) const {
    r = (item % (CH / 2)) * 2;
    i = (item / (CH / 2)) * 8;
  }

  __device__ __forceinline__ void fetch(const T* __restrict__ src, size_t ld, size_t i0, size_t ni, size_t r0,
                                        size_t nr) {
    ok = 0;
    const bool vec_ok = (ld % 8) == 0;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int item = threadIdx.x + q * 256;
      if (item >= NITEM) break;
      int i, r;
      coords(item, i, r);
      const size_t gi = i0 + i;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const size_t gr = r0 + r + u;
        if (vec_ok && gr < nr && gi + 8 <= ni) {
          raw_load(raw[q][u], src + gr * ld + gi);
          ok |= 1u << (2 * q + u);
        }
      }
    }
  }

  __device__ __forceinline__ void commit(T* lds, const T* __restrict__ src, size_t ld, size_t i0, size_t ni,
                                         size_t r0, size_t nr, const View& vw) const {
    const bool view = USE_VIEW && vw.scale != nullptr;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int item = threadIdx.x + q * 256;
      if (item >= NITEM) break;
      int i, r;
      coords(item, i, r);
      const size_t gi = i0 + i;
      const unsigned both = (ok >> (2 * q)) & 3u;
      if (sizeof(T) == 2 && !view && both == 3u) {
        // raw bits straight into (r, r+1) pairs
        const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&raw[q][0]);
        const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&raw[q][1]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t a = w0[e >> 1], b = w1[e >> 1];
          const uint32_t pr = (e & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
          *reinterpret_cast<uint32_t*>(lds + (PERM ? perm64(i + e) : i + e) * LD + r) = pr;
        }
        continue;
      }
      float val[2][8];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const size_t gr = r0 + r + u;
        if (ok & (1u << (2 * q + u))) {
          raw_unpack(raw[q][u], val[u]);
          if (view) {
            float sc[8], sh[8];
            load8(vw.scale + gi, sc);
            load8(vw.shift + gi, sh);
            const float lo = act_lo(vw.act), hi = act_hi(vw.act);
#pragma unroll
            for (int e = 0; e < 8; ++e) val[u][e] = clamp_act(fmaf(val[u][e], sc[e], sh[e]), lo, hi);
          }
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            float x = 0.f;                      // out-of-range elements must stay exactly zero
            if (gr < nr && gi + e < ni) {
              x = to_f32(src[gr * ld + gi + e]);
              if (view) x = act_apply(fmaf(x, vw.scale[gi + e], vw.shift[gi + e]), vw.act);
            }
            val[u][e] = x;
          }
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) lds_put_pair(lds + (PERM ? perm64(i + e) : i + e) * LD + r, val[0][e], val[1][e]);
    }
  }
};

// Branch-free loaders for problems whose extents along the vectorised dimension are multiples of 8
// (every layer of the networks here except the classifier output): a vector is then wholly inside or
// wholly outside the tensor; outside ones are loaded from the base address, which is always valid,
// and zeroed by a select.  The generic loaders above spend most of their instructions on
// per-element bounds branches that never fire for such shapes.
template <typename T, int ROWS, int CH, bool USE_VIEW, bool PERM>
struct VecTileLoader {   // r-contiguous source
  enum { NVEC = ROWS * CH / 8, PER = NVEC / 256, LD = CH + Pad<T>::V };
  static_assert(NVEC % 256 == 0, "tile must divide over 256 threads");
  Raw<T> raw[PER];
  unsigned ok;
  float psc[USE_VIEW ? PER : 1][8], psh[USE_VIEW ? PER : 1][8];   // view vectors requested together with the tile

  // the scale / shift of the channels (= reduction indices) of the vectors that fetch() requests for the same step
  __device__ __forceinline__ void fetch_view(const View& vw, size_t r0, size_t nr) {
    if (!USE_VIEW || !vw.scale) return;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int v = threadIdx.x + q * 256;
      const int r = (v % (CH / 8)) * 8;
      const size_t ch = r0 + r < nr ? r0 + r : 0;
      load8(vw.scale + ch, psc[q]);
      load8(vw.shift + ch, psh[q]);
    }
  }
  // commit with the view vectors that fetch_view requested
  __device__ __forceinline__ void commit_pv(T* lds, int act) const {
    const float lo = act_lo(act), hi = act_hi(act);
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int v = threadIdx.x + q * 256;
      const int i = v / (CH / 8), r = (v % (CH / 8)) * 8;
      const bool in = (ok >> q) & 1u;
      float val[8];
      raw_unpack(raw[q], val);
#pragma unroll
      for (int e = 0; e < 8; ++e) val[e] = in ? clamp_act(fmaf(val[e], psc[USE_VIEW ? q : 0][e], psh[USE_VIEW ? q : 0][e]), lo, hi) : 0.f;
      store8(lds + (PERM ? perm64(i) : i) * LD + r, val);
    }
  }

  __device__ __forceinline__ void fetch(const T* __restrict__ src, size_t ld, size_t i0, size_t ni, size_t r0,
                                        size_t nr) {
    ok = 0;
    // every address first, then the loads back to back: an address computed between two loads can land in a
    // register the compiler still counts as the target of an earlier load, and then each load waits for the one before
    const T* ptr[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int v = threadIdx.x + q * 256;
      const int i = v / (CH / 8), r = (v % (CH / 8)) * 8;
      const size_t gi = i0 + i, gr = r0 + r;
      const bool in = gi < ni && gr < nr;
      ptr[q] = in ? src + gi * ld + gr : src;
      ok |= (in ? 1u : 0u) << q;
    }
#pragma unroll
    for (int q = 0; q < PER; ++q) raw_load(raw[q], ptr[q]);
  }

  __device__ __forceinline__ void commit(T* lds, const T* __restrict__, size_t, size_t, size_t, size_t r0, size_t,
                                         const View& vw) const {
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int v = threadIdx.x + q * 256;
      const int i = v / (CH / 8), r = (v % (CH / 8)) * 8;
      const bool in = (ok >> q) & 1u;
      float val[8];
      raw_unpack(raw[q], val);
      if (USE_VIEW && vw.scale) {
        const size_t ch = in ? r0 + r : 0;
        float sc[8], sh[8];
        load8(vw.scale + ch, sc);
        load8(vw.shift + ch, sh);
        const float lo = act_lo(vw.act), hi = act_hi(vw.act);
#pragma unroll
        for (int e = 0; e < 8; ++e) val[e] = clamp_act(fmaf(val[e], sc[e], sh[e]), lo, hi);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) val[e] = in ? val[e] : 0.f;
      store8(lds + (PERM ? perm64(i) : i) * LD + r, val);
    }
  }

};

template <typename T, int ROWS, int CH, bool USE_VIEW, bool PERM>
struct VecTransLoader {  // i-contiguous source, transposed into (r, r+1) pairs like TransLoader
  enum { NITEM = (ROWS / 8) * (CH / 2), PER = (NITEM + 255) / 256, LD = CH + Pad<T>::V };
  Raw<T> raw[PER][2];
  unsigned ok;
  // the view's scale / shift of this thread's columns: the same for every step of a block (the channel is the tile's
  // i index), so they are loaded once (hold_view) instead of in every commit, where the load could not be hidden
  float vsc[USE_VIEW ? PER : 1][8], vsh[USE_VIEW ? PER : 1][8];
  bool held = false;

  __device__ __forceinline__ void hold_view(const View& vw, size_t i0, size_t ni) {
    if (!USE_VIEW || !vw.scale) return;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int item = threadIdx.x + q * 256;
      const int i = (item / (CH / 2)) * 8;
      const size_t ch = (item < NITEM && i0 + i < ni) ? i0 + i : 0;      // ni is a multiple of 8 here
      load8(vw.scale + ch, vsc[q]);
      load8(vw.shift + ch, vsh[q]);
    }
    held = true;
  }

  __device__ __forceinline__ void fetch(const T* __restrict__ src, size_t ld, size_t i0, size_t ni, size_t r0,
                                        size_t nr) {
    ok = 0;
    const T* ptr[PER][2];                    // every address first, then the loads back to back (see VecTileLoader)
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int item = threadIdx.x + q * 256;
      const int r = (item % (CH / 2)) * 2, i = (item / (CH / 2)) * 8;
      const size_t gi = i0 + i;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const size_t gr = r0 + r + u;
        const bool in = item < NITEM && gr < nr && gi < ni;
        ptr[q][u] = in ? src + gr * ld + gi : src;
        ok |= (in ? 1u : 0u) << (2 * q + u);
      }
    }
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      raw_load(raw[q][0], ptr[q][0]);
      raw_load(raw[q][1], ptr[q][1]);
    }
  }

  __device__ __forceinline__ void commit(T* lds, const T* __restrict__, size_t, size_t i0, size_t, size_t, size_t,
                                         const View& vw) const {
    const bool view = USE_VIEW && vw.scale != nullptr;
#pragma unroll
    for (int q = 0; q < PER; ++q) {
      const int item = threadIdx.x + q * 256;
      if (item >= NITEM) break;
      const int r = (item % (CH / 2)) * 2, i = (item / (CH / 2)) * 8;
      const bool in0 = (ok >> (2 * q)) & 1u, in1 = (ok >> (2 * q + 1)) & 1u;
      if (sizeof(T) == 2 && !view) {
        // raw bits straight into (r, r+1) pairs
        const uint32_t* w0 = reinterpret_cast<const uint32_t*>(&raw[q][0]);
        const uint32_t* w1 = reinterpret_cast<const uint32_t*>(&raw[q][1]);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const uint32_t a = in0 ? w0[e >> 1] : 0u, b = in1 ? w1[e >> 1] : 0u;
          const uint32_t pr = (e & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
          *reinterpret_cast<uint32_t*>(lds + (PERM ? perm64(i + e) : i + e) * LD + r) = pr;
        }
        continue;
      }
      float val[2][8];
      raw_unpack(raw[q][0], val[0]);
      raw_unpack(raw[q][1], val[1]);
      if (view) {
        float sc[8], sh[8];
        if (held) {
#pragma unroll
          for (int e = 0; e < 8; ++e) { sc[e] = vsc[USE_VIEW ? q : 0][e]; sh[e] = vsh[USE_VIEW ? q : 0][e]; }
        } else {
          const size_t ch = (in0 || in1) ? i0 + i : 0;     // same channels for both rows
          load8(vw.scale + ch, sc);
          load8(vw.shift + ch, sh);
        }
        const float lo = act_lo(vw.act), hi = act_hi(vw.act);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          val[0][e] = clamp_act(fmaf(val[0][e], sc[e], sh[e]), lo, hi);
          val[1][e] = clamp_act(fmaf(val[1][e], sc[e], sh[e]), lo, hi);
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e)
        lds_put_pair(lds + (PERM ? perm64(i + e) : i + e) * LD + r, in0 ? val[0][e] : 0.f, in1 ? val[1][e] : 0.f);
    }
  }
};

template <typename T, int ROWS, int CH, bool RC, bool USE_VIEW, bool PERM, bool VEC>
struct LoaderSel { typedef TileLoader<T, ROWS, CH, true, USE_VIEW, PERM> type; };
template <typename T, int ROWS, int CH, bool USE_VIEW, bool PERM>
struct LoaderSel<T, ROWS, CH, false, USE_VIEW, PERM, false> { typedef TransLoader<T, ROWS, CH, USE_VIEW, PERM> type; };
template <typename T, int ROWS, int CH, bool USE_VIEW, bool PERM>
struct LoaderSel<T, ROWS, CH, true, USE_VIEW, PERM, true> { typedef VecTileLoader<T, ROWS, CH, USE_VIEW, PERM> type; };
template <typename T, int ROWS, int CH, bool USE_VIEW, bool PERM>
struct LoaderSel<T, ROWS, CH, false, USE_VIEW, PERM, true> { typedef VecTransLoader<T, ROWS, CH, USE_VIEW, PERM> type; };

// ---- MFMA over one staged chunk of 32 reduction elements starting at column c0 -------
__device__ __forceinline__ void mma32(const bf16_t* xs, const bf16_t* ys, int LD, int irow, int lane, int c0,
                                      f16v acc[2]) {
  const int h = lane >> 5, jl = lane & 31;
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    uint4 a = *reinterpret_cast<const uint4*>(xs + irow * LD + c0 + ks * 16 + h * 8);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      uint4 b = *reinterpret_cast<const uint4*>(ys + (t * 32 + jl) * LD + c0 + ks * 16 + h * 8);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), acc[t], 0, 0, 0);
    }
  }
}

__device__ __forceinline__ void mma32(const float* xs, const float* ys, int LD, int irow, int lane, int c0,
                                      f16v acc[2]) {
  const int h = lane >> 5, jl = lane & 31;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    // lane half h holds r = 8q+4h .. +3; instruction t multiplies r = 8q+t and 8q+4+t
    float4 a = *reinterpret_cast<const float4*>(xs + irow * LD + c0 + q * 8 + h * 4);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      float4 b = *reinterpret_cast<const float4*>(ys + (t * 32 + jl) * LD + c0 + q * 8 + h * 4);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc[t], 0, 0, 0);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc[t], 0, 0, 0);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc[t], 0, 0, 0);
      acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc[t], 0, 0, 0);
    }
  }
}

template <typename T, int MODE, bool SMALL, bool VEC>
__global__ __launch_bounds__(256) void pw_gemm_k(GemmArgs p) {
  constexpr int TI = Shape<SMALL>::TI, CH = Shape<SMALL>::CH;
  constexpr int LD = CH + Pad<T>::V;
  constexpr int STAGE_BYTES = (TI + BJ) * LD * (int)sizeof(T);
  constexpr int CT_BYTES = (SMALL ? 4 : 1) * TI * CLD * 4;
  constexpr int SMEM = STAGE_BYTES > CT_BYTES ? STAGE_BYTES : CT_BYTES;
  __shared__ __attribute__((aligned(16))) char smem[SMEM];
  T* xs = reinterpret_cast<T*>(smem);
  T* ys = xs + TI * LD;
  float* ct = reinterpret_cast<float*>(smem);   // aliases the staging buffers between tiles
  if (MODE == MODE_DGRAD) __builtin_amdgcn_s_setprio(3);   // data-gradient chain: ahead of the weight-gradient stream's waves

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int lb = xcd_logical_block();
  const int jt = lb % p.jtiles;
  const int range = lb / p.jtiles;
  const size_t j0 = (size_t)jt * BJ;
  const T* X = reinterpret_cast<const T*>(p.x);
  const T* Y = reinterpret_cast<const T*>(p.y);

  // reduction extent and the row tiles this block walks
  size_t rbeg = 0, rend;
  int it_beg, it_end;
  if (MODE == MODE_WGRAD) {
    // range = (row tile, split): all row tiles are walked by different blocks, the split picks the pixels
    const int split = range / p.itiles;
    it_beg = range % p.itiles; it_end = it_beg + 1;
    rbeg = (size_t)split * p.mchunk;
    rend = rbeg + p.mchunk < p.M ? rbeg + p.mchunk : p.M;
  } else {
    rend = MODE == MODE_FWD ? p.K : p.N;
    it_beg = range * p.tiles_per_range;
    it_end = it_beg + p.tiles_per_range < p.itiles ? it_beg + p.tiles_per_range : p.itiles;
  }
  const int nchunks = (int)((rend - rbeg + CH - 1) / CH);
  const int nsteps = (it_end - it_beg) * nchunks;

  // operand geometry: leading dimensions and extents
  const size_t ldx = MODE == MODE_FWD ? p.K : p.N;
  const size_t ldy = p.K;
  const size_t ni = MODE == MODE_WGRAD ? (size_t)p.N : p.M;        // extent of i
  const size_t nj = MODE == MODE_FWD ? (size_t)p.N : (size_t)p.K;  // extent of j

  // forward: X = A' (r-contiguous, view), Y = W (r-contiguous)
  // dgrad  : X = dZ (r-contiguous),       Y = W as (j=k, r=n)  (i-contiguous)
  // wgrad  : X = dZ as (i=n, r=m),        Y = A' as (j=k, r=m) (both i-contiguous, view on Y)
  typename LoaderSel<T, TI, CH, MODE != MODE_WGRAD, MODE == MODE_FWD, false, VEC>::type lx;
  typename LoaderSel<T, BJ, CH, MODE == MODE_FWD, MODE == MODE_WGRAD, false, VEC>::type ly;
  // weight gradient: the view vectors of this block's columns stay in registers (the same columns at every step)
  if constexpr (MODE == MODE_WGRAD && VEC) ly.hold_view(p.view, j0, nj);

  f16v acc[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  // output pass mapping: 8 column groups x 32 row lanes
  const int ocg = threadIdx.x & 7, orl = threadIdx.x >> 3;
  float ssum[8] = {0, 0, 0, 0, 0, 0, 0, 0}, ssq[8] = {0, 0, 0, 0, 0, 0, 0, 0};

  if (nsteps > 0) {
    lx.fetch(X, ldx, (size_t)it_beg * TI, ni, rbeg, rend);
    if constexpr (MODE == MODE_FWD && VEC) lx.fetch_view(p.view, rbeg, rend);
    ly.fetch(Y, ldy, j0, nj, rbeg, rend);
  }
  for (int s = 0; s < nsteps; ++s) {
    const int it = it_beg + s / nchunks, kc = s % nchunks;
    const size_t i0 = (size_t)it * TI, r0 = rbeg + (size_t)kc * CH;
    __syncthreads();                       // LDS free: previous multiply / output pass finished
    if constexpr (MODE == MODE_FWD && VEC) {
      if (p.view.scale) lx.commit_pv(xs, p.view.act);
      else lx.commit(xs, X, ldx, i0, ni, r0, rend, p.view);
    } else {
      lx.commit(xs, X, ldx, i0, ni, r0, rend, p.view);
    }
    ly.commit(ys, Y, ldy, j0, nj, r0, rend, p.view);
    __syncthreads();
    if (s + 1 < nsteps) {                  // next chunk travels while this one is multiplied
      const int it2 = it_beg + (s + 1) / nchunks, kc2 = (s + 1) % nchunks;
      lx.fetch(X, ldx, (size_t)it2 * TI, ni, rbeg + (size_t)kc2 * CH, rend);
      if constexpr (MODE == MODE_FWD && VEC) lx.fetch_view(p.view, rbeg + (size_t)kc2 * CH, rend);
      ly.fetch(Y, ldy, j0, nj, rbeg + (size_t)kc2 * CH, rend);
    }
    if (SMALL) mma32(xs, ys, LD, lane & 31, lane, wave * 32, acc);
    else mma32(xs, ys, LD, wave * 32 + (lane & 31), lane, 0, acc);
    if (kc + 1 < nchunks) continue;

    // ---- tile finished: accumulators -> LDS tile -> vector stores ----
    __syncthreads();                       // everyone is done reading the staging buffers
    {
      // register r of lane l is C[8*(r/4) + 4*(l/32) + r%4][l%32]
      const int h = lane >> 5, jl = lane & 31;
      float* base = SMALL ? ct + wave * TI * CLD : ct + wave * 32 * CLD;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          base[(8 * (r / 4) + 4 * h + (r % 4)) * CLD + t * 32 + jl] = acc[t][r];
          acc[t][r] = 0.f;
        }
    }
    __syncthreads();
    const size_t jg = j0 + ocg * 8;
    const bool vec_out = (nj % 8) == 0;
    // residual vectors of all rows of the pass first (see the row-streaming kernel)
    float rpre[SMALL ? 1 : 4][8];
    const bool res_pre = MODE == MODE_DGRAD && p.res != nullptr && vec_out && jg + 8 <= nj;
    if (res_pre) {
#pragma unroll
      for (int q = 0; q < (SMALL ? 1 : 4); ++q) {
        const size_t ig = i0 + orl + q * 32;
        if (ig < ni) load8(reinterpret_cast<const T*>(p.res) + ig * p.K + jg, rpre[q]);
      }
    }
#pragma unroll
    for (int q = 0; q < (SMALL ? 1 : 4); ++q) {
      const int row = orl + q * 32;
      const size_t ig = i0 + row;
      if (ig >= ni || jg >= nj) continue;
      float v[8];
      {
        const float* src = ct + row * CLD + ocg * 8;
        float4 a = *reinterpret_cast<const float4*>(src), b = *reinterpret_cast<const float4*>(src + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        if (SMALL) {
#pragma unroll
          for (int w = 1; w < 4; ++w) {
            const float* s2 = src + w * TI * CLD;
            float4 c = *reinterpret_cast<const float4*>(s2), d = *reinterpret_cast<const float4*>(s2 + 4);
            v[0] += c.x; v[1] += c.y; v[2] += c.z; v[3] += c.w; v[4] += d.x; v[5] += d.y; v[6] += d.z; v[7] += d.w;
          }
        }
      }
      const bool full = vec_out && jg + 8 <= nj;
      if (MODE == MODE_FWD) {
        T* dst = reinterpret_cast<T*>(p.out) + ig * p.N + jg;
        if (p.bias) {
#pragma unroll
          for (int e = 0; e < 8; ++e) if (jg + e < nj) v[e] += p.bias[jg + e];
        }
        if (full) store8(dst, v);
        else for (int e = 0; e < 8 && jg + e < nj; ++e) dst[e] = from_f32<T>(v[e]);
        if (p.stats) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            float sv = round_to<T>(v[e]);   // statistics of the values as stored
            ssum[e] += sv;
            ssq[e] = fmaf(sv, sv, ssq[e]);
          }
        }
      } else if (MODE == MODE_DGRAD) {
        T* dst = reinterpret_cast<T*>(p.out) + ig * p.K + jg;
        if (p.res) {
          const T* rs = reinterpret_cast<const T*>(p.res) + ig * p.K + jg;
          if (full) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += rpre[q][e];      // full implies res_pre
          } else {
            for (int e = 0; e < 8 && jg + e < nj; ++e) v[e] += to_f32(rs[e]);
          }
        }
        if (full) store8(dst, v);
        else for (int e = 0; e < 8 && jg + e < nj; ++e) dst[e] = from_f32<T>(v[e]);
      } else {
        const int split = range / p.itiles;
        float* dst = reinterpret_cast<float*>(p.out) + ((size_t)split * p.N + ig) * p.K + jg;
        if (full) store8(dst, v);
        else for (int e = 0; e < 8 && jg + e < nj; ++e) dst[e] = v[e];
      }
    }
  }

  if (MODE == MODE_FWD && p.stats) {
    // column sums over this block's rows: reduce the 32 row lanes through LDS, one partial per block
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem);      // [32][8 groups][16]
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      red[(orl * 8 + ocg) * 16 + e] = ssum[e];
      red[(orl * 8 + ocg) * 16 + 8 + e] = ssq[e];
    }
    __syncthreads();
    if (threadIdx.x < 128) {
      const int cg = threadIdx.x & 7, e = threadIdx.x >> 3;    // e in 0..15: 0-7 sums, 8-15 squares
      float tot = 0.f;
      for (int rl = 0; rl < 32; ++rl) tot += red[(rl * 8 + cg) * 16 + e];
      const size_t j = j0 + cg * 8 + (e & 7);
      if (j < (size_t)p.N) p.stats[((size_t)range * 2 + (e >> 3)) * p.N + j] = tot;
    }
  }
}


// ---- tall problems: 128 x 64 tiles, rows split over the four wavefronts ----------------
// Double-buffered staging (one barrier per chunk); results go from the MFMA registers
// straight to memory: with the permuted weight tile a lane owns columns 2l and 2l+1, so
// each store instruction writes whole 128-byte (bfloat16) / 256-byte (float) row segments.
__device__ __forceinline__ void store_pair(float* p, float a, float b) { *reinterpret_cast<float2*>(p) = make_float2(a, b); }
__device__ __forceinline__ void store_pair(bf16_t* p, float a, float b) {
  *reinterpret_cast<uint32_t*>(p) = f32x2_to_bf16x2(a, b);
}
__device__ __forceinline__ void store_pair_rounded(float* p, float a, float b, float& ra, float& rb) {
  *reinterpret_cast<float2*>(p) = make_float2(a, b); ra = a; rb = b;
}
__device__ __forceinline__ void store_pair_rounded(bf16_t* p, float a, float b, float& ra, float& rb) {
  const uint32_t v = f32x2_to_bf16x2(a, b);
  *reinterpret_cast<uint32_t*>(p) = v;
  ra = __uint_as_float(v << 16); rb = __uint_as_float(v & 0xffff0000u);
}
__device__ __forceinline__ void load_pair(const float* p, float& a, float& b) { float2 v = *reinterpret_cast<const float2*>(p); a = v.x; b = v.y; }
__device__ __forceinline__ void load_pair(const bf16_t* p, float& a, float& b) {
  uint32_t v = *reinterpret_cast<const uint32_t*>(p);
  a = __uint_as_float(v << 16); b = __uint_as_float(v & 0xffff0000u);
}

// CH = reduction elements staged per step (32 everywhere, see launch_t).
// RES: data gradient with a residual to add (a variant of its own: the sixteen prefetched residual pairs cost
// registers that the plain data gradient should not pay for)
// DEEP: data gradient whose reduction spans at least two steps.  The loads of TWO steps are kept in flight (two
// register sets and the two LDS buffers, addressed statically: the chunk loop is unrolled by two, and a tile with an
// odd number of chunks hands over to a copy of the tile code that starts on the other set).  On this architecture
// loads and stores share one counter and complete out of order with respect to each other, so a wait for "all but
// the youngest n loads" exists only while no store is pending and only if n is the same on every path: the chunk
// loop of a tile has no stores, it is entered after an explicit wait for everything, every step requests its
// successor's successor unconditionally (past the end: a valid tile again, never used), and the tile's stores follow.
template <typename T, int MODE, bool VEC, int CH, bool RES = false, bool DEEP = false>
__global__ __launch_bounds__(256) void pw_gemm_rows_k(GemmArgs p) {
  constexpr int TI = 128;
  constexpr int PD = DEEP ? 2 : 1;
  static_assert(!DEEP || MODE != MODE_FWD, "two steps in flight: data gradient and weight gradient");
  constexpr int LD = CH + Pad<T>::V;
  constexpr int BUF = (TI + BJ) * LD;
  __shared__ __attribute__((aligned(16))) T smem[2 * BUF];
  __shared__ float red[4][64][4];
  if (MODE == MODE_DGRAD) __builtin_amdgcn_s_setprio(3);   // data-gradient chain: ahead of the weight-gradient stream's waves

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int lb = xcd_logical_block();
  const int jt = lb % p.jtiles;
  const int range = lb / p.jtiles;
  const size_t j0 = (size_t)jt * BJ;
  const T* X = reinterpret_cast<const T*>(p.x);
  const T* Y = reinterpret_cast<const T*>(p.y);

  size_t rbeg = 0, rend;
  int it_beg, it_end, split = 0;
  if (MODE == MODE_WGRAD) {
    split = range / p.itiles;
    it_beg = range % p.itiles; it_end = it_beg + 1;
    rbeg = (size_t)split * p.mchunk;
    rend = rbeg + p.mchunk < p.M ? rbeg + p.mchunk : p.M;
  } else {
    rend = MODE == MODE_FWD ? p.K : p.N;
    it_beg = range * p.tiles_per_range;
    it_end = it_beg + p.tiles_per_range < p.itiles ? it_beg + p.tiles_per_range : p.itiles;
  }
  const int nchunks = (int)((rend - rbeg + CH - 1) / CH);

  const size_t ldx = MODE == MODE_FWD ? p.K : p.N;
  const size_t ldy = p.K;
  const size_t ni = MODE == MODE_WGRAD ? (size_t)p.N : p.M;
  const size_t nj = MODE == MODE_FWD ? (size_t)p.N : (size_t)p.K;
  const size_t ldo = nj;                   // leading dimension of the output

  typename LoaderSel<T, TI, CH, MODE != MODE_WGRAD, MODE == MODE_FWD, false, VEC>::type lx[PD];
  typename LoaderSel<T, BJ, CH, MODE == MODE_FWD, MODE == MODE_WGRAD, true, VEC>::type ly[PD];
  // weight gradient: the view vectors of this block's columns stay in registers (the same columns at every step);
  // forward: they are requested together with the tile they belong to (fetch_view)
  if constexpr (MODE == MODE_WGRAD && VEC) {
#pragma unroll
    for (int d = 0; d < PD; ++d) ly[d].hold_view(p.view, j0, nj);
  }

  f16v acc[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  float s0 = 0.f, s1 = 0.f, q0 = 0.f, q1 = 0.f;   // column sums / sums of squares of this lane's two columns

  const int h = lane >> 5, jl = lane & 31;
  const size_t jc = j0 + 2 * jl;                    // this lane's first column
  const bool pair_ok = (ldo % 2) == 0 && jc + 1 < nj;
  float b0 = 0.f, b1 = 0.f;
  if (MODE == MODE_FWD && p.bias) {
    if (jc < nj) b0 = p.bias[jc];
    if (jc + 1 < nj) b1 = p.bias[jc + 1];
  }
  // Have the two values arrive here.  Their first use is in the tile epilogue inside the loop, where the compiler
  // cannot tell how many younger loads are outstanding and waits for all of them: the prefetch of the next tile
  // would be drained before every output pass.
  asm volatile("" ::"v"(b0), "v"(b1));

  const bool pview = MODE == MODE_FWD && VEC && p.view.scale != nullptr;   // view vectors travel with the tile

  // the finished tile with first row i0; the sums are cleared for the next tile
  auto epilogue = [&](const size_t i0) __attribute__((always_inline)) {
    // tile finished: register r of this lane is row 8*(r/4) + 4*h + r%4, columns jc (acc[0]) and jc+1 (acc[1])
    const size_t irow = i0 + wave * 32 + 4 * h;
    if (VEC && i0 + TI <= ni) {
      // all rows inside and an even width: a lane's column pair is wholly in or out, no other bounds
      // tests, one address computation per lane
      if (jc < nj) {
        const size_t obase = (MODE == MODE_WGRAD ? (size_t)split * p.N + irow : irow) * ldo + jc;
        // all sixteen residual pairs are requested before the first store: res and out are not known to be
        // distinct, so loads left between the stores are not moved up and each one waits for memory on its own
        float ra[RES ? 16 : 1], rb[RES ? 16 : 1];
        if (RES) {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            load_pair(reinterpret_cast<const T*>(p.res) + obase + (size_t)(8 * (r / 4) + (r % 4)) * ldo, ra[RES ? r : 0], rb[RES ? r : 0]);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const size_t o = obase + (size_t)(8 * (r / 4) + (r % 4)) * ldo;
          float v0 = acc[0][r], v1 = acc[1][r];
          if (MODE == MODE_FWD) {
            v0 += b0; v1 += b1;
            float a, b;                                         // the values as stored: the statistics use those
            store_pair_rounded(reinterpret_cast<T*>(p.out) + o, v0, v1, a, b);
            if (p.stats) { s0 += a; q0 = fmaf(a, a, q0); s1 += b; q1 = fmaf(b, b, q1); }
          } else if (MODE == MODE_DGRAD) {
            if (RES) { v0 += ra[RES ? r : 0]; v1 += rb[RES ? r : 0]; }
            store_pair(reinterpret_cast<T*>(p.out) + o, v0, v1);
          } else {
            store_pair(reinterpret_cast<float*>(p.out) + o, v0, v1);
          }
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) { acc[0][r] = 0.f; acc[1][r] = 0.f; }
      return;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const size_t ig = irow + 8 * (r / 4) + (r % 4);
      float v0 = acc[0][r], v1 = acc[1][r];
      acc[0][r] = 0.f; acc[1][r] = 0.f;
      if (ig >= ni || jc >= nj) continue;
      if (MODE == MODE_FWD) {
        v0 += b0; v1 += b1;
        T* dst = reinterpret_cast<T*>(p.out) + ig * ldo + jc;
        if (pair_ok) store_pair(dst, v0, v1);
        else { dst[0] = from_f32<T>(v0); if (jc + 1 < nj) dst[1] = from_f32<T>(v1); }
        if (p.stats) {
          float a = round_to<T>(v0), b = round_to<T>(v1);   // statistics of the values as stored
          s0 += a; q0 = fmaf(a, a, q0); s1 += b; q1 = fmaf(b, b, q1);
        }
      } else if (MODE == MODE_DGRAD) {
        T* dst = reinterpret_cast<T*>(p.out) + ig * ldo + jc;
        if (RES) {
          const T* rs = reinterpret_cast<const T*>(p.res) + ig * ldo + jc;
          if (pair_ok) { float ra, rb; load_pair(rs, ra, rb); v0 += ra; v1 += rb; }
          else { v0 += to_f32(rs[0]); if (jc + 1 < nj) v1 += to_f32(rs[1]); }
        }
        if (pair_ok) store_pair(dst, v0, v1);
        else { dst[0] = from_f32<T>(v0); if (jc + 1 < nj) dst[1] = from_f32<T>(v1); }
      } else {
        float* dst = reinterpret_cast<float*>(p.out) + ((size_t)split * p.N + ig) * ldo + jc;
        if (pair_ok) store_pair(dst, v0, v1);
        else { dst[0] = v0; if (jc + 1 < nj) dst[1] = v1; }
      }
    }
  };

  if constexpr (!DEEP) {
    const int nsteps = (it_end - it_beg) * nchunks;
    const bool y_static = nchunks == 1;      // the weight tile never changes: stage it once per buffer
    if (nsteps > 0) {
      lx[0].fetch(X, ldx, (size_t)it_beg * TI, ni, rbeg, rend);
      if constexpr (MODE == MODE_FWD && VEC) { if (pview) lx[0].fetch_view(p.view, rbeg, rend); }
      ly[0].fetch(Y, ldy, j0, nj, rbeg, rend);
    }
    for (int s = 0; s < nsteps; ++s) {
      const int it = it_beg + s / nchunks, kc = s % nchunks;
      const size_t i0 = (size_t)it * TI, r0 = rbeg + (size_t)kc * CH;
      T* xs = smem + (s & 1) * BUF;
      T* ys = xs + TI * LD;
      if constexpr (MODE == MODE_FWD && VEC) {
        if (pview) lx[0].commit_pv(xs, p.view.act);
        else lx[0].commit(xs, X, ldx, i0, ni, r0, rend, p.view);
      } else {
        lx[0].commit(xs, X, ldx, i0, ni, r0, rend, p.view);
      }
      if (!y_static || s < 2) ly[0].commit(ys, Y, ldy, j0, nj, r0, rend, p.view);
      __syncthreads();
      if (s + 1 < nsteps) {
        const int it2 = it_beg + (s + 1) / nchunks, kc2 = (s + 1) % nchunks;
        // the weight tile first: its registers may still be the target of a load the compiler has not seen consumed
        // (its commit is conditional), and the wait for that must not come behind this step's other requests
        if (!y_static || s + 1 < 2) ly[0].fetch(Y, ldy, j0, nj, rbeg + (size_t)kc2 * CH, rend);
        lx[0].fetch(X, ldx, (size_t)it2 * TI, ni, rbeg + (size_t)kc2 * CH, rend);
        if constexpr (MODE == MODE_FWD && VEC) { if (pview) lx[0].fetch_view(p.view, rbeg + (size_t)kc2 * CH, rend); }
      }
  #pragma unroll
      for (int c0 = 0; c0 < CH; c0 += 32) mma32(xs, ys, LD, wave * 32 + jl, lane, c0, acc);
      if (kc + 1 == nchunks) epilogue(i0);
    }
  } else {
    const int ntile = it_end - it_beg;
    auto fetch_step = [&](auto& fx, auto& fy, const int t2, const int kc2) __attribute__((always_inline)) {
      // past the last tile the request is only there to keep the count of loads in flight the same on every path: it
      // repeats one of the last tile's last two chunks, which the caches still hold
      const bool past = t2 >= ntile;
      const size_t r2 = rbeg + (size_t)(past ? nchunks - 2 + kc2 : kc2) * CH;
      fy.fetch(Y, ldy, j0, nj, r2, rend);
      fx.fetch(X, ldx, (size_t)(it_beg + (past ? ntile - 1 : t2)) * TI, ni, r2, rend);
    };
    // chunk kc of tile t from register set / LDS buffer SET, then the request for the step two ahead into the same set
    auto step = [&](auto SET, const int t, const int kc) __attribute__((always_inline)) {
      constexpr int set = decltype(SET)::value;
      const size_t i0 = (size_t)(it_beg + t) * TI, r0 = rbeg + (size_t)kc * CH;
      T* xs = smem + set * BUF;
      T* ys = xs + TI * LD;
      lx[set].commit(xs, X, ldx, i0, ni, r0, rend, p.view);
      ly[set].commit(ys, Y, ldy, j0, nj, r0, rend, p.view);
      __syncthreads();
      int kc2 = kc + 2, t2 = t;
      if (kc2 >= nchunks) { kc2 -= nchunks; ++t2; }
      fetch_step(lx[set], ly[set], t2, kc2);
#pragma unroll
      for (int c0 = 0; c0 < CH; c0 += 32) mma32(xs, ys, LD, wave * 32 + jl, lane, c0, acc);
    };
    // one tile whose chunk 0 sits in set P0
    auto tile_body = [&](auto P0, const int t) __attribute__((always_inline)) {
      constexpr int p0 = decltype(P0)::value;
      // vmcnt(0): the last tile's stores and the two steps requested so far are complete; from here to the end of
      // the chunk loop only loads are pending
      __builtin_amdgcn_s_waitcnt(0x0F70);
      int kc = 0;
      for (; kc + 1 < nchunks; kc += 2) {
        step(std::integral_constant<int, p0>(), t, kc);
        step(std::integral_constant<int, p0 ^ 1>(), t, kc + 1);
      }
      if (kc < nchunks) step(std::integral_constant<int, p0>(), t, kc);
      epilogue((size_t)(it_beg + t) * TI);
    };
    if (ntile > 0) {           // nchunks >= 2 (the host launches this variant only then)
      fetch_step(lx[0], ly[0], 0, 0);
      fetch_step(lx[PD - 1], ly[PD - 1], 0, 1);
    }
    const bool odd = nchunks & 1;
    for (int t = 0; t < ntile;) {
      tile_body(std::integral_constant<int, 0>(), t++);
      if (odd && t < ntile) tile_body(std::integral_constant<int, 1>(), t++);
    }
  }

  if (MODE == MODE_FWD && p.stats) {
    // one partial per block: sum the 8 (wave, half) contributions of every column in a fixed order
    red[wave][lane][0] = s0; red[wave][lane][1] = s1; red[wave][lane][2] = q0; red[wave][lane][3] = q1;
    __syncthreads();
    if (threadIdx.x < 128) {
      const int col = threadIdx.x & 63, sq = threadIdx.x >> 6;   // column within the tile; 0 = sum, 1 = squares
      const int l = col >> 1, t = col & 1;
      float tot = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) tot += red[w][l][2 * sq + t] + red[w][l + 32][2 * sq + t];
      const size_t j = j0 + col;
      if (j < (size_t)p.N) p.stats[((size_t)range * 2 + sq) * p.N + j] = tot;
    }
  }
}

// ---- short problems: 16 x 16 output tiles, operands straight from global memory ----------------
// When M x N is small the layer is pure latency: staged tiles would leave most CUs idle behind a long
// serial reduction.  Here a block owns one 16 x 16 tile, its four wavefronts split the reduction,
// every lane loads its MFMA fragments (G consecutive reduction elements) directly as vectors, and the
// four partial tiles are summed through LDS in a fixed order.
typedef float f4v __attribute__((ext_vector_type(4)));
template <typename T> struct TinyStep;
template <> struct TinyStep<float> { enum { G = 4, KS = 16 }; };
template <> struct TinyStep<bf16_t> { enum { G = 8, KS = 32 }; };

__device__ __forceinline__ void load_frag(const float* p, float* v) {
  float4 a = *reinterpret_cast<const float4*>(p);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
}
__device__ __forceinline__ void load_frag(const bf16_t* p, float* v) { load8(p, v); }
// A fragment as loaded: converted only after every load of a round has been issued.  A conversion next to its
// (conditional) load makes the compiler wait for that one load before it issues the next.
template <typename T> struct FragRaw;
template <> struct FragRaw<float> { float4 v; };
template <> struct FragRaw<bf16_t> { uint4 v; };
__device__ __forceinline__ void frag_load(FragRaw<float>& r, const float* p) { r.v = *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void frag_load(FragRaw<bf16_t>& r, const bf16_t* p) { r.v = *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void frag_zero(FragRaw<float>& r) { r.v = make_float4(0.f, 0.f, 0.f, 0.f); }
__device__ __forceinline__ void frag_zero(FragRaw<bf16_t>& r) { r.v = make_uint4(0u, 0u, 0u, 0u); }
__device__ __forceinline__ void frag_unpack(const FragRaw<float>& r, float* v) { v[0] = r.v.x; v[1] = r.v.y; v[2] = r.v.z; v[3] = r.v.w; }
__device__ __forceinline__ void frag_unpack(const FragRaw<bf16_t>& r, float* v) {
  v[0] = __uint_as_float(r.v.x << 16); v[1] = __uint_as_float(r.v.x & 0xffff0000u);
  v[2] = __uint_as_float(r.v.y << 16); v[3] = __uint_as_float(r.v.y & 0xffff0000u);
  v[4] = __uint_as_float(r.v.z << 16); v[5] = __uint_as_float(r.v.z & 0xffff0000u);
  v[6] = __uint_as_float(r.v.w << 16); v[7] = __uint_as_float(r.v.w & 0xffff0000u);
}

__device__ __forceinline__ f4v tiny_mma(const float* a, const float* b, f4v acc, float) {
#pragma unroll
  for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[e], acc, 0, 0, 0);
  return acc;
}
__device__ __forceinline__ f4v tiny_mma(const float* a, const float* b, f4v acc, bf16_t) {
  uint4 pa, pb;
  pa.x = f32x2_to_bf16x2(a[0], a[1]); pa.y = f32x2_to_bf16x2(a[2], a[3]);
  pa.z = f32x2_to_bf16x2(a[4], a[5]); pa.w = f32x2_to_bf16x2(a[6], a[7]);
  pb.x = f32x2_to_bf16x2(b[0], b[1]); pb.y = f32x2_to_bf16x2(b[2], b[3]);
  pb.z = f32x2_to_bf16x2(b[4], b[5]); pb.w = f32x2_to_bf16x2(b[6], b[7]);
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pa), __builtin_bit_cast(bf16x8, pb), acc, 0, 0, 0);
}

template <typename T, int MODE, int NW>
__device__ __forceinline__ void pw_gemm_tiny_body(const GemmArgs& p, const int bid) {
  constexpr int G = TinyStep<T>::G, KS = TinyStep<T>::KS, U = 4;
  // a block of NW wavefronts works on NW / 4 tiles, four wavefronts each
  constexpr int GROUPS = NW / 4;
  __shared__ float red[GROUPS][4][16][17];
  __shared__ float sred[GROUPS][2][16][17];
  if (MODE == MODE_DGRAD) __builtin_amdgcn_s_setprio(3);   // data-gradient chain: ahead of the weight-gradient stream's waves
  const int grp = (threadIdx.x >> 8), wave = (threadIdx.x >> 6) & 3, lane = threadIdx.x & 63;
  const int tile = bid * GROUPS + grp;
  const bool tile_ok = tile < p.jtiles * p.itiles;
  const int jt = tile % p.jtiles, it = tile / p.jtiles;
  const size_t i0 = (size_t)it * 16;
  const int j0 = jt * 16;
  const int R = MODE == MODE_FWD ? p.K : p.N;       // reduction extent (a multiple of G)
  const int nj = MODE == MODE_FWD ? p.N : p.K;      // output columns
  const int nst = (R + KS - 1) / KS;
  const int sb = wave * nst / 4, se = (wave + 1) * nst / 4;
  const int l16 = lane & 15, kg = (lane >> 4) * G;
  const size_t row = i0 + l16;
  const int col = j0 + l16;
  const bool row_ok = tile_ok && row < p.M, col_ok = tile_ok && col < nj;
  const T* X = reinterpret_cast<const T*>(p.x) + row * (size_t)R;
  const T* W = reinterpret_cast<const T*>(p.y);
  const bool view = MODE == MODE_FWD && p.view.scale != nullptr;
  const float lo = act_lo(p.view.act), hi = act_hi(p.view.act);
  // the output element this thread writes after the reduction; what is added to it there (residual, bias) is
  // requested now: a load at the end of the kernel would be one more round trip on the launch-latency path
  const int orow = (threadIdx.x >> 4) & 15, ocol = threadIdx.x & 15;
  const size_t ig = i0 + orow;
  const int jg = j0 + ocol;
  const bool in = tile_ok && ig < p.M && jg < nj;
  float addend = 0.f;
  if (MODE == MODE_FWD) { if (p.bias && tile_ok && jg < nj) addend = p.bias[jg]; }
  else if (p.res && in) addend = to_f32(reinterpret_cast<const T*>(p.res)[ig * p.K + jg]);

  f4v acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = sb; s < se; s += U) {
    float a[U][G], b[U][G], sc[U][G], sh[U][G];
    FragRaw<T> ar[U], br[U];
    T bs[U][G];                                // data gradient: single elements of W down a column
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = (s + u) * KS + kg;
      const bool ok = s + u < se && k < R;
      frag_zero(ar[u]); frag_zero(br[u]);
#pragma unroll
      for (int e = 0; e < G; ++e) { sc[u][e] = 1.f; sh[u][e] = 0.f; }
      if (ok && row_ok) {
        frag_load(ar[u], X + k);
        if (view) {
          load_frag(p.view.scale + k, sc[u]);
          load_frag(p.view.shift + k, sh[u]);
          if (G == 8) { load_frag(p.view.scale + k + 4, sc[u] + 4); load_frag(p.view.shift + k + 4, sh[u] + 4); }
        }
      }
      if (MODE == MODE_FWD) {
        if (ok && col_ok) frag_load(br[u], W + (size_t)col * p.K + k);
      } else {
        // unconditional, from rows / a column that exist (R is a multiple of G): zeroed below when out of range
        const int kc = ok ? k : 0, cc = col_ok ? col : 0;
#pragma unroll
        for (int e = 0; e < G; ++e) bs[u][e] = W[(size_t)(kc + e) * p.K + cc];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      frag_unpack(ar[u], a[u]);
      if (MODE == MODE_FWD) {
        frag_unpack(br[u], b[u]);
      } else {
        const bool okb = s + u < se && (s + u) * KS + kg < R && col_ok;
#pragma unroll
        for (int e = 0; e < G; ++e) b[u][e] = okb ? to_f32(bs[u][e]) : 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (view) {
        const bool live = s + u < se && (s + u) * KS + kg < R && row_ok;   // padding stays exactly zero
#pragma unroll
        for (int e = 0; e < G; ++e) {
          float y = round_to<T>(clamp_act(fmaf(a[u][e], sc[u][e], sh[u][e]), lo, hi));
          a[u][e] = live ? y : 0.f;
        }
      }
      acc = tiny_mma(a[u], b[u], acc, T());
    }
  }

  // register r of lane l is C[4*(l/16) + r][l%16]
#pragma unroll
  for (int r = 0; r < 4; ++r) red[grp][wave][4 * (lane >> 4) + r][l16] = acc[r];
  __syncthreads();
  asm volatile("" : "+v"(addend));          // first use: its conversion stays here
  const float v0 = red[grp][0][orow][ocol] + red[grp][1][orow][ocol] + red[grp][2][orow][ocol] + red[grp][3][orow][ocol];
  float v = v0;
  if (MODE == MODE_FWD) {
    v += addend;
    if (in) reinterpret_cast<T*>(p.out)[ig * p.N + jg] = from_f32<T>(v);
    if (p.stats) {
      const float sv = in ? round_to<T>(v) : 0.f;     // statistics of the values as stored
      sred[grp][0][orow][ocol] = sv;
      sred[grp][1][orow][ocol] = sv * sv;
      __syncthreads();
      if ((threadIdx.x & 255) < 32 && tile_ok) {
        const int sq = (threadIdx.x >> 4) & 1, c = threadIdx.x & 15;
        float tot = 0.f;
#pragma unroll
        for (int rr = 0; rr < 16; ++rr) tot += sred[grp][sq][rr][c];
        if (j0 + c < p.N) p.stats[((size_t)it * 2 + sq) * p.N + j0 + c] = tot;
      }
    }
  } else {
    if (in) reinterpret_cast<T*>(p.out)[ig * p.K + jg] = from_f32<T>(v + addend);
  }
}

// Weight gradient of a short problem, g_w[n][k] += sum_m dZ[m][n] * A'[m][k], in one launch: a block owns a
// 16 x 16 tile of g_w, its four wavefronts split the pixels and meet in LDS, so there are no partial
// buffers and no second kernel.  A lane's two MFMA operands are single elements of consecutive columns
// (64-byte runs), the per-column scale/shift of the view sit in two registers.  Both storage types use
// the fp32 16x16x4 MFMA: products of bfloat16 values are exact in fp32.
template <typename T, int NW>
__device__ __forceinline__ void pw_wgrad_tiny_body(const GemmArgs& p, const int K_out, const int bid) {
  constexpr int U = 8;
  __shared__ float red[NW][16][17];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int jt = bid % p.jtiles, it = bid / p.jtiles;
  const int l16 = lane & 15, mg = lane >> 4;
  const int n = it * 16 + l16, k = jt * 16 + l16;
  const bool n_ok = n < p.N, k_ok = k < p.K;
  const T* X = reinterpret_cast<const T*>(p.x) + (n_ok ? n : 0);
  const T* Y = reinterpret_cast<const T*>(p.y) + (k_ok ? k : 0);
  const bool view = p.view.scale != nullptr;
  const float sc = view && k_ok ? p.view.scale[k] : 1.f, sh = view && k_ok ? p.view.shift[k] : 0.f;
  const float lo = act_lo(p.view.act), hi = act_hi(p.view.act);
  const size_t M = p.M;
  // the gradient element this thread adds to after the reduction, requested now (see pw_gemm_tiny_body)
  const int orow = (threadIdx.x >> 4) & 15, ocol = threadIdx.x & 15;
  const int on = it * 16 + orow, ok_ = jt * 16 + ocol;
  const bool writer = threadIdx.x < 256 && on < p.N && ok_ < K_out;
  float* dst = reinterpret_cast<float*>(p.out) + (writer ? (size_t)on * K_out + ok_ : 0);
  float g_old = writer ? *dst : 0.f;
  const size_t per = ((M + 4 * NW - 1) / (4 * NW)) * 4;    // pixels per wavefront, a multiple of 4
  const size_t mb = (size_t)wave * per, me = mb + per < M ? mb + per : M;
  f4v acc = {0.f, 0.f, 0.f, 0.f};
  for (size_t m0 = mb; m0 < me; m0 += 4 * U) {
    float x[U], y[U];
    T xr[U], yr[U];                            // converted after all loads of the round are out (see FragRaw)
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t m = m0 + 4 * u + mg;
      const size_t mc = m < me ? m : mb;       // unconditional loads from a valid row (X, Y point at valid columns)
      xr[u] = X[mc * p.N];
      yr[u] = Y[mc * p.K];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const bool ok = m0 + 4 * u + mg < me;
      x[u] = ok && n_ok ? to_f32(xr[u]) : 0.f;
      y[u] = ok && k_ok ? to_f32(yr[u]) : 0.f;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float a = y[u];
      if (view) {
        const bool ok = m0 + 4 * u + mg < me && k_ok;       // padding stays exactly zero
        a = ok ? round_to<T>(clamp_act(fmaf(a, sc, sh), lo, hi)) : 0.f;
      }
      acc = __builtin_amdgcn_mfma_f32_16x16x4f32(x[u], a, acc, 0, 0, 0);
    }
  }
  // register r of lane l is tile element (row 4*(l/16) + r = n, column l%16 = k)
#pragma unroll
  for (int r = 0; r < 4; ++r) red[wave][4 * mg + r][l16] = acc[r];
  __syncthreads();
  asm volatile("" : "+v"(g_old));
  if (writer) {
    float v = 0.f;
#pragma unroll
    for (int q = 0; q < NW; ++q) v += red[q][orow][ocol];
    *dst = g_old + v;
  }
}

template <typename T, int MODE>
__global__ __launch_bounds__(256) void pw_gemm_tiny_k(GemmArgs p) { pw_gemm_tiny_body<T, MODE, 4>(p, xcd_logical_block()); }   // the column tiles of a row panel share an L2
template <typename T>
__global__ __launch_bounds__(256) void pw_wgrad_tiny_k(GemmArgs p, int K_out) { pw_wgrad_tiny_body<T, 4>(p, K_out, blockIdx.x); }
// data gradient and weight gradient of one short layer in one launch: both read the same dZ, their tiles are
// independent, and for these sizes a launch costs more than either of them.  NW wavefronts per block: with many
// pixels the weight-gradient tiles are few and each walks all pixels, so 16 wavefronts share that walk.
template <typename T, int NW>
__global__ __launch_bounds__(64 * NW) void pw_bwd_tiny_k(GemmArgs pd, GemmArgs pw, int K_out, int n_dgrad) {
  if ((int)blockIdx.x < n_dgrad) pw_gemm_tiny_body<T, MODE_DGRAD, NW>(pd, blockIdx.x);
  else pw_wgrad_tiny_body<T, NW>(pw, K_out, blockIdx.x - n_dgrad);
}

// the 16 x 16 kernel serves problems whose output is short (few rows) and whose reduction extent
// allows aligned vector fragments
static bool tiny_ok(int dt, size_t M, int R, int ncols, bool stats) {
  const int G = dt == 0 ? 4 : 8;
  if (M > 2048 || R % G != 0) return false;      // measured: taller problems run faster on the staged kernels
  if ((double)M * R * ncols > 64.0 * 1024 * 1024) return false;   // every block re-reads its operand rows
  if (stats && (M + 15) / 16 > (size_t)kMaxPartials) return false;
  return true;
}

template <int MODE>
static void launch_tiny(int dt, hipStream_t st, GemmArgs& a, int ncols) {
  a.jtiles = (ncols + 15) / 16;
  a.itiles = (int)((a.M + 15) / 16);
  a.nranges = a.itiles;
  a.tiles_per_range = 1;
  unsigned grid = (unsigned)((size_t)a.jtiles * a.itiles);
  if (dt == 0) hipLaunchKernelGGL((pw_gemm_tiny_k<float, MODE>), dim3(grid), dim3(256), 0, st, a);
  else hipLaunchKernelGGL((pw_gemm_tiny_k<bf16_t, MODE>), dim3(grid), dim3(256), 0, st, a);
}

template <typename T, int MODE, bool VEC>
static void launch_t(hipStream_t st, const GemmArgs& a, bool small, unsigned grid) {
  if (small) { hipLaunchKernelGGL((pw_gemm_k<T, MODE, true, VEC>), dim3(grid), dim3(256), 0, st, a); return; }
  const size_t red = MODE == MODE_FWD ? (size_t)a.K : MODE == MODE_DGRAD ? (size_t)a.N : a.mchunk;   // reduction extent of a block
  // Every mode stages 32 reduction elements per step.  64 per step made the weight-gradient kernel itself 5 % faster
  // (half the barriers) but costs 55 KB of LDS per block: next to the data-gradient chain on the other stream the
  // step was 0.9 % slower with it.
  if (MODE == MODE_WGRAD && red > 32)
    hipLaunchKernelGGL((pw_gemm_rows_k<T, MODE, VEC, 32, false, MODE == MODE_WGRAD>), dim3(grid), dim3(256), 0, st, a);
  else if (MODE == MODE_DGRAD && red > 32) {     // at least two steps per tile: two steps' loads in flight
    constexpr bool D = MODE == MODE_DGRAD;
    if (a.res) hipLaunchKernelGGL((pw_gemm_rows_k<T, MODE, VEC, 32, D, D>), dim3(grid), dim3(256), 0, st, a);
    else hipLaunchKernelGGL((pw_gemm_rows_k<T, MODE, VEC, 32, false, D>), dim3(grid), dim3(256), 0, st, a);
  }
  else if (MODE == MODE_DGRAD && a.res) hipLaunchKernelGGL((pw_gemm_rows_k<T, MODE, VEC, 32, MODE == MODE_DGRAD>), dim3(grid), dim3(256), 0, st, a);
  else hipLaunchKernelGGL((pw_gemm_rows_k<T, MODE, VEC, 32>), dim3(grid), dim3(256), 0, st, a);
}

template <int MODE>
static void launch(int dt, hipStream_t st, const GemmArgs& a, bool small) {
  unsigned grid = (unsigned)((size_t)a.jtiles * a.nranges);
  const bool vec = a.K % 8 == 0 && a.N % 8 == 0;   // whole vectors along both weight dimensions
  if (dt == 0) {
    if (vec) launch_t<float, MODE, true>(st, a, small, grid);
    else launch_t<float, MODE, false>(st, a, small, grid);
  } else {
    if (vec) launch_t<bf16_t, MODE, true>(st, a, small, grid);
    else launch_t<bf16_t, MODE, false>(st, a, small, grid);
  }
}

// Row-streaming passes (forward, dgrad): tile shape and the split of the row tiles into ranges.
static void plan_rows(size_t M, int ncols, int R, GemmArgs* a, bool* small) {
  a->jtiles = (ncols + BJ - 1) / BJ;
  size_t big_tiles = (M + 127) / 128;
  // short problems: too few 128-row tiles to fill 256 CUs and a reduction worth splitting
  *small = (big_tiles * a->jtiles < 96 && R >= 128) || (big_tiles * a->jtiles < 512 && R >= 512);
  int TI = *small ? 32 : 128;
  a->itiles = (int)((M + TI - 1) / TI);
  int want = (4096 + a->jtiles - 1) / a->jtiles;          // about 4096 blocks in flight
  if (want > kMaxPartials) want = kMaxPartials;
  if (want < 1) want = 1;
  a->tiles_per_range = (a->itiles + want - 1) / want;
  a->nranges = (a->itiles + a->tiles_per_range - 1) / a->tiles_per_range;
}

void pw_fwd(int dt, hipStream_t st, HView av, const void* w, const float* bias, size_t M, int K, int N,
            void* z, float* stats, int* P_out) {
  GemmArgs a{};
  a.x = av.z; a.y = w; a.view = View{av.z, av.scale, av.shift, av.act};
  a.bias = bias; a.out = z; a.stats = stats; a.M = M; a.K = K; a.N = N;
  KScope ks(st, "pw_fwd", ((double)M * K + (double)M * N + (double)N * K) * (dt == 0 ? 4.0 : 2.0), 2.0 * M * K * N, (long)M, K, N);
  if (tiny_ok(dt, M, K, N, stats != nullptr)) {
    launch_tiny<MODE_FWD>(dt, st, a, N);
    if (P_out) *P_out = a.nranges;
    return;
  }
  if (!bias && pw_deep_ok(dt, M, K, N, false)) { pw_fwd_deep(st, av, w, M, K, N, z, stats, P_out); return; }
  bool small;
  plan_rows(M, N, K, &a, &small);
  if (P_out) *P_out = a.nranges;
  launch<MODE_FWD>(dt, st, a, small);
}

void pw_dgrad(int dt, hipStream_t st, const void* dz, const void* w, const void* res, size_t M, int K,
              int N, void* dA) {
  GemmArgs a{};
  a.x = dz; a.y = w; a.res = res; a.out = dA; a.M = M; a.K = K; a.N = N;
  KScope ks(st, "pw_dgrad", ((double)M * K * (res ? 2.0 : 1.0) + (double)M * N + (double)N * K) * (dt == 0 ? 4.0 : 2.0), 2.0 * M * K * N, (long)M, K, N);
  if (tiny_ok(dt, M, N, K, false)) {
    launch_tiny<MODE_DGRAD>(dt, st, a, K);
    return;
  }
  if (pw_deep_ok(dt, M, N, K, true)) { pw_dgrad_deep(st, dz, w, res, M, K, N, dA); return; }
  bool small;
  plan_rows(M, K, N, &a, &small);
  launch<MODE_DGRAD>(dt, st, a, small);
}

// wgrad: output tiles (N x K) times splits of the pixel range
static void plan_wgrad(size_t M, int K, int N, GemmArgs* a, bool* small) {
  a->jtiles = (K + BJ - 1) / BJ;
  *small = N <= 32;                         // few output rows: 32-row tiles waste less of the MFMA
  int TI = *small ? 32 : 128;
  int CH = *small ? 128 : 32;
  a->itiles = (N + TI - 1) / TI;
  size_t tiles = (size_t)a->itiles * a->jtiles;
  size_t s = (512 + tiles - 1) / tiles;
  size_t smax = (M + 2 * CH - 1) / (2 * CH);      // at least two reduction chunks per split
  if (s > smax) s = smax;
  if (s > (size_t)kMaxPartials) s = kMaxPartials;
  if (s < 1) s = 1;
  size_t mc = (M + s - 1) / s;
  mc = ((mc + CH - 1) / CH) * CH;
  a->mchunk = mc;
  a->nranges = (int)((M + mc - 1) / mc) * a->itiles;
  a->tiles_per_range = 1;
}

size_t pw_wgrad_ws(size_t M, int K, int N) {
  GemmArgs a{};
  bool small;
  plan_wgrad(M, K, N, &a, &small);
  const size_t own = (size_t)(a.nranges / a.itiles) * N * K, tr = pw_wgrad_tr_ws(M, K, N);   // either storage type may run
  return own > tr ? own : tr;
}

void pw_wgrad(int dt, hipStream_t st, const void* dz, HView av, size_t M, int K, int N, float* ws,
              float* g_w, int K_out) {
  GemmArgs a{};
  a.x = dz; a.y = av.z; a.view = View{av.z, av.scale, av.shift, av.act};
  a.out = ws; a.M = M; a.K = K; a.N = N;
  if (M <= 2048) {
    // short problem: straight into g_w, no partials
    KScope ks(st, "pw_wgrad", ((double)M * K + (double)M * N) * (dt == 0 ? 4.0 : 2.0) + (double)N * K * 8, 2.0 * M * K * N, (long)M, K, N);
    a.out = g_w;
    a.jtiles = (K + 15) / 16;
    a.itiles = (N + 15) / 16;
    const unsigned grid = (unsigned)a.jtiles * a.itiles;
    if (dt == 0) hipLaunchKernelGGL(pw_wgrad_tiny_k<float>, dim3(grid), dim3(256), 0, st, a, K_out < 0 ? K : K_out);
    else hipLaunchKernelGGL(pw_wgrad_tiny_k<bf16_t>, dim3(grid), dim3(256), 0, st, a, K_out < 0 ? K : K_out);
    return;
  }
  if (pw_wgrad_tr_ok(dt, M, K, N)) { pw_wgrad_tr(st, dz, av, M, K, N, ws, g_w, K_out); return; }
  bool small;
  plan_wgrad(M, K, N, &a, &small);
  int S = a.nranges / a.itiles;
  {
    KScope ks(st, "pw_wgrad", ((double)M * K + (double)M * N) * (dt == 0 ? 4.0 : 2.0) + (double)S * N * K * 4, 2.0 * M * K * N, (long)M, K, N);
    launch<MODE_WGRAD>(dt, st, a, small);
  }
  // K_out < K: the last K - K_out columns of A are padding and g_w is [N][K_out]
  if (K_out < 0) K_out = K;
  reduce_partials(st, ws, S, (size_t)N * K, K, (size_t)K_out, 1, g_w, K_out);
}

// wgrad then dgrad of one pointwise layer; short problems take one launch for both
void pw_bwd(int dt, hipStream_t st, const void* dz, const void* w, const void* res, HView av, size_t M, int K, int N,
            float* ws, float* g_w, void* dA) {
  if (M <= 2048 && tiny_ok(dt, M, N, K, false)) {
    GemmArgs d{}, g{};
    d.x = dz; d.y = w; d.res = res; d.out = dA; d.M = M; d.K = K; d.N = N;
    d.jtiles = (K + 15) / 16; d.itiles = (int)((M + 15) / 16); d.nranges = d.itiles; d.tiles_per_range = 1;
    g.x = dz; g.y = av.z; g.view = View{av.z, av.scale, av.shift, av.act}; g.out = g_w; g.M = M; g.K = K; g.N = N;
    g.jtiles = (K + 15) / 16; g.itiles = (N + 15) / 16;
    const int nd = d.jtiles * d.itiles, nw = g.jtiles * g.itiles;
    const double es = dt == 0 ? 4.0 : 2.0;
    KScope ks(st, "pw_bwd", ((double)M * K * (res ? 3.0 : 2.0) + (double)M * N + (double)N * K) * es + (double)N * K * 8,
              4.0 * M * K * N, (long)M, K, N);
    if (M > 512) {
      const int nd4 = (nd + 3) / 4;             // four data-gradient tiles per 16-wavefront block
      if (dt == 0) hipLaunchKernelGGL((pw_bwd_tiny_k<float, 16>), dim3(nd4 + nw), dim3(1024), 0, st, d, g, K, nd4);
      else hipLaunchKernelGGL((pw_bwd_tiny_k<bf16_t, 16>), dim3(nd4 + nw), dim3(1024), 0, st, d, g, K, nd4);
    } else {
      if (dt == 0) hipLaunchKernelGGL((pw_bwd_tiny_k<float, 4>), dim3(nd + nw), dim3(256), 0, st, d, g, K, nd);
      else hipLaunchKernelGGL((pw_bwd_tiny_k<bf16_t, 4>), dim3(nd + nw), dim3(256), 0, st, d, g, K, nd);
    }
    return;
  }
  pw_wgrad(dt, st, dz, av, M, K, N, ws, g_w);
  pw_dgrad(dt, st, dz, w, res, M, K, N, dA);
}

}  // namespace ftp
