// Small dense convolutions (3x3 stem, conv1d) and depthwise 3x3, NHWC.
// Inputs are read through a View, so the producer's BatchNorm + activation is
// applied on load and zero padding is inserted after it (a halo cell is 0, not
// act(bn(0))).  Depthwise layers over short tensors (at most 2048 pixels) run whole
// forward / backward sub-chains in one launch (dw_fwd_bn_small_k, dw_bwd_small_k).
#include "dev_common.h"
#include "kernels.h"
#include "bn_pending.h"

namespace ftp {

#define FTP_DISPATCH(dt, ...)                   \
  do {                                          \
    if ((dt) == 0) { typedef float T; __VA_ARGS__; } \
    else { typedef bf16_t T; __VA_ARGS__; }     \
  } while (0)

// g[(j % C) * stride_c + (j / C) * stride_q] += sum_p ws[p * QC + j]   (float64 sum, fixed order)
__global__ void reduce_partials_flat_k(const float* __restrict__ ws, int P, size_t QC, int C, size_t stride_q,
                                       size_t stride_c, int valid_c, float* __restrict__ g) {
  size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= QC || (int)(j % C) >= valid_c) return;
  double s = 0.0;
  for (int p = 0; p < P; ++p) s += (double)ws[(size_t)p * QC + j];
  size_t o = (j % C) * stride_c + (j / C) * stride_q;
  g[o] += (float)s;
}

// many partials: 16 outputs per block, 16 lanes share the partials of one output
__global__ void reduce_partials_wide_k(const float* __restrict__ ws, int P, size_t QC, int C, size_t stride_q,
                                       size_t stride_c, int valid_c, float* __restrict__ g) {
  __shared__ double sm[16][17];
  const int jl = threadIdx.x & 15, lane = threadIdx.x >> 4;
  const size_t j = (size_t)xcd_logical_block() * 16 + jl;     // neighbours read the same lines of the partials: one L2
  double s = 0.0;
  if (j < QC) {
    int p = lane;
    // many partials: sixteen independent loads per round (a round is one trip to memory, and this kernel is nothing but
    // such trips); the sums keep their order
    for (; p + 240 < P; p += 256) {
      float v[16];
#pragma unroll
      for (int u = 0; u < 16; ++u) v[u] = ws[(size_t)(p + 16 * u) * QC + j];
#pragma unroll
      for (int u = 0; u < 16; ++u) s += (double)v[u];
    }
    for (; p + 48 < P; p += 64) {        // four independent loads per round
      float a = ws[(size_t)p * QC + j], b = ws[(size_t)(p + 16) * QC + j];
      float c2 = ws[(size_t)(p + 32) * QC + j], d = ws[(size_t)(p + 48) * QC + j];
      s += (double)a; s += (double)b; s += (double)c2; s += (double)d;
    }
    for (; p < P; p += 16) s += (double)ws[(size_t)p * QC + j];
  }
  sm[lane][jl] = s;
  __syncthreads();
  if (lane == 0 && j < QC && (int)(j % C) < valid_c) {
    double t = 0.0;
#pragma unroll
    for (int l = 0; l < 16; ++l) t += sm[l][jl];
    size_t o = (j % C) * stride_c + (j / C) * stride_q;
    g[o] += (float)t;
  }
}

// columns (j % C) >= valid_c are padding and are skipped
void reduce_partials(hipStream_t st, const float* ws, int P, size_t QC, int C, size_t stride_q,
                     size_t stride_c, float* g, int valid_c) {
  if (valid_c < 0) valid_c = C;
  KScope ks(st, "reduce_partials", ((double)P + 2.0) * QC * 4, (double)P * QC);
  if (P <= 8)
    hipLaunchKernelGGL(reduce_partials_flat_k, dim3((unsigned)((QC + 255) / 256)), dim3(256), 0, st, ws, P, QC, C,
                       stride_q, stride_c, valid_c, g);
  else
    hipLaunchKernelGGL(reduce_partials_wide_k, dim3((unsigned)((QC + 15) / 16)), dim3(256), 0, st, ws, P, QC, C,
                       stride_q, stride_c, valid_c, g);
}

// ======================================================== generic direct conv
static const int kWChunkFloats = 8192;  // LDS weight chunk: 32 KB

int conv_direct_supported(const ConvGeom& g) {
  return g.Cout % 8 == 0 && g.Cout <= 1024 && (size_t)g.Cin * g.Cout <= (size_t)kWChunkFloats;
}

// thread = (output pixel, 8 output channels); weights of a few taps at a time in LDS as [k][Cout]
template <typename T>
__global__ void conv_direct_fwd_k(View in, const T* __restrict__ w, ConvGeom g, int TC, int PPB,
                                  T* __restrict__ z) {
  extern __shared__ float wl[];
  const int CGo = g.Cout / 8;
  const int pl = threadIdx.x / CGo, cg = threadIdx.x % CGo;
  const size_t total = (size_t)g.N * g.Hout * g.Wout;
  const size_t pix = (size_t)blockIdx.x * PPB + pl;
  const bool valid = pix < total;
  int n = 0, ho = 0, wo = 0;
  if (valid) {
    wo = (int)(pix % g.Wout);
    size_t r = pix / g.Wout;
    ho = (int)(r % g.Hout);
    n = (int)(r / g.Hout);
  }
  const int ntaps = g.kh * g.kw, K = ntaps * g.Cin;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int t0 = 0; t0 < ntaps; t0 += TC) {
    const int tcnt = ntaps - t0 < TC ? ntaps - t0 : TC;
    const int kc = tcnt * g.Cin;
    __syncthreads();
    for (int idx = threadIdx.x; idx < kc * g.Cout; idx += blockDim.x) {
      int co = idx / kc, k = idx % kc;
      wl[k * g.Cout + co] = to_f32(w[(size_t)co * K + t0 * g.Cin + k]);
    }
    __syncthreads();
    if (valid) {
      for (int t = 0; t < tcnt; ++t) {
        int tap = t0 + t, i = tap / g.kw, j = tap % g.kw;
        int hi = ho * g.stride + i - g.ph, wi = wo * g.stride + j - g.pw;
        if (hi < 0 || hi >= g.Hin || wi < 0 || wi >= g.Win) continue;
        size_t base = (((size_t)n * g.Hin + hi) * g.Win + wi) * g.Cin;
        for (int ci = 0; ci < g.Cin; ++ci) {
          float xv = view_at<T>(in, base + ci, ci);
          const float* wr = wl + (size_t)(t * g.Cin + ci) * g.Cout + cg * 8;
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] = fmaf(xv, wr[e], acc[e]);
        }
      }
    }
  }
  if (valid) store8(z + pix * g.Cout + cg * 8, acc);
}

void conv_direct_fwd(int dt, hipStream_t st, HView in, const void* w, const ConvGeom& g, void* z) {
  int CGo = g.Cout / 8;
  int PPB = 256 / CGo;
  if (PPB < 1) PPB = 1;
  int TC = kWChunkFloats / (g.Cin * g.Cout);
  if (TC < 1) TC = 1;
  if (TC > g.kh * g.kw) TC = g.kh * g.kw;
  size_t total = (size_t)g.N * g.Hout * g.Wout;
  size_t sm = (size_t)TC * g.Cin * g.Cout * sizeof(float);
  View v{in.z, in.scale, in.shift, in.act};
  KScope ks(st, "conv_direct_fwd", ((double)g.N * g.Hin * g.Win * g.Cin + (double)total * g.Cout + (double)g.kh * g.kw * g.Cin * g.Cout) * (dt == 0 ? 4.0 : 2.0),
            2.0 * total * g.Cout * g.kh * g.kw * g.Cin);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(conv_direct_fwd_k<T>, dim3((unsigned)((total + PPB - 1) / PPB)),
                                      dim3(PPB * CGo), sm, st, v, (const T*)w, g, TC, PPB, (T*)z));
}

// thread = (input pixel, input channel): gathers every (tap, cout) that reaches it
template <typename T>
__global__ void conv_direct_dgrad_k(const T* __restrict__ dz, const T* __restrict__ w, ConvGeom g,
                                    T* __restrict__ dIn) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)g.N * g.Hin * g.Win * g.Cin;
  if (idx >= total) return;
  int ci = (int)(idx % g.Cin);
  size_t r = idx / g.Cin;
  int wi = (int)(r % g.Win);
  r /= g.Win;
  int hi = (int)(r % g.Hin);
  int n = (int)(r / g.Hin);
  const int K = g.kh * g.kw * g.Cin;
  float acc = 0.f;
  for (int i = 0; i < g.kh; ++i) {
    int hn = hi + g.ph - i;
    if (hn < 0 || hn % g.stride) continue;
    int ho = hn / g.stride;
    if (ho >= g.Hout) continue;
    for (int j = 0; j < g.kw; ++j) {
      int wn = wi + g.pw - j;
      if (wn < 0 || wn % g.stride) continue;
      int wo = wn / g.stride;
      if (wo >= g.Wout) continue;
      const T* d = dz + (((size_t)n * g.Hout + ho) * g.Wout + wo) * g.Cout;
      const T* wp = w + (size_t)(i * g.kw + j) * g.Cin + ci;
      for (int co = 0; co < g.Cout; ++co) acc = fmaf(to_f32(d[co]), to_f32(wp[(size_t)co * K]), acc);
    }
  }
  dIn[idx] = from_f32<T>(acc);
}

void conv_direct_dgrad(int dt, hipStream_t st, const void* dz, const void* w, const ConvGeom& g, void* dIn) {
  size_t total = (size_t)g.N * g.Hin * g.Win * g.Cin;
  KScope ks(st, "conv_direct_dgrad", ((double)total + (double)g.N * g.Hout * g.Wout * g.Cout) * (dt == 0 ? 4.0 : 2.0),
            2.0 * g.N * g.Hout * g.Wout * g.Cout * g.kh * g.kw * g.Cin);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(conv_direct_dgrad_k<T>, dim3((unsigned)((total + 255) / 256)), dim3(256),
                                      0, st, (const T*)dz, (const T*)w, g, (T*)dIn));
}

// Weight gradient of a small dense convolution: the input patches are written out once as a
// matrix A[pixel][Kpad] (k = (tap, ci), zero padded to a multiple of 8, producer BatchNorm +
// activation applied), then dW = dZ^T * A runs on the MFMA weight-gradient kernel.
template <typename T>
__global__ void im2col_k(View in, ConvGeom g, int Kpad, T* __restrict__ out) {
  // which tap and input channel column k of the matrix is: worked out once per block (two divisions per column)
  // instead of once per element, packed as (row offset + 1) << 24 | column offset << 16 | channel; 0 = padding column
  extern __shared__ uint32_t taps[];
  const int KG = Kpad / 8, K = g.kh * g.kw * g.Cin;
  for (int k = threadIdx.x; k < Kpad; k += blockDim.x) {
    uint32_t t = 0;
    if (k < K) {
      const int tap = k / g.Cin, ci = k - tap * g.Cin, i = tap / g.kw, j = tap - i * g.kw;
      t = ((uint32_t)(i + 1) << 24) | ((uint32_t)j << 16) | (uint32_t)ci;
    }
    taps[k] = t;
  }
  __syncthreads();
  const size_t total = (size_t)g.N * g.Hout * g.Wout * KG;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int kg = (int)(idx % KG);
    const size_t pix = idx / KG;
    const int wo = (int)(pix % g.Wout);
    const size_t r = pix / g.Wout;
    const int ho = (int)(r % g.Hout), n = (int)(r / g.Hout);
    const int h0 = ho * g.stride - g.ph, w0 = wo * g.stride - g.pw;
    const size_t img = (size_t)n * g.Hin;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t t = taps[kg * 8 + e];
      const int hi = h0 + (int)(t >> 24) - 1, wi = w0 + (int)((t >> 16) & 0xffu), ci = (int)(t & 0xffffu);
      float x = 0.f;
      if (t != 0 && hi >= 0 && hi < g.Hin && wi >= 0 && wi < g.Win)
        x = view_at<T>(in, ((img + hi) * g.Win + wi) * g.Cin + ci, ci);
      v[e] = x;
    }
    store8(out + idx * 8, v);
  }
}

static int direct_kpad(const ConvGeom& g) { return (g.kh * g.kw * g.Cin + 7) / 8 * 8; }

size_t conv_direct_im2col_elems(const ConvGeom& g) { return (size_t)g.N * g.Hout * g.Wout * direct_kpad(g); }

size_t conv_direct_wgrad_ws(const ConvGeom& g) {
  return pw_wgrad_ws((size_t)g.N * g.Hout * g.Wout, direct_kpad(g), g.Cout);
}

void conv_direct_wgrad(int dt, hipStream_t st, const void* dz, HView in, const ConvGeom& g, void* im2col, float* ws,
                       float* g_w, bool patches_ready) {
  const int Kpad = direct_kpad(g), K = g.kh * g.kw * g.Cin;
  const size_t M = (size_t)g.N * g.Hout * g.Wout;
  View v{in.z, in.scale, in.shift, in.act};
  if (!patches_ready) {
    const double es = dt == 0 ? 4.0 : 2.0;
    KScope ks(st, "im2col", ((double)g.N * g.Hin * g.Win * g.Cin + (double)M * Kpad) * es, 0, (long)M, Kpad, g.Cout);
    size_t nvec = M * (Kpad / 8);
    unsigned grid = (unsigned)((nvec + 255) / 256 > 65536 ? 65536 : (nvec + 255) / 256);
    FTP_DISPATCH(dt, hipLaunchKernelGGL(im2col_k<T>, dim3(grid), dim3(256), (size_t)Kpad * sizeof(uint32_t), st, v, g, Kpad, (T*)im2col));
  }
  pw_wgrad(dt, st, dz, HView{im2col, nullptr, nullptr, 0}, M, Kpad, g.Cout, ws, g_w, K);
}

// Forward of a small dense convolution over many pixels (the 224x224 stem) as im2col + MFMA GEMM: the patch
// matrix costs one extra write and read of M x Kpad elements but the GEMM streams at several TB/s and leaves the
// BatchNorm statistics in its epilogue, where the direct kernel issues Cin*kh*kw scalar loads per output vector.
template <typename T>
__global__ void pad_rows_k(const T* __restrict__ w, int rows, int K, int Kpad, T* __restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * Kpad) return;
  const int r = i / Kpad, k = i - r * Kpad;
  out[i] = k < K ? w[(size_t)r * K + k] : from_f32<T>(0.f);
}

// many pixels (the 224x224 stem) or many taps x channels per output (conv1d): the direct kernel's scalar loads lose
int conv_direct_gemm_ok(const ConvGeom& g) {
  const int Kpad = direct_kpad(g);
  return g.Cout % 8 == 0 && (((size_t)g.N * g.Hout * g.Wout >= ((size_t)1 << 18) && Kpad <= 64) || (Kpad >= 40 && Kpad <= 2048));
}
size_t conv_direct_gemm_wpad_elems(const ConvGeom& g) { return (size_t)g.Cout * direct_kpad(g); }

void conv_direct_fwd_gemm(int dt, hipStream_t st, HView in, const void* w, const ConvGeom& g, void* im2col, void* wpad, void* z,
                          float* stats, int* P_out) {
  const int Kpad = direct_kpad(g), K = g.kh * g.kw * g.Cin;
  const size_t M = (size_t)g.N * g.Hout * g.Wout;
  View v{in.z, in.scale, in.shift, in.act};
  {
    const double es = dt == 0 ? 4.0 : 2.0;
    KScope ks(st, "im2col", ((double)g.N * g.Hin * g.Win * g.Cin + (double)M * Kpad) * es, 0, (long)M, Kpad, g.Cout);
    size_t nvec = M * (Kpad / 8);
    unsigned grid = (unsigned)((nvec + 255) / 256 > 65536 ? 65536 : (nvec + 255) / 256);
    FTP_DISPATCH(dt, hipLaunchKernelGGL(im2col_k<T>, dim3(grid), dim3(256), (size_t)Kpad * sizeof(uint32_t), st, v, g, Kpad, (T*)im2col));
    FTP_DISPATCH(dt, hipLaunchKernelGGL(pad_rows_k<T>, dim3((g.Cout * Kpad + 255) / 256), dim3(256), 0, st, (const T*)w, g.Cout, K,
                                        Kpad, (T*)wpad));
  }
  pw_fwd(dt, st, HView{im2col, nullptr, nullptr, 0}, wpad, nullptr, M, Kpad, g.Cout, z, stats, P_out);
}

// Data gradient of a stride-1 dense convolution as a forward convolution of dz with the taps flipped and the
// channel roles swapped: dIn[hi][ci] = sum_{i',j',co} dz[hi - (kh-1-ph) + i'][co] * w[co][kh-1-i'][kw-1-j'][ci],
// run as im2col(dz) x rearranged weights on the MFMA GEMM.
template <typename T>
__global__ void dgrad_weights_k(const T* __restrict__ w, int Cout, int kh, int kw, int Cin, int Kpad, T* __restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= Cin * Kpad) return;
  const int ci = i / Kpad, k = i - ci * Kpad;
  T v = from_f32<T>(0.f);
  if (k < kh * kw * Cout) {
    const int tap = k / Cout, co = k - tap * Cout, ti = tap / kw, tj = tap - ti * kw;
    v = w[(((size_t)co * kh + (kh - 1 - ti)) * kw + (kw - 1 - tj)) * Cin + ci];
  }
  out[i] = v;
}

static ConvGeom dgrad_as_forward(const ConvGeom& g) {
  ConvGeom d = g;
  d.Hin = g.Hout; d.Win = g.Wout; d.Cin = g.Cout;
  d.Hout = g.Hin; d.Wout = g.Win; d.Cout = g.Cin;
  d.stride = 1; d.ph = g.kh - 1 - g.ph; d.pw = g.kw - 1 - g.pw;
  return d;
}

int conv_direct_dgrad_gemm_ok(const ConvGeom& g) {
  if (g.stride != 1 || g.kh - 1 - g.ph < 0 || g.kw - 1 - g.pw < 0) return 0;
  const int Kpad = direct_kpad(dgrad_as_forward(g));
  return Kpad >= 40 && Kpad <= 4096;
}
size_t conv_direct_dgrad_gemm_im2col_elems(const ConvGeom& g) {
  return (size_t)g.N * g.Hin * g.Win * direct_kpad(dgrad_as_forward(g));
}
size_t conv_direct_dgrad_gemm_w_elems(const ConvGeom& g) { return (size_t)g.Cin * direct_kpad(dgrad_as_forward(g)); }

void conv_direct_dgrad_gemm(int dt, hipStream_t st, const void* dz, const void* w, const ConvGeom& g, void* im2col, void* wscratch,
                            void* dIn) {
  const ConvGeom d = dgrad_as_forward(g);
  const int Kpad = direct_kpad(d);
  const size_t M = (size_t)g.N * g.Hin * g.Win;
  View v{dz, nullptr, nullptr, 0};
  {
    const double es = dt == 0 ? 4.0 : 2.0;
    KScope ks(st, "im2col", ((double)g.N * g.Hout * g.Wout * g.Cout + (double)M * Kpad) * es, 0, (long)M, Kpad, g.Cin);
    size_t nvec = M * (Kpad / 8);
    unsigned grid = (unsigned)((nvec + 255) / 256 > 65536 ? 65536 : (nvec + 255) / 256);
    FTP_DISPATCH(dt, hipLaunchKernelGGL(im2col_k<T>, dim3(grid), dim3(256), (size_t)Kpad * sizeof(uint32_t), st, v, d, Kpad, (T*)im2col));
    FTP_DISPATCH(dt, hipLaunchKernelGGL(dgrad_weights_k<T>, dim3((g.Cin * Kpad + 255) / 256), dim3(256), 0, st, (const T*)w, g.Cout,
                                        g.kh, g.kw, g.Cin, Kpad, (T*)wscratch));
  }
  pw_fwd(dt, st, HView{im2col, nullptr, nullptr, 0}, wscratch, nullptr, M, Kpad, g.Cin, dIn, nullptr, nullptr);
}

// ================================================================ depthwise 3x3
// A block owns a slab of CGB*8 channels (128 bytes of every pixel) of one spatial tile.  The input
// patch with its one-pixel halo is staged in LDS once in the tensor's own type, already passed through the
// producer's BatchNorm + activation and with zeros outside the image, so HBM sees every input
// element once per tile.  A thread then owns 4 channels of a horizontal run of 4 pixels: per kernel
// row it reads the 6 (stride 1) or 9 (stride 2) patch vectors under the run once and uses each for
// up to three taps, which cuts the LDS traffic of a pixel-per-thread mapping to a quarter, and it
// keeps the nine weight vectors in registers.  Tiles are numbered so that neighbours, which share
// halo pixels, run on the same XCD and meet in its L2.
struct DwPlan {
  int TH, TW, PH, PW;       // tile of the produced / walked tensor, staged patch
  int CGB, nslab, PPB;      // column groups per slab, slabs, patch pixels staged per pass
  int segw, nseg, spp;      // 4-pixel runs per tile row, per tile, and runs the block covers per pass
  int tiles_h, tiles_w, ntiles, nblocks;
  unsigned m_cgb, m_qb, m_pw, m_segw;   // reciprocals for dw_div (divisors < 64, dividends < 1024)
};
enum { kDwFillNV = 6 };     // passes the patch staging is unrolled for
enum { kDwSegs = 2 };       // 4-pixel runs of a tile a weight-gradient thread keeps the dz of

// x / d for x < 1024, d < 64 with m = 65536 / d + 1: two full-rate instructions instead of the
// ~25-instruction integer division sequence (thread-index decoding was a third of the kernel's VALU work)
static unsigned dw_magic(int d) { return 65536u / (unsigned)d + 1u; }
__device__ __forceinline__ int dw_div(int x, unsigned m) { return (int)(__umul24((unsigned)x, m) >> 16); }

static DwPlan dw_plan(int C, int es, bool half_rows, int out_h, int out_w) {
  DwPlan d;
  const int cgs = C / 8, cap = es == 2 ? 8 : 4;            // 128 bytes of channels per pixel
  d.nslab = (cgs + cap - 1) / cap;
  d.CGB = (cgs + d.nslab - 1) / d.nslab;
  d.PPB = 256 / d.CGB;
  d.spp = 256 / (2 * d.CGB);
  d.TH = half_rows ? 4 : 8;
  d.TW = half_rows ? 8 : 16;     // measured: 8x16 tiles beat 8x8 by 10-25 % (less halo, fewer blocks), 4x8 is best for stride 2
  if (d.TH > out_h) d.TH = out_h;
  if (d.TW > out_w) d.TW = out_w;
  d.segw = (d.TW + 3) / 4;
  d.nseg = d.TH * d.segw;
  d.tiles_h = (out_h + d.TH - 1) / d.TH;
  d.tiles_w = (out_w + d.TW - 1) / d.TW;
  d.ntiles = 0; d.nblocks = 0; d.PH = d.PW = 0;
  d.m_cgb = dw_magic(d.CGB); d.m_qb = dw_magic(2 * d.CGB); d.m_segw = dw_magic(d.segw); d.m_pw = 0;
  return d;
}

// Patch rows h0 .. h0+PH-1, cols w0 .. w0+PW-1 of image n (H x W x C), column groups cg0 .. cg0+CGB-1,
// into LDS as float [PH][PW][CGB][8].  Thread = (pixel lane, column group); fetch() issues all global
// loads, commit() applies the view and writes LDS, so a caller can keep the loads of the next tile
// in flight while it works on the current one.
template <typename T>
struct DwPatch {
  Raw<T> raw[kDwFillNV];
  unsigned ok;
  // image n is at most 2^31 elements: offsets inside it are 32-bit, products of 24-bit factors
  __device__ __forceinline__ void fetch(const T* __restrict__ src, int n, int h0, int w0, const DwPlan& d, int H, int W,
                                        int C, int cg0) {
    ok = 0;
    const int pl = dw_div(threadIdx.x, d.m_cgb), cg = threadIdx.x - pl * d.CGB, gcg = cg0 + cg;
    if (pl >= d.PPB || gcg >= C / 8) return;
    const T* img = src + (size_t)n * H * W * C + gcg * 8;
    const int npix = d.PH * d.PW, dph = dw_div(d.PPB, d.m_pw), dpw = d.PPB - dph * d.PW;
    int ph = dw_div(pl, d.m_pw), pw = pl - ph * d.PW;
    // Offsets first, then the loads back to back and unconditional (a pixel outside the image or the patch reads the
    // image's first pixel and is zeroed in commit): with a branch around each load, and its address computed next to
    // it, every load waited for the one before.
    unsigned off[kDwFillNV];
#pragma unroll
    for (int q = 0; q < kDwFillNV; ++q) {
      const int h = h0 + ph, w = w0 + pw;
      const bool in = pl + q * d.PPB < npix && h >= 0 && h < H && w >= 0 && w < W;
      off[q] = in ? __umul24(__umul24(h, W) + w, C) : 0u;
      ok |= (in ? 1u : 0u) << q;
      ph += dph; pw += dpw;
      if (pw >= d.PW) { pw -= d.PW; ++ph; }
    }
#pragma unroll
    for (int q = 0; q < kDwFillNV; ++q) raw_load(raw[q], img + off[q]);
  }
  __device__ __forceinline__ void commit(T* patch, const View& vw, const DwPlan& d, int cg0) const {
    const int pl = dw_div(threadIdx.x, d.m_cgb), cg = threadIdx.x - pl * d.CGB;
    if (pl >= d.PPB) return;
    const int npix = d.PH * d.PW;
    float sc[8], sh[8];
    const bool view = vw.scale != nullptr && ok != 0;
    if (view) {
      load8(vw.scale + (cg0 + cg) * 8, sc);
      load8(vw.shift + (cg0 + cg) * 8, sh);
    }
    const float lo = act_lo(vw.act), hi = act_hi(vw.act);
    T* dst = patch + (pl * d.CGB + cg) * 8;            // stored in the tensor's own type: the values are already rounded to it
    const int step = d.PPB * d.CGB * 8;
#pragma unroll
    for (int q = 0; q < kDwFillNV; ++q) {
      if (pl + q * d.PPB >= npix) break;
      float val[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      if (ok & (1u << q)) {
        raw_unpack(raw[q], val);
        if (view) {
#pragma unroll
          for (int e = 0; e < 8; ++e) val[e] = clamp_act(fmaf(val[e], sc[e], sh[e]), lo, hi);   // store8 rounds to T
        }
      }
      store8(dst + q * step, val);
    }
  }
};

// the slab's weights as float [9][CGB][8].  All global loads are issued before the first LDS store (at most five
// per thread: 9 * 16 * 8 values over 256 threads): loaded and stored one by one, every round cost a memory round trip
// that nothing else in the block could hide.
template <typename T>
__device__ __forceinline__ void dw_stage_weights(float* wl, const T* __restrict__ w, int C, int cg0, int CGB, unsigned m_cgb) {
  constexpr int NV = 5;
  const int n = 9 * CGB * 8;
  T v[NV];                 // as loaded: a conversion next to its load makes the compiler wait for that load alone
  bool live[NV];
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    const int i = threadIdx.x + q * 256;
    const int e = i & 7, t = dw_div(i >> 3, m_cgb), c8 = (i >> 3) - t * CGB;      // i >> 3 < 160
    const int c = (cg0 + c8) * 8 + e;
    live[q] = i < n && c < C;
    v[q] = w[live[q] ? (size_t)c * 9 + t : 0];
  }
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    const int i = threadIdx.x + q * 256;
    if (i < n) wl[i] = live[q] ? to_f32(v[q]) : 0.f;
  }
}

// out[ho][wo] = sum_{ky,kx} src[ho*S-1+ky][wo*S-1+kx] * w[ky][kx]   (FLIP: w[2-ky][2-kx], which for
// S = 1 is the data gradient with src = dz)
// RL = pixels per run: four at stride 1; two at stride 2, where a run of four keeps 9 patch vectors and 4 sums live
// (111 registers, four resident blocks per CU) and a 4 x 8 tile has work for only 96 of the 256 threads
// STATS (layers with at most kMaxPartials tiles): the block also leaves per-channel sums over its stored outputs, one
// partial per tile ([tile][2][C]).  1: the sum and the sum of squares (what bn_stats would compute in a pass of its
// own).  2, for the data gradient: the output is the gradient dA of the BatchNorm + activation in front of this layer,
// whose conv output zp sits at the same positions; the sums are those of bn_bwd_reduce (dY = dA where the activation
// passes, sum of dY and of dY * zp), so that BatchNorm's backward starts at its finalize.
struct DwPrev { const void* z; const float* scale; const float* shift; int act; };
template <typename T, int S, bool FLIP, int STATS = 0, int RL = (S == 2 ? 2 : 4)>
__global__ __launch_bounds__(256) void dw_conv_k(View in, const T* __restrict__ w, DwPlan d, int Hin, int Win, int Hout,
                                                 int Wout, int C, T* __restrict__ out, float* __restrict__ stats = nullptr,
                                                 DwPrev prev = DwPrev{nullptr, nullptr, nullptr, 0}) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  if (FLIP) __builtin_amdgcn_s_setprio(3);   // data-gradient chain: ahead of the weight-gradient stream's waves
  T* patch = reinterpret_cast<T*>(smem_raw);
  float* wl = reinterpret_cast<float*>(smem_raw + (((size_t)d.PH * d.PW * d.CGB * 8 * sizeof(T) + 15) / 16 * 16));
  const int lb = xcd_logical_block();
  const int slab = lb % d.nslab, tile = lb / d.nslab;     // the slabs of a tile run together: they share cache lines when a slab is not 128 bytes
  const int tw = tile % d.tiles_w, th = (tile / d.tiles_w) % d.tiles_h, n = tile / (d.tiles_w * d.tiles_h);
  const int ho0 = th * d.TH, wo0 = tw * d.TW, cg0 = slab * d.CGB;
  DwPatch<T> lp;
  lp.fetch(reinterpret_cast<const T*>(in.z), n, ho0 * S - 1, wo0 * S - 1, d, Hin, Win, C, cg0);
  dw_stage_weights(wl, w, C, cg0, d.CGB, d.m_cgb);
  lp.commit(patch, in, d, cg0);
  __syncthreads();
  const int QB = 2 * d.CGB, seg0 = dw_div(threadIdx.x, d.m_qb), cq = threadIdx.x - seg0 * QB;
  const int c4 = cq * 4, gc = cg0 * 8 + c4;
  const bool worker = seg0 < d.spp && gc < C;
  if (!STATS && !worker) return;
  float4 wr[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) wr[t] = worker ? ld4(wl + (size_t)(FLIP ? 8 - t : t) * d.CGB * 8 + c4) : make_float4(0.f, 0.f, 0.f, 0.f);
  const int vs = d.CGB * 8;                       // floats per patch pixel
  float4 s1 = make_float4(0.f, 0.f, 0.f, 0.f), s2 = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 psc = make_float4(0.f, 0.f, 0.f, 0.f), psh = psc;
  if (STATS == 2 && worker) { psc = ld4(prev.scale + gc); psh = ld4(prev.shift + gc); }
  const float plo = act_lo(prev.act), phi = act_hi(prev.act);
  for (int sg = worker ? seg0 : d.nseg; sg < d.nseg; sg += d.spp) {
    const int hl = dw_div(sg, d.m_segw), wl0 = (sg - hl * d.segw) * RL;
    const int ho = ho0 + hl;
    if (ho >= Hout) continue;
    float4 zp[RL];
    if (STATS == 2) {                             // requested before the taps are worked off, used after the stores
      const T* zrow = reinterpret_cast<const T*>(prev.z) + ((size_t)n * Hout + ho) * Wout * C + gc;
#pragma unroll
      for (int o = 0; o < RL; ++o) {              // a pixel past the row's end reads the row's first pixel and is not used
        const int wq = wo0 + wl0 + o;
        zp[o] = load4(zrow + (size_t)(wq < Wout ? wq : 0) * C);
      }
    }
    float4 acc[RL];
#pragma unroll
    for (int o = 0; o < RL; ++o) acc[o] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
      const T* row = patch + (size_t)((hl * S + ky) * d.PW + wl0 * S) * vs + c4;
      float4 iv[(RL - 1) * S + 3];
#pragma unroll
      for (int x = 0; x < (RL - 1) * S + 3; ++x) iv[x] = load4(row + (size_t)x * vs);
#pragma unroll
      for (int kx = 0; kx < 3; ++kx)
#pragma unroll
        for (int o = 0; o < RL; ++o) acc[o] = fma4(iv[o * S + kx], wr[ky * 3 + kx], acc[o]);
    }
    T* dst = out + (((size_t)n * Hout + ho) * Wout + wo0 + wl0) * C + gc;
#pragma unroll
    for (int o = 0; o < RL; ++o)
      if (wo0 + wl0 + o < Wout) {
        store4(dst + (size_t)o * C, acc[o]);
        if (STATS) {                              // sums over the values as stored
          float4 r = make_float4(round_to<T>(acc[o].x), round_to<T>(acc[o].y), round_to<T>(acc[o].z), round_to<T>(acc[o].w));
          float4 f = r;
          if (STATS == 2) {
            const float4 y = fma4(zp[o], psc, psh);
            r.x = (y.x > plo && y.x < phi) ? r.x : 0.f; r.y = (y.y > plo && y.y < phi) ? r.y : 0.f;
            r.z = (y.z > plo && y.z < phi) ? r.z : 0.f; r.w = (y.w > plo && y.w < phi) ? r.w : 0.f;
            f = zp[o];
          }
          s1.x += r.x; s1.y += r.y; s1.z += r.z; s1.w += r.w;
          s2 = fma4(r, f, s2);
        }
      }
  }
  if (STATS) {
    // the runs of a channel quad are spread over spp threads: through LDS (the patch is no longer needed), summed in
    // a fixed order by one thread per channel and value
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem_raw);            // [spp][QB][8]
    if (worker) {
      float* r = red + ((size_t)seg0 * QB + cq) * 8;
      r[0] = s1.x; r[1] = s1.y; r[2] = s1.z; r[3] = s1.w; r[4] = s2.x; r[5] = s2.y; r[6] = s2.z; r[7] = s2.w;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < QB * 8; i += 256) {
      const int q = i >> 3, e = i & 7, c = cg0 * 8 + q * 4 + (e & 3);
      if (c >= C) continue;
      float t = 0.f;
      for (int sgi = 0; sgi < d.spp; ++sgi) t += red[((size_t)sgi * QB + q) * 8 + e];
      stats[((size_t)tile * 2 + (e >> 2)) * C + c] = t;
    }
  }
}

// LDS layout: the patch as T [PH][PW][CGB][8], then (16-byte aligned) the weights as float [9][CGB][8]
static size_t dw_patch_bytes(const DwPlan& d, int es) { return (((size_t)d.PH * d.PW * d.CGB * 8 * es) + 15) / 16 * 16; }
static size_t dw_lds_bytes(const DwPlan& d, int es) { return dw_patch_bytes(d, es) + (size_t)9 * d.CGB * 8 * 4; }

// staging is unrolled for kDwFillNV passes; dw_div needs small divisors.  The plans of every shape a model can
// describe satisfy this; if one ever does not, the launch is skipped and the stage call reports it.
static bool dw_check_plan(DwPlan& d, int segs = kDwSegs) {
  if (d.PH * d.PW > kDwFillNV * d.PPB || d.PW > 63 || d.CGB > 16 || d.segw > 32 || d.nseg > segs * d.spp) {
    launch_plan_failed("depthwise tile plan outside the kernels' limits");
    return false;
  }
  d.m_pw = dw_magic(d.PW);
  return true;
}

// the depthwise forward can leave the BatchNorm partial sums itself when its tiles are few enough to be the partials
int dw_fwd_stats_ok(int dt, const ConvGeom& g) {
  const int es = dt == 0 ? 4 : 2;
  const DwPlan d = dw_plan(g.Cout, es, g.stride == 2, g.Hout, g.Wout);
  return (size_t)g.N * d.tiles_h * d.tiles_w <= (size_t)kMaxPartials;
}

void dw_fwd(int dt, hipStream_t st, HView in, const void* w, const ConvGeom& g, void* z, float* stats, int* P_out) {
  const int es = dt == 0 ? 4 : 2, s = g.stride;
  DwPlan d = dw_plan(g.Cout, es, s == 2, g.Hout, g.Wout);
  const int run = s == 2 ? 2 : 4;                // pixels per run, as the kernel's RL
  d.segw = (d.TW + run - 1) / run;
  d.nseg = d.TH * d.segw;
  d.m_segw = dw_magic(d.segw);
  d.PH = (d.TH - 1) * s + 3;
  d.PW = (d.segw * run - 1) * s + 3;             // runs are whole: the patch covers the rounded-up tile width
  d.ntiles = g.N * d.tiles_h * d.tiles_w;
  if (!dw_check_plan(d)) return;
  View v{in.z, in.scale, in.shift, in.act};
  size_t total = (size_t)g.N * g.Hout * g.Wout;
  KScope ks(st, "dw_fwd", ((double)g.N * g.Hin * g.Win * g.Cout + (double)total * g.Cout) * es, 18.0 * total * g.Cout,
            (long)total, g.Cout, g.stride);
  const unsigned grid = (unsigned)d.ntiles * d.nslab;
  if (stats) {
    if (d.ntiles > kMaxPartials) { launch_plan_failed("depthwise forward with statistics: more tiles than partial sums"); return; }
    // the reduction reuses the patch's LDS: [spp][2*CGB][8] floats
    size_t lds = dw_lds_bytes(d, es);
    const size_t red = (size_t)d.spp * 2 * d.CGB * 8 * sizeof(float);
    if (lds < red) lds = red;
    if (s == 1) {
      FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_conv_k<T, 1, false, 1>), dim3(grid), dim3(256), lds, st, v, (const T*)w, d,
                                          g.Hin, g.Win, g.Hout, g.Wout, g.Cout, (T*)z, stats));
    } else {
      FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_conv_k<T, 2, false, 1>), dim3(grid), dim3(256), lds, st, v, (const T*)w, d,
                                          g.Hin, g.Win, g.Hout, g.Wout, g.Cout, (T*)z, stats));
    }
    *P_out = d.ntiles;
    return;
  }
  if (s == 1) {
    FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_conv_k<T, 1, false>), dim3(grid), dim3(256), dw_lds_bytes(d, es), st, v, (const T*)w, d,
                                        g.Hin, g.Win, g.Hout, g.Wout, g.Cout, (T*)z));
  } else {
    FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_conv_k<T, 2, false>), dim3(grid), dim3(256), dw_lds_bytes(d, es), st, v, (const T*)w, d,
                                        g.Hin, g.Win, g.Hout, g.Wout, g.Cout, (T*)z));
  }
}

// ---- short tensors: whole depthwise layers in one launch ------------------------------------------------
// For tensors of a few hundred KB the separate kernels are all launch latency.  Here a block owns 4 channels
// over every pixel: the tensor that is gathered from (input in forward, dz in backward) is staged once in LDS
// as one float4 per pixel (the view applied once per element), so the nine taps are LDS reads and the
// per-channel sums never leave the block.
__device__ __forceinline__ float4 view4(float4 v, const float* sc, const float* sh, float lo, float hi) {
  return make_float4(clamp_act(fmaf(v.x, sc[0], sh[0]), lo, hi), clamp_act(fmaf(v.y, sc[1], sh[1]), lo, hi),
                     clamp_act(fmaf(v.z, sc[2], sh[2]), lo, hi), clamp_act(fmaf(v.w, sc[3], sh[3]), lo, hi));
}
template <typename T> __device__ __forceinline__ float4 round4(float4 v) {
  return make_float4(round_to<T>(v.x), round_to<T>(v.y), round_to<T>(v.z), round_to<T>(v.w));
}

// four channels of one pixel as loaded, converted at the point of use (so the load can stay in flight)
template <typename T> struct Raw4;
template <> struct Raw4<float> { float4 v; };
template <> struct Raw4<bf16_t> { uint2 v; };
__device__ __forceinline__ void raw4_load(Raw4<float>& r, const float* p) { r.v = *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void raw4_load(Raw4<bf16_t>& r, const bf16_t* p) { r.v = *reinterpret_cast<const uint2*>(p); }
__device__ __forceinline__ float4 raw4_unpack(const Raw4<float>& r) { return r.v; }
__device__ __forceinline__ float4 raw4_unpack(const Raw4<bf16_t>& r) {
  return make_float4(__uint_as_float(r.v.x << 16), __uint_as_float(r.v.x & 0xffff0000u), __uint_as_float(r.v.y << 16),
                     __uint_as_float(r.v.y & 0xffff0000u));
}

// Depthwise convolution + BatchNorm statistics + their finalisation (and, when the producer left them pending,
// the finalisation of the input's BatchNorm too).
template <typename T>
__global__ __launch_bounds__(1024) void dw_fwd_bn_small_k(View in, BnPending pend, const T* __restrict__ w, ConvGeom g, size_t M,
                                                          size_t Min, const float* __restrict__ gamma, const float* __restrict__ beta,
                                                          float* mean, float* invstd, float* scale, float* shift,
                                                          float* run_mean, float* run_var, float eps, float momentum,
                                                          T* __restrict__ z) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  float4* tile = reinterpret_cast<float4*>(smem_raw);           // [Min]
  __shared__ float wl[9][4];
  __shared__ float red[16][8];
  __shared__ double pre[32][8];
  __shared__ float insc[2][4];
  // adjacent channel groups share cache lines: keep them on one XCD
  const int C = g.Cout, c0 = xcd_logical_block() * 4, tid = threadIdx.x, nt = blockDim.x, s = g.stride;
  // Everything that depends on nothing is requested first: the input pixels of this block (at most three per thread,
  // raw, from a clamped address), the BatchNorm parameters and running statistics.  They then travel while the pending
  // BatchNorm of the input is finished; the kernel is a chain of memory round trips and little else.
  const T* src = reinterpret_cast<const T*>(in.z);
  Raw4<T> rv[3];
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    const size_t m = (size_t)tid + (size_t)q * nt;
    raw4_load(rv[q], src + (m < Min ? m : 0) * C + c0);
  }
  float bn_g = 0.f, bn_b = 0.f, bn_rm = 0.f, bn_rv = 0.f;
  if (tid < 4) { bn_g = gamma[c0 + tid]; bn_b = beta[c0 + tid]; bn_rm = run_mean[c0 + tid]; bn_rv = run_var[c0 + tid]; }
  if (tid < 36) wl[tid / 4][tid % 4] = to_f32(w[(size_t)(c0 + tid % 4) * 9 + tid / 4]);
  const bool view = in.scale != nullptr;
  if (pend.partial) finish_pending4(pend, C, c0, eps, momentum, pre, insc);
  else if (tid < 4 && view) { insc[0][tid] = in.scale[c0 + tid]; insc[1][tid] = in.shift[c0 + tid]; }
  if (!pend.partial) __syncthreads();
  float sc[4] = {1.f, 1.f, 1.f, 1.f}, sh[4] = {0.f, 0.f, 0.f, 0.f};
  if (view) {
#pragma unroll
    for (int e = 0; e < 4; ++e) { sc[e] = insc[0][e]; sh[e] = insc[1][e]; }
  }
  const float lo = view ? act_lo(in.act) : -INFINITY, hi = view ? act_hi(in.act) : INFINITY;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    const size_t m = (size_t)tid + (size_t)q * nt;
    if (m >= Min) break;
    float4 v = raw4_unpack(rv[q]);
    if (view) v = round4<T>(view4(v, sc, sh, lo, hi));
    tile[m] = v;
  }
  __syncthreads();
  float4 wr[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) wr[t] = make_float4(wl[t][0], wl[t][1], wl[t][2], wl[t][3]);
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (size_t m = tid; m < M; m += nt) {
    const int wo = (int)(m % g.Wout), ho = (int)((m / g.Wout) % g.Hout), n = (int)(m / ((size_t)g.Wout * g.Hout));
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int h = ho * s - 1 + i;
      if (h < 0 || h >= g.Hin) continue;
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const int ww = wo * s - 1 + j;
        if (ww < 0 || ww >= g.Win) continue;
        o = fma4(tile[((size_t)n * g.Hin + h) * g.Win + ww], wr[i * 3 + j], o);
      }
    }
    store4(z + m * C + c0, o);
    const float4 sv = round4<T>(o);               // statistics of the values as stored
    acc[0] += sv.x; acc[1] += sv.y; acc[2] += sv.z; acc[3] += sv.w;
    acc[4] = fmaf(sv.x, sv.x, acc[4]); acc[5] = fmaf(sv.y, sv.y, acc[5]);
    acc[6] = fmaf(sv.z, sv.z, acc[6]); acc[7] = fmaf(sv.w, sv.w, acc[7]);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = wave_sum(acc[e]);
  const int wave = tid >> 6, nw = nt >> 6;
  if ((tid & 63) == 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wave][e] = acc[e];
  }
  __syncthreads();
  // first use of the four values requested at the top: their conversions must not move up to the loads
  asm volatile("" : "+v"(bn_g), "+v"(bn_b), "+v"(bn_rm), "+v"(bn_rv));
  if (tid < 4) {
    const int c = c0 + tid;
    double s0 = 0.0, s1 = 0.0;
    for (int q = 0; q < nw; ++q) { s0 += red[q][tid]; s1 += red[q][4 + tid]; }
    const double Md = (double)M, mu = s0 / Md;
    double var = s1 / Md - mu * mu;
    if (var < 0.0) var = 0.0;
    const double is = 1.0 / sqrt(var + (double)eps);
    const float scv = (float)((double)bn_g * is);
    mean[c] = (float)mu;
    invstd[c] = (float)is;
    scale[c] = scv;
    shift[c] = (float)((double)bn_b - mu * (double)scv);
    const double unb = M > 1 ? var * (Md / (Md - 1.0)) : var;
    run_mean[c] = (float)((1.0 - momentum) * bn_rm + momentum * mu);
    run_var[c] = (float)((1.0 - momentum) * bn_rv + momentum * unb);
  }
}

int dw_fwd_bn_small_ok(const ConvGeom& g) {
  return (size_t)g.N * g.Hout * g.Wout <= 2048 && (size_t)g.N * g.Hin * g.Win <= 3072 && g.Cout >= 32 && g.Cout % 8 == 0;
}

void dw_fwd_bn_small(int dt, hipStream_t st, HView in, const BnPending& pend, const void* w, const ConvGeom& g, const float* gamma,
                     const float* beta, float* mean, float* invstd, float* scale, float* shift, float* run_mean,
                     float* run_var, float eps, float momentum, void* z) {
  const size_t M = (size_t)g.N * g.Hout * g.Wout, Min = (size_t)g.N * g.Hin * g.Win;
  const int es = dt == 0 ? 4 : 2;
  View v{in.z, in.scale, in.shift, in.act};
  KScope ks(st, "dw_fwd_bn_small", ((double)Min * g.Cout + (double)M * g.Cout) * es, 21.0 * M * g.Cout, (long)M, g.Cout, g.stride);
  const int nt = Min > 512 ? 1024 : (Min > 256 ? 512 : 256);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(dw_fwd_bn_small_k<T>, dim3(g.Cout / 4), dim3(nt), Min * 16, st, v, pend, (const T*)w, g, M, Min,
                                      gamma, beta, mean, invstd, scale, shift, run_mean, run_var, eps, momentum, (T*)z));
}

// Backward of a depthwise layer and of the BatchNorm in front of it.  A thread owns input pixels; it gathers the
// dz values that reach a pixel once (from the LDS copy) and uses each twice: times the tap weight for the data
// gradient, times the pixel's own activation for the weight gradient (dW[tap] = sum_p dz[p] * a[p*s-1+tap] is
// the same sum walked from the input side).  The data gradient never leaves the registers: it is gated by the
// activation, reduced into the BatchNorm sums, and after the block-wide reduction turned into the gradient of
// the raw convolution output in front (dz_prev).  Replaces depthwise dgrad + wgrad + partial reduction +
// BatchNorm backward.
template <typename T, int RPT>
__global__ __launch_bounds__(512) void dw_bwd_small_k(const T* __restrict__ dz, BnBwdIn bo, const T* __restrict__ w, View in,
                                                      ConvGeom g, size_t M, size_t Mout, const float* __restrict__ gamma,
                                                      const float* __restrict__ mean, const float* __restrict__ invstd, float* g_w,
                                                      float* g_gamma, float* g_beta, T* __restrict__ dz_prev) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  float4* tile = reinterpret_cast<float4*>(smem_raw);           // dz, [Mout]
  __shared__ float wl[9][4];
  __shared__ float red[8][44];    // [wave][value]
  __builtin_amdgcn_s_setprio(3);             // data-gradient chain: ahead of the weight-gradient stream's waves
  __shared__ float coef[3][4];
  // adjacent channel groups share cache lines: keep them on one XCD
  const int C = g.Cout, c0 = xcd_logical_block() * 4, tid = threadIdx.x, nt = blockDim.x, s = g.stride;
  const T* zin = reinterpret_cast<const T*>(in.z);
  // Everything that depends on nothing is requested first, unconditionally and from clamped addresses: this thread's
  // rows of the layer input, the old weight gradient, and what the finishing threads need after each reduction.
  // The kernel is a chain of memory round trips; these then overlap with the first of them.
  float4 zv[RPT];
#pragma unroll
  for (int q = 0; q < RPT; ++q) {
    const size_t m = tid + (size_t)q * nt;
    zv[q] = load4(zin + (m < M ? m : 0) * C + c0);
  }
  float gw_old = 0.f, f_mu = 0.f, f_is = 0.f, f_g = 0.f, f_gg = 0.f, f_gb = 0.f;
  float f2_mu = 0.f, f2_is = 0.f, f2_g = 0.f, f2_gg = 0.f, f2_gb = 0.f;
  if (tid < 36) gw_old = g_w[(size_t)(c0 + tid % 4) * 9 + tid / 4];
  if (tid >= 64 && tid < 68) {
    const int c = c0 + tid - 64;
    f_mu = mean[c]; f_is = invstd[c]; f_g = gamma[c]; f_gg = g_gamma[c]; f_gb = g_beta[c];
  }
  if (bo.dA && tid < 4) {
    const int c = c0 + tid;
    f2_mu = bo.mean[c]; f2_is = bo.invstd[c]; f2_g = bo.gamma[c]; f2_gg = bo.g_gamma[c]; f2_gb = bo.g_beta[c];
  }
  if (tid < 36) wl[tid / 4][tid % 4] = to_f32(w[(size_t)(c0 + tid % 4) * 9 + tid / 4]);
  float sc[4], sh[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) { sc[e] = in.scale[c0 + e]; sh[e] = in.shift[c0 + e]; }
  const float lo = act_lo(in.act), hi = act_hi(in.act);
  if (bo.dA) {
    // dz is not formed yet: this layer's own BatchNorm backward first (same channels, all pixels: block-local),
    // its result goes straight into the LDS tile and never to memory
    __shared__ float red2[8][8];
    __shared__ float coef2[3][4];
    const T* dA2 = reinterpret_cast<const T*>(bo.dA);
    const T* z2 = reinterpret_cast<const T*>(bo.out.z);
    float sc2[4], sh2[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) { sc2[e] = bo.out.scale[c0 + e]; sh2[e] = bo.out.shift[c0 + e]; }
    const float lo2 = act_lo(bo.out.act), hi2 = act_hi(bo.out.act);
    float4 dy2[RPT], z2v[RPT];
    float b2[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    float4 d2r[RPT];
#pragma unroll
    for (int q = 0; q < RPT; ++q) {
      const size_t m = tid + (size_t)q * nt, mc = m < Mout ? m : 0;
      d2r[q] = load4(dA2 + mc * C + c0);
      z2v[q] = load4(z2 + mc * C + c0);
    }
#pragma unroll
    for (int q = 0; q < RPT; ++q) {
      const size_t m = tid + (size_t)q * nt;
      dy2[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (m >= Mout) { z2v[q] = dy2[q]; continue; }
      const float4 d = d2r[q];
      const float4 zz = z2v[q];
      const float y0 = fmaf(zz.x, sc2[0], sh2[0]), y1 = fmaf(zz.y, sc2[1], sh2[1]), y2 = fmaf(zz.z, sc2[2], sh2[2]),
                  y3 = fmaf(zz.w, sc2[3], sh2[3]);
      float4 v;
      v.x = (y0 > lo2 && y0 < hi2) ? d.x : 0.f;
      v.y = (y1 > lo2 && y1 < hi2) ? d.y : 0.f;
      v.z = (y2 > lo2 && y2 < hi2) ? d.z : 0.f;
      v.w = (y3 > lo2 && y3 < hi2) ? d.w : 0.f;
      dy2[q] = v;
      b2[0] += v.x; b2[1] += v.y; b2[2] += v.z; b2[3] += v.w;
      b2[4] = fmaf(v.x, zz.x, b2[4]); b2[5] = fmaf(v.y, zz.y, b2[5]); b2[6] = fmaf(v.z, zz.z, b2[6]); b2[7] = fmaf(v.w, zz.w, b2[7]);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float r = wave_sum(b2[e]);
      if ((tid & 63) == 0) red2[tid >> 6][e] = r;
    }
    __syncthreads();
    // first use of the values requested at the top: their conversions must not move up to the loads
    asm volatile("" : "+v"(f2_mu), "+v"(f2_is), "+v"(f2_g), "+v"(f2_gg), "+v"(f2_gb));
    if (tid < 4) {
      const int c = c0 + tid;
      double s0 = 0.0, s1 = 0.0;
      for (int q = 0; q < (nt >> 6); ++q) { s0 += red2[q][tid]; s1 += red2[q][4 + tid]; }
      const double mu = f2_mu, is = f2_is, gm = f2_g, Md = (double)Mout;
      const double dbeta = s0, dgamma = is * (s1 - mu * s0);
      bo.g_gamma[c] = f2_gg + (float)dgamma;
      bo.g_beta[c] = f2_gb + (float)dbeta;
      const double k1 = gm * is, k2 = -k1 * is * dgamma / Md, k3 = -k1 * dbeta / Md - k2 * mu;
      coef2[0][tid] = (float)k1; coef2[1][tid] = (float)k2; coef2[2][tid] = (float)k3;
    }
    __syncthreads();
    const float4 k1 = make_float4(coef2[0][0], coef2[0][1], coef2[0][2], coef2[0][3]);
    const float4 k2 = make_float4(coef2[1][0], coef2[1][1], coef2[1][2], coef2[1][3]);
    const float4 k3 = make_float4(coef2[2][0], coef2[2][1], coef2[2][2], coef2[2][3]);
#pragma unroll
    for (int q = 0; q < RPT; ++q) {
      const size_t m = tid + (size_t)q * nt;
      if (m < Mout) tile[m] = round4<T>(fma4(k1, dy2[q], fma4(k2, z2v[q], k3)));   // as a stored dz would read back
    }
  } else {
    for (size_t m = tid; m < Mout; m += nt) tile[m] = load4(dz + m * C + c0);
  }
  __syncthreads();
  float4 wr[9], accw[9], dy[RPT];
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    wr[t] = make_float4(wl[t][0], wl[t][1], wl[t][2], wl[t][3]);
    accw[t] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  float bsum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int q = 0; q < RPT; ++q) {
    const size_t m = tid + (size_t)q * nt;
    dy[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (m >= M) { zv[q] = dy[q]; continue; }
    const int ww = (int)(m % g.Win), h = (int)((m / g.Win) % g.Hin), n = (int)(m / ((size_t)g.Win * g.Hin));
    const float4 y = make_float4(fmaf(zv[q].x, sc[0], sh[0]), fmaf(zv[q].y, sc[1], sh[1]), fmaf(zv[q].z, sc[2], sh[2]),
                                 fmaf(zv[q].w, sc[3], sh[3]));
    const float4 a = round4<T>(make_float4(clamp_act(y.x, lo, hi), clamp_act(y.y, lo, hi), clamp_act(y.z, lo, hi),
                                           clamp_act(y.w, lo, hi)));
    float4 dA = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int hn = h + 1 - i;
      if (hn < 0 || (s == 2 && (hn & 1))) continue;
      const int ho = s == 2 ? hn >> 1 : hn;
      if (ho >= g.Hout) continue;
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const int wn = ww + 1 - j;
        if (wn < 0 || (s == 2 && (wn & 1))) continue;
        const int wo = s == 2 ? wn >> 1 : wn;
        if (wo >= g.Wout) continue;
        const float4 d = tile[((size_t)n * g.Hout + ho) * g.Wout + wo];
        dA = fma4(d, wr[i * 3 + j], dA);
        accw[i * 3 + j] = fma4(d, a, accw[i * 3 + j]);
      }
    }
    dA = round4<T>(dA);                    // the data gradient as the separate kernels would store it
    float4 v;
    v.x = (y.x > lo && y.x < hi) ? dA.x : 0.f;
    v.y = (y.y > lo && y.y < hi) ? dA.y : 0.f;
    v.z = (y.z > lo && y.z < hi) ? dA.z : 0.f;
    v.w = (y.w > lo && y.w < hi) ? dA.w : 0.f;
    dy[q] = v;
    bsum[0] += v.x; bsum[1] += v.y; bsum[2] += v.z; bsum[3] += v.w;
    bsum[4] = fmaf(v.x, zv[q].x, bsum[4]); bsum[5] = fmaf(v.y, zv[q].y, bsum[5]);
    bsum[6] = fmaf(v.z, zv[q].z, bsum[6]); bsum[7] = fmaf(v.w, zv[q].w, bsum[7]);
  }
  // block-wide sums in a fixed order: inside each wave, then the waves in order
  const int wave = tid >> 6, nw = nt >> 6;
  const bool lead = (tid & 63) == 0;
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    const float r0 = wave_sum(accw[t].x), r1 = wave_sum(accw[t].y), r2 = wave_sum(accw[t].z), r3 = wave_sum(accw[t].w);
    if (lead) { red[wave][t * 4 + 0] = r0; red[wave][t * 4 + 1] = r1; red[wave][t * 4 + 2] = r2; red[wave][t * 4 + 3] = r3; }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float r = wave_sum(bsum[e]);
    if (lead) red[wave][36 + e] = r;
  }
  __syncthreads();
  asm volatile("" : "+v"(gw_old), "+v"(f_mu), "+v"(f_is), "+v"(f_g), "+v"(f_gg), "+v"(f_gb));
  if (tid < 36) {
    float tot = 0.f;
    for (int q = 0; q < nw; ++q) tot += red[q][tid];
    g_w[(size_t)(c0 + tid % 4) * 9 + tid / 4] = gw_old + tot;
  } else if (tid >= 64 && tid < 68) {
    const int e = tid - 64, c = c0 + e;
    double s0 = 0.0, s1 = 0.0;
    for (int q = 0; q < nw; ++q) { s0 += red[q][36 + e]; s1 += red[q][40 + e]; }
    const double mu = f_mu, is = f_is, gm = f_g, Md = (double)M;
    const double dbeta = s0, dgamma = is * (s1 - mu * s0);
    g_gamma[c] = f_gg + (float)dgamma;
    g_beta[c] = f_gb + (float)dbeta;
    const double k1 = gm * is, k2 = -k1 * is * dgamma / Md, k3 = -k1 * dbeta / Md - k2 * mu;
    coef[0][e] = (float)k1; coef[1][e] = (float)k2; coef[2][e] = (float)k3;
  }
  __syncthreads();
  const float4 k1 = make_float4(coef[0][0], coef[0][1], coef[0][2], coef[0][3]);
  const float4 k2 = make_float4(coef[1][0], coef[1][1], coef[1][2], coef[1][3]);
  const float4 k3 = make_float4(coef[2][0], coef[2][1], coef[2][2], coef[2][3]);
#pragma unroll
  for (int q = 0; q < RPT; ++q) {
    const size_t m = tid + (size_t)q * nt;
    if (m >= M) continue;
    store4(dz_prev + m * C + c0, fma4(k1, dy[q], fma4(k2, zv[q], k3)));
  }
}

int dw_bwd_small_ok(const ConvGeom& g) {
  return (size_t)g.N * g.Hin * g.Win <= 2048 && g.Cout >= 32 && g.Cout % 8 == 0 && (g.stride == 1 || g.stride == 2);
}

void dw_bwd_small(int dt, hipStream_t st, const void* dz, const BnBwdIn& bo, const void* w, HView in, const ConvGeom& g,
                  const float* gamma, const float* mean, const float* invstd, float* g_w, float* g_gamma, float* g_beta,
                  void* dz_prev) {
  const size_t M = (size_t)g.N * g.Hin * g.Win, Mout = (size_t)g.N * g.Hout * g.Wout;
  const int es = dt == 0 ? 4 : 2;
  View v{in.z, in.scale, in.shift, in.act};
  KScope ks(st, "dw_bwd_small", ((double)M * g.Cout * 2 + (double)Mout * g.Cout) * es, 42.0 * M * g.Cout, (long)M, g.Cout, g.stride);
  const dim3 grid(g.Cout / 4);
  const size_t lds = Mout * 16;
  if (M > 1024) {
    FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_bwd_small_k<T, 4>), grid, dim3(512), lds, st, (const T*)dz, bo, (const T*)w, v, g, M, Mout,
                                        gamma, mean, invstd, g_w, g_gamma, g_beta, (T*)dz_prev));
  } else if (M > 256) {
    FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_bwd_small_k<T, 2>), grid, dim3(M > 512 ? 512 : 256), lds, st, (const T*)dz, bo, (const T*)w,
                                        v, g, M, Mout, gamma, mean, invstd, g_w, g_gamma, g_beta, (T*)dz_prev));
  } else {
    FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_bwd_small_k<T, 1>), grid, dim3(256), lds, st, (const T*)dz, bo, (const T*)w, v, g, M, Mout,
                                        gamma, mean, invstd, g_w, g_gamma, g_beta, (T*)dz_prev));
  }
}

// Stride-2 data gradient over 8 x 8 input tiles: dIn[h][w] = sum over taps (i, j) with h+1-i and w+1-j
// even of dz[(h+1-i)/2][(w+1-j)/2] * w[i][j].  A run of 4 input pixels starting at an even column
// touches three dz columns per dz row.
template <typename T>
__global__ __launch_bounds__(256) void dw_dgrad_s2_k(const T* __restrict__ dz, const T* __restrict__ w, DwPlan d, int Hin,
                                                     int Win, int Hout, int Wout, int C, T* __restrict__ dIn) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  T* patch = reinterpret_cast<T*>(smem_raw);
  float* wl = reinterpret_cast<float*>(smem_raw + (((size_t)d.PH * d.PW * d.CGB * 8 * sizeof(T) + 15) / 16 * 16));
  const int lb = xcd_logical_block();
  const int slab = lb % d.nslab, tile = lb / d.nslab;     // the slabs of a tile run together: they share cache lines when a slab is not 128 bytes
  const int tw = tile % d.tiles_w, th = (tile / d.tiles_w) % d.tiles_h, n = tile / (d.tiles_w * d.tiles_h);
  const int h0 = th * d.TH, w0 = tw * d.TW, cg0 = slab * d.CGB;       // tile origin, even
  __builtin_amdgcn_s_setprio(3);             // data-gradient chain: ahead of the weight-gradient stream's waves
  const int ho_lo = h0 / 2, wo_lo = w0 / 2;
  DwPatch<T> lp;
  View none{nullptr, nullptr, nullptr, 0};
  lp.fetch(dz, n, ho_lo, wo_lo, d, Hout, Wout, C, cg0);
  dw_stage_weights(wl, w, C, cg0, d.CGB, d.m_cgb);
  lp.commit(patch, none, d, cg0);
  __syncthreads();
  const int QB = 2 * d.CGB, seg0 = dw_div(threadIdx.x, d.m_qb), cq = threadIdx.x - seg0 * QB;
  const int c4 = cq * 4, gc = cg0 * 8 + c4;
  if (seg0 >= d.spp || gc >= C) return;
  float4 wr[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) wr[t] = ld4(wl + (size_t)t * d.CGB * 8 + c4);
  const int vs = d.CGB * 8;
  for (int sg = seg0; sg < d.nseg; sg += d.spp) {
    const int hl = dw_div(sg, d.m_segw), wl0 = (sg - hl * d.segw) * 4;
    const int h = h0 + hl;
    if (h >= Hin) continue;
    float4 acc[4];
#pragma unroll
    for (int o = 0; o < 4; ++o) acc[o] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int hn = h + 1 - i;
      if (hn & 1) continue;                        // also skips hn = -1
      const T* row = patch + (size_t)((hn / 2 - ho_lo) * d.PW + wl0 / 2) * vs + c4;
      const float4 d0 = load4(row), d1 = load4(row + vs), d2 = load4(row + 2 * (size_t)vs);
      // pixel 0, 2 (even columns): tap j = 1; pixel 1, 3 (odd): taps j = 0 (next dz column) and j = 2
      acc[0] = fma4(d0, wr[i * 3 + 1], acc[0]);
      acc[1] = fma4(d1, wr[i * 3 + 0], acc[1]);
      acc[1] = fma4(d0, wr[i * 3 + 2], acc[1]);
      acc[2] = fma4(d1, wr[i * 3 + 1], acc[2]);
      acc[3] = fma4(d2, wr[i * 3 + 0], acc[3]);
      acc[3] = fma4(d1, wr[i * 3 + 2], acc[3]);
    }
    T* dst = dIn + (((size_t)n * Hin + h) * Win + w0 + wl0) * C + gc;
#pragma unroll
    for (int o = 0; o < 4; ++o)
      if (w0 + wl0 + o < Win) store4(dst + (size_t)o * C, acc[o]);
  }
}

// the stride-1 data gradient can leave the backward sums of the BatchNorm in front (dw_conv_k, STATS = 2) when its
// tiles are few enough to be the partials
int dw_dgrad_sums_ok(int dt, const ConvGeom& g) {
  if (g.stride != 1) return 0;
  const DwPlan d = dw_plan(g.Cout, dt == 0 ? 4 : 2, false, g.Hin, g.Win);
  return (size_t)g.N * d.tiles_h * d.tiles_w <= (size_t)kMaxPartials;
}

void dw_dgrad(int dt, hipStream_t st, const void* dz, const void* w, const ConvGeom& g, void* dIn, HView prev, float* sums,
              int* P_out) {
  const int es = dt == 0 ? 4 : 2;
  size_t total = (size_t)g.N * g.Hin * g.Win;
  KScope ks(st, "dw_dgrad", ((double)total * g.Cout + (double)g.N * g.Hout * g.Wout * g.Cout) * es, 18.0 * g.N * g.Hout * g.Wout * g.Cout,
            (long)total, g.Cout, g.stride);
  // tiles are in input resolution
  DwPlan d = dw_plan(g.Cout, es, false, g.Hin, g.Win);
  d.ntiles = g.N * d.tiles_h * d.tiles_w;
  const unsigned grid = (unsigned)d.ntiles * d.nslab;
  if (g.stride == 1) {
    // the forward kernel on dz with the weights flipped
    d.PH = d.TH + 2;
    d.PW = d.segw * 4 + 2;
    if (!dw_check_plan(d)) return;
    View v{dz, nullptr, nullptr, 0};
    if (sums) {
      if (d.ntiles > kMaxPartials || !prev.scale) { launch_plan_failed("depthwise data gradient with BatchNorm sums: not for this layer"); return; }
      size_t lds = dw_lds_bytes(d, es);
      const size_t red = (size_t)d.spp * 2 * d.CGB * 8 * sizeof(float);
      if (lds < red) lds = red;
      const DwPrev pv{prev.z, prev.scale, prev.shift, prev.act};
      FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_conv_k<T, 1, true, 2>), dim3(grid), dim3(256), lds, st, v, (const T*)w, d,
                                          g.Hout, g.Wout, g.Hin, g.Win, g.Cout, (T*)dIn, sums, pv));
      *P_out = d.ntiles;
      return;
    }
    FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_conv_k<T, 1, true>), dim3(grid), dim3(256), dw_lds_bytes(d, es), st, v, (const T*)w, d,
                                        g.Hout, g.Wout, g.Hin, g.Win, g.Cout, (T*)dIn));
  } else {
    d.PH = d.TH / 2 + 2;
    d.PW = d.segw * 2 + 2;
    if (!dw_check_plan(d)) return;
    FTP_DISPATCH(dt, hipLaunchKernelGGL(dw_dgrad_s2_k<T>, dim3(grid), dim3(256), dw_lds_bytes(d, es), st, (const T*)dz, (const T*)w,
                                        d, g.Hin, g.Win, g.Hout, g.Wout, g.Cout, (T*)dIn));
  }
}

// dW[c][ky][kx] += sum over output pixels dz[p][c] * in[p*S-1+(ky,kx)][c].  Blocks are persistent over
// tiles; a thread reads the dz of its run straight from global memory (nobody else needs it), keeps
// 9 x 4 sums over all its runs, and the block leaves one partial ws[block][9][C].
// The dz values of a thread's (at most kDwSegs) 4-pixel runs of one tile, requested a whole tile ahead like the
// input patch: a persistent block has few neighbours on its CU to hide a load behind.
template <typename T, int RL = 4, int SEGS = kDwSegs>
struct DwDzRuns {
  Raw4<T> r[SEGS][RL];
  unsigned ok;
  __device__ __forceinline__ void fetch(const T* __restrict__ dz, int tile, const DwPlan& d, int Hout, int Wout, int C,
                                        int seg0, int gc, bool worker) {
    ok = 0;
    if (!worker) return;
    const int tw = tile % d.tiles_w, th = (tile / d.tiles_w) % d.tiles_h, n = tile / (d.tiles_w * d.tiles_h);
    const int ho0 = th * d.TH, wo0 = tw * d.TW;
    // offsets first, then unconditional loads back to back (a pixel outside reads the image's first pixel and is
    // not used): see DwPatch::fetch
    const T* img = dz + (size_t)n * Hout * Wout * C + gc;
    unsigned off[SEGS][RL];
#pragma unroll
    for (int k = 0; k < SEGS; ++k) {
      const int sg = seg0 + k * d.spp;
      const int hl = dw_div(sg < d.nseg ? sg : 0, d.m_segw), wl0 = ((sg < d.nseg ? sg : 0) - hl * d.segw) * RL;
      const int ho = ho0 + hl;
#pragma unroll
      for (int o = 0; o < RL; ++o) {
        const bool in = sg < d.nseg && ho < Hout && wo0 + wl0 + o < Wout;
        off[k][o] = in ? __umul24(__umul24(ho, Wout) + wo0 + wl0 + o, C) : 0u;
        ok |= (in ? 1u : 0u) << (RL * k + o);
      }
    }
#pragma unroll
    for (int k = 0; k < SEGS; ++k)
#pragma unroll
      for (int o = 0; o < RL; ++o) raw4_load(r[k][o], img + off[k][o]);
  }
};

// RL = pixels per run: four at stride 1, two at stride 2 (see dw_conv_k); SEGS = runs of a tile per thread: the 4 x 8
// stride-2 tile has 16 runs, one per thread
template <typename T, int S, int RL = (S == 2 ? 2 : 4), int SEGS = (S == 2 ? 1 : kDwSegs)>
__global__ __launch_bounds__(256) void dw_wgrad_k(const T* __restrict__ dz, View in, DwPlan d, int Hin, int Win, int Hout,
                                                  int Wout, int C, float* __restrict__ ws) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  T* patch = reinterpret_cast<T*>(smem_raw);
  const int lb = xcd_logical_block();
  const int slab = lb % d.nslab, b = lb / d.nslab, cg0 = slab * d.CGB;     // the slabs of a tile run together
  const int QB = 2 * d.CGB, seg0 = dw_div(threadIdx.x, d.m_qb), cq = threadIdx.x - seg0 * QB;
  const int c4 = cq * 4, gc = cg0 * 8 + c4;
  const bool worker = seg0 < d.spp && gc < C;
  const int vs = d.CGB * 8;
  const T* src = reinterpret_cast<const T*>(in.z);
  float4 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) acc[t] = make_float4(0.f, 0.f, 0.f, 0.f);
  DwPatch<T> lp;
  DwDzRuns<T, RL, SEGS> dq[2];
  if (b < d.ntiles) {
    const int tw = b % d.tiles_w, th = (b / d.tiles_w) % d.tiles_h, n = b / (d.tiles_w * d.tiles_h);
    lp.fetch(src, n, th * d.TH * S - 1, tw * d.TW * S - 1, d, Hin, Win, C, cg0);
    dq[0].fetch(dz, b, d, Hout, Wout, C, seg0, gc, worker);
  }
  // two tiles per round so that the two sets of dz registers are addressed statically
  for (int tile0 = b; tile0 < d.ntiles; tile0 += 2 * d.nblocks) {
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      const int tile = tile0 + par * d.nblocks;
      if (tile >= d.ntiles) break;
      __syncthreads();                                       // the previous tile has been consumed
      lp.commit(patch, in, d, cg0);
      __syncthreads();
      const int nt = tile + d.nblocks;
      if (nt < d.ntiles) {
        const int tw2 = nt % d.tiles_w, th2 = (nt / d.tiles_w) % d.tiles_h, n2 = nt / (d.tiles_w * d.tiles_h);
        // the dz runs first: a wait the compiler puts in front of them (their registers were read in the last
        // round's taps) then finds nothing outstanding, instead of the six patch loads
        dq[par ^ 1].fetch(dz, nt, d, Hout, Wout, C, seg0, gc, worker);
        lp.fetch(src, n2, th2 * d.TH * S - 1, tw2 * d.TW * S - 1, d, Hin, Win, C, cg0);
      }
      if (!worker) continue;
      const DwDzRuns<T, RL, SEGS>& cur = dq[par];
#pragma unroll
      for (int k = 0; k < SEGS; ++k) {
        const int sg = seg0 + k * d.spp;
        if (sg >= d.nseg) break;
        if (((cur.ok >> (RL * k)) & ((1u << RL) - 1u)) == 0u) continue;     // the run lies outside the image
        const int hl = dw_div(sg, d.m_segw), wl0 = (sg - hl * d.segw) * RL;
        float4 dv[RL];
#pragma unroll
        for (int o = 0; o < RL; ++o)
          dv[o] = (cur.ok >> (RL * k + o)) & 1u ? raw4_unpack(cur.r[k][o]) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
          const T* row = patch + (size_t)((hl * S + ky) * d.PW + wl0 * S) * vs + c4;
          float4 iv[(RL - 1) * S + 3];
#pragma unroll
          for (int x = 0; x < (RL - 1) * S + 3; ++x) iv[x] = load4(row + (size_t)x * vs);
#pragma unroll
          for (int kx = 0; kx < 3; ++kx)
#pragma unroll
            for (int o = 0; o < RL; ++o) acc[ky * 3 + kx] = fma4(dv[o], iv[o * S + kx], acc[ky * 3 + kx]);
        }
      }
    }
  }
  // sum the runs of every channel quad in a fixed order: red[spp][9][QB] float4
  __syncthreads();
  float4* red = reinterpret_cast<float4*>(smem_raw);
  if (seg0 < d.spp) {
#pragma unroll
    for (int t = 0; t < 9; ++t) red[(seg0 * 9 + t) * QB + cq] = worker ? acc[t] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 9 * QB; i += blockDim.x) {
    const int q = i % QB, t = i / QB;
    if (cg0 * 8 + q * 4 >= C) continue;
    float4 tot = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int r = 0; r < d.spp; ++r) {
      const float4 v = red[(r * 9 + t) * QB + q];
      tot.x += v.x; tot.y += v.y; tot.z += v.z; tot.w += v.w;
    }
    store4(ws + ((size_t)b * 9 + t) * C + cg0 * 8 + q * 4, tot);
  }
}

// ---- depthwise weight gradient without LDS staging: a lane walks down the image ------------------------
// g_w[c][ky][kx] = sum over output pixels of dz[ho][wo][c] * in[ho*S+ky-1][wo*S+kx-1][c].  A lane owns 4 channels and a
// strip of R output columns of one image (R = 2 at stride 1, 1 at stride 2) and walks it from the top row down with
// the input window under the current output pixels in registers ((R-1)*S+3 columns x 3 rows, already through the view,
// as float): per step it brings in S new input rows and R new dz vectors from global memory (requested three steps
// ahead) and does 9 * R four-wide FMAs.  Every input element is converted once per strip it lies under, there is no
// barrier and no LDS traffic inside the walk, and the 36 sums stay in registers over all strips of the lane.
// The lanes of a wavefront (and the wavefronts of a block) take neighbouring strips, so what they request in one
// step is one contiguous stretch of an image row (walking ALONG the rows instead put every lane on a row of its own:
// thousands of 256-byte streams, which the memory served at 2 TB/s).
// The 4-channel groups of a layer are cut into slabs whose widths are powers of two (144 channels = 36 groups =
// 32 + 4), so that gw groups x sw strips fill the 64 lanes of a wavefront exactly; a block's four wavefronts
// take 4 * sw strips of one slab per pass, and the block leaves one partial ws[p][9][C] (its slab's channels).
struct DwMarchSlab { int ch0, gw, sw; int blk0, nblk; };   // first channel, lanes per strip, strips per wavefront; first block, blocks
enum { kDwMarchSlabs = 16, kDwMarchBlocks = 2048, kDwMarchCpl = 2 };   // slabs a layer may need, blocks in all, channels per lane
struct DwMarchArgs {
  const void* dz;
  View in;
  float* ws;
  int Hin, Win, Hout, Wout, C;
  int ncb, nseg, seglen;    // strips side by side, row segments per image (a strip is one segment high), rows per segment
  int nstrips;              // N * nseg * ncb
  int P, nslab;             // partial rows (the most blocks any slab has), slabs
  int nblocks;              // all blocks: the slabs' block ranges one after the other
  DwMarchSlab slab[kDwMarchSlabs];
};

template <int V> struct IntC { static constexpr int value = V; };

// two channels of one pixel as loaded
template <typename T> struct Raw2;
template <> struct Raw2<float> { float2 v; };
template <> struct Raw2<bf16_t> { uint32_t v; };
__device__ __forceinline__ void raw2_load(Raw2<float>& r, const float* p) { r.v = *reinterpret_cast<const float2*>(p); }
__device__ __forceinline__ void raw2_load(Raw2<bf16_t>& r, const bf16_t* p) { r.v = *reinterpret_cast<const uint32_t*>(p); }
__device__ __forceinline__ float2 raw2_unpack(const Raw2<float>& r) { return r.v; }
__device__ __forceinline__ float2 raw2_unpack(const Raw2<bf16_t>& r) {
  return make_float2(__uint_as_float(r.v << 16), __uint_as_float(r.v & 0xffff0000u));
}
// the pair as it reads back after being stored in T (one conversion instruction for both halves)
__device__ __forceinline__ float2 round2(float2 v, float) { return v; }
__device__ __forceinline__ float2 round2(float2 v, bf16_t) {
  const uint32_t u = f32x2_to_bf16x2(v.x, v.y);
  return make_float2(__uint_as_float(u << 16), __uint_as_float(u & 0xffff0000u));
}

template <typename T, int S, bool VIEW>
__global__ __launch_bounds__(256) void dw_wgrad_march_k(DwMarchArgs a) {
  constexpr int R = S == 1 ? 2 : 1;
  constexpr int NCOL = (R - 1) * S + 3;
  __shared__ float2 red[4][9][64];
  // Every slab has blocks in proportion to its work (a narrow tail slab takes many strips per wavefront and needs
  // few): with the same number for all, half the resident blocks of a layer with a tail slab had nothing to do and the
  // wide slabs' blocks took a second round.
  const int lb = xcd_logical_block();
  int si = 0;
  while (si + 1 < a.nslab && lb >= a.slab[si + 1].blk0) ++si;
  const DwMarchSlab sl = a.slab[si];
  const int p = lb - sl.blk0;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int g = lane & (sl.gw - 1), s_l = lane / sl.gw;
  const int c = sl.ch0 + kDwMarchCpl * g;
  const T* src = reinterpret_cast<const T*>(a.in.z);
  const T* dzp = reinterpret_cast<const T*>(a.dz);
  constexpr bool view = VIEW;
  // The walk must be free of branches: only then does the compiler count the loads in flight and wait for the oldest
  // register set alone (with a branch in the loop it waits for all of them).  The heights therefore live in vector
  // registers (a comparison with them is a lane mask, never a jump), and every walk takes a multiple of three steps;
  // the steps behind the last row see dz = 0.
  int hinL = a.Hin, houtL = a.Hout;
  asm volatile("" : "+v"(hinL), "+v"(houtL));
  float2 sc = make_float2(1.f, 1.f), sh = make_float2(0.f, 0.f);
  if (view) {
    sc = *reinterpret_cast<const float2*>(a.in.scale + c);
    sh = *reinterpret_cast<const float2*>(a.in.shift + c);
  }
  const float lo = act_lo(a.in.act), hi = act_hi(a.in.act);
  const float2 zero2 = make_float2(0.f, 0.f);
  float2 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) acc[t] = zero2;
  const unsigned in_row = __umul24(a.Win, a.C), dz_row = __umul24(a.Wout, a.C);

  const int spb = 4 * sl.sw;
  for (int sidx = p * spb + wave * sl.sw + s_l; sidx < a.nstrips; sidx += sl.nblk * spb) {
    const int ns = sidx / a.ncb, cb = sidx - ns * a.ncb;
    const int n = ns / a.nseg, h_beg = (ns - n * a.nseg) * a.seglen;       // a multiple of three: the phases line up
    const int wo0 = cb * R, wi0 = wo0 * S - 1;
    int hendL = h_beg + a.seglen < a.Hout ? h_beg + a.seglen : a.Hout;
    asm volatile("" : "+v"(hendL));
    const T* img = src + (size_t)n * a.Hin * a.Win * a.C + c;
    const T* dimg = dzp + (size_t)n * a.Hout * a.Wout * a.C + c;
    unsigned coff[NCOL], doff[R];
    bool cok[NCOL], dok[R];
#pragma unroll
    for (int r = 0; r < NCOL; ++r) {
      cok[r] = wi0 + r >= 0 && wi0 + r < a.Win;
      coff[r] = cok[r] ? __umul24(wi0 + r, a.C) : 0u;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      dok[r] = wo0 + r < a.Wout;
      doff[r] = dok[r] ? __umul24(wo0 + r, a.C) : 0u;
    }
    float2 win[NCOL][3];
#pragma unroll
    for (int r = 0; r < NCOL; ++r)
#pragma unroll
      for (int y = 0; y < 3; ++y) win[r][y] = zero2;
    // Three steps' loads are in flight (one register set per phase): a lane has nothing else to hide a memory round
    // trip behind, and one step's arithmetic is a fraction of it.
    Raw2<T> rin[3][NCOL][S], rdz[3][R];
    // what output row ho brings in: its S new input rows (y < Hin, else nothing is there) under every column of the
    // strip, and its dz
    auto request_row = [&](auto BUF, const int q, const int y) __attribute__((always_inline)) {
      constexpr int buf = decltype(BUF)::value;
      const unsigned ro = (unsigned)y < (unsigned)hinL ? (unsigned)y * in_row : 0u;
#pragma unroll
      for (int r = 0; r < NCOL; ++r) raw2_load(rin[buf][r][q], img + ro + coff[r]);
    };
    auto request = [&](auto BUF, const int ho) __attribute__((always_inline)) {
      constexpr int buf = decltype(BUF)::value;
      const int y0 = S == 1 ? ho + 1 : 2 * ho;
#pragma unroll
      for (int q = 0; q < S; ++q) request_row(BUF, q, y0 + q);
      const unsigned hr = ho < houtL ? (unsigned)ho * dz_row : 0u;
#pragma unroll
      for (int r = 0; r < R; ++r) raw2_load(rdz[buf][r], dimg + hr + doff[r]);
    };
    auto bring = [&](auto BUF, auto SLOT, const int q, const int y) __attribute__((always_inline)) {
      constexpr int buf = decltype(BUF)::value;
      constexpr int slot = decltype(SLOT)::value;
      const bool yok = (unsigned)y < (unsigned)hinL;
#pragma unroll
      for (int r = 0; r < NCOL; ++r) {
        float2 v = raw2_unpack(rin[buf][r][q]);
        if (view) v = round2(make_float2(clamp_act(fmaf(v.x, sc.x, sh.x), lo, hi), clamp_act(fmaf(v.y, sc.y, sh.y), lo, hi)), T());
        win[r][slot] = (yok && cok[r]) ? v : zero2;       // padding is zero AFTER the view
      }
    };
    // one output row: phase = ho % 3 fixes which window slot holds which input row (row y sits in slot y % 3)
    auto step = [&](auto PH, const int ho) __attribute__((always_inline)) {
      constexpr int ph = decltype(PH)::value;
      constexpr int base = (S * ph + 2) % 3;              // slot of input row ho*S - 1
      if (S == 1) {
        bring(PH, IntC<(ph + 1) % 3>(), 0, ho + 1);
      } else {
        bring(PH, IntC<(2 * ph) % 3>(), 0, 2 * ho);
        bring(PH, IntC<(2 * ph + 1) % 3>(), 1, 2 * ho + 1);
      }
      float2 dv[R];
#pragma unroll
      for (int r = 0; r < R; ++r) dv[r] = (dok[r] && ho < hendL) ? raw2_unpack(rdz[ph][r]) : zero2;
      request(PH, ho + 3);                                 // this register set is free again: the step three ahead
#pragma unroll
      for (int r = 0; r < R; ++r)
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
          for (int kx = 0; kx < 3; ++kx) {
            const float2 w2 = win[r * S + kx][(base + ky) % 3];
            acc[ky * 3 + kx].x = fmaf(dv[r].x, w2.x, acc[ky * 3 + kx].x);
            acc[ky * 3 + kx].y = fmaf(dv[r].y, w2.y, acc[ky * 3 + kx].y);
          }
    };
    // the input rows above the segment's first output row that are under it already: row h_beg*S - 1 (slot 2), and
    // at stride 1 row h_beg as well (slot 0)
    request_row(IntC<0>(), 0, h_beg * S - 1);
    if (S == 1) request_row(IntC<1>(), 0, h_beg);
    bring(IntC<0>(), IntC<2>(), 0, h_beg * S - 1);
    if (S == 1) bring(IntC<1>(), IntC<0>(), 0, h_beg);
    request(IntC<0>(), h_beg);
    request(IntC<1>(), h_beg + 1);
    request(IntC<2>(), h_beg + 2);
    for (int i = 0; i < a.seglen; i += 3) {
      step(IntC<0>(), h_beg + i);
      step(IntC<1>(), h_beg + i + 1);
      step(IntC<2>(), h_beg + i + 2);
    }
  }

  // the block's partial: lanes of one channel group over strips and wavefronts, in a fixed order
#pragma unroll
  for (int t = 0; t < 9; ++t) red[wave][t][lane] = acc[t];
  __syncthreads();
  for (int i = threadIdx.x; i < 9 * sl.gw; i += 256) {
    const int t = i / sl.gw, gg = i - t * sl.gw;
    float2 tot = zero2;
    for (int w = 0; w < 4; ++w)
      for (int q = 0; q < sl.sw; ++q) {
        const float2 v = red[w][t][q * sl.gw + gg];
        tot.x += v.x; tot.y += v.y;
      }
    *reinterpret_cast<float2*>(a.ws + ((size_t)p * 9 + t) * a.C + sl.ch0 + kDwMarchCpl * gg) = tot;
    // the partial rows this slab has no block for (the sum runs over a.P rows for every channel)
    for (int pz = sl.nblk + p; pz < a.P; pz += sl.nblk)
      *reinterpret_cast<float2*>(a.ws + ((size_t)pz * 9 + t) * a.C + sl.ch0 + kDwMarchCpl * gg) = zero2;
  }
}

// slabs (powers of two, widest first) and the number of blocks; false if the layer needs more slabs than the kernel takes
static bool dw_march_plan(const ConvGeom& g, DwMarchArgs* a) {
  int G = g.Cout / kDwMarchCpl, ch = 0, n = 0;
  while (G > 0) {
    int gw = 64;
    while (gw > G) gw >>= 1;
    if (n == kDwMarchSlabs) return false;
    a->slab[n++] = DwMarchSlab{ch, gw, 64 / gw};
    ch += kDwMarchCpl * gw; G -= gw;
  }
  a->nslab = n;
  const int R = g.stride == 1 ? 2 : 1;
  a->ncb = (g.Wout + R - 1) / R;
  // Row segments: a lane's walk is one long chain of dependent steps, so a layer with few strips is cut across its
  // rows until about 2048 wavefronts' worth of lanes exist (cutting further only added partial sums: measured); a segment is a
  // multiple of three rows (the window's phases) and at least 12 rows (its first rows are read twice).
  {
    const double waves = (double)g.N * a->ncb * (g.Cout / kDwMarchCpl) / 64.0;
    int want = (int)(2048.0 / (waves > 1.0 ? waves : 1.0) + 0.999);
    if (want < 1) want = 1;
    int len = (g.Hout + want - 1) / want;
    if (len < 12) len = 12;
    len = (len + 2) / 3 * 3;
    a->seglen = len;
    a->nseg = (g.Hout + len - 1) / len;
  }
  a->nstrips = g.N * a->nseg * a->ncb;
  // blocks per slab: one per pass while all of them fit kDwMarchBlocks, else in proportion to the passes
  long passes[kDwMarchSlabs], total = 0;
  for (int i = 0; i < n; ++i) {
    const int per_pass = 4 * a->slab[i].sw;
    passes[i] = (a->nstrips + per_pass - 1) / per_pass;
    total += passes[i];
  }
  int blk = 0, pmax = 1;
  for (int i = 0; i < n; ++i) {
    long b = total <= kDwMarchBlocks ? passes[i] : (passes[i] * kDwMarchBlocks + total - 1) / total;
    if (b < 1) b = 1;
    if (b > passes[i]) b = passes[i];
    a->slab[i].blk0 = blk;
    a->slab[i].nblk = (int)b;
    blk += (int)b;
    if ((int)b > pmax) pmax = (int)b;
  }
  a->nblocks = blk;
  a->P = pmax;
  a->Hin = g.Hin; a->Win = g.Win; a->Hout = g.Hout; a->Wout = g.Wout; a->C = g.Cout;
  return g.Cout % 8 == 0 && (g.stride == 1 || g.stride == 2);
}

static DwPlan dw_wgrad_plan(const ConvGeom& g, int es, size_t* lds) {
  const int s = g.stride;
  DwPlan d = dw_plan(g.Cout, es, s == 2, g.Hout, g.Wout);
  const int run = s == 2 ? 2 : 4;                // pixels per run, as the kernel's RL
  d.segw = (d.TW + run - 1) / run;
  d.nseg = d.TH * d.segw;
  d.m_segw = dw_magic(d.segw);
  d.PH = (d.TH - 1) * s + 3;
  d.PW = (d.segw * run - 1) * s + 3;
  d.ntiles = g.N * d.tiles_h * d.tiles_w;
  // Persistent blocks over all slabs: fewer than fit the GPU at once next to the other stream's kernels.  The stride-1
  // kernel holds 207 registers (two blocks per CU): with 512 blocks some waited for a place, and a 5 us finalize kernel
  // of the data-gradient chain was measured waiting up to 200 us with them (a trace shows it ending when the first
  // blocks end); 256 leave the weight gradient itself too slow.  The stride-2 kernel holds 149 registers (three blocks
  // per CU): 480 measured best of 384-768.
  const int capn = s == 2 ? 480 : 384;
  const int cap = capn / d.nslab > 1 ? capn / d.nslab : 1;
  d.nblocks = d.ntiles < cap ? d.ntiles : cap;
  size_t a = (size_t)d.PH * d.PW * d.CGB * 8 * es;          // the patch in the tensor's type
  size_t b = (size_t)d.spp * 9 * 2 * d.CGB * 16;
  *lds = a > b ? a : b;
  return d;
}

// ---- depthwise weight gradient, bfloat16: rows staged through LDS ---------------------------------------------
// The marching kernel above reads memory with one 4-byte access per lane.  With a power-of-two channel count a
// wavefront's access is exactly one aligned pixel and it streams at 4.4 - 4.7 TB/s; with 48, 144, 192 ... channels
// (every layer of a width-1.4 MobileNetV2) pixels straddle cache lines and a narrow tail slab needs accesses of its
// own: 2.1 - 3.4 TB/s, although the arithmetic alone would take a quarter of the time (measured with all rows
// redirected to one cached row).  Here the memory side is decoupled from the channel count: a block owns a band of
// WB output columns of one image (all channels of a slab of at most 256) and walks down a segment of its rows; the
// S new input rows of a step and the dz row are contiguous runs of several KB in memory, fetched with 16-byte
// vectors a step ahead, put through the view once, and kept in an LDS ring of rows; a thread owns one channel QUAD
// and every NCG-th column of the band and reads its nine taps from the ring (8-byte LDS reads, no bounds logic: the
// ring holds zeros where the image ends).  One barrier per step; one fp32 partial [9][C] per block at the end.
enum { kDwRowsNV = 4, kDwRowsDzNV = 2, kDwRowsMaxCpt = 4 };
struct DwRowsArgs {
  const bf16_t* dz;
  const bf16_t* in;
  const float* scale;
  const float* shift;
  int act;
  float* ws;
  int Hin, Win, Hout, Wout, C;
  int CS, nslab;            // channels per slab (a multiple of 8), slabs
  int Q, NCG, CPT, WB;      // channel quads of a slab, column groups, columns per thread and step, columns per band
  int WIN;                  // input columns under a band
  int bands, nseg, seglen;  // bands across, row segments per image, output rows per segment
  int P;                    // blocks (= partials) per slab: N * bands * nseg
};

template <int S, bool VIEW>
__global__ __launch_bounds__(256) void dw_wgrad_rows_k(DwRowsArgs a) {
  constexpr int RING = S == 1 ? 4 : 5;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  const int tid = threadIdx.x;
  const int lb = xcd_logical_block();
  const int si = lb % a.nslab, pb = lb / a.nslab;             // the slabs of a band run side by side
  const int band = pb % a.bands, rest = pb / a.bands, seg = rest % a.nseg, n = rest / a.nseg;
  const int c0 = si * a.CS, cs = a.C - c0 < a.CS ? a.C - c0 : a.CS;      // this slab's channels
  const int CS = a.CS, WIN = a.WIN, WB = a.WB;
  const int wb0 = band * WB, wi0 = wb0 * S - 1;
  const int h0 = seg * a.seglen, h1 = h0 + a.seglen < a.Hout ? h0 + a.seglen : a.Hout;
  const int rowElems = WIN * CS;                               // one ring slot
  bf16_t* ring = reinterpret_cast<bf16_t*>(smem_raw);          // [RING][WIN][CS]
  bf16_t* dzs = ring + RING * rowElems;                        // [2][WB][CS]
  const bf16_t* img = a.in + (size_t)n * a.Hin * a.Win * a.C + c0;
  const bf16_t* dimg = a.dz + (size_t)n * a.Hout * a.Wout * a.C + c0;
  const int VR = CS / 8;                                       // vectors per pixel of the slab
  const int nin = WIN * VR, ndz = WB * VR;                     // vectors per input row, per dz row

  // ---- staging: vector v of a row is (column v / VR, channels 8 * (v % VR) ..); a thread's vectors are the same
  // in every row, so their offsets are worked out once ----
  float* vsc = reinterpret_cast<float*>(dzs + 2 * WB * CS);    // [CS] scale, [CS] shift of the view
  if (VIEW) {
    for (int i = tid; i < CS; i += 256) {
      vsc[i] = i < cs ? a.scale[c0 + i] : 0.f;
      vsc[CS + i] = i < cs ? a.shift[c0 + i] : 0.f;
    }
  }
  int goff[kDwRowsNV], loff[kDwRowsNV];                        // offset inside an image row (-1: nothing there), inside a ring slot
#pragma unroll
  for (int q = 0; q < kDwRowsNV; ++q) {
    const int v = tid + q * 256;
    const int col = v / VR, ch = (v - col * VR) * 8, wi = wi0 + col;
    loff[q] = col * CS + ch;
    goff[q] = (v < nin && wi >= 0 && wi < a.Win && ch < cs) ? wi * a.C + ch : -1;
  }
  int dgoff[kDwRowsDzNV], dloff[kDwRowsDzNV];
#pragma unroll
  for (int q = 0; q < kDwRowsDzNV; ++q) {
    const int v = tid + q * 256;
    const int col = v / VR, ch = (v - col * VR) * 8;
    dloff[q] = col * CS + ch;
    dgoff[q] = (v < ndz && wb0 + col < a.Wout && ch < cs) ? (wb0 + col) * a.C + ch : -1;
  }
  const int nq = (nin + 255) / 256;                            // passes a row takes (uniform)
  uint4 rin[S][kDwRowsNV], rdz[kDwRowsDzNV];
  unsigned okin[S], okdz;
  // an input row y of the image; the ring holds zeros outside the image and past the slab's channels
  auto fetch_row = [&](uint4* r, unsigned& ok, const int y) __attribute__((always_inline)) {
    ok = 0;
    const bool yin = y >= 0 && y < a.Hin;
    const bf16_t* rowp = img + (size_t)(yin ? y : 0) * a.Win * a.C;
#pragma unroll
    for (int q = 0; q < kDwRowsNV; ++q) {
      if (q >= nq) break;
      const bool in = yin && goff[q] >= 0;
      r[q] = *reinterpret_cast<const uint4*>(rowp + (in ? goff[q] : 0));
      ok |= (in ? 1u : 0u) << q;
    }
  };
  auto commit_row = [&](const uint4* r, const unsigned ok, const int y) __attribute__((always_inline)) {
    bf16_t* dst = ring + ((y + RING) % RING) * rowElems;
    const float lo = act_lo(a.act), hi = act_hi(a.act);
#pragma unroll
    for (int q = 0; q < kDwRowsNV; ++q) {
      if (q >= nq) break;
      if (tid + q * 256 >= nin) break;
      uint4 o = make_uint4(0u, 0u, 0u, 0u);
      if (ok & (1u << q)) {
        o = r[q];
        if (VIEW) {
          Raw<bf16_t> raw; raw.a = o;
          float f[8], sc[8], sh[8];
          raw_unpack(raw, f);
          const int ch = loff[q] % CS;
          load8(vsc + ch, sc);
          load8(vsc + CS + ch, sh);
#pragma unroll
          for (int e = 0; e < 8; ++e) f[e] = clamp_act(fmaf(f[e], sc[e], sh[e]), lo, hi);
          o.x = f32x2_to_bf16x2(f[0], f[1]); o.y = f32x2_to_bf16x2(f[2], f[3]);
          o.z = f32x2_to_bf16x2(f[4], f[5]); o.w = f32x2_to_bf16x2(f[6], f[7]);
        }
      }
      *reinterpret_cast<uint4*>(dst + loff[q]) = o;
    }
  };
  auto fetch_dz = [&](const int ho) __attribute__((always_inline)) {
    okdz = 0;
    const bf16_t* rowp = dimg + (size_t)(ho < h1 ? ho : h0) * a.Wout * a.C;
#pragma unroll
    for (int q = 0; q < kDwRowsDzNV; ++q) {
      if (q * 256 >= ndz) break;
      const bool in = dgoff[q] >= 0 && ho < h1;
      rdz[q] = *reinterpret_cast<const uint4*>(rowp + (in ? dgoff[q] : 0));
      okdz |= (in ? 1u : 0u) << q;
    }
  };
  auto commit_dz = [&](const int ho) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < kDwRowsDzNV; ++q) {
      if (tid + q * 256 >= ndz) break;
      *reinterpret_cast<uint4*>(dzs + (ho & 1) * WB * CS + dloff[q]) = (okdz & (1u << q)) ? rdz[q] : make_uint4(0u, 0u, 0u, 0u);
    }
  };

  // ---- this thread's work: channel quad q4 of the slab, columns cgi + j * NCG of the band ----
  const int q4 = tid % a.Q, cgi = tid / a.Q;
  const bool worker = cgi < a.NCG && q4 * 4 < cs;
  float4 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) acc[t] = make_float4(0.f, 0.f, 0.f, 0.f);

  if (VIEW) __syncthreads();                                   // the view vectors are in LDS
  // rows above the first step's new ones
  if (S == 1) {
    fetch_row(rin[0], okin[0], h0 - 1);
    commit_row(rin[0], okin[0], h0 - 1);
    fetch_row(rin[0], okin[0], h0);
    commit_row(rin[0], okin[0], h0);
  } else {
    fetch_row(rin[0], okin[0], 2 * h0 - 1);
    commit_row(rin[0], okin[0], 2 * h0 - 1);
  }
  // the new rows of step ho: S == 1: row ho + 1; S == 2: rows 2 ho and 2 ho + 1
  auto fetch_step = [&](const int ho) __attribute__((always_inline)) {
#pragma unroll
    for (int r = 0; r < S; ++r) fetch_row(rin[r], okin[r], S == 1 ? ho + 1 : 2 * ho + r);
    fetch_dz(ho);
  };
  fetch_step(h0);
  for (int ho = h0; ho < h1; ++ho) {
#pragma unroll
    for (int r = 0; r < S; ++r) commit_row(rin[r], okin[r], S == 1 ? ho + 1 : 2 * ho + r);
    commit_dz(ho);
    __syncthreads();          // also: every thread is done with the step before last, whose ring slots are written next
    fetch_step(ho + 1);       // past the segment: rows of the image that are simply not used (dz past h1 is zero)
    if (worker) {
      const bf16_t* dzr = dzs + (ho & 1) * WB * CS + q4 * 4;
      const bf16_t* rows[3];
#pragma unroll
      for (int ky = 0; ky < 3; ++ky) rows[ky] = ring + ((ho * S - 1 + ky + RING) % RING) * rowElems + q4 * 4;
#pragma unroll
      for (int j = 0; j < kDwRowsMaxCpt; ++j) {
        if (j >= a.CPT) break;
        const int lc = cgi + j * a.NCG;                        // column of the band
        const float4 d = load4(dzr + lc * CS);
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
          const bf16_t* row = rows[ky] + (lc * S) * CS;
#pragma unroll
          for (int kx = 0; kx < 3; ++kx) acc[ky * 3 + kx] = fma4(d, load4(row + kx * CS), acc[ky * 3 + kx]);
        }
      }
    }
  }
  // ---- the block's partial: the column groups of a channel quad in a fixed order ----
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem_raw);             // [NCG][9][CS]
  if (worker) {
#pragma unroll
    for (int t = 0; t < 9; ++t) *reinterpret_cast<float4*>(red + ((size_t)cgi * 9 + t) * CS + q4 * 4) = acc[t];
  }
  __syncthreads();
  for (int i = tid; i < 9 * cs; i += 256) {
    const int t = i / cs, c = i - t * cs;
    float tot = 0.f;
    for (int g = 0; g < a.NCG; ++g) tot += red[((size_t)g * 9 + t) * CS + c];
    a.ws[((size_t)pb * 9 + t) * a.C + c0 + c] = tot;
  }
}

static bool dw_rows_plan(const ConvGeom& g, DwRowsArgs* a, size_t* lds) {
  const int S = g.stride, C = g.Cout;
  if (C % 8 || (S != 1 && S != 2) || g.kh != 3 || g.kw != 3) return false;
  a->nslab = (C + 255) / 256;
  a->CS = ((C + a->nslab - 1) / a->nslab + 7) / 8 * 8;
  a->Q = a->CS / 4;
  a->NCG = 256 / a->Q;
  if (a->NCG < 1) return false;
  if (a->NCG > g.Wout) a->NCG = g.Wout;
  // columns per thread and step
  // ring rows of about 8 KB at stride 2, 4 KB at stride 1, and about 1024 / 2048 blocks: measured on the 112 x 112 layers
  const double row_bytes = S == 2 ? 8192.0 : 4096.0, want_blocks = S == 2 ? 1024.0 : 2048.0;
  int cpt = (int)(row_bytes / ((double)a->NCG * S * a->CS * 2) + 0.5);
  if (cpt < 1) cpt = 1;
  if (cpt > kDwRowsMaxCpt) cpt = kDwRowsMaxCpt;
  while (cpt > 1 && a->NCG * (cpt - 1) >= g.Wout) --cpt;
  a->CPT = cpt;
  a->WB = a->NCG * cpt;
  a->WIN = (a->WB - 1) * S + 3;
  a->bands = (g.Wout + a->WB - 1) / a->WB;
  while (a->CPT > 1 && ((size_t)a->WIN * (a->CS / 8) > (size_t)kDwRowsNV * 256 || (size_t)a->WB * (a->CS / 8) > (size_t)kDwRowsDzNV * 256)) {
    --a->CPT;
    a->WB = a->NCG * a->CPT;
    a->WIN = (a->WB - 1) * S + 3;
    a->bands = (g.Wout + a->WB - 1) / a->WB;
  }
  if ((size_t)a->WIN * (a->CS / 8) > (size_t)kDwRowsNV * 256 || (size_t)a->WB * (a->CS / 8) > (size_t)kDwRowsDzNV * 256) return false;
  // row segments, at least 8 rows each
  const double blocks = (double)g.N * a->bands * a->nslab;
  int want = (int)(want_blocks / (blocks > 1.0 ? blocks : 1.0) + 0.999);
  if (want < 1) want = 1;
  int len = (g.Hout + want - 1) / want;
  if (len < 8) len = 8;
  if (len > g.Hout) len = g.Hout;
  a->seglen = len;
  a->nseg = (g.Hout + len - 1) / len;
  a->P = g.N * a->bands * a->nseg;
  a->Hin = g.Hin; a->Win = g.Win; a->Hout = g.Hout; a->Wout = g.Wout; a->C = C;
  const int RING = S == 1 ? 4 : 5;
  const size_t stage = ((size_t)RING * a->WIN + 2 * (size_t)a->WB) * a->CS * sizeof(bf16_t) + 2 * (size_t)a->CS * sizeof(float);
  const size_t red = (size_t)a->NCG * 9 * a->CS * sizeof(float);
  *lds = stage > red ? stage : red;
  return *lds <= 64 * 1024 && a->P <= 65535;
}

size_t dw_wgrad_ws(const ConvGeom& g) {
  size_t lds;
  DwPlan d = dw_wgrad_plan(g, 4, &lds);          // the float plan has at least as many slabs, the bound holds for both
  DwPlan e = dw_wgrad_plan(g, 2, &lds);
  size_t n = (size_t)(d.nblocks > e.nblocks ? d.nblocks : e.nblocks);
  DwMarchArgs m{};
  if (dw_march_plan(g, &m) && (size_t)m.P > n) n = m.P;
  DwRowsArgs r{};
  size_t rl;
  if (dw_rows_plan(g, &r, &rl) && (size_t)r.P > n) n = r.P;
  return n * 9 * g.Cout;
}

void dw_wgrad(int dt, hipStream_t st, const void* dz, HView in, const ConvGeom& g, float* ws, float* g_w) {
  const int es = dt == 0 ? 4 : 2;
  {
    DwRowsArgs r{};
    size_t lds;
    // Where it pays (measured, all layer shapes of the two MobileNetV2 widths): images of 112 x 112 and more whose channel
    // count the marching kernel has to cut into a wide slab and a narrow tail.  Power-of-two channel counts, and the
    // smaller images (too few rows per block to hide the step's barrier behind), stay with the marching kernel.
    DwMarchArgs mm{};
    const bool tail = dw_march_plan(g, &mm) && mm.nslab > 1;
    if (dt == 1 && tail && (size_t)g.Hin * g.Win >= (size_t)112 * 112 && dw_rows_plan(g, &r, &lds)) {
      r.dz = (const bf16_t*)dz; r.in = (const bf16_t*)in.z; r.scale = in.scale; r.shift = in.shift; r.act = in.act; r.ws = ws;
      {
        KScope ks(st, "dw_wgrad", ((double)g.N * g.Hin * g.Win * g.Cout + (double)g.N * g.Hout * g.Wout * g.Cout) * es + (double)r.P * 9 * g.Cout * 4,
                  18.0 * g.N * g.Hout * g.Wout * g.Cout, (long)g.N * g.Hout * g.Wout, g.Cout, g.stride);
        const dim3 grid((unsigned)r.P * r.nslab), block(256);
        if (g.stride == 1) {
          if (in.scale) hipLaunchKernelGGL((dw_wgrad_rows_k<1, true>), grid, block, lds, st, r);
          else hipLaunchKernelGGL((dw_wgrad_rows_k<1, false>), grid, block, lds, st, r);
        } else {
          if (in.scale) hipLaunchKernelGGL((dw_wgrad_rows_k<2, true>), grid, block, lds, st, r);
          else hipLaunchKernelGGL((dw_wgrad_rows_k<2, false>), grid, block, lds, st, r);
        }
      }
      reduce_partials(st, ws, r.P, (size_t)9 * g.Cout, g.Cout, 1, 9, g_w);
      return;
    }
  }
  DwMarchArgs m{};
  if (dw_march_plan(g, &m)) {
    m.dz = dz; m.in = View{in.z, in.scale, in.shift, in.act}; m.ws = ws;
    {
      KScope ks(st, "dw_wgrad", ((double)g.N * g.Hin * g.Win * g.Cout + (double)g.N * g.Hout * g.Wout * g.Cout) * es + (double)m.P * 9 * g.Cout * 4,
                18.0 * g.N * g.Hout * g.Wout * g.Cout, (long)g.N * g.Hout * g.Wout, g.Cout, g.stride);
      const unsigned grid = (unsigned)m.nblocks;
      const bool vw = in.scale != nullptr;
      if (g.stride == 1) {
        if (vw) { FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_wgrad_march_k<T, 1, true>), dim3(grid), dim3(256), 0, st, m)); }
        else { FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_wgrad_march_k<T, 1, false>), dim3(grid), dim3(256), 0, st, m)); }
      } else {
        if (vw) { FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_wgrad_march_k<T, 2, true>), dim3(grid), dim3(256), 0, st, m)); }
        else { FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_wgrad_march_k<T, 2, false>), dim3(grid), dim3(256), 0, st, m)); }
      }
    }
    reduce_partials(st, ws, m.P, (size_t)9 * g.Cout, g.Cout, 1, 9, g_w);
    return;
  }
  size_t lds;
  DwPlan d = dw_wgrad_plan(g, es, &lds);
  if (!dw_check_plan(d, g.stride == 2 ? 1 : kDwSegs)) return;     // also: the runs of a tile whose dz a thread holds
  View v{in.z, in.scale, in.shift, in.act};
  {
    KScope ks(st, "dw_wgrad", ((double)g.N * g.Hin * g.Win * g.Cout + (double)g.N * g.Hout * g.Wout * g.Cout) * es + (double)d.nblocks * 9 * g.Cout * 4,
              18.0 * g.N * g.Hout * g.Wout * g.Cout, (long)g.N * g.Hout * g.Wout, g.Cout, g.stride);
    const unsigned grid = (unsigned)d.nblocks * d.nslab;
    if (g.stride == 1) {
      FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_wgrad_k<T, 1>), dim3(grid), dim3(256), lds, st, (const T*)dz, v, d, g.Hin, g.Win,
                                          g.Hout, g.Wout, g.Cout, ws));
    } else {
      FTP_DISPATCH(dt, hipLaunchKernelGGL((dw_wgrad_k<T, 2>), dim3(grid), dim3(256), lds, st, (const T*)dz, v, d, g.Hin, g.Win,
                                          g.Hout, g.Wout, g.Cout, ws));
    }
  }
  reduce_partials(st, ws, d.nblocks, (size_t)9 * g.Cout, g.Cout, 1, 9, g_w);
}

}  // namespace ftp
