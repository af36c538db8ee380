// Small dense convolutions (3x3 stem, conv1d) and depthwise 3x3, NHWC.
// Inputs are read through a View, so the producer's BatchNorm + activation is
// applied on load and zero padding is inserted after it (a halo cell is 0, not
// act(bn(0))).
#include "dev_common.h"
#include "kernels.h"

namespace ftp {

#define FTP_DISPATCH(dt, ...)                   \
  do {                                          \
    if ((dt) == 0) { typedef float T; __VA_ARGS__; } \
    else { typedef bf16_t T; __VA_ARGS__; }     \
  } while (0)

// g[(j % C) * stride_c + (j / C) * stride_q] += sum_p ws[p * QC + j]
__global__ void reduce_partials_k(const float* __restrict__ ws, int P, size_t QC, int C, size_t stride_q,
                                  size_t stride_c, float* __restrict__ g) {
  size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= QC) return;
  double s = 0.0;
  for (int p = 0; p < P; ++p) s += (double)ws[(size_t)p * QC + j];
  size_t o = (j % C) * stride_c + (j / C) * stride_q;
  g[o] += (float)s;
}

void reduce_partials(hipStream_t st, const float* ws, int P, size_t QC, int C, size_t stride_q,
                     size_t stride_c, float* g) {
  KScope ks(st, "reduce_partials", ((double)P + 2.0) * QC * 4, (double)P * QC);
  hipLaunchKernelGGL(reduce_partials_k, dim3((unsigned)((QC + 255) / 256)), dim3(256), 0, st, ws, P, QC, C,
                     stride_q, stride_c, g);
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

// thread = (k = (tap, ci), 8 output channels); block = a chunk of output pixels
template <typename T>
__global__ void conv_direct_wgrad_k(const T* __restrict__ dz, View in, ConvGeom g, int KPB, size_t ppc,
                                    float* __restrict__ ws) {
  const int CGo = g.Cout / 8;
  const int cg = threadIdx.x % CGo;
  const int k = blockIdx.y * KPB + threadIdx.x / CGo;
  const int K = g.kh * g.kw * g.Cin;
  if (k >= K) return;
  const int tap = k / g.Cin, ci = k % g.Cin, i = tap / g.kw, j = tap % g.kw;
  const size_t total = (size_t)g.N * g.Hout * g.Wout;
  size_t p0 = (size_t)blockIdx.x * ppc, p1 = p0 + ppc < total ? p0 + ppc : total;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (size_t pix = p0; pix < p1; ++pix) {
    int wo = (int)(pix % g.Wout);
    size_t r = pix / g.Wout;
    int ho = (int)(r % g.Hout), n = (int)(r / g.Hout);
    int hi = ho * g.stride + i - g.ph, wi = wo * g.stride + j - g.pw;
    if (hi < 0 || hi >= g.Hin || wi < 0 || wi >= g.Win) continue;
    float xv = view_at<T>(in, (((size_t)n * g.Hin + hi) * g.Win + wi) * g.Cin + ci, ci);
    float d[8];
    load8(dz + pix * g.Cout + cg * 8, d);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = fmaf(xv, d[e], acc[e]);
  }
  store8(ws + ((size_t)blockIdx.x * K + k) * g.Cout + cg * 8, acc);
}

static void direct_wgrad_shape(const ConvGeom& g, int* S, size_t* ppc) {
  size_t total = (size_t)g.N * g.Hout * g.Wout;
  size_t c = (total + 511) / 512;
  if (c < 64) c = 64;
  *ppc = c;
  *S = (int)((total + c - 1) / c);
}

size_t conv_direct_wgrad_ws(const ConvGeom& g) {
  int S; size_t ppc;
  direct_wgrad_shape(g, &S, &ppc);
  return (size_t)S * g.kh * g.kw * g.Cin * g.Cout;
}

void conv_direct_wgrad(int dt, hipStream_t st, const void* dz, HView in, const ConvGeom& g, float* ws,
                       float* g_w) {
  int S; size_t ppc;
  direct_wgrad_shape(g, &S, &ppc);
  int CGo = g.Cout / 8, KPB = 256 / CGo, K = g.kh * g.kw * g.Cin;
  if (KPB < 1) KPB = 1;
  View v{in.z, in.scale, in.shift, in.act};
  {
    KScope ks(st, "conv_direct_wgrad", ((double)g.N * g.Hin * g.Win * g.Cin + (double)g.N * g.Hout * g.Wout * g.Cout) * (dt == 0 ? 4.0 : 2.0) + (double)S * K * g.Cout * 4,
              2.0 * g.N * g.Hout * g.Wout * g.Cout * K);
    FTP_DISPATCH(dt, hipLaunchKernelGGL(conv_direct_wgrad_k<T>, dim3(S, (K + KPB - 1) / KPB), dim3(KPB * CGo), 0,
                                        st, (const T*)dz, v, g, KPB, ppc, ws));
  }
  reduce_partials(st, ws, S, (size_t)K * g.Cout, g.Cout, 1, (size_t)K, g_w);
}

// ================================================================ depthwise 3x3
// rows = pixels, thread = 8 channels; the block's slab of weights sits in LDS as [tap][channel]
template <typename T>
__device__ __forceinline__ void dw_load_weights(const T* __restrict__ w, int C, int W, float* wl) {
  int c_base = blockIdx.y * W * 8;
  for (int idx = threadIdx.x; idx < 9 * W * 8; idx += blockDim.x) {
    int tap = idx / (W * 8), cl = idx % (W * 8);
    int c = c_base + cl;
    wl[idx] = c < C ? to_f32(w[(size_t)c * 9 + tap]) : 0.f;
  }
  __syncthreads();
}

template <typename T>
__global__ void dw_fwd_k(View in, const T* __restrict__ w, ConvGeom g, int W, int R, size_t rpb,
                         T* __restrict__ z) {
  extern __shared__ float wl[];
  const int C = g.Cout;
  dw_load_weights(w, C, W, wl);
  int tx = threadIdx.x % W, ty = threadIdx.x / W;
  int cg = blockIdx.y * W + tx;
  if (cg >= C / 8) return;
  const int c0 = cg * 8;
  const size_t total = (size_t)g.N * g.Hout * g.Wout;
  size_t m0 = (size_t)blockIdx.x * rpb, m1 = m0 + rpb < total ? m0 + rpb : total;
  for (size_t m = m0 + ty; m < m1; m += R) {
    int wo = (int)(m % g.Wout);
    size_t r = m / g.Wout;
    int ho = (int)(r % g.Hout), n = (int)(r / g.Hout);
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      int hi = ho * g.stride + i - 1;
      if (hi < 0 || hi >= g.Hin) continue;
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        int wi = wo * g.stride + j - 1;
        if (wi < 0 || wi >= g.Win) continue;
        float v[8];
        view_load8<T>(in, (((size_t)n * g.Hin + hi) * g.Win + wi) * C + c0, c0, v);
        const float* wr = wl + (i * 3 + j) * W * 8 + tx * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(v[e], wr[e], acc[e]);
      }
    }
    store8(z + m * C + c0, acc);
  }
}

static RowTile dw_tile(size_t rows, int C) {
  // weight slab in LDS is 9*W*8 floats: keep W <= 64 (18 KB)
  RowTile t;
  int CG = C / 8;
  t.nslab = (CG + 63) / 64;
  t.W = (CG + t.nslab - 1) / t.nslab;
  t.R = 256 / t.W;
  size_t want = (rows + 2047) / 2048;
  size_t rpb = ((want + t.R - 1) / t.R) * t.R;
  if (rpb < (size_t)t.R * 2) rpb = (size_t)t.R * 2;
  t.rows_per_block = rpb;
  t.P = (int)((rows + rpb - 1) / rpb);
  return t;
}

void dw_fwd(int dt, hipStream_t st, HView in, const void* w, const ConvGeom& g, void* z) {
  size_t total = (size_t)g.N * g.Hout * g.Wout;
  RowTile t = dw_tile(total, g.Cout);
  View v{in.z, in.scale, in.shift, in.act};
  size_t sm = (size_t)9 * t.W * 8 * sizeof(float);
  KScope ks(st, "dw_fwd", ((double)g.N * g.Hin * g.Win * g.Cout + (double)total * g.Cout) * (dt == 0 ? 4.0 : 2.0), 18.0 * total * g.Cout);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(dw_fwd_k<T>, dim3(t.P, t.nslab), dim3(t.W * t.R), sm, st, v, (const T*)w, g,
                                      t.W, t.R, t.rows_per_block, (T*)z));
}

// gather form: every input pixel collects the (at most 9) outputs it fed
template <typename T>
__global__ void dw_dgrad_k(const T* __restrict__ dz, const T* __restrict__ w, ConvGeom g, int W, int R,
                           size_t rpb, T* __restrict__ dIn) {
  extern __shared__ float wl[];
  const int C = g.Cout;
  dw_load_weights(w, C, W, wl);
  int tx = threadIdx.x % W, ty = threadIdx.x / W;
  int cg = blockIdx.y * W + tx;
  if (cg >= C / 8) return;
  const int c0 = cg * 8;
  const size_t total = (size_t)g.N * g.Hin * g.Win;
  size_t m0 = (size_t)blockIdx.x * rpb, m1 = m0 + rpb < total ? m0 + rpb : total;
  for (size_t m = m0 + ty; m < m1; m += R) {
    int wi = (int)(m % g.Win);
    size_t r = m / g.Win;
    int hi = (int)(r % g.Hin), n = (int)(r / g.Hin);
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      int hn = hi + 1 - i;
      if (hn < 0 || (hn % g.stride) != 0) continue;
      int ho = hn / g.stride;
      if (ho >= g.Hout) continue;
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        int wn = wi + 1 - j;
        if (wn < 0 || (wn % g.stride) != 0) continue;
        int wo = wn / g.stride;
        if (wo >= g.Wout) continue;
        float d[8];
        load8(dz + (((size_t)n * g.Hout + ho) * g.Wout + wo) * C + c0, d);
        const float* wr = wl + (i * 3 + j) * W * 8 + tx * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(d[e], wr[e], acc[e]);
      }
    }
    store8(dIn + m * C + c0, acc);
  }
}

void dw_dgrad(int dt, hipStream_t st, const void* dz, const void* w, const ConvGeom& g, void* dIn) {
  size_t total = (size_t)g.N * g.Hin * g.Win;
  RowTile t = dw_tile(total, g.Cout);
  size_t sm = (size_t)9 * t.W * 8 * sizeof(float);
  KScope ks(st, "dw_dgrad", ((double)total * g.Cout + (double)g.N * g.Hout * g.Wout * g.Cout) * (dt == 0 ? 4.0 : 2.0), 18.0 * g.N * g.Hout * g.Wout * g.Cout);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(dw_dgrad_k<T>, dim3(t.P, t.nslab), dim3(t.W * t.R), sm, st, (const T*)dz,
                                      (const T*)w, g, t.W, t.R, t.rows_per_block, (T*)dIn));
}

// per-channel, per-tap sums over all output pixels: thread partials -> LDS -> ws[P][9][C]
template <typename T>
__global__ void dw_wgrad_k(const T* __restrict__ dz, View in, ConvGeom g, int W, int R, size_t rpb,
                           float* __restrict__ ws) {
  extern __shared__ float smem[];
  const int C = g.Cout;
  int tx = threadIdx.x % W, ty = threadIdx.x / W;
  int cg = blockIdx.y * W + tx;
  const bool live = cg < C / 8;
  const int c0 = cg * 8;
  float acc[72];
#pragma unroll
  for (int e = 0; e < 72; ++e) acc[e] = 0.f;
  if (live) {
    const size_t total = (size_t)g.N * g.Hout * g.Wout;
    size_t m0 = (size_t)blockIdx.x * rpb, m1 = m0 + rpb < total ? m0 + rpb : total;
    for (size_t m = m0 + ty; m < m1; m += R) {
      int wo = (int)(m % g.Wout);
      size_t r = m / g.Wout;
      int ho = (int)(r % g.Hout), n = (int)(r / g.Hout);
      float d[8];
      load8(dz + m * C + c0, d);
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        int hi = ho * g.stride + i - 1;
        if (hi < 0 || hi >= g.Hin) continue;
#pragma unroll
        for (int j = 0; j < 3; ++j) {
          int wi = wo * g.stride + j - 1;
          if (wi < 0 || wi >= g.Win) continue;
          float v[8];
          view_load8<T>(in, (((size_t)n * g.Hin + hi) * g.Win + wi) * C + c0, c0, v);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[(i * 3 + j) * 8 + e] = fmaf(d[e], v[e], acc[(i * 3 + j) * 8 + e]);
        }
      }
    }
  }
  // reduce across the R rows of the block, 3 taps (24 values) at a time
#pragma unroll
  for (int part = 0; part < 3; ++part) {
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 24; ++e) smem[(e * R + ty) * W + tx] = acc[part * 24 + e];
    __syncthreads();
    if (ty == 0 && live) {
#pragma unroll
      for (int t = 0; t < 3; ++t) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float s = 0.f;
          for (int r = 0; r < R; ++r) s += smem[((t * 8 + e) * R + r) * W + tx];
          o[e] = s;
        }
        store8(ws + ((size_t)blockIdx.x * 9 + part * 3 + t) * C + c0, o);
      }
    }
  }
}

static RowTile dw_wgrad_tile(const ConvGeom& g) {
  size_t total = (size_t)g.N * g.Hout * g.Wout;
  RowTile t = dw_tile(total, g.Cout);
  size_t want = (total + kMaxPartials - 1) / kMaxPartials;
  size_t rpb = ((want + t.R - 1) / t.R) * t.R;
  if (rpb < (size_t)t.R * 2) rpb = (size_t)t.R * 2;
  t.rows_per_block = rpb;
  t.P = (int)((total + rpb - 1) / rpb);
  return t;
}

size_t dw_wgrad_ws(const ConvGeom& g) { return (size_t)dw_wgrad_tile(g).P * 9 * g.Cout; }

void reduce_partials(hipStream_t st, const float* ws, int P, size_t QC, int C, size_t stride_q,
                     size_t stride_c, float* g);

void dw_wgrad(int dt, hipStream_t st, const void* dz, HView in, const ConvGeom& g, float* ws, float* g_w) {
  RowTile t = dw_wgrad_tile(g);
  View v{in.z, in.scale, in.shift, in.act};
  size_t sm = (size_t)24 * t.R * t.W * sizeof(float);
  {
    KScope ks(st, "dw_wgrad", ((double)g.N * g.Hin * g.Win * g.Cout + (double)g.N * g.Hout * g.Wout * g.Cout) * (dt == 0 ? 4.0 : 2.0) + (double)t.P * 9 * g.Cout * 4,
              18.0 * g.N * g.Hout * g.Wout * g.Cout);
    FTP_DISPATCH(dt, hipLaunchKernelGGL(dw_wgrad_k<T>, dim3(t.P, t.nslab), dim3(t.W * t.R), sm, st, (const T*)dz, v,
                                        g, t.W, t.R, t.rows_per_block, ws));
  }
  reduce_partials(st, ws, t.P, (size_t)9 * g.Cout, g.Cout, 1, 9, g_w);
}

}  // namespace ftp
