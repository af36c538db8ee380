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
  const size_t j = (size_t)blockIdx.x * 16 + jl;
  double s = 0.0;
  if (j < QC) {
    int p = lane;
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
  const int KG = Kpad / 8, K = g.kh * g.kw * g.Cin;
  const size_t total = (size_t)g.N * g.Hout * g.Wout * KG;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const int kg = (int)(idx % KG);
    const size_t pix = idx / KG;
    const int wo = (int)(pix % g.Wout);
    const size_t r = pix / g.Wout;
    const int ho = (int)(r % g.Hout), n = (int)(r / g.Hout);
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = kg * 8 + e;
      float x = 0.f;
      if (k < K) {
        const int tap = k / g.Cin, ci = k % g.Cin, i = tap / g.kw, j = tap % g.kw;
        const int hi = ho * g.stride + i - g.ph, wi = wo * g.stride + j - g.pw;
        if (hi >= 0 && hi < g.Hin && wi >= 0 && wi < g.Win)
          x = view_at<T>(in, (((size_t)n * g.Hin + hi) * g.Win + wi) * g.Cin + ci, ci);
      }
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
                       float* g_w) {
  const int Kpad = direct_kpad(g), K = g.kh * g.kw * g.Cin;
  const size_t M = (size_t)g.N * g.Hout * g.Wout;
  View v{in.z, in.scale, in.shift, in.act};
  {
    const double es = dt == 0 ? 4.0 : 2.0;
    KScope ks(st, "im2col", ((double)g.N * g.Hin * g.Win * g.Cin + (double)M * Kpad) * es, 0, (long)M, Kpad, g.Cout);
    size_t nvec = M * (Kpad / 8);
    unsigned grid = (unsigned)((nvec + 255) / 256 > 65536 ? 65536 : (nvec + 255) / 256);
    FTP_DISPATCH(dt, hipLaunchKernelGGL(im2col_k<T>, dim3(grid), dim3(256), 0, st, v, g, Kpad, (T*)im2col));
  }
  pw_wgrad(dt, st, dz, HView{im2col, nullptr, nullptr, 0}, M, Kpad, g.Cout, ws, g_w, K);
}

// ================================================================ depthwise 3x3
// A block owns a slab of CGB*8 channels and walks spatial output tiles (TH x TW).  For every
// tile the input patch with its one-pixel halo is staged in LDS once, already passed through the
// producer's BatchNorm + activation and with zeros outside the image, so HBM sees every input
// element once per tile and the nine taps are served from LDS.  Threads keep the slab's weights
// in registers; per-channel BatchNorm sums (forward) and weight-gradient sums (wgrad) accumulate
// over all tiles of the block and leave as one partial per block.
struct DwPlan {
  int TH, TW, PH, PW;       // output tile, staged patch (input resolution)
  int CGB, nslab, PPB;      // column groups per slab, slabs, pixels per pass (blockDim = CGB*PPB)
  int tiles_h, tiles_w, ntiles, nblocks;
  size_t lds_bytes;
};

static DwPlan dw_plan(const ConvGeom& g, int es, int out_h, int out_w, int max_blocks) {
  DwPlan d;
  const int cgs = g.Cout / 8, cap = es == 2 ? 8 : 4;       // 128 bytes of channels per pixel
  d.nslab = (cgs + cap - 1) / cap;
  d.CGB = (cgs + d.nslab - 1) / d.nslab;
  d.PPB = 256 / d.CGB;
  d.TH = g.stride == 1 ? 8 : 4;
  d.TW = 8;
  if (d.TH > out_h) d.TH = out_h;
  if (d.TW > out_w) d.TW = out_w;
  d.tiles_h = (out_h + d.TH - 1) / d.TH;
  d.tiles_w = (out_w + d.TW - 1) / d.TW;
  d.ntiles = g.N * d.tiles_h * d.tiles_w;
  d.nblocks = d.ntiles < max_blocks ? d.ntiles : max_blocks;
  d.PH = d.PW = 0;
  d.lds_bytes = 0;
  return d;
}

// Rows h0..h0+PH-1, cols w0..w0+PW-1 of image n (H x W x C), channel groups cg0..cg0+CGB-1, as
// LDS array [PH][PW][CGB][8].  fetch() issues the global loads into registers, commit() applies the
// view and writes LDS, so the loads of the next tile are in flight while the current one is used.
template <typename T, bool VIEW, int NV>
struct PatchLoader {
  Raw<T> raw[NV];
  unsigned ok;
  __device__ __forceinline__ void fetch(const T* __restrict__ src, int n, int h0, int w0, int PH, int PW, int H, int W,
                                        int C, int cg0, int CGB) {
    ok = 0;
    const int total = PH * PW * CGB, cgs = C / 8;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int v = threadIdx.x + q * blockDim.x;
      if (v < total) {
        const int cg = v % CGB, pix = v / CGB, pw = pix % PW, ph = pix / PW;
        const int h = h0 + ph, w = w0 + pw, gcg = cg0 + cg;
        if (h >= 0 && h < H && w >= 0 && w < W && gcg < cgs) {
          raw_load(raw[q], src + (((size_t)n * H + h) * W + w) * C + gcg * 8);
          ok |= 1u << q;
        }
      }
    }
  }
  __device__ __forceinline__ void commit(float* lds, const View& vw, int PH, int PW, int cg0, int CGB) const {
    const int total = PH * PW * CGB;
#pragma unroll
    for (int q = 0; q < NV; ++q) {
      const int v = threadIdx.x + q * blockDim.x;
      if (v < total) {
        float val[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (ok & (1u << q)) {
          raw_unpack(raw[q], val);
          if (VIEW && vw.scale) {
            const int c = (cg0 + v % CGB) * 8;
            float sc[8], sh[8];
            load8(vw.scale + c, sc);
            load8(vw.shift + c, sh);
            const float lo = act_lo(vw.act), hi = act_hi(vw.act);
#pragma unroll
            for (int e = 0; e < 8; ++e) val[e] = round_to<T>(clamp_act(fmaf(val[e], sc[e], sh[e]), lo, hi));
          }
        }
        store8(lds + (size_t)v * 8, val);
      }
    }
  }
};
enum { kDwPatchNV = 5, kDwTileNV = 2 };

// Forward: one block = one spatial tile x one channel slab.  Many small blocks per CU hide the
// HBM latency; weights of the slab sit in LDS next to the patch.
template <typename T>
__global__ __launch_bounds__(256) void dw_fwd_k(View in, const T* __restrict__ w, ConvGeom g, DwPlan d, T* __restrict__ z) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  const int C = g.Cout, cgs = C / 8, s = g.stride;
  const int PH = (d.TH - 1) * s + 3, PW = (d.TW - 1) * s + 3;
  float* patch = reinterpret_cast<float*>(smem_raw);      // float in LDS: converted once, no unpacking per tap
  float* wl = patch + (size_t)PH * PW * d.CGB * 8;        // [9][CGB][8]
  const int cg = threadIdx.x % d.CGB, pl = threadIdx.x / d.CGB;
  const int cg0 = blockIdx.y * d.CGB, gcg = cg0 + cg;
  const int tile = blockIdx.x;
  const int tw = tile % d.tiles_w, th = (tile / d.tiles_w) % d.tiles_h, n = tile / (d.tiles_w * d.tiles_h);
  const int ho0 = th * d.TH, wo0 = tw * d.TW;
  for (int i = threadIdx.x; i < 9 * d.CGB * 8; i += blockDim.x) {
    const int e = i % 8, c8 = (i / 8) % d.CGB, t = i / (8 * d.CGB);
    const int c = (cg0 + c8) * 8 + e;
    wl[i] = c < C ? to_f32(w[(size_t)c * 9 + t]) : 0.f;
  }
  {
    // thread = (pixel lane pl, column group cg); pixel index advances by PPB per pass
    const int npix = PH * PW, h0 = ho0 * s - 1, w0 = wo0 * s - 1;
    const int dph = d.PPB / PW, dpw = d.PPB % PW;
    int ph = pl / PW, pw = pl % PW;
    for (int pix = pl; pix < npix; pix += d.PPB) {
      const int h = h0 + ph, ww = w0 + pw;
      float val[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      if (h >= 0 && h < g.Hin && ww >= 0 && ww < g.Win && gcg < cgs)
        view_load8<T>(in, (((size_t)n * g.Hin + h) * g.Win + ww) * C + gcg * 8, gcg * 8, val);
      store8(patch + ((size_t)pix * d.CGB + cg) * 8, val);
      ph += dph; pw += dpw;
      if (pw >= PW) { pw -= PW; ++ph; }
    }
  }
  __syncthreads();
  if (gcg >= cgs) return;
  const int dhl = d.PPB / d.TW, dwl = d.PPB % d.TW;
  int hl = pl / d.TW, wl_ = pl % d.TW;
  for (int p = pl; p < d.TH * d.TW; p += d.PPB, hl += dhl, wl_ += dwl) {
    if (wl_ >= d.TW) { wl_ -= d.TW; ++hl; }
    const int ho = ho0 + hl, wo = wo0 + wl_;
    if (ho >= g.Hout || wo >= g.Wout) continue;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        float v[8], wr[8];
        load8(patch + ((size_t)((hl * s + i) * PW + wl_ * s + j) * d.CGB + cg) * 8, v);
        load8(wl + ((i * 3 + j) * d.CGB + cg) * 8, wr);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(v[e], wr[e], acc[e]);
      }
    store8(z + (((size_t)n * g.Hout + ho) * g.Wout + wo) * C + gcg * 8, acc);
  }
}

void dw_fwd(int dt, hipStream_t st, HView in, const void* w, const ConvGeom& g, void* z) {
  const int es = dt == 0 ? 4 : 2;
  DwPlan d = dw_plan(g, es, g.Hout, g.Wout, 1 << 30);
  View v{in.z, in.scale, in.shift, in.act};
  size_t total = (size_t)g.N * g.Hout * g.Wout;
  KScope ks(st, "dw_fwd", ((double)g.N * g.Hin * g.Win * g.Cout + (double)total * g.Cout) * es, 18.0 * total * g.Cout,
            (long)total, g.Cout, g.stride);
  int PH = (d.TH - 1) * g.stride + 3, PW = (d.TW - 1) * g.stride + 3;
  size_t lds = (size_t)PH * PW * d.CGB * 8 * 4 + (size_t)9 * d.CGB * 8 * 4;
  FTP_DISPATCH(dt, hipLaunchKernelGGL(dw_fwd_k<T>, dim3(d.ntiles, d.nslab), dim3(d.CGB * d.PPB), lds, st,
                                      v, (const T*)w, g, d, (T*)z));
}

// dIn tile (input resolution) from a staged dz patch: dIn[h][w] = sum_{i,j} dz[(h+1-i)/s][(w+1-j)/s] * w[i][j]
template <typename T>
__global__ __launch_bounds__(256) void dw_dgrad_k(const T* __restrict__ dz, const T* __restrict__ w, ConvGeom g, DwPlan d, T* __restrict__ dIn) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  const int C = g.Cout, cgs = C / 8, s = g.stride;
  float* patch = reinterpret_cast<float*>(smem_raw);
  float* wl = patch + (size_t)d.PH * d.PW * d.CGB * 8;    // [9][CGB][8]
  const int cg = threadIdx.x % d.CGB, pl = threadIdx.x / d.CGB;
  const int cg0 = blockIdx.y * d.CGB, gcg = cg0 + cg;
  const int tile = blockIdx.x;
  const int tw = tile % d.tiles_w, th = (tile / d.tiles_w) % d.tiles_h, n = tile / (d.tiles_w * d.tiles_h);
  const int h0 = th * d.TH, w0 = tw * d.TW;                 // input-resolution tile origin (even)
  // dz rows that can reach input rows h0 .. h0+TH-1: ho = (h+1-i)/s, i in 0..2
  const int ho_lo = s == 1 ? h0 - 1 : h0 / 2, wo_lo = s == 1 ? w0 - 1 : w0 / 2;
  for (int i = threadIdx.x; i < 9 * d.CGB * 8; i += blockDim.x) {
    const int e = i % 8, c8 = (i / 8) % d.CGB, t = i / (8 * d.CGB);
    const int c = (cg0 + c8) * 8 + e;
    wl[i] = c < C ? to_f32(w[(size_t)c * 9 + t]) : 0.f;
  }
  {
    const int npix = d.PH * d.PW;
    const int dph = d.PPB / d.PW, dpw = d.PPB % d.PW;
    int ph = pl / d.PW, pw = pl % d.PW;
    for (int pix = pl; pix < npix; pix += d.PPB) {
      const int ho = ho_lo + ph, wo = wo_lo + pw;
      float val[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      if (ho >= 0 && ho < g.Hout && wo >= 0 && wo < g.Wout && gcg < cgs)
        load8(dz + (((size_t)n * g.Hout + ho) * g.Wout + wo) * C + gcg * 8, val);
      store8(patch + ((size_t)pix * d.CGB + cg) * 8, val);
      ph += dph; pw += dpw;
      if (pw >= d.PW) { pw -= d.PW; ++ph; }
    }
  }
  __syncthreads();
  if (gcg >= cgs) return;
  const int dhl = d.PPB / d.TW, dwl = d.PPB % d.TW;
  int hl = pl / d.TW, wl_ = pl % d.TW;
  for (int p = pl; p < d.TH * d.TW; p += d.PPB, hl += dhl, wl_ += dwl) {
    if (wl_ >= d.TW) { wl_ -= d.TW; ++hl; }
    const int h = h0 + hl, ww = w0 + wl_;
    if (h >= g.Hin || ww >= g.Win) continue;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int hn = h + 1 - i;
      if (hn < 0 || (s == 2 && (hn & 1))) continue;
      const int ho = hn / s;
      if (ho >= g.Hout) continue;
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        const int wn = ww + 1 - j;
        if (wn < 0 || (s == 2 && (wn & 1))) continue;
        const int wo = wn / s;
        if (wo >= g.Wout) continue;
        float v[8], wr[8];
        load8(patch + ((size_t)((ho - ho_lo) * d.PW + (wo - wo_lo)) * d.CGB + cg) * 8, v);
        load8(wl + ((i * 3 + j) * d.CGB + cg) * 8, wr);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf(v[e], wr[e], acc[e]);
      }
    }
    store8(dIn + (((size_t)n * g.Hin + h) * g.Win + ww) * C + gcg * 8, acc);
  }
}

void dw_dgrad(int dt, hipStream_t st, const void* dz, const void* w, const ConvGeom& g, void* dIn) {
  const int es = dt == 0 ? 4 : 2;
  // tiles are in input resolution; for stride 2 an 8x8 input tile needs a 5x5 dz patch
  ConvGeom gi = g;
  gi.stride = 1;
  DwPlan d = dw_plan(gi, es, g.Hin, g.Win, 1 << 30);
  if (g.stride == 1) { d.PH = d.TH + 2; d.PW = d.TW + 2; }
  else { d.PH = d.TH / 2 + 2; d.PW = d.TW / 2 + 2; }
  size_t total = (size_t)g.N * g.Hin * g.Win;
  KScope ks(st, "dw_dgrad", ((double)total * g.Cout + (double)g.N * g.Hout * g.Wout * g.Cout) * es, 18.0 * g.N * g.Hout * g.Wout * g.Cout,
            (long)total, g.Cout, g.stride);
  size_t lds = (size_t)d.PH * d.PW * d.CGB * 8 * 4 + (size_t)9 * d.CGB * 8 * 4;
  FTP_DISPATCH(dt, hipLaunchKernelGGL(dw_dgrad_k<T>, dim3(d.ntiles, d.nslab), dim3(d.CGB * d.PPB), lds, st, (const T*)dz,
                                      (const T*)w, g, d, (T*)dIn));
}

// dW[c][tap] += sum over pixels dz[p][c] * in[p*s + tap][c]: input patch and dz tile in LDS, thread =
// (column group, tap, pixel part); the block's sums over all its tiles leave as one partial ws[block][9][C]
template <typename T>
__global__ __launch_bounds__(256) void dw_wgrad_k(const T* __restrict__ dz, View in, ConvGeom g, DwPlan d, int parts, float* __restrict__ ws) {
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  const int C = g.Cout, cgs = C / 8, s = g.stride;
  const int PH = (d.TH - 1) * s + 3, PW = (d.TW - 1) * s + 3;
  const size_t psz = (size_t)PH * PW * d.CGB * 8, tsz = (size_t)d.TH * d.TW * d.CGB * 8;
  const int cg0 = blockIdx.y * d.CGB;
  // accumulate role: cg fastest, then tap, then part
  const int acg = threadIdx.x % d.CGB, atap = (threadIdx.x / d.CGB) % 9, apart = threadIdx.x / (d.CGB * 9);
  const bool worker = apart < parts && cg0 + acg < cgs;
  const int ti = atap / 3, tj = atap % 3;
  View none{nullptr, nullptr, nullptr, 0};
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  PatchLoader<T, true, kDwPatchNV> lp;
  PatchLoader<T, false, kDwTileNV> lt;
  const T* src = reinterpret_cast<const T*>(in.z);
  int it = 0;
  if ((int)blockIdx.x < d.ntiles) {
    const int tile = blockIdx.x;
    const int tw = tile % d.tiles_w, th = (tile / d.tiles_w) % d.tiles_h, n = tile / (d.tiles_w * d.tiles_h);
    lp.fetch(src, n, th * d.TH * s - 1, tw * d.TW * s - 1, PH, PW, g.Hin, g.Win, C, cg0, d.CGB);
    lt.fetch(dz, n, th * d.TH, tw * d.TW, d.TH, d.TW, g.Hout, g.Wout, C, cg0, d.CGB);
  }
  for (int tile = blockIdx.x; tile < d.ntiles; tile += gridDim.x, ++it) {
    float* patch = reinterpret_cast<float*>(smem_raw);
    float* dzt = patch + psz;
    __syncthreads();                                       // the previous tile has been consumed
    lp.commit(patch, in, PH, PW, cg0, d.CGB);
    lt.commit(dzt, none, d.TH, d.TW, cg0, d.CGB);          // zero outside the image
    __syncthreads();
    const int nt = tile + gridDim.x;
    if (nt < d.ntiles) {
      const int tw2 = nt % d.tiles_w, th2 = (nt / d.tiles_w) % d.tiles_h, n2 = nt / (d.tiles_w * d.tiles_h);
      lp.fetch(src, n2, th2 * d.TH * s - 1, tw2 * d.TW * s - 1, PH, PW, g.Hin, g.Win, C, cg0, d.CGB);
      lt.fetch(dz, n2, th2 * d.TH, tw2 * d.TW, d.TH, d.TW, g.Hout, g.Wout, C, cg0, d.CGB);
    }
    if (!worker) continue;
    for (int p = apart; p < d.TH * d.TW; p += parts) {
      const int hl = p / d.TW, wl = p % d.TW;
      float dv[8], v[8];
      load8(dzt + ((size_t)p * d.CGB + acg) * 8, dv);
      load8(patch + ((size_t)((hl * s + ti) * PW + wl * s + tj) * d.CGB + acg) * 8, v);
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] = fmaf(dv[e], v[e], acc[e]);
    }
  }
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem_raw);          // [parts][9][CGB][8]
  if (apart < parts) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[((apart * 9 + atap) * d.CGB + acg) * 8 + e] = worker ? acc[e] : 0.f;
  }
  __syncthreads();
  if (apart == 0 && cg0 + acg < cgs) {
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float t = 0.f;
      for (int r = 0; r < parts; ++r) t += red[((r * 9 + atap) * d.CGB + acg) * 8 + e];
      o[e] = t;
    }
    store8(ws + ((size_t)blockIdx.x * 9 + atap) * C + (cg0 + acg) * 8, o);
  }
}

static DwPlan dw_wgrad_plan(const ConvGeom& g, int es, int* parts, size_t* lds) {
  DwPlan d = dw_plan(g, es, g.Hout, g.Wout, kMaxPartials);
  *parts = 256 / (d.CGB * 9);
  int PH = (d.TH - 1) * g.stride + 3, PW = (d.TW - 1) * g.stride + 3;
  size_t a = ((size_t)PH * PW + (size_t)d.TH * d.TW) * d.CGB * 8 * 4;   // float tiles
  size_t b = (size_t)*parts * 9 * d.CGB * 8 * 4;
  *lds = a > b ? a : b;
  return d;
}

size_t dw_wgrad_ws(const ConvGeom& g) { return (size_t)kMaxPartials * 9 * g.Cout; }


void dw_wgrad(int dt, hipStream_t st, const void* dz, HView in, const ConvGeom& g, float* ws, float* g_w) {
  const int es = dt == 0 ? 4 : 2;
  int parts; size_t lds;
  DwPlan d = dw_wgrad_plan(g, es, &parts, &lds);
  View v{in.z, in.scale, in.shift, in.act};
  {
    KScope ks(st, "dw_wgrad", ((double)g.N * g.Hin * g.Win * g.Cout + (double)g.N * g.Hout * g.Wout * g.Cout) * es + (double)d.nblocks * 9 * g.Cout * 4,
              18.0 * g.N * g.Hout * g.Wout * g.Cout, (long)g.N * g.Hout * g.Wout, g.Cout, g.stride);
    FTP_DISPATCH(dt, hipLaunchKernelGGL(dw_wgrad_k<T>, dim3(d.nblocks, d.nslab), dim3(256), lds, st, (const T*)dz, v, g, d, parts, ws));
  }
  reduce_partials(st, ws, d.nblocks, (size_t)9 * g.Cout, g.Cout, 1, 9, g_w);
}

}  // namespace ftp
