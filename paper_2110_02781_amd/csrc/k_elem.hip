// BatchNorm statistics / apply / backward, pooling, softmax cross-entropy,
// SGD-momentum and small utility kernels.  All are HBM-bound streaming kernels:
// each thread moves 8 consecutive channels (16 or 32 bytes) per access, rows
// are walked so that a block touches contiguous memory, and per-channel sums
// are reduced in a fixed order (per thread -> LDS across the block -> float64
// across blocks), so results are run-to-run deterministic.  Short tensors (at most
// 2048 rows) use one-launch variants in which a block owns 4 channels over all rows.
#include "dev_common.h"
#include "kernels.h"
#include "bn_pending.h"

namespace ftp {

#define FTP_DISPATCH(dt, ...)                   \
  do {                                          \
    if ((dt) == 0) { typedef float T; __VA_ARGS__; } \
    else { typedef bf16_t T; __VA_ARGS__; }     \
  } while (0)

static RowTile rowtile_with(size_t M, int CG, int nslab, int max_partials) {
  RowTile t;
  t.nslab = nslab;
  t.W = (CG + t.nslab - 1) / t.nslab;
  t.R = 256 / t.W;
  if (t.R < 1) t.R = 1;
  size_t want = (M + max_partials - 1) / max_partials;        // rows per block so that P <= max
  size_t rpb = ((want + t.R - 1) / t.R) * t.R;
  size_t min_rpb = (size_t)t.R * 4;                            // at least 4 iterations per block
  if (min_rpb < (size_t)kBnMinRows) min_rpb = ((kBnMinRows + t.R - 1) / t.R) * t.R;
  if (rpb < min_rpb) rpb = min_rpb;
  t.rows_per_block = rpb;
  t.P = (int)((M + rpb - 1) / rpb);
  if (t.P < 1) t.P = 1;
  return t;
}

RowTile make_rowtile(size_t M, int C, int max_partials) {
  const int CG = C / 8;
  RowTile t = rowtile_with(M, CG, (CG + 255) / 256, max_partials);
  // Few rows and many channels (6 K x 1344): the rows alone give too few blocks for 256 CUs, so the channels are cut
  // into slabs as well, down to 8 column groups (one 128-byte line per row and slab), until there are about 1024 blocks.
  // Only where the ROWS are what limits the blocks (P stopped by the minimum rows per block, not by max_partials).
  while (t.P < 256 && t.P < max_partials / 2 && (size_t)t.P * t.nslab < 1024 && (CG + t.nslab) / (t.nslab + 1) >= 8)
    t = rowtile_with(M, CG, t.nslab + 1, max_partials);
  return t;
}

// Column sums of a block: v[0..16) of thread (tx = column group, ty = row lane) are 8 sums and 8 second
// sums for channels cg*8..+7.  They go through LDS; then every (value, column group) pair gets its own
// thread, which adds the R row lanes in order and stores straight into partial[2][C] (the serial tail of
// one thread per column group doing all 16 values cost more than the streaming loop for short blocks).
__device__ __forceinline__ void reduce_rows_to_partial(const float (&v)[16], int tx, int ty, int W, int R, int cg0, int C,
                                                       float* smem, float* __restrict__ partial) {
#pragma unroll
  for (int e = 0; e < 16; ++e) smem[(e * R + ty) * W + tx] = v[e];
  __syncthreads();
  for (int i = threadIdx.x; i < 16 * W; i += blockDim.x) {
    const int e = i / W, x = i - e * W;
    if ((cg0 + x) * 8 >= C) continue;
    float s = 0.f;
    for (int r = 0; r < R; ++r) s += smem[(e * R + r) * W + x];
    partial[(size_t)(e >> 3) * C + (cg0 + x) * 8 + (e & 7)] = s;
  }
}

// ------------------------------------------------------------------ bn_stats
template <typename T>
__global__ void bn_stats_k(const T* __restrict__ z, size_t M, int C, int W, int R, size_t rpb,
                           float* __restrict__ partial) {
  extern __shared__ float smem[];
  int tx = threadIdx.x % W, ty = threadIdx.x / W;
  int cg = blockIdx.y * W + tx;
  float acc[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  if (cg < C / 8) {
    size_t m0 = (size_t)blockIdx.x * rpb, m1 = m0 + rpb < M ? m0 + rpb : M;
    // four rows per round: the loads are issued together, the sums keep a fixed order
    for (size_t m = m0 + ty; m < m1; m += 4 * (size_t)R) {
      Raw<T> rv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (m + (size_t)u * R < m1) raw_load(rv[u], z + (m + (size_t)u * R) * C + cg * 8);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (m + (size_t)u * R >= m1) break;
        float v[8];
        raw_unpack(rv[u], v);
#pragma unroll
        for (int e = 0; e < 8; ++e) { acc[e] += v[e]; acc[8 + e] = fmaf(v[e], v[e], acc[8 + e]); }
      }
    }
  }
  reduce_rows_to_partial(acc, tx, ty, W, R, blockIdx.y * W, C, smem, partial + (size_t)blockIdx.x * 2 * C);
}

void bn_stats(int dt, hipStream_t st, const void* z, size_t M, int C, float* partial, int* P_out) {
  RowTile t = make_rowtile(M, C, kBnPartials);
  {
    KScope ks(st, "bn_stats", (double)M * C * (dt == 0 ? 4.0 : 2.0), 3.0 * M * C);
    dim3 grid(t.P, t.nslab), block(t.W * t.R);
    size_t sm = (size_t)16 * t.R * t.W * sizeof(float);
    FTP_DISPATCH(dt, hipLaunchKernelGGL(bn_stats_k<T>, grid, block, sm, st, (const T*)z, M, C, t.W, t.R,
                                        t.rows_per_block, partial));
  }
  *P_out = t.P;
}

// Sum partial[p][q][c] over p in float64; kFinCh channels per block, kFinLanes lanes per channel
// (few channels per block: a layer has only C / kFinCh blocks and the partial walk is pure latency).
enum { kFinCh = 8, kFinLanes = 256 / kFinCh };
template <int Q>
__device__ __forceinline__ void sum_partials(const float* __restrict__ partial, int P, int C, int c,
                                             int lane, double (&out)[Q], double* smem) {
  double s[Q];
#pragma unroll
  for (int q = 0; q < Q; ++q) s[q] = 0.0;
  if (c < C) {
    // sixteen partials per round (all of them, for up to 512 partials): the loads are independent and unconditional
    // (past the end: the round's first partial again, not added), the sums keep their order; a round costs one trip to
    // memory, and this kernel is nothing but such trips
    constexpr int U = 16;
    for (int p = lane; p < P; p += U * kFinLanes) {
      float v[U][Q];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int pp = p + kFinLanes * u < P ? p + kFinLanes * u : p;
#pragma unroll
        for (int q = 0; q < Q; ++q) v[u][q] = partial[((size_t)pp * Q + q) * C + c];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (p + kFinLanes * u < P) {
#pragma unroll
          for (int q = 0; q < Q; ++q) s[q] += (double)v[u][q];
        }
      }
    }
  }
  int cl = threadIdx.x % kFinCh;
#pragma unroll
  for (int q = 0; q < Q; ++q) smem[(q * kFinLanes + lane) * kFinCh + cl] = s[q];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < Q; ++q) {
    // four chains of eight in a fixed order instead of one of thirty-two dependent float64 additions
    double t[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int l = 0; l < kFinLanes; ++l) t[l & 3] += smem[(q * kFinLanes + l) * kFinCh + cl];
    out[q] = (t[0] + t[1]) + (t[2] + t[3]);
  }
}

__global__ void bn_finalize_k(const float* __restrict__ partial, int P, size_t M, int C,
                              const float* __restrict__ gamma, const float* __restrict__ beta,
                              float* mean, float* invstd, float* scale, float* shift, float* run_mean,
                              float* run_var, float eps, float momentum) {
  __shared__ double smem[2 * kFinLanes * kFinCh];
  int cl = threadIdx.x % kFinCh, lane = threadIdx.x / kFinCh;
  int c = xcd_logical_block() * kFinCh + cl;     // neighbours read the same lines of the partials: one L2
  double s[2];
  sum_partials<2>(partial, P, C, c, lane, s, smem);
  if (lane == 0 && c < C) {
    double mu = s[0] / (double)M;
    double var = s[1] / (double)M - mu * mu;
    if (var < 0.0) var = 0.0;
    double is = 1.0 / sqrt(var + (double)eps);
    float sc = (float)((double)gamma[c] * is);
    mean[c] = (float)mu;
    invstd[c] = (float)is;
    scale[c] = sc;
    shift[c] = (float)((double)beta[c] - mu * (double)sc);
    double unb = M > 1 ? var * ((double)M / (double)(M - 1)) : var;
    run_mean[c] = (float)((1.0 - momentum) * run_mean[c] + momentum * mu);
    run_var[c] = (float)((1.0 - momentum) * run_var[c] + momentum * unb);
  }
}

void bn_finalize(hipStream_t st, const float* partial, int P, size_t M, int C, const float* gamma,
                 const float* beta, float* mean, float* invstd, float* scale, float* shift,
                 float* run_mean, float* run_var, float eps, float momentum) {
  KScope ks(st, "bn_finalize", (double)P * 2 * C * 4 + 8.0 * C * 4, 0);
  hipLaunchKernelGGL(bn_finalize_k, dim3((C + kFinCh - 1) / kFinCh), dim3(256), 0, st, partial, P, M, C, gamma, beta,
                     mean, invstd, scale, shift, run_mean, run_var, eps, momentum);
}

// ------------------------------------------------------------- bn backward
// dY = dA where the activation (compile-time ACT) passes, else 0
template <int ACT>
__device__ __forceinline__ float act_gate(float d, float z, float sc, float sh) {
  if (ACT == ACT_NONE) return d;
  const float y = fmaf(z, sc, sh);
  if (ACT == ACT_RELU) return y > 0.f ? d : 0.f;
  return (y > 0.f && y < 6.f) ? d : 0.f;
}

#define FTP_DISPATCH_ACT(dt, act, ...)                                        \
  do {                                                                        \
    if ((act) == ACT_NONE) { constexpr int ACT = ACT_NONE; FTP_DISPATCH(dt, __VA_ARGS__); }        \
    else if ((act) == ACT_RELU) { constexpr int ACT = ACT_RELU; FTP_DISPATCH(dt, __VA_ARGS__); }   \
    else { constexpr int ACT = ACT_RELU6; FTP_DISPATCH(dt, __VA_ARGS__); }    \
  } while (0)

template <typename T, int ACT>
__global__ void bn_bwd_reduce_k(const T* __restrict__ dA, const T* __restrict__ z, size_t M, int C,
                                const float* __restrict__ scale, const float* __restrict__ shift,
                                int W, int R, size_t rpb, float* __restrict__ partial) {
  extern __shared__ float smem[];
  __builtin_amdgcn_s_setprio(3);     // data-gradient chain: ahead of the weight-gradient stream's waves on a shared SIMD
  int tx = threadIdx.x % W, ty = threadIdx.x / W;
  int cg = blockIdx.y * W + tx;
  float acc[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  if (cg < C / 8) {
    float sc[8], sh[8];
    load8(scale + cg * 8, sc);
    load8(shift + cg * 8, sh);
    size_t m0 = (size_t)blockIdx.x * rpb, m1 = m0 + rpb < M ? m0 + rpb : M;
    // four rows per round: the loads are issued together, the sums keep a fixed order
    for (size_t m = m0 + ty; m < m1; m += 4 * (size_t)R) {
      Raw<T> rd[4], rv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (m + (size_t)u * R < m1) {
          raw_load(rd[u], dA + (m + (size_t)u * R) * C + cg * 8);
          raw_load(rv[u], z + (m + (size_t)u * R) * C + cg * 8);
        }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (m + (size_t)u * R >= m1) break;
        float d[8], v[8];
        raw_unpack(rd[u], d);
        raw_unpack(rv[u], v);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float dy = act_gate<ACT>(d[e], v[e], sc[e], sh[e]);
          acc[e] += dy;
          acc[8 + e] = fmaf(dy, v[e], acc[8 + e]);
        }
      }
    }
  }
  reduce_rows_to_partial(acc, tx, ty, W, R, blockIdx.y * W, C, smem, partial + (size_t)blockIdx.x * 2 * C);
}

void bn_bwd_reduce(int dt, hipStream_t st, const void* dA, const void* z, size_t M, int C,
                   const float* scale, const float* shift, int act, float* partial, int* P_out) {
  RowTile t = make_rowtile(M, C, kBnPartials);
  {
    KScope ks(st, "bn_bwd_reduce", 2.0 * M * C * (dt == 0 ? 4.0 : 2.0), 6.0 * M * C, (long)M, C, act);
    dim3 grid(t.P, t.nslab), block(t.W * t.R);
    size_t sm = (size_t)16 * t.R * t.W * sizeof(float);
    FTP_DISPATCH_ACT(dt, act, hipLaunchKernelGGL((bn_bwd_reduce_k<T, ACT>), grid, block, sm, st, (const T*)dA, (const T*)z, M,
                                                 C, scale, shift, t.W, t.R, t.rows_per_block, partial));
  }
  *P_out = t.P;
}

__global__ void bn_bwd_finalize_k(const float* __restrict__ partial, int P, size_t M, int C,
                                  const float* __restrict__ gamma, const float* __restrict__ mean,
                                  const float* __restrict__ invstd, float* g_gamma, float* g_beta,
                                  float* coef) {
  __shared__ double smem[2 * kFinLanes * kFinCh];
  // data-gradient chain.  Without this its few waves are the youngest on SIMDs that the weight-gradient stream's
  // long-running waves keep busy, and issue goes to the oldest wave first: measured 190 us instead of 5 next to a
  // persistent depthwise weight-gradient kernel
  __builtin_amdgcn_s_setprio(3);
  int cl = threadIdx.x % kFinCh, lane = threadIdx.x / kFinCh;
  int c = xcd_logical_block() * kFinCh + cl;     // neighbours read the same lines of the partials: one L2
  double s[2];
  sum_partials<2>(partial, P, C, c, lane, s, smem);
  if (lane == 0 && c < C) {
    double mu = mean[c], is = invstd[c], g = gamma[c];
    double dbeta = s[0];
    double dgamma = is * (s[1] - mu * s[0]);
    g_gamma[c] += (float)dgamma;
    g_beta[c] += (float)dbeta;
    double k1 = g * is;
    double k2 = -k1 * is * dgamma / (double)M;
    double k3 = -k1 * dbeta / (double)M - k2 * mu;
    coef[c] = (float)k1;
    coef[C + c] = (float)k2;
    coef[2 * C + c] = (float)k3;
  }
}

void bn_bwd_finalize(hipStream_t st, const float* partial, int P, size_t M, int C, const float* gamma,
                     const float* mean, const float* invstd, float* g_gamma, float* g_beta, float* coef) {
  KScope ks(st, "bn_bwd_finalize", (double)P * 2 * C * 4 + 10.0 * C * 4, 0);
  hipLaunchKernelGGL(bn_bwd_finalize_k, dim3((C + kFinCh - 1) / kFinCh), dim3(256), 0, st, partial, P, M, C, gamma, mean,
                     invstd, g_gamma, g_beta, coef);
}

// thread = (column group, row lane): coefficients stay in registers, rows advance by R
template <typename T, int ACT>
__global__ void bn_bwd_apply_k(const T* __restrict__ dA, const T* __restrict__ z, size_t M, int C,
                               const float* __restrict__ scale, const float* __restrict__ shift,
                               const float* __restrict__ coef, int W, int R, size_t rpb, T* __restrict__ dz) {
  __builtin_amdgcn_s_setprio(3);     // data-gradient chain: ahead of the weight-gradient stream's waves on a shared SIMD
  const int tx = threadIdx.x % W, ty = threadIdx.x / W;
  const int cg = blockIdx.y * W + tx;
  if (cg >= C / 8) return;
  const int c = cg * 8;
  float sc[8], sh[8], k1[8], k2[8], k3[8];
  if (ACT != ACT_NONE) { load8(scale + c, sc); load8(shift + c, sh); }
  load8(coef + c, k1); load8(coef + C + c, k2); load8(coef + 2 * C + c, k3);
  const size_t m0 = (size_t)blockIdx.x * rpb, m1 = m0 + rpb < M ? m0 + rpb : M;
  for (size_t m = m0 + ty; m < m1; m += 2 * (size_t)R) {
    Raw<T> rd[2], rv[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
      if (m + (size_t)u * R < m1) {
        raw_load(rd[u], dA + (m + (size_t)u * R) * C + c);
        raw_load(rv[u], z + (m + (size_t)u * R) * C + c);
      }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (m + (size_t)u * R >= m1) break;
      float d[8], v[8], o[8];
      raw_unpack(rd[u], d);
      raw_unpack(rv[u], v);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float dy = act_gate<ACT>(d[e], v[e], sc[e], sh[e]);
        o[e] = fmaf(k1[e], dy, fmaf(k2[e], v[e], k3[e]));
      }
      store8(dz + (m + (size_t)u * R) * C + c, o);
    }
  }
}

static inline int flat_grid(size_t n, int block) {
  size_t g = (n + block - 1) / block;
  if (g > 65536) g = 65536;
  if (g < 1) g = 1;
  return (int)g;
}

void bn_bwd_apply(int dt, hipStream_t st, const void* dA, const void* z, size_t M, int C,
                  const float* scale, const float* shift, int act, const float* coef, void* dz) {
  KScope ks(st, "bn_bwd_apply", 3.0 * M * C * (dt == 0 ? 4.0 : 2.0), 6.0 * M * C, (long)M, C, act);
  RowTile t = make_rowtile(M, C, 1 << 14);       // no partials here: many short blocks
  dim3 grid(t.P, t.nslab), block(t.W * t.R);
  FTP_DISPATCH_ACT(dt, act, hipLaunchKernelGGL((bn_bwd_apply_k<T, ACT>), grid, block, 0, st, (const T*)dA, (const T*)z, M, C,
                                               scale, shift, coef, t.W, t.R, t.rows_per_block, (T*)dz));
}

// BatchNorm backward for short tensors in ONE launch: a block owns 4 channels over all M rows, so it
// can reduce, finalize and apply without any other block (the three-kernel path needs two grid-wide
// dependencies, i.e. two extra launches, which dominate when the tensor is a few hundred KB).
// Every thread keeps its rows in registers: one trip to memory, then reduce, then apply.
template <typename T, int RPT>
__global__ __launch_bounds__(1024) void bn_bwd_small_k(const T* __restrict__ dA, const T* __restrict__ z, size_t M, int C,
                                                       const float* __restrict__ scale, const float* __restrict__ shift, int act,
                                                       const float* __restrict__ gamma, const float* __restrict__ mean,
                                                       const float* __restrict__ invstd, float* g_gamma, float* g_beta,
                                                       T* __restrict__ dz) {
  __builtin_amdgcn_s_setprio(3);     // data-gradient chain: ahead of the weight-gradient stream's waves on a shared SIMD
  __shared__ float red[16][8];    // [wave][value]
  __shared__ float coef[3][4];
  const int c0 = xcd_logical_block() * 4, tid = threadIdx.x, nt = blockDim.x;   // RPT * nt >= M; neighbours share an XCD
  // requested with the rows: what the four finishing threads need after the reduction
  float f_mu = 0.f, f_is = 0.f, f_g = 0.f, f_gg = 0.f, f_gb = 0.f;
  if (tid < 4) { f_mu = mean[c0 + tid]; f_is = invstd[c0 + tid]; f_g = gamma[c0 + tid]; f_gg = g_gamma[c0 + tid]; f_gb = g_beta[c0 + tid]; }
  float4 d[RPT], v[RPT];
#pragma unroll
  for (int q = 0; q < RPT; ++q) {       // unconditional, from a clamped row: rows past M are masked where they are used
    const size_t m = tid + (size_t)q * nt, mc = m < M ? m : 0;
    d[q] = load4(dA + mc * C + c0);
    v[q] = load4(z + mc * C + c0);
  }
  float sc[4], sh[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) { sc[e] = scale[c0 + e]; sh[e] = shift[c0 + e]; }
  const float lo = act_lo(act), hi = act_hi(act);
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int q = 0; q < RPT; ++q) {
    const float y0 = fmaf(v[q].x, sc[0], sh[0]), y1 = fmaf(v[q].y, sc[1], sh[1]), y2 = fmaf(v[q].z, sc[2], sh[2]),
                y3 = fmaf(v[q].w, sc[3], sh[3]);
    const bool live = tid + (size_t)q * nt < M;
    float4 dy;                              // rows past M count as zeros
    dy.x = (live && y0 > lo && y0 < hi) ? d[q].x : 0.f;
    dy.y = (live && y1 > lo && y1 < hi) ? d[q].y : 0.f;
    dy.z = (live && y2 > lo && y2 < hi) ? d[q].z : 0.f;
    dy.w = (live && y3 > lo && y3 < hi) ? d[q].w : 0.f;
    d[q] = dy;
    acc[0] += dy.x; acc[1] += dy.y; acc[2] += dy.z; acc[3] += dy.w;
    acc[4] = fmaf(dy.x, v[q].x, acc[4]); acc[5] = fmaf(dy.y, v[q].y, acc[5]);
    acc[6] = fmaf(dy.z, v[q].z, acc[6]); acc[7] = fmaf(dy.w, v[q].w, acc[7]);
  }
  // fixed-shape reduction: inside each wave, then the waves in order
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = wave_sum(acc[e]);
  const int wave = tid >> 6, nw = nt >> 6;
  if ((tid & 63) == 0) {
#pragma unroll
    for (int e = 0; e < 8; ++e) red[wave][e] = acc[e];
  }
  __syncthreads();
  // first use of the five values requested at the top: their conversions must not move up to the loads
  asm volatile("" : "+v"(f_mu), "+v"(f_is), "+v"(f_g), "+v"(f_gg), "+v"(f_gb));
  if (tid < 4) {
    const int c = c0 + tid;
    double s0 = 0.0, s1 = 0.0;
    for (int w = 0; w < nw; ++w) { s0 += red[w][tid]; s1 += red[w][4 + tid]; }
    const double mu = f_mu, is = f_is, g = f_g, Md = (double)M;
    const double dbeta = s0, dgamma = is * (s1 - mu * s0);
    g_gamma[c] = f_gg + (float)dgamma;
    g_beta[c] = f_gb + (float)dbeta;
    const double k1 = g * is, k2 = -k1 * is * dgamma / Md, k3 = -k1 * dbeta / Md - k2 * mu;
    coef[0][tid] = (float)k1; coef[1][tid] = (float)k2; coef[2][tid] = (float)k3;
  }
  __syncthreads();
  const float4 k1 = make_float4(coef[0][0], coef[0][1], coef[0][2], coef[0][3]);
  const float4 k2 = make_float4(coef[1][0], coef[1][1], coef[1][2], coef[1][3]);
  const float4 k3 = make_float4(coef[2][0], coef[2][1], coef[2][2], coef[2][3]);
#pragma unroll
  for (int q = 0; q < RPT; ++q) {
    const size_t m = tid + (size_t)q * nt;
    if (m >= M) continue;
    store4(dz + m * C + c0, fma4(k1, d[q], fma4(k2, v[q], k3)));
  }
}

int bn_bwd_small_ok(size_t M, int C) { return M <= 2048 && C >= 16 && C % 4 == 0; }

void bn_bwd_small(int dt, hipStream_t st, const void* dA, const void* z, size_t M, int C, const float* scale,
                  const float* shift, int act, const float* gamma, const float* mean, const float* invstd,
                  float* g_gamma, float* g_beta, void* dz) {
  KScope ks(st, "bn_bwd_small", 3.0 * M * C * (dt == 0 ? 4.0 : 2.0), 12.0 * M * C, (long)M, C);
  const int nt = M > 512 ? 1024 : (M > 256 ? 512 : 256);
  if (M > 1024) {
    FTP_DISPATCH(dt, hipLaunchKernelGGL((bn_bwd_small_k<T, 2>), dim3(C / 4), dim3(nt), 0, st, (const T*)dA, (const T*)z, M, C, scale,
                                        shift, act, gamma, mean, invstd, g_gamma, g_beta, (T*)dz));
  } else {
    FTP_DISPATCH(dt, hipLaunchKernelGGL((bn_bwd_small_k<T, 1>), dim3(C / 4), dim3(nt), 0, st, (const T*)dA, (const T*)z, M, C, scale,
                                        shift, act, gamma, mean, invstd, g_gamma, g_beta, (T*)dz));
  }
}

template <typename T>
__global__ void bn_apply_k(View in, size_t nvec, int CG, const T* __restrict__ res, T* __restrict__ out) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (size_t)gridDim.x * blockDim.x) {
    int c = (int)(i % CG) * 8;
    float v[8];
    view_load8<T>(in, i * 8, c, v);
    if (res) {
      float r[8];
      load8(res + i * 8, r);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += r[e];
    }
    store8(out + i * 8, v);
  }
}

void bn_apply(int dt, hipStream_t st, HView in, size_t M, int C, const void* res, void* out) {
  size_t nvec = M * (size_t)(C / 8);
  KScope ks(st, "bn_apply", (res ? 3.0 : 2.0) * M * C * (dt == 0 ? 4.0 : 2.0), 3.0 * M * C);
  View v{in.z, in.scale, in.shift, in.act};
  FTP_DISPATCH(dt, hipLaunchKernelGGL(bn_apply_k<T>, dim3(flat_grid(nvec, 256)), dim3(256), 0, st, v, nvec,
                                      C / 8, (const T*)res, (T*)out));
}

// Finish a BatchNorm whose statistics are still partial sums and materialise its output (+ residual) in ONE
// launch, for short tensors: a block owns 4 channels over all rows.
template <typename T>
__global__ __launch_bounds__(1024) void bn_finalize_apply_small_k(BnPending pend, const T* __restrict__ z, size_t M, int C, int act,
                                                                  float eps, float momentum, const T* __restrict__ res,
                                                                  T* __restrict__ out) {
  __shared__ double pre[32][8];
  __shared__ float insc[2][4];
  const int c0 = xcd_logical_block() * 4, tid = threadIdx.x, nt = blockDim.x;
  // the rows of this thread (at most two: M <= 2048 with 1024 threads, else one) and their residuals are requested
  // before the statistics are finished, so the two round trips overlap
  float4 zv[2], rv[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const size_t m = (size_t)tid + (size_t)q * nt, mc = m < M ? m : 0;
    zv[q] = load4(z + mc * C + c0);
    rv[q] = load4((res ? res : z) + mc * C + c0);      // unconditional: without a residual the row itself, not used
  }
  finish_pending4(pend, C, c0, eps, momentum, pre, insc);
  float sc[4], sh[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) { sc[e] = insc[0][e]; sh[e] = insc[1][e]; }
  const float lo = act_lo(act), hi = act_hi(act);
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const size_t m = (size_t)tid + (size_t)q * nt;
    if (m >= M) break;
    float4 v = zv[q];
    v.x = round_to<T>(clamp_act(fmaf(v.x, sc[0], sh[0]), lo, hi));
    v.y = round_to<T>(clamp_act(fmaf(v.y, sc[1], sh[1]), lo, hi));
    v.z = round_to<T>(clamp_act(fmaf(v.z, sc[2], sh[2]), lo, hi));
    v.w = round_to<T>(clamp_act(fmaf(v.w, sc[3], sh[3]), lo, hi));
    if (res) { v.x += rv[q].x; v.y += rv[q].y; v.z += rv[q].z; v.w += rv[q].w; }
    store4(out + m * C + c0, v);
  }
}

int bn_finalize_apply_small_ok(size_t M, int C) { return M <= 2048 && C % 4 == 0; }

void bn_finalize_apply_small(int dt, hipStream_t st, const BnPending& pend, const void* z, size_t M, int C, int act, float eps,
                             float momentum, const void* res, void* out) {
  KScope ks(st, "bn_fin_apply_small", (res ? 3.0 : 2.0) * M * C * (dt == 0 ? 4.0 : 2.0) + (double)pend.P * 2 * C * 4, 3.0 * M * C);
  const int nt = M > 512 ? 1024 : (M > 256 ? 512 : 256);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(bn_finalize_apply_small_k<T>, dim3(C / 4), dim3(nt), 0, st, pend, (const T*)z, M, C, act, eps,
                                      momentum, (const T*)res, (T*)out));
}

// ------------------------------------------------------------------ pooling
// block = (image n, group of 8 channels); 64 lanes walk the positions, fixed-order sum through LDS
template <typename T>
__global__ __launch_bounds__(64) void gap_fwd_k(View in, int N, int HW, int CG, T* __restrict__ out) {
  __shared__ float red[64][8];
  const int i = blockIdx.x, n = i / CG, cg = i % CG, lane = threadIdx.x;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int p = lane; p < HW; p += 64) {
    float v[8];
    view_load8<T>(in, ((size_t)n * HW + p) * CG * 8 + cg * 8, cg * 8, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += v[e];
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[lane][e] = acc[e];
  __syncthreads();
  if (lane < 8) {
    float s = 0.f;
    for (int l = 0; l < 64; ++l) s += red[l][lane];
    float o = s * (1.f / (float)HW);
    out[(size_t)i * 8 + lane] = from_f32<T>(o);
  }
}

void gap_fwd(int dt, hipStream_t st, HView in, int N, int HW, int C, void* out) {
  View v{in.z, in.scale, in.shift, in.act};
  int n = N * (C / 8);
  KScope ks(st, "gap_fwd", ((double)N * HW * C + (double)N * C) * (dt == 0 ? 4.0 : 2.0), 3.0 * N * HW * C);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(gap_fwd_k<T>, dim3(n), dim3(64), 0, st, v, N, HW, C / 8, (T*)out));
}

template <typename T>
__global__ void gap_bwd_k(const T* __restrict__ dOut, size_t nvec, int HW, int CG, T* __restrict__ dIn) {
  float inv = 1.f / (float)HW;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (size_t)gridDim.x * blockDim.x) {
    size_t n = i / ((size_t)HW * CG);
    int cg = (int)(i % CG);
    float v[8];
    load8(dOut + (n * CG + cg) * 8, v);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= inv;
    store8(dIn + i * 8, v);
  }
}

void gap_bwd(int dt, hipStream_t st, const void* dOut, int N, int HW, int C, void* dIn) {
  size_t nvec = (size_t)N * HW * (C / 8);
  KScope ks(st, "gap_bwd", ((double)N * HW * C + (double)N * C) * (dt == 0 ? 4.0 : 2.0), 1.0 * N * HW * C);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(gap_bwd_k<T>, dim3(flat_grid(nvec, 256)), dim3(256), 0, st,
                                      (const T*)dOut, nvec, HW, C / 8, (T*)dIn));
}

// ----------------------------------------------------- softmax cross-entropy
__device__ __forceinline__ float block_reduce_256(float v, bool is_max, float* smem) {
  int tid = threadIdx.x;
  smem[tid] = v;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) smem[tid] = is_max ? fmaxf(smem[tid], smem[tid + s]) : smem[tid] + smem[tid + s];
    __syncthreads();
  }
  float r = smem[0];
  __syncthreads();
  return r;
}

template <typename T>
__global__ void softmax_ce_k(const T* __restrict__ logits, const int32_t* __restrict__ labels, int B,
                             int classes, float* __restrict__ row_loss, T* __restrict__ dlogits) {
  __shared__ float smem[256];
  int b = blockIdx.x;
  const T* row = logits + (size_t)b * classes;
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < classes; j += 256) mx = fmaxf(mx, to_f32(row[j]));
  mx = block_reduce_256(mx, true, smem);
  float s = 0.f;
  for (int j = threadIdx.x; j < classes; j += 256) s += expf(to_f32(row[j]) - mx);
  s = block_reduce_256(s, false, smem);
  int lab = labels[b];
  const bool lab_ok = lab >= 0 && lab < classes;   // an invalid label yields a NaN loss, never a stray read
  float invB = 1.f / (float)B, invs = 1.f / s;
  for (int j = threadIdx.x; j < classes; j += 256) {
    float p = expf(to_f32(row[j]) - mx) * invs;
    dlogits[(size_t)b * classes + j] = from_f32<T>((p - (j == lab ? 1.f : 0.f)) * invB);
  }
  if (threadIdx.x == 0) row_loss[b] = lab_ok ? -(to_f32(row[lab]) - mx - logf(s)) : NAN;
}

__global__ void mean_rows_k(const float* __restrict__ row_loss, int B, float* __restrict__ loss) {
  __shared__ float smem[256];
  float s = 0.f;
  for (int i = threadIdx.x; i < B; i += 256) s += row_loss[i];
  s = block_reduce_256(s, false, smem);
  if (threadIdx.x == 0) *loss = s / (float)B;
}

void softmax_ce(int dt, hipStream_t st, const void* logits, const int32_t* labels, int B, int classes,
                float* row_loss, void* dlogits, float* loss) {
  KScope ks(st, "softmax_ce", 2.0 * B * classes * (dt == 0 ? 4.0 : 2.0), 8.0 * B * classes);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(softmax_ce_k<T>, dim3(B), dim3(256), 0, st, (const T*)logits, labels, B,
                                      classes, row_loss, (T*)dlogits));
  hipLaunchKernelGGL(mean_rows_k, dim3(1), dim3(256), 0, st, row_loss, B, loss);
}

// block = 16 output columns x 16 row lanes; the row lanes' sums meet in LDS in a fixed order
template <typename T>
__global__ __launch_bounds__(256) void bias_grad_k(const T* __restrict__ d, int B, int Nout, float* __restrict__ g) {
  __shared__ float red[16][17];
  const int jl = threadIdx.x & 15, lane = threadIdx.x >> 4;
  const int j = blockIdx.x * 16 + jl;
  float s = 0.f;
  if (j < Nout)
    for (int b = lane; b < B; b += 16) s += to_f32(d[(size_t)b * Nout + j]);
  red[lane][jl] = s;
  __syncthreads();
  if (lane == 0 && j < Nout) {
    float t = 0.f;
#pragma unroll
    for (int l = 0; l < 16; ++l) t += red[l][jl];
    g[j] += t;
  }
}

void bias_grad(int dt, hipStream_t st, const void* d, int B, int Nout, float* g_bias) {
  KScope ks(st, "bias_grad", (double)B * Nout * (dt == 0 ? 4.0 : 2.0) + 8.0 * Nout, 1.0 * B * Nout);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(bias_grad_k<T>, dim3((Nout + 15) / 16), dim3(256), 0, st, (const T*)d, B, Nout, g_bias));
}

// -------------------------------------------------------------------- SGD
__global__ void sgd_update_k(float* __restrict__ w, float* __restrict__ g, float* __restrict__ v,
                             bf16_t* __restrict__ w_lp, size_t n, float lr, float mu, float wd) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    float wi = w[i];
    float gi = fmaf(wd, wi, g[i]);
    float vi = fmaf(mu, v[i], gi);
    wi = fmaf(-lr, vi, wi);
    w[i] = wi;
    v[i] = vi;
    g[i] = 0.f;
    if (w_lp) w_lp[i] = f32_to_bf16(wi);
  }
}

void sgd_update(hipStream_t st, float* w, float* g, float* v, void* w_lp, size_t n, float lr, float mu,
                float wd) {
  KScope ks(st, "sgd_update", (w_lp ? 26.0 : 24.0) * n, 6.0 * n);
  hipLaunchKernelGGL(sgd_update_k, dim3(flat_grid(n, 256)), dim3(256), 0, st, w, g, v, (bf16_t*)w_lp, n, lr,
                     mu, wd);
}

// w[i] = (src[0][i] + src[1][i] + ... ) / n, summed in the order given; optional bfloat16 copy
__global__ void aggregate_k(float* __restrict__ w, bf16_t* __restrict__ w_lp, AggSources src, int n, size_t count) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) {
    float acc = src.p[0][i];
    for (int j = 1; j < n; ++j) acc += src.p[j][i];
    acc = acc / (float)n;
    w[i] = acc;
    if (w_lp) w_lp[i] = from_f32<bf16_t>(acc);
  }
}

void aggregate_weights(hipStream_t st, float* w, void* w_lp, const AggSources& src, int n, size_t count) {
  KScope ks(st, "aggregate", (double)count * (4.0 * (n + 1) + (w_lp ? 2.0 : 0.0)), (double)count * n);
  hipLaunchKernelGGL(aggregate_k, dim3(flat_grid(count, 256)), dim3(256), 0, st, w, (bf16_t*)w_lp, src, n, count);
}

__global__ void fill_zero_k(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0u;
}

void fill_zero(hipStream_t st, void* p, size_t bytes) {
  KScope ks(st, "fill_zero", (double)bytes, 0);
  size_t n = (bytes + 3) / 4;  // buffers are allocated in multiples of 256 bytes
  hipLaunchKernelGGL(fill_zero_k, dim3(flat_grid(n, 256)), dim3(256), 0, st, (uint32_t*)p, n);
}

// plain 16-byte-per-thread copy of known size: the yardstick hardware traffic counters are scaled by
__global__ void calibration_copy_k(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

void calibration_copy(hipStream_t st, const void* src, void* dst, size_t bytes) {
  size_t n = bytes / 16;
  KScope ks(st, "calibration_copy", 2.0 * n * 16, 0);
  hipLaunchKernelGGL(calibration_copy_k, dim3(flat_grid(n, 256)), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n);
}

template <typename T>
__global__ void f32_to_storage_k(const float* __restrict__ src, T* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = from_f32<T>(src[i]);
}

void f32_to_storage(int dt, hipStream_t st, const float* src, void* dst, size_t n) {
  KScope ks(st, "f32_to_storage", (4.0 + (dt == 0 ? 4.0 : 2.0)) * n, 0);
  FTP_DISPATCH(dt, hipLaunchKernelGGL(f32_to_storage_k<T>, dim3(flat_grid(n, 256)), dim3(256), 0, st, src,
                                      (T*)dst, n));
}

}  // namespace ftp
