// Backward of a narrow-to-wide pointwise layer (the expand layer of an inverted residual block: K input channels,
// N = t*K output channels) in ONE pass over its tensors, bfloat16.
//
// Layer by layer the backward of such a layer moves the wide [M][N] tensors seven times: the BatchNorm backward
// reads dA and z and writes dz, the data gradient reads dz, the weight gradient reads dz again.  Here a block takes
// 64 rows at a time, forms their dz = k1*dA*act'(scale*z+shift) + k2*z + k3 once, into LDS, and uses it from there
// for both products:
//     dIn[m][k]  = sum_n dz[m][n] * W[n][k]  (+ res[m][k])     reduction over the layer's own channels
//     dW[n][k]  += sum_m dz[m][n] * A[m][k]                    reduction over the rows
// so the wide tensors are read once (dA, z) and never written.  The second product needs both operands with the rows
// as the contiguous index of a lane's MFMA fragment while memory and LDS hold them channel-contiguous: the LDS
// transpose read of gfx950 (ds_read_b64_tr_b16: sixteen lanes hand in the addresses of sixteen 4-element rows and
// get the 16 x 4 block back transposed) delivers exactly that, without a repacking pass.  The weight-gradient sums
// of a block stay in its MFMA accumulators over all its row tiles; it leaves one fp32 partial [N][K].
// Only layers whose N x K accumulators fit the registers of a block take this path (N <= 320, K <= 48: the layers
// with the largest tensors); the rest keep the layer-by-layer kernels.
#include "dev_common.h"
#include "kernels.h"
#include "mfma_frag.h"

namespace ftp {

enum { kFusedBlocks = 256 };   // blocks: one per CU (two where the partials allow, or where 32-row tiles leave the registers for it)

struct FusedArgs {
  const bf16_t* dA;      // [M][N] gradient of the activated output
  const bf16_t* z;       // [M][N] raw convolution output
  const float* scale;    // [N] BatchNorm scale / shift of z (decide the activation's on / off)
  const float* shift;
  const float* coef;     // [3][N]: dz = k1 * dY + k2 * z + k3
  const bf16_t* w;       // [N][K]
  const bf16_t* a;       // [M][K] the layer's input as stored
  const bf16_t* res;     // [M][K] added to dIn, or nullptr
  bf16_t* dIn;           // [M][K]
  float* ws;             // [P][N][K] partial weight gradients
  size_t M;
  int K, N, NP, KP;      // NP, KP: N rounded up to 32, K rounded up to 16 (LDS tiles, zero padded)
  int ntiles;
};

// NTW: 16-wide tiles of N per wavefront (4 * NTW * 16 >= N), KT: 16-wide tiles of K; IT: passes of the elementwise
// stage (256 threads cover 256 / (N/8) rows per pass)
// ROWS: rows per tile, 64 or 32 (the wide layers: ten 16-byte vectors each of dA and z in flight per thread for a 64-row
// tile put the kernel above 256 registers, one block per CU; with 32 rows two blocks fit and hide each other's phases)
template <int ACT, int NTW, int KT, int IT, bool RES, int ROWS>
__global__ __launch_bounds__(256) void pw_bwd_fused_k(FusedArgs p) {
  constexpr int kFusedRows = ROWS;
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  __builtin_amdgcn_s_setprio(3);              // data-gradient chain
  const int LDN = p.NP + 8, LDK = p.KP + 8;
  bf16_t* sDz = reinterpret_cast<bf16_t*>(smem_raw);           // [64][LDN]
  bf16_t* sA = sDz + kFusedRows * LDN;                          // [64][LDK]
  bf16_t* sWt = sA + kFusedRows * LDK;                          // [KP][LDN]: W transposed
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l16 = lane & 15, G = lane >> 4;
  const int N = p.N, K = p.K;
  const int CG = N / 8, RP = 256 / CG;        // column groups, rows per elementwise pass
  const int cg = tid % CG, er = tid / CG;     // this thread's column group and first row
  const bool ew = er < RP;
  const int c = cg * 8;

  // ---- once per block: zero the padding, stage W transposed -------------------------------------------------
  for (int i = tid; i < kFusedRows * LDN; i += 256) sDz[i] = 0;
  for (int i = tid; i < kFusedRows * LDK; i += 256) sA[i] = 0;
  for (int i = tid; i < p.KP * LDN; i += 256) sWt[i] = 0;
  __syncthreads();
  for (int i = tid; i < N * (K / 8); i += 256) {
    const int n = i / (K / 8), k8 = (i - n * (K / 8)) * 8;
    const uint4 v = *reinterpret_cast<const uint4*>(p.w + (size_t)n * K + k8);
    const uint32_t wds[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) sWt[(k8 + e) * LDN + n] = (bf16_t)((wds[e >> 1] >> ((e & 1) * 16)) & 0xffffu);
  }
  float sc[8], sh[8], k1[8], k2[8], k3[8];
  {
    const int cc = ew ? c : 0;
    if (ACT != ACT_NONE) { load8(p.scale + cc, sc); load8(p.shift + cc, sh); }
    load8(p.coef + cc, k1); load8(p.coef + N + cc, k2); load8(p.coef + 2 * N + cc, k3);
  }

  // the input tile: rows x K/8 vectors over the 256 threads (at most 2 each: K/8 <= 6, 384 vectors for 64 rows)
  const int AV = kFusedRows * (K / 8);
  Raw<bf16_t> rd[IT], rz[IT], ra[2];
  auto fetch = [&](const int tile) __attribute__((always_inline)) {
    const size_t m0 = (size_t)tile * kFusedRows;
#pragma unroll
    for (int q = 0; q < IT; ++q) {
      const int r = er + q * RP;
      const size_t m = m0 + r;
      const bool in = ew && r < kFusedRows && m < p.M;
      const size_t off = in ? m * N + c : 0;
      raw_load(rd[q], p.dA + off);
      raw_load(rz[q], p.z + off);
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int i = tid + q * 256;
      const int r = i / (K / 8), k8 = (i - r * (K / 8)) * 8;
      const size_t m = m0 + r;
      const bool in = i < AV && m < p.M;
      raw_load(ra[q], p.a + (in ? m * K + k8 : 0));
    }
  };

  f4v_t accw[NTW][KT];
#pragma unroll
  for (int i = 0; i < NTW; ++i)
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) accw[i][kt] = f4v_t{0.f, 0.f, 0.f, 0.f};
  const int NT = N / 16;

  int tile = blockIdx.x;
  if (tile < p.ntiles) fetch(tile);
  for (; tile < p.ntiles; tile += gridDim.x) {
    const size_t m0 = (size_t)tile * kFusedRows;
    __syncthreads();                                   // the previous tile's products have read the LDS tiles
    // ---- dz of this tile into LDS, and the input tile ----
#pragma unroll
    for (int q = 0; q < IT; ++q) {
      const int r = er + q * RP;
      if (ew && r < kFusedRows) {
        float d[8], v[8], o[8];
        raw_unpack(rd[q], d);
        raw_unpack(rz[q], v);
        const bool live = m0 + r < p.M;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float dy = d[e];
          if (ACT != ACT_NONE) {
            const float y = fmaf(v[e], sc[e], sh[e]);
            dy = (y > 0.f && (ACT == ACT_RELU || y < 6.f)) ? dy : 0.f;
          }
          o[e] = live ? fmaf(k1[e], dy, fmaf(k2[e], v[e], k3[e])) : 0.f;
        }
        store8(sDz + r * LDN + c, o);
      }
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int i = tid + q * 256;
      if (i < AV) {
        const int r = i / (K / 8), k8 = (i - r * (K / 8)) * 8;
        uint4 v = ra[q].a;
        if (m0 + r >= p.M) v = make_uint4(0u, 0u, 0u, 0u);
        *reinterpret_cast<uint4*>(sA + r * LDK + k8) = v;
      }
    }
    __syncthreads();
    if (tile + (int)gridDim.x < p.ntiles) fetch(tile + gridDim.x);     // travels during the products

    // ---- data gradient: rows 16*wave .. +15, D'[k][row] = sum_n W^T[k][n] * dz[row][n] ----
    {
      // 64 rows: one 16-row tile per wavefront; 32 rows: two wavefronts share a row tile and split the k-tiles
      constexpr int RT = kFusedRows / 16, WPT = 4 / RT;
      const int R0 = (wave % RT) * 16, kpart = wave / RT;
      const size_t m = m0 + R0 + l16;
      float rs[KT][4];
      if (RES) {
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
          const int k = kt * 16 + G * 4;
          uint2 u = make_uint2(0u, 0u);
          if (m < p.M && k < K && kt % WPT == kpart) u = *reinterpret_cast<const uint2*>(p.res + m * K + k);
          rs[kt][0] = __uint_as_float(u.x << 16); rs[kt][1] = __uint_as_float(u.x & 0xffff0000u);
          rs[kt][2] = __uint_as_float(u.y << 16); rs[kt][3] = __uint_as_float(u.y & 0xffff0000u);
        }
      }
      f4v_t accd[KT];
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) accd[kt] = f4v_t{0.f, 0.f, 0.f, 0.f};
      for (int n0 = 0; n0 < p.NP; n0 += 32) {
        const bf16x8_t b = lds_frag(sDz + (R0 + l16) * LDN + n0 + G * 8);
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
          if (kt % WPT != kpart) continue;                 // uniform over the wavefront
          const bf16x8_t a = lds_frag(sWt + (kt * 16 + l16) * LDN + n0 + G * 8);
          accd[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, accd[kt], 0, 0, 0);
        }
      }
      // lane: row R0 + l16, columns kt*16 + 4*G .. +3
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        const int k = kt * 16 + G * 4;
        if (m < p.M && k < K && kt % WPT == kpart) {
          float v0 = accd[kt][0], v1 = accd[kt][1], v2 = accd[kt][2], v3 = accd[kt][3];
          if (RES) { v0 += rs[kt][0]; v1 += rs[kt][1]; v2 += rs[kt][2]; v3 += rs[kt][3]; }
          uint2 u;
          u.x = f32x2_to_bf16x2(v0, v1);
          u.y = f32x2_to_bf16x2(v2, v3);
          *reinterpret_cast<uint2*>(p.dIn + m * K + k) = u;
        }
      }
    }

    // ---- weight gradient: this wavefront's n-tiles, D[n][k] += sum_rows dz[row][n] * A[row][k] ----
#pragma unroll
    for (int s = 0; s < kFusedRows / 32; ++s) {
      bf16x8_t bk[KT];
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) bk[kt] = lds_frag_tr(sA, LDK, s * 32 + G * 8, kt * 16, l16);
#pragma unroll
      for (int i = 0; i < NTW; ++i) {
        const int nt = wave + 4 * i;
        if (nt < NT) {
          const bf16x8_t an = lds_frag_tr(sDz, LDN, s * 32 + G * 8, nt * 16, l16);
#pragma unroll
          for (int kt = 0; kt < KT; ++kt) accw[i][kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(an, bk[kt], accw[i][kt], 0, 0, 0);
        }
      }
    }
  }

  // ---- the block's partial: register r of lane l is D[nt*16 + 4*G + r][kt*16 + l16] ----
  float* out = p.ws + (size_t)blockIdx.x * N * K;
#pragma unroll
  for (int i = 0; i < NTW; ++i) {
    const int nt = wave + 4 * i;
    if (nt >= NT) continue;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      const int k = kt * 16 + l16;
      if (k >= K) continue;
#pragma unroll
      for (int r = 0; r < 4; ++r) out[(size_t)(nt * 16 + 4 * G + r) * K + k] = accw[i][kt][r];
    }
  }
}

// ---- host side ---------------------------------------------------------------------------------------------
struct FusedPlan { int NTW, KT, IT, NP, KP, ntiles, P, rows; size_t lds; };

static bool fused_plan(size_t M, int K, int N, FusedPlan* f) {
  if (N % 16 || K % 8 || N < 64 || N > 320 || K > 48 || M <= 2048 || N < 2 * K) return false;
  const int NT = N / 16, CG = N / 8;
  f->NTW = (NT + 3) / 4;
  f->KT = (K + 15) / 16;
  f->NP = (N + 31) / 32 * 32;
  f->KP = f->KT * 16;
  const int RP = 256 / CG;
  // 64-row tiles unless their elementwise stage needs more than eight passes per thread (the 288-channel layers: more
  // than 256 registers).  Measured in a step: this rule 7.50 ms, 32 rows from seven passes on (the 192-channel layers
  // too) 7.53 ms, 64 rows everywhere 7.55 ms.
  const int kFusedRows = (64 + RP - 1) / RP > 8 ? 32 : 64;
  f->rows = kFusedRows;
  f->IT = (kFusedRows + RP - 1) / RP;
  f->ntiles = (int)((M + kFusedRows - 1) / kFusedRows);
  // one block per CU, two where the partials stay below ~4 % of what the layer moves
  const double layer_bytes = (double)M * (2.0 * N + 3.0 * K) * 2.0;
  const int cap = (kFusedRows == 32 || 2.0 * kFusedBlocks * N * K * 8.0 <= 0.25 * layer_bytes) ? 2 * kFusedBlocks : kFusedBlocks;
  f->P = f->ntiles < cap ? f->ntiles : cap;
  f->lds = ((size_t)kFusedRows * (f->NP + 8) + (size_t)kFusedRows * (f->KP + 8) + (size_t)f->KP * (f->NP + 8)) * 2;
  if (kFusedRows * (K / 8) > 512) return false;
  return f->NTW <= 5 && f->KT <= 3 && f->IT <= (kFusedRows == 32 ? 6 : 8);
}

int pw_bwd_fused_ok(int dt, size_t M, int K, int N, HView a) {
  FusedPlan f;
  return dt == 1 && a.scale == nullptr && fused_plan(M, K, N, &f);
}

size_t pw_bwd_fused_ws(size_t M, int K, int N) {
  FusedPlan f;
  if (!fused_plan(M, K, N, &f)) return 0;
  return (size_t)f.P * N * K;
}

template <int ACT, int NTW, int KT, int IT, int ROWS>
static void fused_launch(hipStream_t st, const FusedArgs& a, const FusedPlan& f) {
  if (a.res) hipLaunchKernelGGL((pw_bwd_fused_k<ACT, NTW, KT, IT, true, ROWS>), dim3(f.P), dim3(256), f.lds, st, a);
  else hipLaunchKernelGGL((pw_bwd_fused_k<ACT, NTW, KT, IT, false, ROWS>), dim3(f.P), dim3(256), f.lds, st, a);
}

template <int ACT, int NTW, int KT>
static void fused_launch_it(hipStream_t st, const FusedArgs& a, const FusedPlan& f) {
  // passes of the elementwise stage: the tile's rows over 256 / (N/8) rows per pass (at most 8, see fused_plan)
  if (f.rows == 32) fused_launch<ACT, NTW, KT, 6, 32>(st, a, f);
  else if (f.IT <= 4) fused_launch<ACT, NTW, KT, 4, 64>(st, a, f);
  else if (f.IT <= 6) fused_launch<ACT, NTW, KT, 6, 64>(st, a, f);
  else fused_launch<ACT, NTW, KT, 8, 64>(st, a, f);
}

template <int ACT>
static void fused_launch_shape(hipStream_t st, const FusedArgs& a, const FusedPlan& f) {
  if (f.NTW <= 2 && f.KT <= 1) fused_launch_it<ACT, 2, 1>(st, a, f);
  else if (f.NTW <= 3 && f.KT <= 2) fused_launch_it<ACT, 3, 2>(st, a, f);
  else fused_launch_it<ACT, 5, 3>(st, a, f);
}

void pw_bwd_fused(hipStream_t st, const void* dA, HView out, const float* coef, const void* w, const void* a_in,
                  const void* res, size_t M, int K, int N, float* ws, float* g_w, void* dIn, hipStream_t st_sum,
                  hipEvent_t ev_sum) {
  FusedPlan f;
  if (!fused_plan(M, K, N, &f)) { launch_plan_failed("fused pointwise backward called for a shape it does not take"); return; }
  FusedArgs a{};
  a.dA = (const bf16_t*)dA; a.z = (const bf16_t*)out.z; a.scale = out.scale; a.shift = out.shift; a.coef = coef;
  a.w = (const bf16_t*)w; a.a = (const bf16_t*)a_in; a.res = (const bf16_t*)res; a.dIn = (bf16_t*)dIn; a.ws = ws;
  a.M = M; a.K = K; a.N = N; a.NP = f.NP; a.KP = f.KP; a.ntiles = f.ntiles;
  {
    KScope ks(st, "pw_bwd_fused", ((double)M * N * 2.0 + (double)M * K * (res ? 3.0 : 2.0)) * 2.0 + (double)f.P * N * K * 4.0,
              4.0 * M * K * N, (long)M, K, N);
    if (out.act == ACT_NONE) fused_launch_shape<ACT_NONE>(st, a, f);
    else if (out.act == ACT_RELU) fused_launch_shape<ACT_RELU>(st, a, f);
    else fused_launch_shape<ACT_RELU6>(st, a, f);
  }
  if (st_sum != st) {                 // the partial sums are summed on another stream, behind the kernel
    if (hipEventRecord(ev_sum, st) != hipSuccess || hipStreamWaitEvent(st_sum, ev_sum, 0) != hipSuccess) {
      launch_plan_failed("fused pointwise backward: could not order the partial sums behind the kernel");
      return;
    }
  }
  reduce_partials(st_sum, ws, f.P, (size_t)N * K, K, (size_t)K, 1, g_w, K);
}

}  // namespace ftp

// ---- weight gradient of a pointwise layer, bfloat16, operands staged as they lie in memory --------------------
// g_w[n][k] += sum_m dZ[m][n] * A'[m][k]: both MFMA operands need the rows m as the contiguous index of a lane's
// fragment while dZ and A hold channels contiguously.  A block stages 64-row chunks of a 128-column strip of dZ and a
// 64-column strip of A (through the view) into LDS with plain 16-byte copies and reads them back with the LDS
// transpose read (lds_frag_tr): no repacking pass (the layer-by-layer kernel spends most of its instructions
// interleaving row pairs).  The rows are split over blocks; every block leaves one fp32 partial of its
// 128 x 64 tile, summed by reduce_partials in a fixed order.
namespace ftp {

enum { kWgN = 128, kWgK = 64, kWgRows = 64 };

struct WgTrArgs {
  const bf16_t* dz;     // [M][N]
  const bf16_t* a;      // [M][K]
  const float* scale;   // view of A (nullptr: stored activated)
  const float* shift;
  int act;
  float* ws;            // [S][N][K]
  size_t M, mchunk;     // rows per split (a multiple of 64)
  int K, N, itiles, jtiles;
};

template <bool VIEW>
__global__ __launch_bounds__(256) void pw_wgrad_tr_k(WgTrArgs p) {
  constexpr int LDN = kWgN + 8, LDK = kWgK + 8;
  __shared__ __attribute__((aligned(16))) bf16_t sZ[2][kWgRows * LDN];
  __shared__ __attribute__((aligned(16))) bf16_t sA[2][kWgRows * LDK];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l16 = lane & 15, G = lane >> 4;
  const int lb = xcd_logical_block();
  const int jt = lb % p.jtiles, rest = lb / p.jtiles, it = rest % p.itiles, split = rest / p.itiles;
  const int n0 = it * kWgN, k0 = jt * kWgK;
  const size_t mb = (size_t)split * p.mchunk, me = mb + p.mchunk < p.M ? mb + p.mchunk : p.M;
  const int N = p.N, K = p.K;

  // staging map: dZ chunk = 64 rows x 16 vectors (4 per thread), A chunk = 64 rows x 8 vectors (2 per thread)
  const int zc = (tid & 15) * 8, zr = tid >> 4;         // + 16 rows per pass
  const int ac = (tid & 7) * 8, ar = tid >> 3;          // + 32 rows per pass
  const bool zc_ok = n0 + zc < N, ac_ok = k0 + ac < K;
  float sc[8], sh[8];
  if (VIEW) { load8(p.scale + (ac_ok ? k0 + ac : 0), sc); load8(p.shift + (ac_ok ? k0 + ac : 0), sh); }
  const float lo = act_lo(p.act), hi = act_hi(p.act);

  Raw<bf16_t> rz[4], ra[2];
  auto fetch = [&](const size_t m0) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const size_t m = m0 + zr + 16 * q;
      raw_load(rz[q], p.dz + ((zc_ok && m < me) ? m * N + n0 + zc : 0));
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const size_t m = m0 + ar + 32 * q;
      raw_load(ra[q], p.a + ((ac_ok && m < me) ? m * K + k0 + ac : 0));
    }
  };
  auto commit = [&](const int buf, const size_t m0) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const size_t m = m0 + zr + 16 * q;
      uint4 v = rz[q].a;
      if (!(zc_ok && m < me)) v = make_uint4(0u, 0u, 0u, 0u);
      *reinterpret_cast<uint4*>(&sZ[buf][(zr + 16 * q) * LDN + zc]) = v;
    }
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const size_t m = m0 + ar + 32 * q;
      const bool in = ac_ok && m < me;
      if (VIEW) {
        float v[8];
        raw_unpack(ra[q], v);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = in ? clamp_act(fmaf(v[e], sc[e], sh[e]), lo, hi) : 0.f;   // padding stays zero
        store8(&sA[buf][(ar + 32 * q) * LDK + ac], v);
      } else {
        uint4 v = ra[q].a;
        if (!in) v = make_uint4(0u, 0u, 0u, 0u);
        *reinterpret_cast<uint4*>(&sA[buf][(ar + 32 * q) * LDK + ac]) = v;
      }
    }
  };

  // wavefront w: n-tiles 2w, 2w+1 of the strip (16 columns each), all four k-tiles
  f4v_t acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f4v_t{0.f, 0.f, 0.f, 0.f};

  const int nchunks = (int)((me - mb + kWgRows - 1) / kWgRows);
  if (nchunks > 0) fetch(mb);
  for (int ch = 0; ch < nchunks; ++ch) {
    const int buf = ch & 1;
    commit(buf, mb + (size_t)ch * kWgRows);
    __syncthreads();                      // chunk ch is in LDS; the other buffer's readers finished before their next commit
    if (ch + 1 < nchunks) fetch(mb + (size_t)(ch + 1) * kWgRows);
#pragma unroll
    for (int s = 0; s < kWgRows / 32; ++s) {
      bf16x8_t bk[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) bk[j] = lds_frag_tr(sA[buf], LDK, s * 32 + G * 8, j * 16, l16);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const bf16x8_t an = lds_frag_tr(sZ[buf], LDN, s * 32 + G * 8, (2 * wave + i) * 16, l16);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(an, bk[j], acc[i][j], 0, 0, 0);
      }
    }
  }
  // register r of lane l: D[n = tile*16 + 4*G + r][k = j*16 + l16]
  float* out = p.ws + (size_t)split * N * K;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + j * 16 + l16;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int n = n0 + (2 * wave + i) * 16 + 4 * G + r;
        if (n < N && k < K) out[(size_t)n * K + k] = acc[i][j][r];
      }
    }
}

static bool wg_tr_plan(size_t M, int K, int N, WgTrArgs* a, int* S) {
  if (K % 8 || N % 8 || M <= 2048 || N < 48) return false;     // a 128-column strip of a narrower dZ is mostly padding: measured slower
  a->itiles = (N + kWgN - 1) / kWgN;
  a->jtiles = (K + kWgK - 1) / kWgK;
  const size_t tiles = (size_t)a->itiles * a->jtiles;
  // about 512 blocks: with 1024 the kernel itself takes the same time, but twice the partial tiles are written and
  // summed afterwards (more than the operands themselves for the layers with large weight matrices)
  size_t s = (512 + tiles - 1) / tiles;
  const size_t smax = (M + 2 * kWgRows - 1) / (2 * kWgRows);
  if (s > smax) s = smax;
  if (s > (size_t)kMaxPartials) s = kMaxPartials;
  if (s < 1) s = 1;
  size_t mc = (M + s - 1) / s;
  mc = (mc + kWgRows - 1) / kWgRows * kWgRows;
  a->mchunk = mc;
  *S = (int)((M + mc - 1) / mc);
  return true;
}

int pw_wgrad_tr_ok(int dt, size_t M, int K, int N) {
  WgTrArgs a{};
  int S;
  return dt == 1 && wg_tr_plan(M, K, N, &a, &S);
}
size_t pw_wgrad_tr_ws(size_t M, int K, int N) {
  WgTrArgs a{};
  int S;
  if (!wg_tr_plan(M, K, N, &a, &S)) return 0;
  return (size_t)S * N * K;
}
void pw_wgrad_tr(hipStream_t st, const void* dz, HView av, size_t M, int K, int N, float* ws, float* g_w, int K_out) {
  WgTrArgs a{};
  int S = 1;
  if (!wg_tr_plan(M, K, N, &a, &S)) { launch_plan_failed("transposing weight gradient called for a shape it does not take"); return; }
  a.dz = (const bf16_t*)dz; a.a = (const bf16_t*)av.z; a.scale = av.scale; a.shift = av.shift; a.act = av.act;
  a.ws = ws; a.M = M; a.K = K; a.N = N;
  {
    KScope ks(st, "pw_wgrad", ((double)M * K + (double)M * N) * 2.0 + (double)S * N * K * 4, 2.0 * M * K * N, (long)M, K, N);
    const unsigned grid = (unsigned)(a.itiles * a.jtiles * S);
    if (av.scale) hipLaunchKernelGGL(pw_wgrad_tr_k<true>, dim3(grid), dim3(256), 0, st, a);
    else hipLaunchKernelGGL(pw_wgrad_tr_k<false>, dim3(grid), dim3(256), 0, st, a);
  }
  if (K_out < 0) K_out = K;
  reduce_partials(st, ws, S, (size_t)N * K, K, (size_t)K_out, 1, g_w, K_out);
}

}  // namespace ftp
