// Pointwise layers with a LONG reduction and few rows, bfloat16: the project layers (forward) and the expand layers
// (data gradient) of the low-resolution inverted residual blocks, 6 K - 25 K rows against a reduction of 256 - 1800
// channels.  Their tensors are small (they stay in the memory-side cache) and their arithmetic intensity is at the
// MFMA / HBM balance, so what they need is a GEMM that keeps the matrix cores fed, not a streaming kernel:
//   * a block owns a (32*S) x (32*T) output tile (S = 2 or 4, T = 2 .. 5) and walks the whole reduction in steps of 64,
//     its four wavefronts in a 2 x 2 arrangement of (16*S) x (16*T) sub-tiles of v_mfma_f32_16x16x32_bf16;
//   * both operands go through double-buffered LDS (one barrier per step); the 16-byte vectors of the next two
//     steps are on their way from memory into registers while the current step is multiplied (a layer has about one
//     block per CU and a round trip to memory takes several steps: what hides it is bytes in flight per block);
//   * the weights of the data gradient are stored [reduction][column]: they are staged as they lie in memory and
//     read back through the LDS transpose read, so neither mode repacks anything;
//   * the weight operand is the MFMA's first operand: a lane then holds four CONSECUTIVE output columns of one row
//     and stores (and adds the residual, and sums the BatchNorm statistics of) 8-byte groups.
// Forward applies the producer's BatchNorm + activation to the rows on their way into LDS and leaves the column sums of
// the stored output (one partial per row tile, summed in a fixed order) for the BatchNorm that follows.
#include "dev_common.h"
#include "kernels.h"
#include "mfma_frag.h"

namespace ftp {

enum { kDeepKS = 64, kDeepLD = kDeepKS + 8, kDeepMaxR = 2048 };
enum { DEEP_FWD = 0, DEEP_FWD_VIEW = 1, DEEP_DGRAD = 2, DEEP_DGRAD_RES = 3 };

struct DeepArgs {
  const bf16_t* x;      // [M][R]: A as stored (forward) or dZ (data gradient)
  const bf16_t* y;      // W[N][K]: forward [column][reduction], data gradient [reduction][column]
  const float* scale;   // forward: view of x, indexed by the reduction channel (DEEP_FWD_VIEW)
  const float* shift;
  const bf16_t* res;    // [M][NC] added to the result (DEEP_DGRAD_RES)
  bf16_t* out;          // [M][NC]
  float* stats;         // forward: [row tiles][2][NC] column sums of the stored output and of its squares, or nullptr
  int act;
  int M, R, NC;         // rows, reduction extent, output columns
  int jtiles;           // column tiles; the grid is jtiles * row tiles
};

template <int S, int T, int MODE>
__global__ __launch_bounds__(256) void pw_gemm_deep_k(DeepArgs p) {
  constexpr bool DG = MODE >= DEEP_DGRAD;
  constexpr int BM = 32 * S, BN = 32 * T, LD = kDeepLD, LDY = BN + 8;
  constexpr int XS = BM * LD;                               // elements of one x buffer
  constexpr int YS = DG ? kDeepKS * LDY : BN * LD;          // elements of one y buffer
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  bf16_t* xs = reinterpret_cast<bf16_t*>(smem_raw);         // [2][BM][LD]
  bf16_t* ys = xs + 2 * XS;                                 // [2][BN][LD] or [2][64][LDY]
  float* vw = reinterpret_cast<float*>(ys + 2 * YS);        // forward with a view: scale[RP], shift[RP], RP = R rounded up to 64
  if (DG) __builtin_amdgcn_s_setprio(3);                    // data-gradient chain

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l16 = lane & 15, G = lane >> 4;
  const int wm = wave >> 1, wn = wave & 1;
  const int lb = xcd_logical_block();
  const int jt = lb % p.jtiles, it = lb / p.jtiles;
  const int m0 = it * BM, j0 = jt * BN;
  const int M = p.M, R = p.R, NC = p.NC;

  // ---- loaders: S vectors of x and T vectors of y per thread and step ----
  // Both operands are read through buffer descriptors (base, size): a load whose byte offset lies outside the tensor
  // returns zeros, so a vector outside the operand (rows past M, columns past NC, reduction elements past R) is
  // requested at an offset past the end instead of being selected away afterwards: no selects and no branches between a
  // load and its use, one 32-bit offset register per vector, and the only waits in the loop are the counted ones in
  // front of each step.  Through the view a zero row becomes act(shift): such rows (past M) are never stored and are
  // masked out of the statistics; past R the weights are zero, so the products vanish.
  const int xkv = (tid & 7) * 8, xrow = tid >> 3;           // x: 8 threads cover the 64 reduction elements of a row
  // steps in flight: two.  A third costs about a hundred registers here, and two resident blocks per CU, which hide each
  // other's barrier and LDS phases, measured worth more than the third step.
  constexpr int D = 2;
  constexpr uint32_t kPast = 0x80000000u;                   // beyond any operand here (they are smaller than 2 GiB), also after adding a step
  struct Set { uint4 x[S]; uint4 y[T]; };
  Set set[D];
  const int RP = (R + kDeepKS - 1) / kDeepKS * kDeepKS;
  const __amdgpu_buffer_rsrc_t bx = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(p.x), 0, (int)((size_t)M * R * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t by = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(p.y), 0, (int)((size_t)R * NC * 2), 0x00020000);
  uint32_t ox[S], oy[T];                                    // byte offsets of this thread's vectors at step 0
#pragma unroll
  for (int q = 0; q < S; ++q) {
    const int m = m0 + xrow + q * 32;
    ox[q] = m < M ? (uint32_t)(m * R + xkv) * 2u : kPast;
  }
#pragma unroll
  for (int q = 0; q < T; ++q) {
    if (!DG) {
      const int j = j0 + xrow + q * 32;
      oy[q] = j < NC ? (uint32_t)(j * R + xkv) * 2u : kPast;
    } else {
      const int v = tid + q * 256;
      const int j = j0 + (v % (4 * T)) * 8;
      oy[q] = j < NC ? (uint32_t)((v / (4 * T)) * NC + j) * 2u : kPast;
    }
  }
  if (MODE == DEEP_FWD_VIEW) {
    for (int i = tid; i < RP; i += 256) {
      vw[i] = i < R ? p.scale[i] : 0.f;
      vw[RP + i] = i < R ? p.shift[i] : 0.f;
    }
  }
  typedef uint32_t u4v_t __attribute__((ext_vector_type(4)));
  auto ld = [&](const __amdgpu_buffer_rsrc_t rs, const uint32_t off) __attribute__((always_inline)) {
    const u4v_t v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
  };
  auto fetch = [&](Set& f, const int r0) __attribute__((always_inline)) {
    const bool kin = r0 + xkv < R;
#pragma unroll
    for (int q = 0; q < S; ++q) f.x[q] = ld(bx, kin ? ox[q] + (uint32_t)r0 * 2u : kPast);
#pragma unroll
    for (int q = 0; q < T; ++q) {
      if (!DG) {
        f.y[q] = ld(by, kin ? oy[q] + (uint32_t)r0 * 2u : kPast);
      } else {
        const int v = tid + q * 256;
        f.y[q] = ld(by, r0 + v / (4 * T) < R ? oy[q] + (uint32_t)(r0 * NC) * 2u : kPast);
      }
    }
  };
  auto commit = [&](const Set& f, const int r0, bf16_t* xb, bf16_t* yb) __attribute__((always_inline)) {
    const float lo = act_lo(p.act), hi = act_hi(p.act);
    float vsc[8], vsh[8];
    if (MODE == DEEP_FWD_VIEW) {           // r0 + xkv < RP: the steps stop at RP
      load8(vw + r0 + xkv, vsc);
      load8(vw + RP + r0 + xkv, vsh);
    }
#pragma unroll
    for (int q = 0; q < S; ++q) {
      uint4 v = f.x[q];
      if (MODE == DEEP_FWD_VIEW) {
        Raw<bf16_t> raw;
        raw.a = v;
        float t[8];
        raw_unpack(raw, t);
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = clamp_act(fmaf(t[e], vsc[e], vsh[e]), lo, hi);
        v.x = f32x2_to_bf16x2(t[0], t[1]); v.y = f32x2_to_bf16x2(t[2], t[3]);
        v.z = f32x2_to_bf16x2(t[4], t[5]); v.w = f32x2_to_bf16x2(t[6], t[7]);
      }
      *reinterpret_cast<uint4*>(xb + (xrow + q * 32) * LD + xkv) = v;
    }
#pragma unroll
    for (int q = 0; q < T; ++q) {
      if (!DG) {
        *reinterpret_cast<uint4*>(yb + (xrow + q * 32) * LD + xkv) = f.y[q];
      } else {
        const int i = tid + q * 256;
        *reinterpret_cast<uint4*>(yb + (i / (4 * T)) * LDY + (i % (4 * T)) * 8) = f.y[q];
      }
    }
  };

  f4v_t acc[S][T];
#pragma unroll
  for (int a = 0; a < S; ++a)
#pragma unroll
    for (int b = 0; b < T; ++b) acc[a][b] = f4v_t{0.f, 0.f, 0.f, 0.f};

  // one step: set -> LDS buffer s % 2, barrier (which also says that everyone has finished multiplying the step before
  // last, this buffer's previous contents), the set's next request (D steps ahead; past the end: zeros), multiply
  auto step = [&](Set& f, const int s) __attribute__((always_inline)) {
    bf16_t* xb = xs + (s & 1) * XS;
    bf16_t* yb = ys + (s & 1) * YS;
    commit(f, s * kDeepKS, xb, yb);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);   // the requests stay here, D steps ahead of their use (the scheduler would move them down to it)
    fetch(f, (s + D) * kDeepKS);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < kDeepKS / 32; ++ks) {
      bf16x8_t xf[S], yf[T];
#pragma unroll
      for (int a = 0; a < S; ++a) xf[a] = lds_frag(xb + (wm * 16 * S + a * 16 + l16) * LD + ks * 32 + G * 8);
#pragma unroll
      for (int b = 0; b < T; ++b) {
        if (DG) yf[b] = lds_frag_tr(yb, LDY, ks * 32 + G * 8, wn * 16 * T + b * 16, l16);
        else yf[b] = lds_frag(yb + (wn * 16 * T + b * 16 + l16) * LD + ks * 32 + G * 8);
      }
#pragma unroll
      for (int a = 0; a < S; ++a)
#pragma unroll
        for (int b = 0; b < T; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(yf[b], xf[a], acc[a][b], 0, 0, 0);
    }
  };

  const int nsteps = RP / kDeepKS;
#pragma unroll
  for (int d = 0; d < D; ++d) {
    fetch(set[d], d * kDeepKS);
    // the sets are requested in order: a wait for set d is then a wait for "all but the youngest loads" on every path
    __builtin_amdgcn_sched_barrier(0);
  }
  if (MODE == DEEP_FWD_VIEW) __syncthreads();                        // the view vectors are in LDS
  // whole groups of D steps without a branch inside (a path from the middle of a group back to the loop head would
  // turn every wait at the head into a wait for all loads), then the remaining steps
  int s0 = 0;
  for (; s0 + D <= nsteps; s0 += D) {
#pragma unroll
    for (int d = 0; d < D; ++d) step(set[d], s0 + d);
  }
#pragma unroll
  for (int d = 0; d + 1 < D; ++d)
    if (s0 + d < nsteps) step(set[d], s0 + d);

  // ---- results: acc[a][b][e] is out[m0 + wm*16S + 16a + l16][j0 + wn*16T + 16b + 4G + e] ----
  float s1[T][4], s2[T][4];
#pragma unroll
  for (int b = 0; b < T; ++b)
#pragma unroll
    for (int e = 0; e < 4; ++e) { s1[b][e] = 0.f; s2[b][e] = 0.f; }
  uint2 rs[S][T];
  if (MODE == DEEP_DGRAD_RES) {          // all residual groups are requested before the first store
#pragma unroll
    for (int a = 0; a < S; ++a)
#pragma unroll
      for (int b = 0; b < T; ++b) {
        const int m = m0 + wm * 16 * S + a * 16 + l16, j = j0 + wn * 16 * T + b * 16 + 4 * G;
        const bool in = m < M && j < NC;
        rs[a][b] = *reinterpret_cast<const uint2*>(p.res + (in ? (size_t)m * NC + j : 0));
      }
  }
#pragma unroll
  for (int a = 0; a < S; ++a)
#pragma unroll
    for (int b = 0; b < T; ++b) {
      const int m = m0 + wm * 16 * S + a * 16 + l16, j = j0 + wn * 16 * T + b * 16 + 4 * G;
      float v0 = acc[a][b][0], v1 = acc[a][b][1], v2 = acc[a][b][2], v3 = acc[a][b][3];
      if (MODE == DEEP_DGRAD_RES) {
        v0 += __uint_as_float(rs[a][b].x << 16); v1 += __uint_as_float(rs[a][b].x & 0xffff0000u);
        v2 += __uint_as_float(rs[a][b].y << 16); v3 += __uint_as_float(rs[a][b].y & 0xffff0000u);
      }
      uint2 u;
      u.x = f32x2_to_bf16x2(v0, v1);
      u.y = f32x2_to_bf16x2(v2, v3);
      if (m < M && j < NC) *reinterpret_cast<uint2*>(p.out + (size_t)m * NC + j) = u;
      if (!DG) {                         // statistics of the values as stored; columns past NC are exact zeros, rows past M are masked
        if (m >= M) u = make_uint2(0u, 0u);
        const float r0v = __uint_as_float(u.x << 16), r1v = __uint_as_float(u.x & 0xffff0000u);
        const float r2v = __uint_as_float(u.y << 16), r3v = __uint_as_float(u.y & 0xffff0000u);
        s1[b][0] += r0v; s1[b][1] += r1v; s1[b][2] += r2v; s1[b][3] += r3v;
        s2[b][0] = fmaf(r0v, r0v, s2[b][0]); s2[b][1] = fmaf(r1v, r1v, s2[b][1]);
        s2[b][2] = fmaf(r2v, r2v, s2[b][2]); s2[b][3] = fmaf(r3v, r3v, s2[b][3]);
      }
    }
  if (!DG && p.stats) {
    // sum over the 16 rows a 16-lane group holds (butterflies inside the group), then the two wavefronts that share
    // the columns through LDS in a fixed order: one partial per row tile
    __syncthreads();                     // the staging buffers are free
    float* red = reinterpret_cast<float*>(smem_raw);       // [2 (wm)][2 (sum, squares)][BN]
#pragma unroll
    for (int b = 0; b < T; ++b)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float a1 = s1[b][e], a2 = s2[b][e];
        a1 += dpp_move<0xB1>(a1); a1 += dpp_move<0x4E>(a1); a1 += dpp_move<0x141>(a1); a1 += dpp_move<0x140>(a1);
        a2 += dpp_move<0xB1>(a2); a2 += dpp_move<0x4E>(a2); a2 += dpp_move<0x141>(a2); a2 += dpp_move<0x140>(a2);
        if (l16 == 0) {
          const int col = wn * 16 * T + b * 16 + 4 * G + e;
          red[(wm * 2 + 0) * BN + col] = a1;
          red[(wm * 2 + 1) * BN + col] = a2;
        }
      }
    __syncthreads();
    for (int i = tid; i < 2 * BN; i += 256) {
      const int which = i / BN, col = i - which * BN;
      const int j = j0 + col;
      if (j < NC) p.stats[((size_t)it * 2 + which) * NC + j] = red[which * BN + col] + red[(2 + which) * BN + col];
    }
  }
}

// ---- host side ---------------------------------------------------------------------------------------------
struct DeepPlan { int S, T, itiles, jtiles; size_t lds; };

// rows M, reduction extent R, output columns NC
static bool deep_plan(size_t M, int R, int NC, bool dgrad, DeepPlan* d) {
  if (M <= 2048 || M > 65536 || R < 192 || R > kDeepMaxR || R % 8 || NC % 8 || NC < 32) return false;
  // column tile: the width (96, 128 or 160; 64 for narrow outputs) that pads the fewest columns, the wider on ties
  int T = 2;
  if (NC > 64) {
    int best = 1 << 30;
    for (int t = 5; t >= 3; --t) {
      const int padded = (NC + 32 * t - 1) / (32 * t) * (32 * t);
      if (padded < best) { best = padded; T = t; }
    }
  }
  d->T = T;
  d->jtiles = (NC + 32 * T - 1) / (32 * T);
  // 128-row tiles when they still give every CU two blocks, 64-row tiles otherwise
  d->S = ((M + 127) / 128) * d->jtiles >= 512 ? 4 : 2;
  d->itiles = (int)((M + 32 * d->S - 1) / (32 * d->S));
  if (d->itiles > kMaxPartials) return false;
  const size_t xs = (size_t)32 * d->S * kDeepLD, ys = dgrad ? (size_t)kDeepKS * (32 * T + 8) : (size_t)32 * T * kDeepLD;
  d->lds = 2 * (xs + ys) * sizeof(bf16_t) + (dgrad ? 0 : 2 * (size_t)((R + kDeepKS - 1) / kDeepKS * kDeepKS) * sizeof(float));
  const size_t red = (size_t)4 * 32 * T * sizeof(float);
  if (d->lds < red) d->lds = red;
  return true;
}

int pw_deep_ok(int dt, size_t M, int R, int NC, bool dgrad) {
  DeepPlan d;
  return dt == 1 && deep_plan(M, R, NC, dgrad, &d);
}

template <int S, int T>
static void deep_launch_mode(hipStream_t st, const DeepArgs& a, const DeepPlan& d, int mode) {
  const dim3 grid((unsigned)d.itiles * d.jtiles), block(256);
  switch (mode) {
    case DEEP_FWD: hipLaunchKernelGGL((pw_gemm_deep_k<S, T, DEEP_FWD>), grid, block, d.lds, st, a); break;
    case DEEP_FWD_VIEW: hipLaunchKernelGGL((pw_gemm_deep_k<S, T, DEEP_FWD_VIEW>), grid, block, d.lds, st, a); break;
    case DEEP_DGRAD: hipLaunchKernelGGL((pw_gemm_deep_k<S, T, DEEP_DGRAD>), grid, block, d.lds, st, a); break;
    default: hipLaunchKernelGGL((pw_gemm_deep_k<S, T, DEEP_DGRAD_RES>), grid, block, d.lds, st, a); break;
  }
}

static void deep_launch(hipStream_t st, const DeepArgs& a, const DeepPlan& d, int mode) {
  if (d.S == 2) {
    switch (d.T) {
      case 2: deep_launch_mode<2, 2>(st, a, d, mode); break;
      case 3: deep_launch_mode<2, 3>(st, a, d, mode); break;
      case 4: deep_launch_mode<2, 4>(st, a, d, mode); break;
      default: deep_launch_mode<2, 5>(st, a, d, mode); break;
    }
  } else {
    switch (d.T) {
      case 2: deep_launch_mode<4, 2>(st, a, d, mode); break;
      case 3: deep_launch_mode<4, 3>(st, a, d, mode); break;
      case 4: deep_launch_mode<4, 4>(st, a, d, mode); break;
      default: deep_launch_mode<4, 5>(st, a, d, mode); break;
    }
  }
}

// z[M][N] = A'[M][K] * W[N][K]^T; stats as in pw_fwd (P_out = partials written)
void pw_fwd_deep(hipStream_t st, HView av, const void* w, size_t M, int K, int N, void* z, float* stats, int* P_out) {
  DeepPlan d;
  if (!deep_plan(M, K, N, false, &d)) { launch_plan_failed("long-reduction pointwise forward called for a shape it does not take"); return; }
  DeepArgs a{};
  a.x = (const bf16_t*)av.z; a.y = (const bf16_t*)w; a.scale = av.scale; a.shift = av.shift; a.act = av.act;
  a.out = (bf16_t*)z; a.stats = stats; a.M = (int)M; a.R = K; a.NC = N; a.jtiles = d.jtiles;
  if (P_out) *P_out = d.itiles;
  deep_launch(st, a, d, av.scale ? DEEP_FWD_VIEW : DEEP_FWD);
}

// dA[M][K] = dZ[M][N] * W[N][K] (+ res)
void pw_dgrad_deep(hipStream_t st, const void* dz, const void* w, const void* res, size_t M, int K, int N, void* dA) {
  DeepPlan d;
  if (!deep_plan(M, N, K, true, &d)) { launch_plan_failed("long-reduction pointwise data gradient called for a shape it does not take"); return; }
  DeepArgs a{};
  a.x = (const bf16_t*)dz; a.y = (const bf16_t*)w; a.res = (const bf16_t*)res; a.out = (bf16_t*)dA;
  a.M = (int)M; a.R = N; a.NC = K; a.jtiles = d.jtiles;
  deep_launch(st, a, d, res ? DEEP_DGRAD_RES : DEEP_DGRAD);
}

}  // namespace ftp
