// Device helper shared by the short-tensor kernels: finishing BatchNorm statistics that a producer left as
// partial sums, for the four channels a block owns.
#pragma once
#include "dev_common.h"
#include "kernels.h"

namespace ftp {

// finish pending BatchNorm statistics for channels c0..c0+3 (first 256 threads), result in insc[2][4]
__device__ __forceinline__ void finish_pending4(const BnPending& pend, int C, int c0, float eps, float momentum, double (*pre)[8],
                                                float (*insc)[4]) {
  const int tid = threadIdx.x;
  // what the last four threads need at the end is requested now, and the partials four at a time from clamped
  // addresses: this runs at the head of kernels that are a chain of memory round trips and little else
  float p_g = 0.f, p_b = 0.f, p_rm = 0.f, p_rv = 0.f;
  if (tid < 4) { p_g = pend.gamma[c0 + tid]; p_b = pend.beta[c0 + tid]; p_rm = pend.run_mean[c0 + tid]; p_rv = pend.run_var[c0 + tid]; }
  if (tid < 256) {
    const int v = tid & 7, lane = tid >> 3;           // 4 sums, 4 second sums; 32 lanes each
    double t = 0.0;
    for (int q0 = lane; q0 < pend.P; q0 += 128) {
      float x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int q = q0 + 32 * u;
        x[u] = pend.partial[((size_t)(q < pend.P ? q : 0) * 2 + (v >> 2)) * C + c0 + (v & 3)];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) t += q0 + 32 * u < pend.P ? (double)x[u] : 0.0;
    }
    pre[lane][v] = t;
  }
  __syncthreads();
  // first use of the four values requested at the top: their conversions must not move up to the loads
  asm volatile("" : "+v"(p_g), "+v"(p_b), "+v"(p_rm), "+v"(p_rv));
  if (tid < 4) {
    const int c = c0 + tid;
    double s0 = 0.0, s1 = 0.0;
    for (int l = 0; l < 32; ++l) { s0 += pre[l][tid]; s1 += pre[l][4 + tid]; }
    const double Md = (double)pend.M, mu = s0 / Md;
    double var = s1 / Md - mu * mu;
    if (var < 0.0) var = 0.0;
    const double is = 1.0 / sqrt(var + (double)eps);
    const float scv = (float)((double)p_g * is);
    const float shv = (float)((double)p_b - mu * (double)scv);
    pend.mean[c] = (float)mu;
    pend.invstd[c] = (float)is;
    pend.scale[c] = scv;
    pend.shift[c] = shv;
    const double unb = pend.M > 1 ? var * (Md / (Md - 1.0)) : var;
    pend.run_mean[c] = (float)((1.0 - momentum) * p_rm + momentum * mu);
    pend.run_var[c] = (float)((1.0 - momentum) * p_rv + momentum * unb);
    insc[0][tid] = scv;
    insc[1][tid] = shv;
  }
  __syncthreads();
}

}  // namespace ftp
