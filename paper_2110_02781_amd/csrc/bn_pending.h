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
  if (tid < 256) {
    const int v = tid & 7, lane = tid >> 3;           // 4 sums, 4 second sums; 32 lanes each
    double t = 0.0;
    for (int q = lane; q < pend.P; q += 32) t += (double)pend.partial[((size_t)q * 2 + (v >> 2)) * C + c0 + (v & 3)];
    pre[lane][v] = t;
  }
  __syncthreads();
  if (tid < 4) {
    const int c = c0 + tid;
    double s0 = 0.0, s1 = 0.0;
    for (int l = 0; l < 32; ++l) { s0 += pre[l][tid]; s1 += pre[l][4 + tid]; }
    const double Md = (double)pend.M, mu = s0 / Md;
    double var = s1 / Md - mu * mu;
    if (var < 0.0) var = 0.0;
    const double is = 1.0 / sqrt(var + (double)eps);
    const float scv = (float)((double)pend.gamma[c] * is);
    const float shv = (float)((double)pend.beta[c] - mu * (double)scv);
    pend.mean[c] = (float)mu;
    pend.invstd[c] = (float)is;
    pend.scale[c] = scv;
    pend.shift[c] = shv;
    const double unb = pend.M > 1 ? var * (Md / (Md - 1.0)) : var;
    pend.run_mean[c] = (float)((1.0 - momentum) * pend.run_mean[c] + momentum * mu);
    pend.run_var[c] = (float)((1.0 - momentum) * pend.run_var[c] + momentum * unb);
    insc[0][tid] = scv;
    insc[1][tid] = shv;
  }
  __syncthreads();
}

}  // namespace ftp
