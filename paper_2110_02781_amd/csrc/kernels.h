// Host-side launch interface of the HIP kernels.  All functions enqueue work on
// `st` and return immediately; none allocates.  `dt` selects the storage type
// of activations / activation gradients / working weights (0 = float,
// 1 = bfloat16); statistics, weight gradients and accumulators are fp32.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ftp {

// Optional per-launch timing (diagnostics for benchmarks): when tracing is on, a
// KScope brackets one kernel launch with two HIP events on the launch stream and
// records the kernel family, the bytes the launch must move at least (each operand
// once) and its floating-point operations.
struct KScope {
  KScope(hipStream_t st, const char* name, double alg_bytes, double flops, long d0 = -1, long d1 = -1, long d2 = -1);
  ~KScope();
  int slot;
  hipStream_t st;
};

// A launcher that finds its own launch plan outside what its kernel was written for skips the launch and says so here;
// the stage call that enqueued it returns an error (launch_plan_failure_take returns the text once, or nullptr).
void launch_plan_failed(const char* what);
const char* launch_plan_failure_take();

struct HView {  // same layout as the device-side View
  const void* z;
  const float* scale;
  const float* shift;
  int act;
};

// BatchNorm statistics that have been reduced to partial[P][2][C] but not finalised yet
struct BnPending {
  const float* partial;
  int P;
  size_t M;
  const float* gamma;
  const float* beta;
  float *mean, *invstd, *scale, *shift, *run_mean, *run_var;
};

// a BatchNorm backward still to be done: gradient dA of the activated output `out`
struct BnBwdIn {
  const void* dA;
  HView out;
  const float *gamma, *mean, *invstd;
  float *g_gamma, *g_beta;
};

struct ConvGeom {
  int N, Hin, Win, Cin, Hout, Wout, Cout, kh, kw, stride, ph, pw;
};

// Launch shape for kernels that walk a [M][C] tensor by rows, 8 channels per thread.
struct RowTile {
  int W;                  // column groups handled by one block
  int R;                  // rows handled per block iteration
  int nslab;              // grid.y
  size_t rows_per_block;
  int P;                  // grid.x = number of row chunks = number of partials
};
RowTile make_rowtile(size_t M, int C, int max_partials);
enum { kMaxPartials = 512 };
// row-streaming BatchNorm reductions: more, shorter blocks (occupancy); each block covers >= kBnMinRows rows so
// the partials stay small next to the tensor
enum { kBnPartials = 512, kBnMinRows = 32 };

// ---- BatchNorm ---------------------------------------------------------------
// partial[P][2][C] <- per-chunk sums of z and z*z
void bn_stats(int dt, hipStream_t st, const void* z, size_t M, int C, float* partial, int* P_out);
// mean/invstd/scale/shift (each [C]) from the partials; updates running stats
void bn_finalize(hipStream_t st, const float* partial, int P, size_t M, int C, const float* gamma,
                 const float* beta, float* mean, float* invstd, float* scale, float* shift,
                 float* run_mean, float* run_var, float eps, float momentum);
// partial[P][2][C] <- sums of dY and dY*z with dY = dA * act'(scale*z+shift)
void bn_bwd_reduce(int dt, hipStream_t st, const void* dA, const void* z, size_t M, int C,
                   const float* scale, const float* shift, int act, float* partial, int* P_out);
// g_gamma += dgamma, g_beta += dbeta; coef[3][C] for dz = k1*dY + k2*z + k3
void bn_bwd_finalize(hipStream_t st, const float* partial, int P, size_t M, int C, const float* gamma,
                     const float* mean, const float* invstd, float* g_gamma, float* g_beta, float* coef);
// dz (may alias dA) = k1*dA*act'(y) + k2*z + k3
void bn_bwd_apply(int dt, hipStream_t st, const void* dA, const void* z, size_t M, int C,
                  const float* scale, const float* shift, int act, const float* coef, void* dz);
// the three steps above in one launch for short tensors (bn_bwd_small_ok); dz must not alias dA
int bn_bwd_small_ok(size_t M, int C);
void bn_bwd_small(int dt, hipStream_t st, const void* dA, const void* z, size_t M, int C, const float* scale,
                  const float* shift, int act, const float* gamma, const float* mean, const float* invstd,
                  float* g_gamma, float* g_beta, void* dz);
// out = act(scale*z+shift) (+ res)
void bn_apply(int dt, hipStream_t st, HView in, size_t M, int C, const void* res, void* out);

// finalize the pending statistics of z and write act(scale*z+shift) (+ res), one launch, short tensors
int bn_finalize_apply_small_ok(size_t M, int C);
void bn_finalize_apply_small(int dt, hipStream_t st, const BnPending& pend, const void* z, size_t M, int C, int act, float eps,
                             float momentum, const void* res, void* out);

// ---- pooling, loss, optimiser ---------------------------------------------------
void gap_fwd(int dt, hipStream_t st, HView in, int N, int HW, int C, void* out);
void gap_bwd(int dt, hipStream_t st, const void* dOut, int N, int HW, int C, void* dIn);
// per-row loss into row_loss[B], dlogits[B][classes] = (softmax - onehot)/B, then mean into *loss
void softmax_ce(int dt, hipStream_t st, const void* logits, const int32_t* labels, int B, int classes,
                float* row_loss, void* dlogits, float* loss);
// g_bias[j] += sum_b d[b][j]
void bias_grad(int dt, hipStream_t st, const void* d, int B, int Nout, float* g_bias);
// g += wd*w; v = mu*v+g; w -= lr*v; g = 0; optional working copy w_lp (bfloat16)
void sgd_update(hipStream_t st, float* w, float* g, float* v, void* w_lp, size_t n, float lr, float mu,
                float wd);
// weight aggregation: w = mean of up to 8 stashed versions (fp32, summed in order), optional bfloat16 copy
struct AggSources { const float* p[8]; };
void aggregate_weights(hipStream_t st, float* w, void* w_lp, const AggSources& src, int n, size_t count);
void fill_zero(hipStream_t st, void* p, size_t bytes);
void calibration_copy(hipStream_t st, const void* src, void* dst, size_t bytes);
void f32_to_storage(int dt, hipStream_t st, const float* src, void* dst, size_t n);

// ---- generic small dense convolution (stem 3x3, conv1d) ---------------------------
int conv_direct_supported(const ConvGeom& g);
void conv_direct_fwd(int dt, hipStream_t st, HView in, const void* w, const ConvGeom& g, void* z);
// many pixels, few taps: im2col + GEMM with the BatchNorm statistics in its epilogue (conv_direct_gemm_ok);
// im2col: conv_direct_im2col_elems(g) elements, wpad: conv_direct_gemm_wpad_elems(g) elements of scratch
int conv_direct_gemm_ok(const ConvGeom& g);
size_t conv_direct_gemm_wpad_elems(const ConvGeom& g);
void conv_direct_fwd_gemm(int dt, hipStream_t st, HView in, const void* w, const ConvGeom& g, void* im2col, void* wpad, void* z,
                          float* stats, int* P_out);
void conv_direct_dgrad(int dt, hipStream_t st, const void* dz, const void* w, const ConvGeom& g, void* dIn);
// stride-1 data gradient as im2col(dz) x flipped weights on the GEMM (conv_direct_dgrad_gemm_ok); scratch sizes in elements
int conv_direct_dgrad_gemm_ok(const ConvGeom& g);
size_t conv_direct_dgrad_gemm_im2col_elems(const ConvGeom& g);
size_t conv_direct_dgrad_gemm_w_elems(const ConvGeom& g);
void conv_direct_dgrad_gemm(int dt, hipStream_t st, const void* dz, const void* w, const ConvGeom& g, void* im2col, void* wscratch,
                            void* dIn);
// g_w[Cout][kh][kw][Cin] += dW; im2col: scratch of conv_direct_im2col_elems(g) activation elements
size_t conv_direct_wgrad_ws(const ConvGeom& g);  // floats of workspace needed
size_t conv_direct_im2col_elems(const ConvGeom& g);
// patches_ready: im2col already holds this layer's patch matrix (left there by conv_direct_fwd_gemm on the same input)
void conv_direct_wgrad(int dt, hipStream_t st, const void* dz, HView in, const ConvGeom& g, void* im2col, float* ws,
                       float* g_w, bool patches_ready = false);
// g[(j % C) * stride_c + (j / C) * stride_q] += sum_p ws[p * QC + j]; columns j % C >= valid_c skipped (-1: none)
void reduce_partials(hipStream_t st, const float* ws, int P, size_t QC, int C, size_t stride_q, size_t stride_c,
                     float* g, int valid_c = -1);

// ---- depthwise 3x3 ----------------------------------------------------------------
// stats != nullptr (only if dw_fwd_stats_ok): the kernel also writes the BatchNorm partial sums [*P_out][2][C] of z
int dw_fwd_stats_ok(int dt, const ConvGeom& g);
void dw_fwd(int dt, hipStream_t st, HView in, const void* w, const ConvGeom& g, void* z, float* stats = nullptr,
            int* P_out = nullptr);
// convolution + BatchNorm statistics + finalize in one launch for short tensors (dw_fwd_bn_small_ok)
int dw_fwd_bn_small_ok(const ConvGeom& g);
// pend.partial != nullptr: the BatchNorm of the input is still partial sums (pw_fwd's epilogue); the kernel
// finishes it for the channels it owns (writes the per-channel vectors and the running statistics)
void dw_fwd_bn_small(int dt, hipStream_t st, HView in, const BnPending& pend, const void* w, const ConvGeom& g, const float* gamma,
                     const float* beta, float* mean, float* invstd, float* scale, float* shift, float* run_mean,
                     float* run_var, float eps, float momentum, void* z);
// depthwise dgrad + wgrad + the BatchNorm backward of the layer in front, one launch, short tensors
// (dw_bwd_small_ok): dz_prev = gradient of the raw output of the convolution that feeds `in`
int dw_bwd_small_ok(const ConvGeom& g);
// bo.dA != nullptr: dz is not formed yet; the kernel first runs the BatchNorm backward of the depthwise layer's own
// output (bo: gradient of the activated output, the output view, its BatchNorm vectors and gradient slots)
void dw_bwd_small(int dt, hipStream_t st, const void* dz, const BnBwdIn& bo, const void* w, HView in, const ConvGeom& g,
                  const float* gamma, const float* mean, const float* invstd, float* g_w, float* g_gamma, float* g_beta,
                  void* dz_prev);
// sums != nullptr (only if dw_dgrad_sums_ok and prev is a view): the kernel also leaves the partial sums
// [*P_out][2][C] that bn_bwd_reduce would compute for the BatchNorm + activation `prev` in front of this layer
int dw_dgrad_sums_ok(int dt, const ConvGeom& g);
void dw_dgrad(int dt, hipStream_t st, const void* dz, const void* w, const ConvGeom& g, void* dIn, HView prev = HView{},
              float* sums = nullptr, int* P_out = nullptr);
size_t dw_wgrad_ws(const ConvGeom& g);
void dw_wgrad(int dt, hipStream_t st, const void* dz, HView in, const ConvGeom& g, float* ws, float* g_w);

// ---- pointwise / fully connected GEMMs (MFMA) ---------------------------------------
// Z[M][N] = A'[M][K] * W[N][K]^T (+ bias[N]); when stats != nullptr also writes the per-column
// partial sums stats[P][2][N] of the stored Z and Z*Z (same layout as bn_stats), P into *P_out
void pw_fwd(int dt, hipStream_t st, HView a, const void* w, const float* bias, size_t M, int K, int N,
            void* z, float* stats, int* P_out);
// dA[M][K] = dZ[M][N] * W[N][K] (+ res[M][K])
void pw_dgrad(int dt, hipStream_t st, const void* dz, const void* w, const void* res, size_t M, int K,
              int N, void* dA);
// g_w[N][K] += dZ[M][N]^T * A'[M][K]
size_t pw_wgrad_ws(size_t M, int K, int N);
// K_out >= 0: g_w is [N][K_out] and the last K - K_out columns of A are zero padding
void pw_wgrad(int dt, hipStream_t st, const void* dz, HView a, size_t M, int K, int N, float* ws,
              float* g_w, int K_out = -1);

// Narrow-to-wide pointwise layer (K inputs, N >= 2K outputs, bfloat16, input stored activated), whole backward behind
// the BatchNorm reductions in one pass: dz = k1*dA*act'(out) + k2*z + k3 formed per row tile on chip,
// dIn = dz * W (+ res), g_w += dz^T * A.  coef: [3][N] from bn_bwd_finalize.  ws: pw_bwd_fused_ws(M, K, N) floats.
// The kernel's partial weight gradients are summed on st_sum; if that is not st, ev_sum orders the sum behind the kernel.
int pw_bwd_fused_ok(int dt, size_t M, int K, int N, HView a);
size_t pw_bwd_fused_ws(size_t M, int K, int N);
void pw_bwd_fused(hipStream_t st, const void* dA, HView out, const float* coef, const void* w, const void* a_in,
                  const void* res, size_t M, int K, int N, float* ws, float* g_w, void* dIn, hipStream_t st_sum,
                  hipEvent_t ev_sum);


// bfloat16 pointwise layers with a long reduction (>= 192) and 2 K - 64 K rows: forward (A' * W^T, BatchNorm partial sums
// as pw_fwd leaves them) and data gradient (dZ * W (+ res)) on 2 x 2 wavefront tiles of 16x16x32 MFMAs; pw_fwd and
// pw_dgrad dispatch to them.  R = reduction extent, NC = output columns.
int pw_deep_ok(int dt, size_t M, int R, int NC, bool dgrad);
void pw_fwd_deep(hipStream_t st, HView a, const void* w, size_t M, int K, int N, void* z, float* stats, int* P_out);
void pw_dgrad_deep(hipStream_t st, const void* dz, const void* w, const void* res, size_t M, int K, int N, void* dA);
// the weight gradient for bfloat16 layers with more than 2048 rows: operands staged untransposed, transposed on the
// way out of LDS (pw_wgrad dispatches to it; ws: pw_wgrad_tr_ws floats)
int pw_wgrad_tr_ok(int dt, size_t M, int K, int N);
size_t pw_wgrad_tr_ws(size_t M, int K, int N);
void pw_wgrad_tr(hipStream_t st, const void* dz, HView a, size_t M, int K, int N, float* ws, float* g_w, int K_out);

// wgrad (g_w +=) then dgrad (dA =) of one layer on one stream; one launch for short problems
void pw_bwd(int dt, hipStream_t st, const void* dz, const void* w, const void* res, HView a, size_t M, int K, int N,
            float* ws, float* g_w, void* dA);

}  // namespace ftp
