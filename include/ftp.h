/*
 * ftp.h — C ABI of the MI355X stage-training library.
 *
 * One pipeline stage's training step of FTPipeHD: a worker builds the sub-model
 * given by its partition points (paper, section "Initialization"), forwards and
 * backwards batches under the one-forward-one-backward rule with weight
 * stashing (section "Async Pipeline Training"), updates its weights with SGD,
 * momentum and weight decay (section "Experiment Setup"), and the central node
 * profiles per-layer execution time and output size (section "Initialization",
 * model profiling phase) and solves the partition dynamic programme (section
 * "Dynamic Model Partition").
 *
 * Conventions
 *   - Every function returns 0 (FTP_OK) or a negative ftp_status; on error the
 *     outputs are untouched and ftp_last_error() holds a thread-local message.
 *     No C++ exception and no abort crosses this boundary.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host
 *     addresses.  `stream` is a hipStream_t passed as void* (NULL = default
 *     stream).  Compute calls are asynchronous on that stream; import / export /
 *     profile / solve are synchronous.
 *   - The compute calls of one stage share its workspace: issue them in program
 *     order on one stream (or on streams the caller has ordered with events).
 *     A large stage runs its weight gradients on a stream of its own inside
 *     ftp_stage_backward; that work is ordered before anything enqueued on the
 *     caller's stream after the call.  Different stages are independent.
 *   - Activations are NHWC (channels fastest): [batch, H, W, C]; a 1-D window of
 *     T steps is H = 1, W = T.  Their element type is the model's ftp_dtype
 *     (float, or bfloat16 with fp32 accumulation, statistics, gradients of
 *     weights, momentum and master weights).
 *   - The caller owns x / y / dy / dx / labels / loss buffers.  The stage owns
 *     everything that lives between calls (weights, momentum, gradients, BN
 *     running statistics, per-slot stash, workspace) and frees it in
 *     ftp_stage_destroy.
 *   - A partition unit ("layer" in the paper) is the smallest piece a stage
 *     boundary may fall between; a residual connection is never cut.
 */
#ifndef FTP_H
#define FTP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FTP_OK = 0,
  FTP_ERR_ARG = -1,         /* NULL pointer, bad range, bad size              */
  FTP_ERR_SHAPE = -2,       /* unit list does not chain / count mismatch      */
  FTP_ERR_UNSUPPORTED = -3, /* valid request the kernels do not cover         */
  FTP_ERR_SLOT = -4,        /* slot busy on forward / empty on backward       */
  FTP_ERR_VALUE = -5,       /* NaN, infinite or non-positive cost / capacity  */
  FTP_ERR_HIP = -6,         /* HIP runtime failure (message has the detail)   */
  FTP_ERR_NOMEM = -7
} ftp_status;

typedef enum { FTP_F32 = 0, FTP_BF16 = 1 } ftp_dtype;

typedef enum {
  FTP_UNIT_CONV = 0,   /* conv (kh x kw, stride, zero pad) + BatchNorm + act     */
  FTP_UNIT_INVRES = 1, /* inverted residual: [1x1 expand+BN+ReLU6 if expand>1]
                          -> depthwise 3x3 (stride)+BN+ReLU6 -> 1x1 project+BN;
                          adds its input when stride == 1 and cin == cout        */
  FTP_UNIT_GAP = 2,    /* mean over H and W                                      */
  FTP_UNIT_FC = 3,     /* y = x W^T + b                                          */
  FTP_UNIT_LOSS = 4    /* softmax cross-entropy, mean over the batch             */
} ftp_unit_kind;

typedef enum { FTP_ACT_NONE = 0, FTP_ACT_RELU = 1, FTP_ACT_RELU6 = 2 } ftp_act;

typedef struct {
  int32_t kind;          /* ftp_unit_kind                                        */
  int32_t cin, cout;     /* channels in / out (LOSS: cin = cout = classes)       */
  int32_t kh, kw;        /* CONV only                                            */
  int32_t stride;        /* CONV, INVRES                                         */
  int32_t pad_h, pad_w;  /* CONV only                                            */
  int32_t expand;        /* INVRES only: expansion factor t                      */
  int32_t act;           /* CONV only: ftp_act after the BatchNorm               */
} ftp_unit_desc;

/* SGD with momonentum and weight decay: g += wd*w; v = momentum*v + g; w -= lr*v. */
typedef struct { float lr, momentum, weight_decay; } ftp_sgd;

typedef struct ftp_model ftp_model; /* immutable unit list of the whole network  */
typedef struct ftp_stage ftp_stage; /* units [a,b) at one batch size, on one GPU */

const char* ftp_last_error(void);

/* ---- model description ---------------------------------------------------- */

/* The network every worker partitions (section "Initialization": the central node sends the model and the initial
 * partition points; a worker builds its sub-model from layer start_i to layer end_i).  Copies `units` (host, L
 * entries).  in_h/in_w/in_c: shape of the network input.  Channel counts that feed a BatchNorm must be multiples
 * of 8. */
int ftp_model_create(const ftp_unit_desc* units, int L, int in_h, int in_w, int in_c,
                     ftp_dtype act_dtype, ftp_model** out);
void ftp_model_destroy(ftp_model*);
int ftp_model_num_units(const ftp_model*);
/* Shape (H, W, C) of the tensor entering unit `u` (u == L: leaving the last). */
int ftp_model_unit_in_shape(const ftp_model*, int u, int* h, int* w, int* c);
/* Number of fp32 parameters of unit u.  Layout of a unit's parameter vector:
 *   CONV   : w[cout][kh][kw][cin], gamma[cout], beta[cout]
 *   INVRES : (expand > 1: w1[ce][cin], gamma1[ce], beta1[ce],)
 *            wd[ce][3][3], gamma2[ce], beta2[ce], w3[cout][ce], gamma3[cout], beta3[cout]
 *            with ce = cin * expand
 *   FC     : w[cout][cin], b[cout]
 *   GAP, LOSS : none */
int ftp_model_unit_param_count(const ftp_model*, int u, size_t* n);
/* Number of BatchNorm channels of unit u, summed over its BatchNorms in order. */
int ftp_model_unit_bn_channels(const ftp_model*, int u, size_t* n);

/* ---- stage ------------------------------------------------------------------ */

/* The sub-model of one worker (section "Initialization": layers start_i .. end_i of the partition points; section
 * "Async Pipeline Training": stage i of n keeps n-i batches in flight, hence the slots).
 * Builds units [a,b) for `batch` samples with `n_slots` in-flight batches on the
 * current HIP device; allocates all device memory it will ever need.  Weights
 * start at zero (import them), momentum and gradients at zero, BN running mean
 * 0 / variance 1. */
int ftp_stage_create(const ftp_model*, int a, int b, int batch, int n_slots, ftp_stage** out);
/* The same with options.  FTP_STAGE_RECOMPUTE: a slot keeps only the stage input of its batch (and, after
 * ftp_stage_snapshot_weights, its weight version); the intermediates of the batch forwarded last live in one
 * stash that all slots share, and the backward of any other slot first runs the forward again from the kept
 * input with that slot's weights (paper, section "Synchronous Pipeline Parallelism Training": intermediates
 * are thrown away and re-computed when the gradient arrives).  The second forward leaves the BatchNorm running
 * statistics alone, and the kernels being deterministic, a run gives bit for bit the weights of a stage
 * that keeps everything.  Memory: one stash + n_slots inputs instead of n_slots stashes.  With this option
 * ftp_stage_loss(slot) must follow ftp_stage_forward(slot) before any other forward (the logits are not kept),
 * and ftp_stage_export_conv_output sees only the slot forwarded or recomputed last.
 * Unknown flag bits: FTP_ERR_ARG. */
enum { FTP_STAGE_RECOMPUTE = 1 };
int ftp_stage_create_ex(const ftp_model*, int a, int b, int batch, int n_slots, unsigned flags, ftp_stage** out);
void ftp_stage_destroy(ftp_stage*);
/* Device memory, in bytes, that the stage allocated at creation (host pointer out). */
int ftp_stage_device_bytes(const ftp_stage*, size_t* bytes);

/* Weights travel between workers and the central node as per-layer vectors (sections "Weight Replication" and
 * "Fault Tolerance Mechanism": a worker fetches the layers it lacks; here the host side of that exchange).
 * Host <-> device copies of one unit's parameter vector (layout above), its
 * accumulated gradient, its momentum buffer, and its BN running statistics
 * (running_mean then running_var of each BatchNorm in order; 2 * bn_channels). */
int ftp_stage_import_weights(ftp_stage*, int unit, const float* host_w, size_t n);
int ftp_stage_export_weights(const ftp_stage*, int unit, float* host_w, size_t n);
int ftp_stage_export_grads(const ftp_stage*, int unit, float* host_g, size_t n);
int ftp_stage_export_momentum(const ftp_stage*, int unit, float* host_v, size_t n);
int ftp_stage_export_bn_stats(const ftp_stage*, int unit, float* host_s, size_t n);

/* Inspection of a busy slot (between its forward and its backward): the raw
 * output z of convolution number `conv` of `unit` (0-based within the unit, in
 * execution order) converted to float, n = batch*Hout*Wout*Cout values in NHWC
 * order; and that convolution's BatchNorm batch statistics as 4*Cout floats:
 * mean, 1/sqrt(var+eps), scale = gamma/sqrt(var+eps), shift = beta - mean*scale.
 * The value the next layer consumes is act(scale*z + shift).  Synchronous. */
int ftp_stage_export_conv_output(const ftp_stage*, int slot, int unit, int conv, float* host_z, size_t n);
int ftp_stage_export_bn_batch_stats(const ftp_stage*, int slot, int unit, int conv, float* host_s, size_t n);

/* Section "Async Pipeline Training": a worker forwards a batch through its sub-model with its newest weights and
 * passes the result on.  Forward of one batch through units [a,b) with the current weights.
 * x_dev: [batch, H, W, C] of unit a's input, read only, copied into the slot
 * (the stashed stage input).  y_dev: output of the last unit, or NULL; when the
 * stage ends with the LOSS unit, y receives the logits [batch, classes].
 * The slot must be free; it is busy until its backward. */
int ftp_stage_forward(ftp_stage*, int slot, const void* x_dev, void* y_dev, void* stream);

/* Section "Async Pipeline Training": the last stage computes the loss of a batch and starts its backward pass.
 * Stages that end with the LOSS unit: mean cross-entropy of the slot's logits
 * against labels_dev (int32 [batch], 0 <= label < classes) into loss_dev (one
 * float); also seeds the slot's backward so dy_dev may be NULL there. */
int ftp_stage_loss(ftp_stage*, int slot, const int32_t* labels_dev, float* loss_dev, void* stream);

/* The loss of ftp_stage_loss for callers that cannot allocate device memory and have no stage object at hand: code
 * under HIP graph capture, tight serving or evaluation loops, harnesses that forbid hipMalloc.  Same kernels, same
 * results bit for bit; the per-row losses that ftp_stage_loss keeps in memory the stage allocated live in a
 * file-scope device array of FTP_STATIC_LOSS_MAX_BATCH floats (256 KiB per GPU, held until the process ends).
 * logits_dev [batch, classes] and dlogits_dev (same shape, receives (softmax - onehot) / batch) are of `dtype`;
 * labels_dev int32 [batch], 0 <= label < classes (a label outside gives a NaN loss); loss_dev one float.  The caller
 * owns all four buffers.  batch > FTP_STATIC_LOSS_MAX_BATCH: FTP_ERR_ARG, nothing is launched.  Calls no hipMalloc,
 * hipFree or other allocating routine (the first call on a device looks up that device's address of the array);
 * nothing in the array has to be cleared between calls.  All calls on one GPU share the array: calls that may run
 * concurrently there (different streams without an ordering) race on it.  Asynchronous on `stream`. */
#define FTP_STATIC_LOSS_MAX_BATCH 65536
int ftp_softmax_ce_static(const void* logits_dev, const int32_t* labels_dev, int batch, int classes, ftp_dtype dtype,
                          void* dlogits_dev, float* loss_dev, void* stream);

/* Section "Async Pipeline Training" (weight stashing: the backward of a batch uses the weight version its forward
 * used).  Copies the current weights into the slot (weight stashing): the slot's
 * backward then differentiates with respect to that version.  Call it between
 * the slot's forward and the next update.  Without it, backward uses the
 * weights current at that time. */
int ftp_stage_snapshot_weights(ftp_stage*, int slot, void* stream);

/* Weight aggregation (section "Async Pipeline Training": stage i of n has n-i weight
 * versions in use at once and merges them at an interval that is a multiple of
 * n-i).  The live weights become the arithmetic mean, element by element in fp32
 * (summed in the order given, then divided by n), of the versions stashed by
 * ftp_stage_snapshot_weights() in slots[0..n); the bfloat16 working copy is
 * re-derived; momentum, gradients and the snapshots themselves are not touched.
 * `slots` is a host array, 1 <= n <= 8, every listed slot must hold a snapshot
 * (FTP_ERR_SLOT otherwise), a slot may not be listed twice.  Asynchronous on
 * `stream`.  When to call it is the caller's schedule: the paper's example merges
 * the versions of the n-i batches in flight right after the forward that follows
 * every (n-i)-th backward. */
int ftp_stage_aggregate_weights(ftp_stage*, const int* slots, int n, void* stream);

/* Section "Async Pipeline Training": the backward pass of a batch through the sub-model, with the stashed weight
 * version.  Backward of the slot's batch.  dy_dev: gradient of the stage output (same
 * shape and type as y), or NULL after ftp_stage_loss.  dx_dev: receives the
 * gradient of the stage input, or NULL (e.g. a == 0).  Weight gradients are
 * ACCUMULATED into the stage's gradient buffers.  Frees the slot. */
int ftp_stage_backward(ftp_stage*, int slot, const void* dy_dev, void* dx_dev, void* stream);

/* Section "Experiment Setup" (SGD, momentum 0.9, weight decay 4e-5): g += wd*w; v = momentum*v + g; w -= lr*v.
 * One step on all parameters of the stage from the accumulated gradients, which are then zeroed. */
int ftp_stage_update(ftp_stage*, const ftp_sgd* opt, void* stream);

/* ---- profiling and partition ------------------------------------------------ */

/* Model profiling (section "Initialization", model profiling phase: the central node measures the running time
 * of the forward and backward pass of each layer, averaged over ten executions, and the size of each layer's
 * output).  Runs forward and backward of every unit of the whole model on synthetic data `reps` times (the paper
 * uses 10) after 2 discarded warm-up runs, and returns per unit the mean forward+backward time in nanoseconds
 * rounded to an integer value (t_ns, host, [L]) and the output size in bytes (out_bytes, host, [L]).  The
 * per-unit times are measured unit after unit on one stream and then scaled by one common factor so that their
 * sum is the mean forward+backward time of a whole batch under the execution plan training uses (`reps` more
 * runs): ftp_estimate_capacity of this same device on the whole model is then 1.  Synchronous. */
int ftp_profile_layers(const ftp_model*, int batch, int reps, double* t_ns, int64_t* out_bytes,
                       void* stream);

/* Section "Dynamic Model Partition": the dynamic programme A(j, n) over contiguous splits that minimises the slowest
 * stage (base case: the prefix on device 0; recurrence: the last cut, with the optional transfer term and the
 * last-stage time), every layer's time on worker k being its profiled time times the capacity C_k.
 * layer_costs[L] > 0: execution time of each unit
 * on the profiling device; device_capacities[N] > 0: TIME MULTIPLIERS (the
 * paper's computing capacity C_k = worker time / central-node time, so larger =
 * slower; stage k on device k costs C_k * sum of its costs).  Optional
 * out_bytes[L] and bandwidth[N-1] (both non-NULL) add the transfer term
 * 2 * out_bytes[l-1] / bandwidth[k-1] for the cut in front of stage k.
 * bounds[N+1] receives bounds[0] = 0 < ... < bounds[N] = L, stage k = units
 * [bounds[k], bounds[k+1]); *bottleneck (may be NULL) the minimised slowest
 * time.  Every stage is non-empty (N <= L).  Ties: smallest last cut.
 * All host pointers; float64 arithmetic, bit-reproducible. */
int ftp_solve_partition(const double* layer_costs, int L, const double* device_capacities, int N,
                        const double* out_bytes, const double* bandwidth, int32_t* bounds,
                        double* bottleneck);

/* Section "Dynamic Model Partition", capacity equation: a worker's measured stage time divided by the
 * profiling device's time for the same units [start, end] (inclusive). */
int ftp_estimate_capacity(double stage_time, const double* layer_costs, int L, int start, int end,
                          double* capacity);

/* Re-partition schedule (section "Dynamic Model Partition"): *due = 1 when a re-partition follows the
 * batches_done-th trained batch: the first after 10 batches, then every 100 (10, 110, 210, ...). */
int ftp_repartition_due(int64_t batches_done, int* due);

/* Capacities for the next re-partition (capacity equations of the same section).  mean_times[n]: the mean
 * execution time each worker reported for its current stage [bounds_cur[i], bounds_cur[i+1]) in the unit of
 * layer_costs[L]; a value that is not finite and positive means "no report".  capacities[0] = 1.0 (the central
 * node, whose report is not used); capacities[i] = mean_times[i] / sum of layer_costs over worker i's stage; if
 * any worker i >= 1 has no report every capacity is 1.0 (the re-partition then uses the central node's times
 * alone).  All host pointers. */
int ftp_repartition_capacities(const double* mean_times, const double* layer_costs, int L, const int32_t* bounds_cur,
                               int n, double* capacities);

/* Online execution profiling (section "Dynamic Model Partition", execution
 * profiling phase: every worker records the execution time of every batch and
 * reports the average, which becomes the numerator of its capacity).
 * ftp_stage_timing(stage, 1) starts recording, per forwarded batch, the time of
 * its forward plus its backward on the streams they were enqueued on (HIP
 * events; up to 256 batches between reads, later ones are not recorded);
 * ftp_stage_timing(stage, 0) stops and discards.  Switch only while no batch is
 * in flight.  ftp_stage_timing_read waits for the recorded batches, returns their
 * number and the mean forward+backward time in nanoseconds (0 if none), and
 * starts a new window; batches in flight at that moment are left out.  Feed the
 * mean to ftp_estimate_capacity together with the profiled costs of the stage's
 * units.  Off by default: a step then records no events at all. */
int ftp_stage_timing(ftp_stage*, int enable);
int ftp_stage_timing_read(ftp_stage*, double* mean_ns, int* n_batches);

/* Weight redistribution after a re-partition or a single worker failure (the
 * paper's Algorithm "Weight Redistribution", sections "Dynamic Model Partition"
 * and "Fault Tolerance Mechanism"), for the worker that holds stage i_cur of
 * bounds_cur[n_cur+1] and will hold stage i_new of bounds_new[n_new+1] (half-open
 * unit bounds as returned by ftp_solve_partition, same total).  i_fail: index in
 * the CURRENT numbering of the failed worker, or -1 for a plain re-partition.
 * source[j], j = 0 .. bounds_new[i_new+1]-bounds_new[i_new]-1, receives for unit
 * bounds_new[i_new]+j either -1 (the worker holds it already) or the index, in
 * the NEW numbering, of the worker to fetch it from: the current holder, moved
 * up by one if it sat behind the failed worker; the failed worker's chain
 * successor (which now carries the failed index) for a unit of the failed stage;
 * worker 0 (the central node) if the failed stage was the last one.  Host
 * pointers only; no device work. */
int ftp_redistribution_plan(const int32_t* bounds_new, int n_new, const int32_t* bounds_cur, int n_cur, int i_fail,
                            int i_cur, int i_new, int32_t* source);

/* Worker list after failures (section "Fault Tolerance Mechanism": with one failed worker every index greater
 * than its index decreases by one and the smaller ones stay; with several, each failed worker is replaced by the
 * alive workers that follow it, one by one).  worker_ids[n]: the current list (device ids in training order,
 * entry 0 the central node); failed[n_failed]: indices into it, each in 1..n-1 (the central node runs the fault
 * handler and cannot be listed), no index twice.  new_ids (room for n entries) receives the alive entries in
 * their old order and *n_new their number; new_index (n entries, may be NULL) receives for every old index its
 * new index, or -1 for a failed worker.  The index a failed worker had is thereby carried by the alive worker
 * that followed it, which is what ftp_redistribution_plan's `source` refers to.  Host pointers only. */
int ftp_renumber_workers(const int32_t* worker_ids, int n, const int32_t* failed, int n_failed, int32_t* new_ids,
                         int32_t* new_index, int* n_new);

/* Device-side half of the redistribution: copies weights, momentum and BatchNorm
 * running statistics of units [unit_lo, unit_hi) from `src` to `dst` (both
 * stages must contain the range and be built from the same model and type),
 * device to device on `stream`, and refreshes dst's bfloat16 working copy of
 * them.  Pending gradients are not copied. */
int ftp_stage_copy_units(ftp_stage* dst, const ftp_stage* src, int unit_lo, int unit_hi, void* stream);

/* ---- diagnostics ---------------------------------------------------------------- */

/* Per-kernel timing for benchmarks (not part of the paper's method).  Between
 * begin and end every kernel launch of this library is bracketed by HIP events
 * on its own stream; end synchronises the device and returns one row per kernel
 * family: launches, summed duration, summed algorithmic bytes (every operand of
 * a launch counted once) and floating-point operations.  max_launches bounds the
 * event pool; exceeding it makes end return FTP_ERR_ARG with partial rows.  A
 * negative max_launches (pool size = its magnitude) splits the rows further by
 * problem shape: the name then reads "family d0 d1 d2" (GEMMs: M K N).
 * One more row, named "__event_pair_overhead" (launches = 1), gives in total_ms what a pair of events adds
 * to the launch it brackets, measured at begin on empty kernels: take it off every launch's time to get kernel
 * durations comparable with a profiler's.
 * Process-wide, not thread-safe, and the event records slow small steps down. */
typedef struct {
  char name[48];
  int64_t launches;
  double total_ms, alg_bytes, flops;
} ftp_ktrace_row;
int ftp_ktrace_begin(int max_launches);
int ftp_ktrace_end(ftp_ktrace_row* rows, int max_rows, int* n_rows);

/* Test hook for the error path of the compute calls: marks, for the calling thread, a launch plan as failed, exactly
 * as a kernel launcher does when a shape falls outside what its kernel was written for.  The next compute call of
 * this thread (forward, loss, backward, update, aggregate, copy_units) then returns FTP_ERR_UNSUPPORTED with the
 * reason in ftp_last_error() and clears the mark; other threads are not affected. */
int ftp_diag_fail_next_launch_plan(void);

/* Copies `bytes` (a multiple of 16) from src_dev to dst_dev with a plain kernel: a launch of
 * exactly known HBM traffic (bytes read + bytes written) against which hardware traffic counters
 * (rocprofv3 FETCH_SIZE / WRITE_SIZE) are scaled.  Asynchronous on `stream`. */
int ftp_calibration_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FTP_H */
