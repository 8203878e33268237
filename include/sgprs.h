/*
 * sgprs.h -- C ABI of the MI355X (gfx950) stage-computation library under SGPRS.
 *
 * SGPRS (the paper's "Task Model" and "Real-Time Scheduler Design" sections)
 * splits each periodic DNN task tau_i into stages tau_i^j and runs the stages
 * on a context pool CP = {cp_1 .. cp_np} of n_p spatial GPU partitions with a
 * fixed number of compute units each.  This library is the part the
 * partitions execute: the pool itself (CU-masked HIP streams) and the six
 * stages of the paper's benchmark task, ResNet18 on a 224x224 input
 * ("Simulation Results"), as hand-written HIP kernels.  The scheduler that
 * decides which stage goes to which partition is host logic at the end of this
 * header (sgprs_sched_*); it launches nothing by itself.
 *
 * Conventions
 *  - Every call returns an int status: SGPRS_OK (0) or a negative SGPRS_ERR_*.
 *    Nothing throws across the ABI.  sgprs_last_error() gives a thread-local
 *    text for the last failure on the calling thread.
 *  - Handles (sgprs_pool_t, sgprs_task_t) are opaque, owned by the library,
 *    released by the matching *_destroy.
 *  - "DEVICE" pointers are device memory owned by the caller (for instance
 *    torch.Tensor.data_ptr()); they must stay valid until the partition the
 *    work was queued on has been synchronised.  "HOST" pointers are ordinary
 *    host memory, read or written before the call returns.
 *  - All *_run and per-operator calls only ENQUEUE work on the partition's
 *    stream and return; arguments are validated first, so a failing call
 *    enqueues nothing.
 *  - Activation layout is NHWC (channels fastest) in the call's dtype.
 *    SGPRS_BF16 means bf16 storage with fp32 accumulation and an fp32
 *    epilogue; results are rounded to bf16 (nearest, ties to even) on store.
 *  - A CU mask never changes results, only speed: for a given tensor shape the
 *    arithmetic order depends on the partition's CU count only through the
 *    split-K factor, whose second pass sums in a fixed order.
 */
#ifndef SGPRS_H
#define SGPRS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sgprs_pool sgprs_pool_t;
typedef struct sgprs_task sgprs_task_t;

typedef enum { SGPRS_F32 = 0, SGPRS_BF16 = 1 } sgprs_dtype_t;

enum {
    SGPRS_OK = 0,
    SGPRS_ERR_INVALID_ARG = -1,
    SGPRS_ERR_NO_DEVICE = -2,
    SGPRS_ERR_HIP = -3,
    SGPRS_ERR_OOM = -4,
    SGPRS_ERR_UNSUPPORTED = -5,
    SGPRS_ERR_OVERSUBSCRIBED = -6
};

/* pool flags */
enum {
    SGPRS_POOL_OVERSUBSCRIBE = 1u, /* allow n_p * cus > total CUs: masks wrap and overlap */
    SGPRS_POOL_BLOCKED_LAYOUT = 2u /* mask bit = xcd * cus_per_xcd + cu instead of the
                                      default cu * n_xcd + xcd (see sgprs_build_cu_mask) */
};

#define SGPRS_MAX_MASK_WORDS 16 /* 512 CUs */
#define SGPRS_RESNET18_CONVS 20
#define SGPRS_RESNET18_STAGES 6

const char *sgprs_status_string(int status);
const char *sgprs_last_error(void);
/* major*10000 + minor*100 + patch */
int sgprs_version(void);

/* ------------------------------------------------------------------ pool --
 * Context pool CP of the paper's task model: n_p partitions, each restricted
 * to `cus_per_partition` compute units through hipExtStreamCreateWithCUMask.
 * The paper's "sm SMs for each" context becomes "cus CUs for each" stream.
 * Over-subscription (sum of partition sizes above the GPU's CU count, the
 * paper's SGPRS_os variants) needs SGPRS_POOL_OVERSUBSCRIBE. */

/* HOST-only helper, needs no GPU.  Fills `words` (n_words uint32, bit i of the
 * whole vector = CU-mask bit i) with the mask of partition `partition`.
 * Every partition takes cus/n_xcd CUs on EACH of the n_xcd accelerator dies,
 * slots [partition*cus/n_xcd, (partition+1)*cus/n_xcd) modulo the die's CU
 * count, so that the hardware's round-robin of workgroups over dies stays
 * balanced.  blocked_layout selects how (die, slot) maps to a bit.
 * Errors: INVALID_ARG if total_cus % n_xcd, cus % n_xcd, cus outside
 * [n_xcd, total_cus], partition < 0, or n_words too small. */
int sgprs_build_cu_mask(int total_cus, int n_xcd, int cus, int partition, int blocked_layout,
                        uint32_t *words, int n_words);

/* Creates n_p partitions of cus_per_partition CUs on `device`.  cus must be a
 * multiple of the die count.  NO_DEVICE if there is no usable GPU,
 * OVERSUBSCRIBED if n_p*cus exceeds the device without the flag. */
int sgprs_pool_create(int device, int n_p, int cus_per_partition, unsigned flags,
                      sgprs_pool_t **out);
/* Same with caller-chosen masks: masks[p*words_per_mask .. +words_per_mask) HOST.
 * Mask bit i selects a CU of die i % n_xcd; INVALID_ARG for a mask that selects
 * no CU at all or leaves one of the dies without a CU (workgroups are handed to
 * the dies in turn, so such a stream could not run). */
int sgprs_pool_create_masks(int device, int n_p, const uint32_t *masks, int words_per_mask,
                            sgprs_pool_t **out);
/* Synchronises and destroys all partition streams. */
int sgprs_pool_destroy(sgprs_pool_t *pool);
/* Any output pointer may be NULL. */
int sgprs_pool_info(const sgprs_pool_t *pool, int *n_p, int *cus_per_partition, int *total_cus,
                    int *n_xcd);
/* Number of CUs in one partition's mask. */
int sgprs_pool_partition_cus(const sgprs_pool_t *pool, int partition, int *cus);
int sgprs_pool_get_mask(const sgprs_pool_t *pool, int partition, uint32_t *words, int n_words);
/* The partition's hipStream_t (for events or torch.cuda.ExternalStream); NULL on error. */
void *sgprs_pool_stream(const sgprs_pool_t *pool, int partition);
int sgprs_partition_sync(sgprs_pool_t *pool, int partition);
int sgprs_pool_sync(sgprs_pool_t *pool);
/* Diagnostic: runs `n_blocks` (<= 65536) one-wave workgroups on the partition,
 * each spinning ~spin_cycles clock ticks, and records where each ran:
 * out[2*b] = accelerator die id, out[2*b+1] = hardware id register (CU, shader
 * array and engine fields).  out: DEVICE uint32[2*n_blocks].  Used to check
 * the mask-bit -> die mapping by measurement. */
int sgprs_partition_probe(sgprs_pool_t *pool, int partition, int n_blocks, int spin_cycles,
                          uint32_t *out);
/* Diagnostic: the same probe, but recorded into a HIP graph by stream capture
 * and launched as a graph on the partition's stream (synchronous).  Shows
 * whether graph launches keep to the partition's CUs, which sgprs_task_run
 * relies on when it replays a captured task. */
int sgprs_partition_probe_graph(sgprs_pool_t *pool, int partition, int n_blocks, int spin_cycles,
                                uint32_t *out);
/* Diagnostic: the sustained matrix-core rate of the partition.  One 512-thread
 * workgroup per CU runs `steps` (1..1e6) rounds of 18 k-steps; per k-step every
 * wavefront reads four 16-byte fragments per lane from LDS and issues four
 * MFMA 32x32x16 bf16 (the inner loop of the 3x3 convolution kernel without its
 * global loads): 2 * 32*32*16 * 4 * 18 * 8 * steps FLOP per CU.  random_data
 * != 0 fills the fragments with pseudo-random bf16 values instead of 1.0 (the
 * clock the chip sustains depends on it).  out: DEVICE uint64[3], written by
 * workgroup 0: elapsed ticks of the 100 MHz constant-rate counter, elapsed
 * shader clocks, a checksum.  Time the launch with events on the partition's
 * stream for the aggregate rate. */
int sgprs_mfma_probe(sgprs_pool_t *pool, int partition, int random_data, int steps, uint64_t *out);
/* Diagnostic: the sustained rate of the load path the convolution kernels use
 * (16-byte buffer loads straight into LDS).  One 512-thread workgroup per CU
 * reads 64 KiB per iteration, `iters` (1..1e6) times, cycling through its own
 * region of region_bytes (a power of two, 16 KiB..1 GiB) of buf: workgroup b
 * uses buf + (b * region_bytes) % buf_bytes (buf DEVICE, 16-byte aligned,
 * buf_bytes a multiple of region_bytes).  With all regions together inside the
 * L2s this measures L2 -> LDS, with more it measures what lies behind them.
 * out: DEVICE uint32[CUs of the partition]; workgroup b writes the sum of the
 * 16384 32-bit words its last iteration left in LDS.  Moves CUs * iters *
 * 65536 bytes; time the launch with events on the partition's stream. */
int sgprs_load_probe(sgprs_pool_t *pool, int partition, const void *buf, size_t buf_bytes,
                     size_t region_bytes, int iters, uint32_t *out);

/* -------------------------------------------------------- per-operator ----
 * The operators of the paper's "GPU Speedup Analysis": convolution, max
 * pooling and the remaining ResNet18 operations.  All tensors DEVICE, NHWC. */

typedef struct {
    int n, h, w;        /* batch, input height, width */
    int cin, cout;      /* channels */
    int r, s;           /* kernel height, width (r == s: 1, 3 or 7) */
    int stride, pad;
    int dtype;          /* sgprs_dtype_t */
    int relu;           /* 1: ReLU after scale/shift(+residual) */
} sgprs_conv_desc_t;

/* HOST helper: folded inference BN, scale = gamma/sqrt(var+eps),
 * shift = beta - mean*scale, computed in fp64, returned as fp32. */
int sgprs_fold_bn(const float *gamma, const float *beta, const float *mean, const float *var,
                  float eps, int c, float *scale, float *shift);
/* HOST helpers: size of, and conversion to, the packed weight layout the conv
 * kernels read.  w_oihw: [cout][cin][r][s] fp32.  Packed: [cout][K'] in the
 * call's dtype (bf16 rounded to nearest even), K' ordered (r, s, c) for
 * cin % 32 == 0, and a zero-padded 7 x 32 tap-row layout for the 3-channel
 * 7x7 stride-2 stem.  UNSUPPORTED for any other shape. */
int sgprs_conv_packed_weight_bytes(const sgprs_conv_desc_t *d, size_t *bytes);
int sgprs_pack_conv_weights(const sgprs_conv_desc_t *d, const float *w_oihw, void *w_packed,
                            size_t bytes);
int sgprs_unpack_conv_weights(const sgprs_conv_desc_t *d, const void *w_packed, size_t bytes,
                              float *w_oihw);
/* Split-K scratch needed on a partition of partition_cus CUs (0 when the
 * launch is not split). */
int sgprs_conv2d_workspace(const sgprs_conv_desc_t *d, int partition_cus, size_t *bytes);
/* Which kernel sgprs_conv2d would launch for this shape on a partition of
 * partition_cus CUs, with or without a residual (host logic only, nothing is
 * enqueued).  family: 0 implicit GEMM, 1 LDS-patch 3x3, 2 stride-2 LDS-patch
 * 3x3, 3 row-streaming 3x3 (64 -> 64 channels, 56-pixel rows), 4 the 7x7 stem;
 * detail: the tile variant, or the output rows per stream and job of family 3. */
int sgprs_conv2d_plan(const sgprs_conv_desc_t *d, int partition_cus, int has_residual, int *family,
                      int *detail);
/* y = act( scale[k] * conv(x, w)[.,k] + shift[k] (+ residual) ).
 * x: [n][h][w][cin]; w_packed: DEVICE copy of the packed weights; scale, shift:
 * DEVICE fp32[cout]; residual: NULL or [n][p][q][cout] in dtype; y: same shape.
 * workspace: DEVICE, at least sgprs_conv2d_workspace() bytes (may be NULL if 0).
 * x, residual and y must not overlap. */
int sgprs_conv2d(const sgprs_conv_desc_t *d, const void *x, const void *w_packed,
                 const float *scale, const float *shift, const void *residual, void *y,
                 void *workspace, size_t workspace_bytes, sgprs_pool_t *pool, int partition);
/* Measurement hook, process-wide (atomic settings, read by every thread that plans a
 * launch; launches already planned keep their plan): which convolution kernel
 * sgprs_conv2d and the stages pick for 3x3 bf16 layers.  kind -1: automatic
 * (default); 0: implicit GEMM only; 1: the stride-1 LDS-patch kernel with the
 * given tile variant (0..4) and split factor where the shape allows it; 2:
 * automatic, but implicit-GEMM launches use tile variant `variant` (0..3)
 * wherever it divides cout, with split-K factor `splits` (0: planner's choice);
 * 3: automatic, plus the stride-2 LDS-patch kernel (not chosen otherwise) with
 * tile variant `variant` (0: 256 rows, 1: 128 rows) wherever the shape allows
 * it; variant 2 switches it off again; 4: automatic, but stage 0 of a bf16
 * task uses the 4-slot stem+pool kernel instead of the packed-row one; 5:
 * automatic, but without the row-streaming kernel of the 64 -> 64 layers. */
int sgprs_conv_tuning_override(int kind, int variant, int splits);
/* Max pooling 3x3, stride 2, pad 1 (padding never wins): [n][h][w][c] ->
 * [n][(h-1)/2+1][(w-1)/2+1][c].  c % 8 == 0 (bf16) or c % 4 == 0 (fp32). */
int sgprs_maxpool2d(int dtype, int n, int h, int w, int c, const void *x, void *y,
                    sgprs_pool_t *pool, int partition);
/* y = max(0, scale[c]*x + shift[c]) over `pixels` rows of c channels. */
int sgprs_bn_relu(int dtype, size_t pixels, int c, const void *x, const float *scale,
                  const float *shift, void *y, sgprs_pool_t *pool, int partition);
/* y = a + b, followed by ReLU if relu != 0; `count` elements (multiple of 8). */
int sgprs_add_relu(int dtype, size_t count, const void *a, const void *b, void *y, int relu,
                   sgprs_pool_t *pool, int partition);
/* Global average pool over hw positions, then FC: x [n][hw][cin] (dtype),
 * w [cout][cin] (dtype, DEVICE), bias NULL or fp32[cout], logits fp32 [n][cout].
 * workspace: DEVICE fp32[n*cin] for the pooled vectors.  cin is 512, 1024 or 2048.
 * Up to 8 images with cin 512 or 1024 take one fused launch that leaves the
 * workspace untouched; its logits are bit-identical to the two-kernel path's. */
int sgprs_avgpool_fc(int dtype, int n, int hw, int cin, int cout, const void *x, const void *w,
                     const float *bias, float *logits, float *workspace, sgprs_pool_t *pool,
                     int partition);
/* Global average pool alone (paper: the average-pooling row of the GPU speedup
 * analysis): pooled[n][c] = mean over the hw positions of x[n][hw][c], fp32,
 * summed in a fixed order (the first half of sgprs_avgpool_fc, same kernels,
 * same bits as its workspace).  c in {512, 1024, 2048}; x and pooled DEVICE,
 * 16-byte aligned, distinct.  UNSUPPORTED beyond 65535 images or 2^31 elements. */
int sgprs_global_avgpool(int dtype, int n, int hw, int c, const void *x, float *pooled,
                         sgprs_pool_t *pool, int partition);

/* The same operator for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  The pooled vectors go to a 512 KiB array that is part of
 * the library's device image (one copy per GPU, held until the process ends);
 * its address is looked up on the first call on a device, and no call
 * allocates or frees anything.  n * cin must not exceed 131072 (64 * 2048)
 * values: UNSUPPORTED beyond that.  Every call on a GPU shares that GPU's
 * array, which keeps the last call's contents: calls that overlap in time on
 * one GPU (different partitions, or threads) race on it, so serialise them.
 * Nothing in it needs clearing: each call overwrites the n * cin values it
 * reads.  Logits are bit-identical to sgprs_avgpool_fc's. */
int sgprs_avgpool_fc_static(int dtype, int n, int hw, int cin, int cout, const void *x,
                            const void *w, const float *bias, float *logits, sgprs_pool_t *pool,
                            int partition);

/* ------------------------------------------------------------------ task --
 * Task tau_i = one ResNet18 instance, split into the paper's six stages:
 *   0 conv7x7/2+BN+ReLU+maxpool3x3/2, 1..4 layer1..layer4 (two BasicBlocks
 *   each, 1x1/2 projection shortcut at the head of layers 2-4), 5 global
 *   average pool + FC.
 * Creating a task is the offline phase: BN folding, rounding to dtype, weight
 * packing and upload happen there. */

typedef struct {
    /* HOST fp32, forward order: stem; layer1.{0,1}.conv{1,2}; then for layers
     * 2..4: L.0.conv1, L.0.conv2, L.0.downsample, L.1.conv1, L.1.conv2 */
    const float *conv_w[SGPRS_RESNET18_CONVS]; /* OIHW */
    const float *bn_gamma[SGPRS_RESNET18_CONVS];
    const float *bn_beta[SGPRS_RESNET18_CONVS];
    const float *bn_mean[SGPRS_RESNET18_CONVS];
    const float *bn_var[SGPRS_RESNET18_CONVS];
    const float *fc_w; /* [1000][512] */
    const float *fc_b; /* [1000] or NULL */
    float bn_eps;
} sgprs_resnet18_params_t;

/* Allocates device weights and an activation workspace for up to max_batch
 * images.  A task is not re-entrant: one run in flight at a time. */
int sgprs_task_create_resnet18(int device, int dtype, int max_batch,
                               const sgprs_resnet18_params_t *host_params, sgprs_task_t **out);
int sgprs_task_destroy(sgprs_task_t *task);
/* Number of stages (6), or a negative status. */
int sgprs_task_num_stages(const sgprs_task_t *task);
/* Byte sizes and logical N,C,H,W of a stage's input and output at `batch`.
 * Stage 5's output is fp32 [batch][1000] whatever the dtype.  Outputs nullable. */
int sgprs_task_stage_io(const sgprs_task_t *task, int stage, int batch, size_t *in_bytes,
                        size_t *out_bytes, int in_nchw[4], int out_nchw[4]);
/* Stage tau_i^j on partition cp_p: in/out DEVICE, NHWC in the task's dtype. */
int sgprs_stage_run(sgprs_task_t *task, int stage, int batch, const void *in, void *out,
                    sgprs_pool_t *pool, int partition);
/* All six stages in order.  partition_per_stage == NULL: all on `partition`;
 * otherwise HOST int[6] and consecutive stages on different partitions are
 * chained with events.  in: [batch][224][224][3]; logits: fp32 [batch][1000].
 * The call returns once everything is queued; completion is observed on the
 * last stage's partition.  When all stages run on one partition, per-kernel
 * timing is off and graph replay applies (sgprs_task_set_graph_replay), the
 * second call with the same (batch, in, logits, pool, partition) records the
 * kernels into a HIP graph and later calls replay it:
 * one host call per inference.  The buffers are read and written at replay
 * time as usual; only the pointers are fixed. */
int sgprs_task_run(sgprs_task_t *task, int batch, const void *in, float *logits,
                   sgprs_pool_t *pool, int partition, const int *partition_per_stage);
/* DEVICE pointer to the task-owned buffer holding stage j's output (j in 0..4)
 * after sgprs_task_run; NULL on error. */
const void *sgprs_task_stage_output(const sgprs_task_t *task, int stage);
/* Per-kernel timing for measurement.  With profiling on, every kernel launch
 * of a stage is bracketed by events on the partition stream (this adds
 * latency; keep it off when timing throughput).  After synchronising,
 * sgprs_task_kernel_times returns, for the last run of each stage, one record
 * per launch: HOST arrays of length *count (in: capacity).  kind: 0 conv
 * implicit GEMM, 1 stem conv, 2 split-K reduce, 3 max-pool, 4 avg-pool, 5 FC
 * (variant 2, 3: avg-pool and FC in one launch; 4: the FC on the matrix cores),
 * 6 BN+ReLU, 7 add+ReLU, 8 LDS-patch 3x3 conv, 9 fused stem conv + max-pool
 * (variant 2: the bf16 kernel with packed input rows),
 * 10 two implicit-GEMM convolutions of one input in a single launch, 11 the
 * stride-2 LDS-patch 3x3 conv (variant + 4: together with the 1x1 shortcut),
 * 12 the row-streaming 3x3 conv of the 64 -> 64 layers.
 * flops/bytes are the algorithmic work of the launch. */
int sgprs_task_set_profiling(sgprs_task_t *task, int on);
/* Graph replay of sgprs_task_run (see there): mode 1 always, 0 never (every
 * call enqueues its kernels one by one), -1 automatic (default): batches of up
 * to 8 images.  A replay costs about 5 us of GPU time and saves 50-90 us of
 * host time: it pays when one host thread feeds several partitions with short
 * inferences.  Graphs already captured are kept. */
int sgprs_task_set_graph_replay(sgprs_task_t *task, int mode);
int sgprs_task_kernel_times(sgprs_task_t *task, int stage, int *count, int *kind, int *variant,
                            float *ms, double *flops, double *bytes);
/* Name of the kernel instantiation behind (kind, variant), for matching
 * profiler rows; points into a small ring of static buffers (copy it before
 * asking for more than eight names). */
const char *sgprs_kernel_name(int kind, int variant);

/* ------------------------------------------------------------ scheduler --
 * The paper's scheduler ("Real-Time Scheduler Design"), host logic only: it
 * launches nothing and reads no clock; the caller reports releases and
 * completions with their times (seconds, any origin) and asks which stage may
 * start.  Not thread-safe: one thread drives one scheduler.
 *
 * Offline phase, at sgprs_sched_add_task ("Two Level Priority Assignment",
 * "WCET and Virtual Deadline Assignment"): the last stage of a task is high
 * priority, the others low; stage j's relative deadline is
 * D * C^j / sum_k C^k (C = wcet, D = rel_deadline).
 * Online phase ("Absolute Deadline Assignment", "Context Assignment", "Stage
 * Queuing"): stage j of a job released at r has the absolute deadline
 * r + D^0 + .. + D^j.  On release a stage is assigned to a context: one with an
 * empty queue (waiting or running stages) first; else, among the contexts
 * where now + backlog + C^j <= deadline (backlog = WCETs waiting plus what is
 * left of the running ones), the one with the fewest stages queued; else the
 * one with the smallest backlog; ties to the lowest index.  A context runs up
 * to lanes_per_context stages at once (the paper: 4), the first lanes/2 lanes
 * for high-priority stages, the rest for medium and low ones (one lane: shared
 * by all).  A low-priority stage whose predecessor completed after its
 * deadline is medium.  A free lane takes, of the waiting stages of its class,
 * the highest level, then the earliest deadline, then the earliest release. */
typedef struct sgprs_sched sgprs_sched_t;
typedef struct {
    int task, job, stage;   /* what to run */
    int context, lane;      /* where: lane < lanes_per_context */
    int level;              /* 0 high, 1 medium, 2 low */
    double deadline;        /* absolute */
    double wcet;
} sgprs_dispatch_t;
typedef struct {
    long long jobs_released, jobs_completed, jobs_missed; /* missed: last stage completed after r + D */
    long long stages_completed, stages_missed;
} sgprs_sched_stats_t;

/* n_contexts in [1,64], lanes_per_context in [1,8]. */
int sgprs_sched_create(int n_contexts, int lanes_per_context, sgprs_sched_t **out);
void sgprs_sched_destroy(sgprs_sched_t *sched);
/* wcet: HOST double[n_stages], all > 0 (seconds); period, rel_deadline > 0.
 * *task_id receives the task's index (0, 1, ...). */
int sgprs_sched_add_task(sgprs_sched_t *sched, int n_stages, const double *wcet, double period,
                         double rel_deadline, int *task_id);
/* The task's relative virtual deadlines: HOST double[capacity >= n_stages]. */
int sgprs_sched_virtual_deadlines(const sgprs_sched_t *sched, int task, int capacity, double *out);
/* A job of `task` is released at `now`: its first stage is queued.  *job_id
 * (may be NULL) receives the job's number (0, 1, ... per task). */
int sgprs_sched_release(sgprs_sched_t *sched, int task, double now, int *job_id);
/* Returns 1 and fills *out if a waiting stage may start at `now` (its lane is
 * then busy until sgprs_sched_complete), 0 if none can, < 0 on error.  Call it
 * until it returns 0.  Contexts and lanes are scanned in index order. */
int sgprs_sched_next(sgprs_sched_t *sched, double now, sgprs_dispatch_t *out);
/* The running stage (task, job, stage) completed at `now`: its lane is free,
 * the deadline is checked (*missed, may be NULL: 1 if now > deadline), and the
 * job's next stage, if any, is released at `now`.  Error if it is not running. */
int sgprs_sched_complete(sgprs_sched_t *sched, int task, int job, int stage, double now, int *missed);
int sgprs_sched_get_stats(const sgprs_sched_t *sched, sgprs_sched_stats_t *out);
/* Run loop only (sgprs_sched_run_periodic): at most max_busy lanes have a stage
 * in flight at once; further stages wait in the scheduler's queues even if their
 * lane is free.  Default 4: on MI355X more than four CU-masked streams busy at
 * once cut the throughput of all of them by more than half, whatever their
 * size (idle ones cost nothing).  0: no limit.  The scheduler's decisions
 * (sgprs_sched_next) are not affected. */
int sgprs_sched_set_max_busy(sgprs_sched_t *sched, int max_busy);

/* The periodic-release experiment of "Simulation Results" on the real pool.
 * tasks[i] (HOST array of n_tasks handles, n_tasks = the scheduler's task
 * count, stage counts equal) is the DNN behind the scheduler's task i;
 * inputs[i] / logits[i] are its DEVICE input and fp32 logits buffers for
 * `batch` images.  Lane l of context c is partition c * lanes + l of `pool`,
 * which must have at least n_contexts * lanes partitions (give the lanes of a
 * context the same CU mask; contexts may overlap: an over-subscribed pool).
 * Job k of task i is released at offsets[i] + k * period_i (offsets HOST
 * double[n_tasks] or NULL = 0) while that is < duration_s seconds on the host's
 * steady clock; the calling thread releases jobs, takes the scheduler's
 * decisions and polls one event per lane for completions until every job has
 * finished; the launches themselves (sgprs_stage_run and the event record) are
 * made by one helper thread per lane (up to 16 lanes; beyond that by the calling
 * thread), which the call creates and joins.  A
 * job released while the task's previous job is still in flight is dropped
 * (a task holds one job's activations) and counts as a miss.
 * report: elapsed_s = max(duration_s, time of the last completion), fps =
 * completed jobs / elapsed_s, dmr = (missed + dropped) / releases, response
 * times from release to completion of the last stage.  Blocking; the
 * scheduler must have no job in flight when called. */
typedef struct {
    double elapsed_s;
    long long releases, dropped;
    sgprs_sched_stats_t sched; /* of this run only */
    double fps, dmr;
    double mean_response_s, max_response_s;
} sgprs_run_report_t;
int sgprs_sched_run_periodic(sgprs_sched_t *sched, sgprs_pool_t *pool, sgprs_task_t *const *tasks,
                             int n_tasks, const void *const *inputs, float *const *logits, int batch,
                             const double *offsets, double duration_s, sgprs_run_report_t *report);

/* Static, purely spatial execution of the task model's pool (every task keeps
 * one partition: the comparison shape of "Simulation Results"): task i runs
 * `rounds` inferences of `batch` images on partition partition_of_task[i]
 * (HOST int[n_tasks]) through sgprs_task_run; inputs[i] / logits[i] DEVICE as
 * there.  The calling thread hands out one inference at a time per task,
 * round-robin, keeps at most max_busy partitions busy at once (0: no limit; see
 * sgprs_sched_set_max_busy for why 4 is the useful value on MI355X), and polls
 * one event per task.  Blocking; *elapsed_s (may be NULL) receives the wall time
 * from the first launch to the last completion.  Tasks sharing a partition run
 * one after the other. */
int sgprs_pool_run_static(sgprs_pool_t *pool, sgprs_task_t *const *tasks, int n_tasks,
                          const void *const *inputs, float *const *logits, int batch,
                          const int *partition_of_task, int rounds, int max_busy, double *elapsed_s);

#ifdef __cplusplus
}
#endif
#endif /* SGPRS_H */
