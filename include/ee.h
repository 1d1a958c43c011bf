/*
 * ee.h -- C ABI of the MI355X (gfx950) early-exit serving library.
 *
 * The library runs the data-parallel hot path of exit-aware batched serving of early-exit
 * CNNs: a backbone segment over a batch of in-flight samples, the exit head after it, the
 * compaction of survivors with refill of the freed batch slots, and the stream driver that
 * strings them together with the paper's exit-aware preemptive scheduler.
 *
 * Conventions for every call
 *   - returns EE_OK (0) or a negative ee_status; never throws, never aborts;
 *   - "device" pointers are GPU global memory owned by the caller (16-byte aligned); "host"
 *     pointers are ordinary process memory; "device-visible" means either device memory or
 *     pinned host memory;
 *   - device work is enqueued on the HIP stream given to ee_create and is asynchronous unless
 *     stated otherwise: device outputs are valid once the caller has synchronised that stream;
 *   - no device or pinned memory is allocated after ee_create (ee_lanes excepted, which adds a
 *     lane's workspace): activation workspaces are sized for b_max at
 *     creation, as the paper pre-allocates its buffers for the largest activation matrix at
 *     B_max (Sec. III-B, "Overhead").  ee_serve_stream and ee_schedule_sim keep their queues in
 *     ordinary host containers that may grow during a call;
 *   - activations are NHWC, dense [slot][H][W][C], slot-major; int8 networks use int8
 *     activations, bf16 networks raw bfloat16 (uint16_t);
 *   - a ctx must not be used from two threads at once.
 */
#ifndef EE_H
#define EE_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ee_ctx ee_ctx;

typedef enum {
    EE_OK = 0,
    EE_ERR_ARG = -1,          /* NULL pointer, index or batch size out of range, misaligned pointer */
    EE_ERR_SHAPE = -2,        /* blob whose tensor shapes do not chain */
    EE_ERR_UNSUPPORTED = -3,  /* dtype or layer kind the library does not carry */
    EE_ERR_DEVICE = -4,       /* HIP error (no device, allocation or launch failure) */
    EE_ERR_OVERFLOW = -5      /* a size does not fit the library's limits */
} ee_status;

typedef enum { EE_I8 = 0, EE_BF16 = 1 } ee_dtype;

const char* ee_strerror(int status);

/* Host-only validation of a network blob (layout: the header comment of csrc/net.cpp).
 * Needs no GPU.  EE_ERR_SHAPE if the layer shapes do not chain. */
int ee_blob_check(const void* model_blob, size_t blob_bytes);

/* Parse the blob, repack the weights for the matrix cores into device memory and size the
 * workspace for b_max slots (1..1024).  `dtype` must match the blob.  `hip_stream` is a
 * hipStream_t (NULL = the default stream).  The blob may be freed after the call.
 * EE_ERR_OVERFLOW if b_max samples of some layer's tensor reach 2 GiB (the kernels address a
 * batch tensor with 32-bit byte offsets). */
int ee_create(const void* model_blob, size_t blob_bytes, int b_max, int dtype, void* hip_stream, ee_ctx** out);
int ee_destroy(ee_ctx* ctx);

/* Number of segments and per-sample byte sizes entering / leaving each (arrays of >= 8). */
int ee_query(const ee_ctx* ctx, int* n_stages, int64_t* stage_in_bytes, int64_t* stage_out_bytes);

/* ProcUntilExit of Algorithm 1, backbone part: all layers of segment `stage` (0-based) on slots
 * [0, b_act).  Every CONV layer is the GEMM  R x P . P x C  of Sec. II-C with the batch appended
 * along the row dimension (R-batching, Sec. III-A).
 *   act_in   device, [b_act][Hi][Wi][Ci]   (read only)
 *   act_out  device, [b_act][Ho][Wo][Co]   (written); must not alias act_in
 * b_act == 0 is a no-op.  EE_ERR_ARG for stage / b_act out of range or NULL / misaligned pointers. */
int ee_stage_forward(ee_ctx* ctx, int stage, int b_act, const void* act_in, void* act_out);

/* Exit head of segment `stage` on act[b_act][H][W][C]: global average pool, FC, softmax top-1
 * confidence compared with `thr` (Sec. IV "Benchmarks": softmax top-1 as confidence; a sample
 * leaves at the first exit whose confidence reaches the threshold).  At the last exit every
 * sample leaves and `thr` is ignored.  Per-slot device outputs:
 *   label[b_act] int32, conf[b_act] float, score[b_act] int64, exit_flag[b_act] uint8 (1 = leaves).
 * int8 networks: score is the integer softmax denominator S (confidence = 2^30 / S) and the
 * decision is S <= floor(2^30 / thr); bf16 networks: score is 0 and the decision conf >= thr. */
int ee_exit_head(ee_ctx* ctx, int stage, int b_act, const void* act, float thr,
                 int32_t* label, float* conf, int64_t* score, uint8_t* exit_flag);

/* For callers that cannot allocate device memory or may not trigger an allocation: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The same computation, arguments and outputs
 * as ee_exit_head, but the head's scratch memory (pooled sums, partial rows of the float pooling, logits) lies
 * in a fixed array of EE_STATIC_SCRATCH_BYTES that is part of the library image (one copy per GPU, held until
 * the process ends) instead of the context's workspace; the call allocates nothing, on the host or the device,
 * and what it clears it clears with a kernel, not a memset node.  EE_ERR_OVERFLOW when
 *   4 * b_act * (C + n_cls)  (+ 4 * b_act * splits * C for bf16 networks whose pooling is split)
 * rounded up to 256-byte blocks exceeds the array; EE_ERR_DEVICE when the array's address cannot be found.
 * All calls on one GPU share the array, from every context: calls that overlap on one GPU (different
 * streams or threads) race and must be serialised by the caller.  ee_last_logits does not see this call. */
#define EE_STATIC_SCRATCH_BYTES (4 * 1024 * 1024)
int ee_exit_head_static(ee_ctx* ctx, int stage, int b_act, const void* act, float thr,
                        int32_t* label, float* conf, int64_t* score, uint8_t* exit_flag);
int ee_static_scratch_bytes(void);

/* The logits the most recent ee_exit_head call computed, [b_act][n_cls] int32 (int8 networks) or
 * float (bf16 networks), copied to host memory.  Synchronous; for verification. */
int ee_last_logits(ee_ctx* ctx, int b_act, void* host_out);

/* B_rem = B_act - B_exit and B_merged = B_rem + B_incr of Algorithm 1: stable compaction of the
 * survivors (exit_flag == 0) of act_src[b_act] into act_dst[0, B_rem), then the b_incr samples of
 * refill_act appended at act_dst[B_rem, B_rem + b_incr); ids travel the same way.  All tensors
 * have the per-sample shape of segment `stage`'s output.  act_dst must hold b_act + b_incr
 * (<= b_max) samples and must not alias act_src / refill_act.
 *   exit_flag, act_src, ids_src, refill_act, refill_ids   device (read only)
 *   act_dst, ids_dst                                       device (written)
 *   b_rem_out, b_merged_out                                device-visible int (written), may be NULL */
int ee_compact_refill(ee_ctx* ctx, int stage, int b_act, const uint8_t* exit_flag,
                      const void* act_src, void* act_dst, const int32_t* ids_src, int32_t* ids_dst,
                      const void* refill_act, const int32_t* refill_ids, int b_incr,
                      int* b_rem_out, int* b_merged_out);

/* Set-up call for ee_serve_stream with lanes > 1: makes the context hold n lanes (1..4), i.e. allocates the workspace and the
 * HIP stream (default priority) of the lanes it does not have yet.  Returns the number of lanes or a negative status. */
int ee_lanes(ee_ctx* ctx, int n);

/* ---- stream serving: Algorithm 1 with the criterion of Eq. (3) / Eq. (4) ------------------- */
typedef struct { int64_t n; const int64_t* arrival_ns; /* host, non-decreasing */ } ee_trace;

typedef struct {
    int32_t b_max;          /* <= the ctx's b_max */
    int32_t clock;          /* 0: wall clock (latencies are measurements); 1: virtual clock driven by lut_ns */
    int64_t t_slo_ns;       /* latency SLO T_SLO; < 0 = none (infinite slack) */
    const int64_t* lut_ns;  /* host, [n_stages][b_max]: time of segment s (with its exit head) entered with
                               B = column + 1 samples (Sec. III-B, "Exit-Level Latency Prediction") */
    int32_t min_incr;       /* smallest B_incr worth a preemption; 1 = Algorithm 1 as printed */
    int32_t refill;         /* 0: model-level batching (no preemption); 1: Algorithm 1; 2: stage pools (below) */
    int64_t t_timeout_ns;   /* refill = 0: batch-forming window T_timeout of adaptive batching <B_max, T_timeout> (Sec. II-D):
                               a full batch is issued at once, an incomplete one when the oldest queued request has waited
                               this long; <= 0: whatever is queued is issued at once.  B_max = 1 is the SERIAL baseline. */
    int32_t lanes;          /* refill = 2: steps that may be in flight at once, 1..4 (0 = 1), at most what ee_lanes made */
    int32_t zero_copy;      /* 1: survivors of an exit are not moved (Sec. III-A: only the addressing changes): the samples of a batch
                               stay in the slots the segment wrote and the next segment gathers them through a slot table;
                               0: the compaction kernel copies them into a dense batch.  Results and schedule are the same.
                               EE_ERR_UNSUPPORTED unless ee_zero_copy_supported; with refill = 2 at most two lanes. */
} ee_serve_opts;

/* 1 when the context can serve with zero_copy = 1: b_max <= 256 and every tensor that crosses a segment boundary is read
 * and written by the general matrix-core convolution kernel only; else 0. */
int ee_zero_copy_supported(const ee_ctx* ctx);

/* refill = 2, stage pools, is an extension that is not in the paper.  Algorithm 1 keeps one active batch
 * and lets newcomers catch up with it (Sec. III-B, non-recursive by design); here the survivors of exit i
 * wait, first in first out, in a pool in front of segment i+1, and every step runs ONE segment on the front
 * min(n, b_max) samples of one level (level 0 = the arrival queue):
 *   - preferred: the deepest level holding a full batch of b_max; else the deepest non-empty pool; else the
 *     queue; else the server idles until the next arrival;
 *   - with t_slo_ns >= 0 a pool i goes first when its oldest sample still meets the SLO if segments i..|E|
 *     run now but not if the preferred step runs first: T_rest < T_slack and not T_first + T_rest < T_slack,
 *     T_slack as in Eq. (3), T_rest and T_first from lut_ns at the entering batch sizes; the deepest such pool
 *     whose successor pool is not full (its survivors need room there).
 * With lanes > 1 up to that many steps run concurrently on the GPU, each on a stream of its own: at most one step per
 * level is in flight, a level whose successor pool holds a full batch does not run, and while some step is in flight
 * an idle lane only starts full batches.  events: aux of EE_EV_PROC is the lane.
 * A pool never holds more than 2 b_max - 1 samples.  min_incr is not used.  stats: rounds = launches of
 * segment 0, criterion_evals / preemptions = evaluations of the SLO rule / times it changed the choice;
 * events: EE_EV_PROC per launch, EE_EV_CRITERION (stage = pool, b = its batch, aux = 1 if it goes first). */

typedef struct { int32_t exit_idx; int32_t label; float conf; int32_t pad_; int64_t score; int64_t latency_ns; } ee_result;

typedef struct { int64_t t_ns; int32_t kind; int32_t stage; int32_t b; int32_t aux; } ee_event;
enum { EE_EV_ROUND = 1, EE_EV_PROC = 2, EE_EV_PROC_CATCHUP = 3, EE_EV_CRITERION = 4, EE_EV_MERGE = 5 };

typedef struct {
    int64_t rounds, criterion_evals, preemptions, end_time_ns;
    int64_t seg_runs[8], seg_samples[8];   /* per segment: runs (main + catch-up) and samples entered */
    int64_t n_events;
} ee_serve_stats;

/* Synchronous.  Serves trace->n requests; request k is row k of input_pool (device,
 * [n][H][W][C], resident before the call) and its result is results[k] (host): results are
 * stored by sample id, not in completion order (Sec. III-B, "Overhead").  stats and events
 * may be NULL.  EE_ERR_ARG for decreasing arrival times, b_max out of range or refill outside 0..2. */
int ee_serve_stream(ee_ctx* ctx, const ee_trace* trace, const void* input_pool, const ee_serve_opts* opts,
                    ee_result* results, ee_serve_stats* stats, ee_event* events, int64_t max_events);

/* The same scheduler with the network replaced by a table: forced_exit[k] (host) is the 0-based
 * exit at which request k leaves.  Touches no GPU; opts->clock must be 1. */
int ee_schedule_sim(int n_stages, const ee_trace* trace, const int32_t* forced_exit, const ee_serve_opts* opts,
                    ee_result* results, ee_serve_stats* stats, ee_event* events, int64_t max_events);

/* Design-time latency table (Sec. III-B, "Exit-Level Latency Prediction"): runs segment s with its
 * exit head for every B = 1..b_max, `reps` times each, and stores the mean time in
 * lut_ns[s * b_max + B - 1] (host).  Synchronous; activations are whatever the workspace holds. */
int ee_measure_lut(ee_ctx* ctx, int reps, int64_t* lut_ns);

/* Design-time measurement of one layer alone (Sec. III-B builds its latency tables the same way, ahead of time): layer
 * `layer` of the network on `b` samples of the context's workspace, `reps` launches back to back between two HIP events
 * after two warm-up launches; *us_out = mean microseconds per launch (host), *ops_out = 2 * MACs and *bytes_out = the
 * algorithmic HBM bytes of one launch (may be NULL).  cfg = 0 uses the layer's table entry, else that kernel
 * configuration (as in ee_config_set); cfg = 0x20000 times the fused inverted-residual block headed by `layer` (its
 * layers' operations and bytes; EE_ERR_ARG when the layer heads none).  Synchronous; overwrites workspace
 * activations.  EE_ERR_DEVICE when the configuration does not exist for this layer. */
int ee_time_layer(ee_ctx* ctx, int layer, int b, int cfg, int reps, double* us_out, double* ops_out, double* bytes_out);

/* ---- kernel timing (HIP events on the library's stream) ------------------------------------ */
enum { EE_K_CONV_MFMA = 0, EE_K_CONV_FIRST = 1, EE_K_CONV_DIRECT = 2, EE_K_DEPTHWISE = 3, EE_K_MAXPOOL = 4,
       EE_K_PAD_INPUT = 5, EE_K_GAP = 6, EE_K_FC = 7, EE_K_SOFTMAX = 8, EE_K_COMPACT = 9, EE_K_ADMIT = 10,
       EE_K_CONV_STREAM = 11,   /* matrix-core layers whose operands come straight from global memory (thin and streaming kernels) */
       EE_K_COUNT = 12 };
typedef struct { int64_t launches; double ms; double ops; double bytes; } ee_kernel_stat;
/* enable = 1 brackets every kernel launch with a pair of HIP events; ee_profile_read synchronises,
 * adds the elapsed times up per kernel class into stats[EE_K_COUNT] (host) and, when per_layer is not
 * NULL, per layer of the network into per_layer[number of layers] (host), then resets the counters.
 * ops = 2 * MACs of the launches, bytes = their algorithmic HBM traffic (each operand once). */
int ee_profile_enable(ee_ctx* ctx, int enable);
/* creates event pairs ahead of time so that a timed region does not pay for their creation */
int ee_profile_reserve(ee_ctx* ctx, int64_t n_pairs);
int ee_profile_read(ee_ctx* ctx, ee_kernel_stat* stats, ee_kernel_stat* per_layer);
const char* ee_kernel_name(int kernel_class);

/* Tuning / test control of the convolution tiling, process-wide: 0 = chosen per layer and active
 * batch size (default), 1 = 128x128, 2 = 128x64, 3 = 64x64, 4 = 64x128 (output pixels x output channels
 * per workgroup), 7 = the streaming kernel for the layers it covers (many pixels, a reduction of at most nine
 * 32-byte blocks, at most 64 output channels; other layers keep the default).  A whole configuration word as
 * in ee_config_set (tile | reduction step << 4 | ring stages << 8 | wavefront groups << 12) forces that one on
 * every matrix-core layer; a ring deeper than LDS allows runs with the deepest that fits.  Results never depend
 * on it.  Returns the previous setting, EE_ERR_ARG if out of range. */
int ee_tune_conv_tile(int cfg);

/* Kernel-configuration table, one entry per (convolution layer, active-batch bucket 2^k): the GPU
 * counterpart of the run-time look-up the paper keeps per layer and batch size (Sec. III-A, the
 * configuration buffer of the Fluid Batching engine).  ee_autotune times the candidate workgroup tiles,
 * reduction steps and LDS ring depths of every matrix-core convolution on the context's own workspace
 * (`reps` launches per candidate, synchronous, overwrites the workspace activations) and keeps the
 * fastest; until it is called the configuration is chosen from the layer shape alone.  Results never
 * depend on the table.  ee_config_table copies layer `layer`'s entries to cfg_out[0..n) (host) and
 * returns how many the layer has (0 = not tuned or not a matrix-core convolution); an entry is
 * tile | step << 4 | stages << 8 | groups << 12 with tile 1: 128x128, 2: 128x64, 3: 64x64, 4: 64x128 (pixels x
 * channels), step 1: 64, 2: 128, 3: 256 bytes of the reduction axis per stage, groups 0: one group of 4
 * wavefronts, 2 or 4: that many groups sharing the reduction of a tile; the entry 7 alone selects the streaming
 * kernel.  EE_ERR_ARG for bad arguments. */
int ee_autotune(ee_ctx* ctx, int reps);
int ee_config_table(const ee_ctx* ctx, int layer, int* cfg_out, int n);
/* Loads a stored table for layer `layer` (n <= 16 entries as ee_config_table returns them; n = 0 clears it):
 * the table is design-time data, as the paper's look-up tables are.  EE_ERR_ARG for a layer that is not a
 * matrix-core convolution, an entry outside the encoding, or the entry 7 for a layer the streaming kernel does not
 * cover; an entry that names a tile combination the library does not have makes the launch that would use it fail
 * with EE_ERR_DEVICE. */
int ee_config_set(ee_ctx* ctx, int layer, const int* cfg, int n);

/* Fused layer pairs.  A matrix-core convolution without residual whose 64, 128 or 256 output channels are read by
 * one layer only, the next, a 1x1 stride-1 convolution (conv2 -> conv3 of a bottleneck block), can run as ONE
 * launch that keeps the intermediate tensor in LDS; results are those of the two separate kernels, bit for bit on
 * the int8 path.  ee_pair_count: how many layers of the network head such a pair.  ee_pair_mode: 0 = never fuse,
 * 1 = as the table says (default; until ee_autotune has run: fused below 32 samples, configuration by shape; it then
 * times every fused configuration against the two best separate kernels per batch bucket), 2 = fuse every pair.
 * ee_pair_table: like ee_config_table for the fused launch of the pair headed by `layer`; an entry is
 * rows | step << 4 | stages << 8 with rows 1: 128, 2: 64 pixels per workgroup, step 1: 64, 2: 128 bytes, or 0 = the
 * two layers run separately for that bucket.  EE_ERR_ARG for bad arguments. */
int ee_pair_count(const ee_ctx* ctx);
int ee_pair_mode(ee_ctx* ctx, int mode);
int ee_pair_table(const ee_ctx* ctx, int layer, int* cfg_out, int n);
/* Loads a stored fused-pair table (as ee_config_set; EE_ERR_ARG when `layer` heads no pair). */
int ee_pair_set(ee_ctx* ctx, int layer, const int* cfg, int n);

/* Fused inverted-residual blocks (int8).  A 1x1 stride-1 convolution without residual (the expansion), the 3x3 depthwise
 * layer with padding 1 that alone reads it and the 1x1 stride-1 convolution (the projection, with or without residual) that
 * alone reads that can run as ONE launch in which the expanded tensor exists only in LDS, 32 channels at a time; results
 * are those of the three separate kernels, bit for bit.  Covered: input channels a multiple of 8 up to 160, output
 * channels a multiple of 8 up to 160, depthwise stride 1 or 2.  A 3x3 depthwise layer that no such block covers and the 1x1
 * convolution that alone reads it are fused the same way (a block without expansion, headed by the depthwise layer; its
 * channels a multiple of 16).  ee_ir_count: how many layers of the network head such a
 * block.  ee_ir_mode: 0 = never fuse, 1 = as the table says (default; nothing is fused until ee_autotune has timed the
 * fused launch against the three tuned layers per batch bucket, or a table was loaded), 2 = fuse every block.
 * ee_ir_table / ee_ir_set: the table of the block headed by `layer`, one entry per batch bucket, 1 = fused, 0 = separate
 * (ee_ir_set: EE_ERR_ARG when `layer` heads no block).
 * Bottleneck blocks of the same three-layer shape (int8) go through the same switches and tables with a kernel of their own: a
 * 1x1 stride-1 convolution from 64 or 256 to 64 channels, the 3x3 stride-1 convolution with padding 1 (64 -> 64) that alone
 * reads it, and the 1x1 stride-1 convolution to 256 channels (with or without residual) that alone reads that; as a segment's
 * last layers the launch also pools for the exit head and writes through the slot table of zero-copy compaction.  Where the
 * residual is a 1x1 stride-1 convolution of the block's own 64-channel input and that convolution is the layer right in
 * front of the block, the convolution heads a block of four layers, tuned against that convolution followed by the block of
 * three.  The same switches and tables cover the first layers of a ResNet-style network (int8): a 7x7 stride-2 convolution
 * of a 3-channel image to 64 channels and the 3x3 stride-2 max-pool with padding 1 that alone reads it run as one launch (a block
 * of two layers headed by the convolution).  ee_ir_layers: the number of layers of the block headed by `layer` (2, 3 or 4), 0
 * when it heads none. */
int ee_ir_count(const ee_ctx* ctx);
int ee_ir_layers(const ee_ctx* ctx, int layer);
int ee_ir_mode(ee_ctx* ctx, int mode);
int ee_ir_table(const ee_ctx* ctx, int layer, int* cfg_out, int n);
int ee_ir_set(ee_ctx* ctx, int layer, const int* cfg, int n);

/* Host copy of the 256-entry table round(2^30 * 2^(-i/256)) used by the integer softmax. */
const uint32_t* ee_exp2_table(void);

#ifdef __cplusplus
}
#endif
#endif
