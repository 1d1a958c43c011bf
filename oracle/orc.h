/*
 * CPU oracle for the staged early-exit forward pass and exit-aware preemptive serving.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, obviously-correct reference used by
 * the tests, the smoke check and the benchmark's CPU-baseline leg.  It shares no code
 * with the GPU library and must never be called from the product path.
 *
 * Every function is the textbook definition written as naive loops:
 *   - convolution = the GEMM  R x P . P x C -> R x C  over Toeplitz matrices that the paper
 *     uses to describe every CONV/FC layer (Sec. II-C, Fig. "computation of a convolutional
 *     layer, mapped as GEMM"), evaluated directly (orc_conv_acc_i8) and, as an independent
 *     second formulation, by materialising the Toeplitz matrix (orc_conv_acc_i8_toeplitz);
 *   - the exit head = global average pool, FC, softmax top-1 confidence compared with a
 *     threshold (Sec. IV "Benchmarks": softmax top-1 as confidence metric);
 *   - serving = Algorithm 1 with the SLO criterion of Eq. (3) and Eq. (4) on a virtual clock
 *     driven by the exit-level latency table (Sec. III-B "Exit-Level Latency Prediction").
 *
 * Integer path: int8 activations/weights, int32 accumulators (computed in int64 and checked
 * to fit), power-of-two requantisation with round-half-up.  bf16 path: double accumulation,
 * one rounding to float, bf16 round-to-nearest-even after every layer.
 *
 * Parity status: all functions are pinned by tests/test_oracle_*.py (closed forms, brute
 * force, the paper's scheduling-timeline example).  Wall-clock latencies are measurements
 * and therefore "parity unpinned"; the oracle only implements the virtual clock.
 */
#ifndef ORC_H
#define ORC_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_OK = 0, ORC_ERR_ARG = -1, ORC_ERR_SHAPE = -2, ORC_ERR_UNSUPPORTED = -3, ORC_ERR_OVERFLOW = -5 };

/* ---- int8 primitives (NHWC) ------------------------------------------------------- */
int orc_conv_acc_i8(const int8_t* x, int n, int h, int w, int ci, const int8_t* wt, const int32_t* bias,
                    int co, int kh, int kw, int stride, int pad, int32_t* acc);
int orc_conv_acc_i8_toeplitz(const int8_t* x, int n, int h, int w, int ci, const int8_t* wt,
                             const int32_t* bias, int co, int kh, int kw, int stride, int pad, int32_t* acc);
/* the same two with `pad` rows and `pad_w` columns of zero padding (kernels that are not square) */
int orc_conv_acc_i8_hw(const int8_t* x, int n, int h, int w, int ci, const int8_t* wt, const int32_t* bias,
                       int co, int kh, int kw, int stride, int pad, int pad_w, int32_t* acc);
int orc_conv_acc_i8_toeplitz_hw(const int8_t* x, int n, int h, int w, int ci, const int8_t* wt,
                                const int32_t* bias, int co, int kh, int kw, int stride, int pad, int pad_w, int32_t* acc);
int orc_dwconv_acc_i8(const int8_t* x, int n, int h, int w, int c, const int8_t* wt, const int32_t* bias,
                      int kh, int kw, int stride, int pad, int32_t* acc);
int orc_requant_i8(const int32_t* acc, const int8_t* res, int64_t count, int shift, int res_shift,
                   int lo, int hi, int8_t* y);
int orc_maxpool_i8(const int8_t* x, int n, int h, int w, int c, int k, int stride, int pad, int8_t* y);
int orc_avgpool_i8(const int8_t* x, int n, int h, int w, int c, int k, int stride, int pad, int8_t* y);
int orc_gap_i8(const int8_t* x, int n, int h, int w, int c, int gap_shift, int32_t* sums, int8_t* g);
int orc_fc_i8(const int8_t* g, int n, int c, const int8_t* wfc, const int32_t* bfc, int n_cls, int32_t* a);
int orc_softmax_top1_i8(const int32_t* a, int n, int n_cls, int frac_bits, int32_t* label, int64_t* score);
int64_t orc_score_threshold(float thr);
const uint32_t* orc_exp2_table(void);

/* ---- bf16 primitives (tensors are raw bf16 bit patterns) --------------------------- */
int orc_conv_bf16(const uint16_t* x, int n, int h, int w, int ci, const uint16_t* wt, const float* bias,
                  int co, int kh, int kw, int stride, int pad, const uint16_t* res, float f_lo, float f_hi,
                  uint16_t* y);
int orc_dwconv_bf16(const uint16_t* x, int n, int h, int w, int c, const uint16_t* wt, const float* bias,
                    int kh, int kw, int stride, int pad, float f_lo, float f_hi, uint16_t* y);
int orc_maxpool_bf16(const uint16_t* x, int n, int h, int w, int c, int k, int stride, int pad, uint16_t* y);
int orc_avgpool_bf16(const uint16_t* x, int n, int h, int w, int c, int k, int stride, int pad, uint16_t* y);
int orc_conv_bf16_hw(const uint16_t* x, int n, int h, int w, int ci, const uint16_t* wt, const float* bias,
                     int co, int kh, int kw, int stride, int pad, int pad_w, const uint16_t* res, float f_lo, float f_hi,
                     uint16_t* y);
int orc_head_bf16(const uint16_t* x, int n, int h, int w, int c, const uint16_t* wfc, const float* bfc,
                  int n_cls, float logit_scale, float* logits, int32_t* label, float* conf);
uint16_t orc_f32_to_bf16(float v);
float orc_bf16_to_f32(uint16_t b);

/* ---- network level ------------------------------------------------------------------ */
typedef struct { int32_t exit_idx; int32_t label; float conf; int32_t pad_; int64_t score; int64_t latency_ns; } orc_result;

int orc_blob_check(const void* blob, size_t bytes);
/* per-sample byte sizes entering / leaving each segment and the stored exit thresholds (arrays of 8) */
int orc_query(const void* blob, size_t bytes, int* n_stages, int64_t* stage_in_bytes, int64_t* stage_out_bytes, float* thr);
int orc_stage_forward(const void* blob, size_t bytes, int stage, int b_act, const void* act_in, void* act_out);
/* logits (optional, may be NULL): [b_act][n_cls] int32 (int8 nets) or float (bf16 nets). */
int orc_exit_head(const void* blob, size_t bytes, int stage, int b_act, const void* act, float thr,
                  int32_t* label, float* conf, int64_t* score, uint8_t* exit_flag, void* logits);
int orc_compact_refill(int64_t sample_bytes, int b_act, const uint8_t* exit_flag, const void* act_src,
                       void* act_dst, const int32_t* ids_src, int32_t* ids_dst, const void* refill_act,
                       const int32_t* refill_ids, int b_incr, int* b_rem_out, int* b_merged_out);
/* every sample on its own through the segments until it exits (thresholds from the blob) */
int orc_forward_alone(const void* blob, size_t bytes, int64_t n, const void* inputs, orc_result* results);

/* worker threads of the parallel loops over samples (timing the oracle on one core); 0 = the default again */
int orc_set_threads(int n);

/* ---- Algorithm 1 on a virtual clock -------------------------------------------------- */
typedef struct {
    int32_t b_max;
    int32_t clock;       /* must be 1 (virtual) for the oracle */
    int64_t t_slo_ns;    /* < 0: no SLO (infinite slack) */
    const int64_t* lut_ns;  /* [n_stages][b_max]: time of segment s entered with B = col+1 samples */
    int32_t min_incr;    /* smallest catch-up batch worth a preemption; 1 = as in the paper */
    int32_t refill;      /* 0 = model-level batching, 1 = Algorithm 1, 2 = stage pools (an extension, see orc_serve.c) */
    int64_t t_timeout_ns; /* refill = 0: batch-forming window of adaptive batching (Sec. II-D); <= 0: batches are issued at once */
    int32_t lanes;       /* refill = 2: steps that may be in flight at once, 1..4 (0 = 1) */
    int32_t pad_;
} orc_serve_opts;

typedef struct { int64_t t_ns; int32_t kind; int32_t stage; int32_t b; int32_t aux; } orc_event;
enum { ORC_EV_ROUND = 1, ORC_EV_PROC = 2, ORC_EV_PROC_CATCHUP = 3, ORC_EV_CRITERION = 4, ORC_EV_MERGE = 5 };

typedef struct {
    int64_t rounds, criterion_evals, preemptions, end_time_ns;
    int64_t seg_runs[8], seg_samples[8];   /* per segment: launches (main + catch-up) and samples entered */
    int64_t n_events;
} orc_serve_stats;

/* forced_exit: NULL = run the network; otherwise forced_exit[id] is the (0-based) exit at which
   sample id leaves and no tensor is touched (scheduler-only runs).  n_stages_forced gives |E| then. */
int orc_serve_stream(const void* blob, size_t bytes, int64_t n, const int64_t* arrival_ns, const void* input_pool,
                     const orc_serve_opts* opts, const int32_t* forced_exit, int n_stages_forced,
                     orc_result* results, orc_serve_stats* stats, orc_event* events, int64_t max_events);

#ifdef __cplusplus
}
#endif
#endif
