/*
 * CPU oracle, network level: blob parsing, one backbone segment, one exit head, slot
 * compaction / refill, and the batch-of-one staged forward.  TEST INFRASTRUCTURE ONLY.
 *
 * An early-exit network (Sec. II-B) is a backbone cut into segments; after segment i an exit
 * head produces a softmax top-1 confidence, and a sample leaves at the first exit whose
 * confidence reaches the threshold (Sec. IV "Benchmarks"); the last exit takes everyone.
 */
#include "orc.h"

#include <stdlib.h>
#include <string.h>

#pragma pack(push, 1)
typedef struct {
    char magic[8]; int32_t version, dtype, n_stages, n_ops, in_h, in_w, in_c, n_classes;
    int64_t stages_off, ops_off, exits_off, data_off, total_bytes; char reserved[48];
} blob_header;
typedef struct { int32_t first_op, n_ops, n_tensors, out_tensor, out_h, out_w, out_c, reserved; } blob_stage;
typedef struct {
    int32_t kind, src, dst, res, h_in, w_in, c_in, h_out, w_out, c_out, kh, kw, stride, pad, shift, res_shift, lo, hi;
    float f_lo, f_hi; int64_t w_off, b_off;
    int32_t pad_w, c_off, c_tot, reserved;   /* columns of padding; the op writes channels [c_off, c_off + c_out) of a c_tot-channel tensor */
} blob_op;
typedef struct {
    int32_t h, w, c, n_cls, gap_shift, frac_bits; float logit_scale, thr; int64_t w_off, b_off; char reserved[16];
} blob_exit;
#pragma pack(pop)

typedef struct {
    const unsigned char* base; size_t bytes;
    const blob_header* hd; const blob_stage* st; const blob_op* op; const blob_exit* ex;
} net_view;

enum { KIND_CONV = 0, KIND_DWCONV = 1, KIND_MAXPOOL = 2, KIND_AVGPOOL = 3 };

static int view_blob(const void* blob, size_t bytes, net_view* v)
{
    if (!blob || bytes < sizeof(blob_header)) return ORC_ERR_ARG;
    v->base = (const unsigned char*)blob; v->bytes = bytes;
    v->hd = (const blob_header*)blob;
    if (memcmp(v->hd->magic, "EENETv2\0", 8) != 0 || v->hd->version != 2) return ORC_ERR_ARG;
    if (v->hd->dtype != 0 && v->hd->dtype != 1) return ORC_ERR_UNSUPPORTED;
    if ((size_t)v->hd->total_bytes > bytes || v->hd->n_stages <= 0 || v->hd->n_stages > 8 || v->hd->n_ops < 0) return ORC_ERR_ARG;
    v->st = (const blob_stage*)(v->base + v->hd->stages_off);
    v->op = (const blob_op*)(v->base + v->hd->ops_off);
    v->ex = (const blob_exit*)(v->base + v->hd->exits_off);
    return ORC_OK;
}

static void stage_in_shape(const net_view* v, int s, int* h, int* w, int* c)
{
    if (s == 0) { *h = v->hd->in_h; *w = v->hd->in_w; *c = v->hd->in_c; }
    else { *h = v->st[s - 1].out_h; *w = v->st[s - 1].out_w; *c = v->st[s - 1].out_c; }
}

/* Shapes must chain: every op reads a tensor that has been written with the dims it states and writes either a
 * new tensor or a channel slice of a concatenation tensor; the stage output has the dims the stage record and
 * the exit head state. */
int orc_blob_check(const void* blob, size_t bytes)
{
    net_view v;
    int rc = view_blob(blob, bytes, &v);
    if (rc) return rc;
    const int esz = v.hd->dtype == 0 ? 1 : 2;
    for (int s = 0; s < v.hd->n_stages; ++s) {
        const blob_stage* st = &v.st[s];
        if (st->n_tensors < 1 || st->n_tensors > 256 || st->first_op < 0 || st->first_op + st->n_ops > v.hd->n_ops) return ORC_ERR_SHAPE;
        int th[256], tw[256], tc[256], filled[256];    /* filled: channels written so far; 0 = not written yet */
        static _Thread_local int sl_off[256][32], sl_len[256][32];   /* the slices written so far, per tensor */
        int n_sl[256];
        memset(filled, 0, sizeof filled);
        memset(n_sl, 0, sizeof n_sl);
        stage_in_shape(&v, s, &th[0], &tw[0], &tc[0]);
        filled[0] = tc[0];
        for (int k = 0; k < st->n_ops; ++k) {
            const blob_op* o = &v.op[st->first_op + k];
            if (o->kind < 0 || o->kind > KIND_AVGPOOL) return ORC_ERR_UNSUPPORTED;
            if (o->src < 0 || o->src >= st->n_tensors || o->dst < 1 || o->dst >= st->n_tensors || o->dst == o->src) return ORC_ERR_SHAPE;
            if (filled[o->src] == 0 || filled[o->src] != tc[o->src]) return ORC_ERR_SHAPE;        /* read before it is complete */
            if (o->h_in != th[o->src] || o->w_in != tw[o->src] || o->c_in != tc[o->src]) return ORC_ERR_SHAPE;
            if (o->stride <= 0 || o->kh <= 0 || o->kw <= 0 || o->pad < 0 || o->pad_w < 0) return ORC_ERR_SHAPE;
            if (o->h_out != (o->h_in + 2 * o->pad - o->kh) / o->stride + 1 || o->w_out != (o->w_in + 2 * o->pad_w - o->kw) / o->stride + 1)
                return ORC_ERR_SHAPE;
            if (o->h_out <= 0 || o->w_out <= 0 || o->c_out <= 0) return ORC_ERR_SHAPE;
            if (o->kind != KIND_CONV && (o->c_out != o->c_in || o->pad != o->pad_w || o->kh != o->kw)) return ORC_ERR_SHAPE;
            if (o->c_off < 0 || o->c_tot < o->c_off + o->c_out) return ORC_ERR_SHAPE;
            if (filled[o->dst] == 0) { th[o->dst] = o->h_out; tw[o->dst] = o->w_out; tc[o->dst] = o->c_tot; }
            else if (th[o->dst] != o->h_out || tw[o->dst] != o->w_out || tc[o->dst] != o->c_tot || o->c_tot == o->c_out) return ORC_ERR_SHAPE;
            for (int j = 0; j < n_sl[o->dst]; ++j)          /* slices of one tensor must not overlap */
                if (o->c_off < sl_off[o->dst][j] + sl_len[o->dst][j] && sl_off[o->dst][j] < o->c_off + o->c_out) return ORC_ERR_SHAPE;
            if (n_sl[o->dst] >= 32) return ORC_ERR_SHAPE;
            sl_off[o->dst][n_sl[o->dst]] = o->c_off; sl_len[o->dst][n_sl[o->dst]] = o->c_out; n_sl[o->dst]++;
            filled[o->dst] += o->c_out;
            if (filled[o->dst] > o->c_tot) return ORC_ERR_SHAPE;
            if (o->res >= 0) {
                if (o->kind != KIND_CONV || o->res >= st->n_tensors || o->c_tot != o->c_out || filled[o->res] == 0 || filled[o->res] != tc[o->res]) return ORC_ERR_SHAPE;
                if (th[o->res] != o->h_out || tw[o->res] != o->w_out || tc[o->res] != o->c_out) return ORC_ERR_SHAPE;
            }
            if (o->kind == KIND_CONV || o->kind == KIND_DWCONV) {
                const int64_t nw = (int64_t)o->c_out * o->kh * o->kw * (o->kind == KIND_DWCONV ? 1 : o->c_in);
                if (o->w_off < v.hd->data_off || (size_t)(o->w_off + nw * esz) > bytes) return ORC_ERR_SHAPE;
                if (o->b_off < v.hd->data_off || (size_t)(o->b_off + 4 * (int64_t)o->c_out) > bytes) return ORC_ERR_SHAPE;
            }
        }
        const int next = st->n_tensors;
        for (int t = 0; t < st->n_tensors; ++t)
            if (filled[t] == 0 || filled[t] != tc[t]) return ORC_ERR_SHAPE;                         /* every tensor is written, and completely */
        if (next != st->n_tensors || st->out_tensor < 0 || st->out_tensor >= next) return ORC_ERR_SHAPE;
        if (th[st->out_tensor] != st->out_h || tw[st->out_tensor] != st->out_w || tc[st->out_tensor] != st->out_c) return ORC_ERR_SHAPE;
        const blob_exit* e = &v.ex[s];
        if (e->h != st->out_h || e->w != st->out_w || e->c != st->out_c || e->n_cls != v.hd->n_classes || e->n_cls <= 0) return ORC_ERR_SHAPE;
        if ((size_t)(e->w_off + (int64_t)e->n_cls * e->c * esz) > bytes || (size_t)(e->b_off + 4 * (int64_t)e->n_cls) > bytes) return ORC_ERR_SHAPE;
    }
    return ORC_OK;
}

/* One backbone segment on slots [0, b_act): act_in[b][Hi][Wi][Ci] -> act_out[b][Ho][Wo][Co].
 * Layers run one after the other over the whole batch; samples never interact (batching only
 * appends rows to the activation matrix, Sec. III-A). */
int orc_stage_forward(const void* blob, size_t bytes, int stage, int b_act, const void* act_in, void* act_out)
{
    net_view v;
    int rc = orc_blob_check(blob, bytes);
    if (rc) return rc;
    view_blob(blob, bytes, &v);
    if (stage < 0 || stage >= v.hd->n_stages || b_act < 0 || (!act_in && b_act) || (!act_out && b_act)) return ORC_ERR_ARG;
    if (b_act == 0) return ORC_OK;
    const blob_stage* st = &v.st[stage];
    const int esz = v.hd->dtype == 0 ? 1 : 2;
    void* tens[256];
    memset(tens, 0, sizeof tens);
    tens[0] = (void*)act_in;
    int32_t* acc = NULL;
    for (int k = 0; k < st->n_ops && rc == ORC_OK; ++k) {
        const blob_op* o = &v.op[st->first_op + k];
        const int64_t out_elems = (int64_t)b_act * o->h_out * o->w_out * o->c_out;
        const int64_t rows = (int64_t)b_act * o->h_out * o->w_out;
        const int sliced = o->c_tot != o->c_out;
        if (!tens[o->dst]) {                               /* first writer: the whole tensor, c_tot channels per pixel */
            tens[o->dst] = (o->dst == st->out_tensor) ? act_out : malloc((size_t)(rows * o->c_tot * esz));
            if (!tens[o->dst]) { rc = ORC_ERR_ARG; break; }
        }
        /* a slice is computed densely, then copied into its channels of the concatenation tensor */
        void* dst = sliced ? malloc((size_t)(out_elems * esz)) : tens[o->dst];
        if (!dst) { rc = ORC_ERR_ARG; break; }
        const void* src = tens[o->src];
        const void* res = o->res >= 0 ? tens[o->res] : NULL;
        const void* wt = v.base + o->w_off;
        const void* bs = v.base + o->b_off;
        if (v.hd->dtype == 0) {
            if (o->kind == KIND_MAXPOOL) {
                rc = orc_maxpool_i8((const int8_t*)src, b_act, o->h_in, o->w_in, o->c_in, o->kh, o->stride, o->pad, (int8_t*)dst);
            } else if (o->kind == KIND_AVGPOOL) {
                rc = orc_avgpool_i8((const int8_t*)src, b_act, o->h_in, o->w_in, o->c_in, o->kh, o->stride, o->pad, (int8_t*)dst);
            } else {
                acc = (int32_t*)realloc(acc, sizeof(int32_t) * (size_t)out_elems);
                if (!acc) { rc = ORC_ERR_ARG; break; }
                if (o->kind == KIND_CONV)
                    rc = orc_conv_acc_i8_hw((const int8_t*)src, b_act, o->h_in, o->w_in, o->c_in, (const int8_t*)wt, (const int32_t*)bs,
                                            o->c_out, o->kh, o->kw, o->stride, o->pad, o->pad_w, acc);
                else
                    rc = orc_dwconv_acc_i8((const int8_t*)src, b_act, o->h_in, o->w_in, o->c_in, (const int8_t*)wt, (const int32_t*)bs,
                                           o->kh, o->kw, o->stride, o->pad, acc);
                if (rc == ORC_OK)
                    rc = orc_requant_i8(acc, (const int8_t*)res, out_elems, o->shift, o->res_shift, o->lo, o->hi, (int8_t*)dst);
            }
        } else {
            if (o->kind == KIND_MAXPOOL)
                rc = orc_maxpool_bf16((const uint16_t*)src, b_act, o->h_in, o->w_in, o->c_in, o->kh, o->stride, o->pad, (uint16_t*)dst);
            else if (o->kind == KIND_AVGPOOL)
                rc = orc_avgpool_bf16((const uint16_t*)src, b_act, o->h_in, o->w_in, o->c_in, o->kh, o->stride, o->pad, (uint16_t*)dst);
            else if (o->kind == KIND_CONV)
                rc = orc_conv_bf16_hw((const uint16_t*)src, b_act, o->h_in, o->w_in, o->c_in, (const uint16_t*)wt, (const float*)bs,
                                      o->c_out, o->kh, o->kw, o->stride, o->pad, o->pad_w, (const uint16_t*)res, o->f_lo, o->f_hi, (uint16_t*)dst);
            else
                rc = orc_dwconv_bf16((const uint16_t*)src, b_act, o->h_in, o->w_in, o->c_in, (const uint16_t*)wt, (const float*)bs,
                                     o->kh, o->kw, o->stride, o->pad, o->f_lo, o->f_hi, (uint16_t*)dst);
        }
        if (sliced) {
            if (rc == ORC_OK)
                for (int64_t r = 0; r < rows; ++r)
                    memcpy((char*)tens[o->dst] + (r * o->c_tot + o->c_off) * esz, (const char*)dst + r * o->c_out * esz, (size_t)(o->c_out * esz));
            free(dst);
        }
    }
    free(acc);
    for (int t = 1; t < st->n_tensors; ++t)
        if (tens[t] && tens[t] != act_out) free(tens[t]);
    return rc;
}

/* Exit head of segment `stage` on act[b_act][H][W][C]: GAP -> FC -> softmax top-1 -> compare.
 * At the last exit every sample leaves whatever its confidence. */
int orc_exit_head(const void* blob, size_t bytes, int stage, int b_act, const void* act, float thr,
                  int32_t* label, float* conf, int64_t* score, uint8_t* exit_flag, void* logits)
{
    net_view v;
    int rc = orc_blob_check(blob, bytes);
    if (rc) return rc;
    view_blob(blob, bytes, &v);
    if (stage < 0 || stage >= v.hd->n_stages || b_act < 0) return ORC_ERR_ARG;
    if (b_act == 0) return ORC_OK;
    if (!act || !label || !conf || !score || !exit_flag) return ORC_ERR_ARG;
    const blob_exit* e = &v.ex[stage];
    const int last = stage == v.hd->n_stages - 1;
    if (v.hd->dtype == 0) {
        int8_t* g = (int8_t*)malloc((size_t)b_act * e->c);
        int32_t* a = logits ? (int32_t*)logits : (int32_t*)malloc(sizeof(int32_t) * (size_t)b_act * e->n_cls);
        if (!g || !a) { free(g); if (!logits) free(a); return ORC_ERR_ARG; }
        rc = orc_gap_i8((const int8_t*)act, b_act, e->h, e->w, e->c, e->gap_shift, NULL, g);
        if (!rc) rc = orc_fc_i8(g, b_act, e->c, (const int8_t*)(v.base + e->w_off), (const int32_t*)(v.base + e->b_off), e->n_cls, a);
        if (!rc) rc = orc_softmax_top1_i8(a, b_act, e->n_cls, e->frac_bits, label, score);
        if (!rc) {
            const int64_t s_thr = orc_score_threshold(thr);
            for (int b = 0; b < b_act; ++b) {
                conf[b] = (float)(1073741824.0 / (double)score[b]);
                exit_flag[b] = (uint8_t)(last || score[b] <= s_thr);
            }
        }
        free(g);
        if (!logits) free(a);
    } else {
        rc = orc_head_bf16((const uint16_t*)act, b_act, e->h, e->w, e->c, (const uint16_t*)(v.base + e->w_off),
                           (const float*)(v.base + e->b_off), e->n_cls, e->logit_scale, (float*)logits, label, conf);
        if (!rc)
            for (int b = 0; b < b_act; ++b) {
                score[b] = 0;
                exit_flag[b] = (uint8_t)(last || conf[b] >= thr);
            }
    }
    return rc;
}

/* Survivors (exit_flag == 0) keep their relative order and move to slots [0, B_rem); the
 * b_incr refill samples follow in the order given: B_merged = B_rem + B_incr (Sec. III-B,
 * "Preemption Mechanism").  Source and destination must not overlap. */
int orc_compact_refill(int64_t sample_bytes, int b_act, const uint8_t* exit_flag, const void* act_src,
                       void* act_dst, const int32_t* ids_src, int32_t* ids_dst, const void* refill_act,
                       const int32_t* refill_ids, int b_incr, int* b_rem_out, int* b_merged_out)
{
    if (sample_bytes <= 0 || b_act < 0 || b_incr < 0 || (b_act && (!exit_flag || !act_src)) || (b_incr && !refill_act)) return ORC_ERR_ARG;
    if (!act_dst && (b_act || b_incr)) return ORC_ERR_ARG;
    int b_rem = 0;
    for (int b = 0; b < b_act; ++b) {
        if (exit_flag[b]) continue;
        memcpy((char*)act_dst + (int64_t)b_rem * sample_bytes, (const char*)act_src + (int64_t)b * sample_bytes, (size_t)sample_bytes);
        if (ids_dst && ids_src) ids_dst[b_rem] = ids_src[b];
        ++b_rem;
    }
    for (int k = 0; k < b_incr; ++k) {
        memcpy((char*)act_dst + (int64_t)(b_rem + k) * sample_bytes, (const char*)refill_act + (int64_t)k * sample_bytes, (size_t)sample_bytes);
        if (ids_dst && refill_ids) ids_dst[b_rem + k] = refill_ids[k];
    }
    if (b_rem_out) *b_rem_out = b_rem;
    if (b_merged_out) *b_merged_out = b_rem + b_incr;
    return ORC_OK;
}

static int64_t stage_bytes(const net_view* v, int s, int out)
{
    int h, w, c;
    if (out) { h = v->st[s].out_h; w = v->st[s].out_w; c = v->st[s].out_c; }
    else stage_in_shape(v, s, &h, &w, &c);
    return (int64_t)h * w * c * (v->hd->dtype == 0 ? 1 : 2);
}

int orc_query(const void* blob, size_t bytes, int* n_stages, int64_t* stage_in_bytes, int64_t* stage_out_bytes, float* thr)
{
    net_view v;
    int rc = orc_blob_check(blob, bytes);
    if (rc) return rc;
    view_blob(blob, bytes, &v);
    if (n_stages) *n_stages = v.hd->n_stages;
    for (int s = 0; s < v.hd->n_stages; ++s) {
        if (stage_in_bytes) stage_in_bytes[s] = stage_bytes(&v, s, 0);
        if (stage_out_bytes) stage_out_bytes[s] = stage_bytes(&v, s, 1);
        if (thr) thr[s] = v.ex[s].thr;
    }
    return ORC_OK;
}

/* Each sample alone (B = 1) through segment 1, exit 1, segment 2, ... until it exits, with the
 * thresholds stored in the blob.  latency_ns is left 0. */
int orc_forward_alone(const void* blob, size_t bytes, int64_t n, const void* inputs, orc_result* results)
{
    net_view v;
    int rc = orc_blob_check(blob, bytes);
    if (rc) return rc;
    view_blob(blob, bytes, &v);
    if (n < 0 || (n && (!inputs || !results))) return ORC_ERR_ARG;
    const int64_t in_bytes = stage_bytes(&v, 0, 0);
    int64_t max_bytes = in_bytes;
    for (int s = 0; s < v.hd->n_stages; ++s)
        if (stage_bytes(&v, s, 1) > max_bytes) max_bytes = stage_bytes(&v, s, 1);
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t k = 0; k < n; ++k) {
        void* cur = malloc((size_t)max_bytes);
        void* nxt = malloc((size_t)max_bytes);
        if (!cur || !nxt) { fail = ORC_ERR_ARG; free(cur); free(nxt); continue; }
        memcpy(cur, (const char*)inputs + k * in_bytes, (size_t)in_bytes);
        for (int s = 0; s < v.hd->n_stages; ++s) {
            int r = orc_stage_forward(blob, bytes, s, 1, cur, nxt);
            int32_t label; float conf; int64_t score; uint8_t flag = 0;
            if (!r) r = orc_exit_head(blob, bytes, s, 1, nxt, v.ex[s].thr, &label, &conf, &score, &flag, NULL);
            if (r) { fail = r; break; }
            if (flag) {
                results[k].exit_idx = s; results[k].label = label; results[k].conf = conf; results[k].pad_ = 0;
                results[k].score = score; results[k].latency_ns = 0;
                break;
            }
            void* t = cur; cur = nxt; nxt = t;
        }
        free(cur); free(nxt);
    }
    return fail;
}

/* worker threads the parallel loops over samples use (0 = the OpenMP default again) */
#ifdef _OPENMP
#include <omp.h>
static int orc_default_threads = 0;
int orc_set_threads(int n)
{
    if (!orc_default_threads) orc_default_threads = omp_get_max_threads();
    omp_set_num_threads(n > 0 ? n : orc_default_threads);
    return omp_get_max_threads();
}
#else
int orc_set_threads(int n) { (void)n; return 1; }
#endif
