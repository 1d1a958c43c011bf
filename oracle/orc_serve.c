/*
 * CPU oracle, serving: Algorithm 1 (exit-aware preemptive scheduling) on a virtual clock.
 * TEST INFRASTRUCTURE ONLY.
 *
 * Notation follows Sec. III-B: B_act active batch, B_exit samples leaving at an exit,
 * B_rem = B_act - B_exit, B_slack = B_max - B_rem, B_incr = min(N_Q, B_slack),
 * B_merged = B_rem + (catch-up survivors), T_slack (Eq. 3), T_overhead (Eq. 4).
 *
 * Readings where the algorithm as printed is silent or cannot run as written:
 *   - the printed loop stops before the last segment; here the last segment is processed too
 *     and everyone left exits there;
 *   - B_incr = 0 (empty queue) ends the refill loop (it would spin forever otherwise);
 *   - B_rem = 0 ends the round: there is no "oldest active sample" to compute T_slack for;
 *   - the latency table is indexed by segment and by the batch size ENTERING the segment and a
 *     segment's time includes its exit head; T_{0:i} of Eq. 4 = segments 1..i at B_incr,
 *     the second term = segments i+1..|E| at the upper bound B_rem + B_incr;
 *   - the server idles until the next arrival when the queue is empty;
 *   - requests are taken from the head of the queue (FIFO), results are stored by sample id.
 *
 * Baselines of the evaluation (Sec. V-A): refill = 0 is model-level batching; with t_timeout_ns > 0 it is adaptive
 * batching <B_max, T_timeout> (Sec. II-D); SERIAL is B_max = 1.
 *
 * Second policy (opts->refill == 2), an extension that is NOT in the paper: stage pools.  Where
 * Algorithm 1 holds one active batch and lets newcomers catch up with it, here the survivors of
 * exit i wait in a pool in front of segment i+1, and a segment is launched on a full batch of
 * B_max whenever some pool (or the arrival queue, level 0) holds that many.  See serve_pooled().
 */
#include "orc.h"

#include <stdlib.h>
#include <string.h>

typedef struct {
    const void* blob; size_t bytes;
    int n_stages, b_max;
    int64_t n; const int64_t* arrival; const char* pool;
    const orc_serve_opts* opts; const int32_t* forced;
    orc_result* results; orc_serve_stats* stats; orc_event* events; int64_t max_events;
    int64_t now, next_arrival /* first id not yet admitted */, q_head /* first id still queued */, done;
    int64_t sample_bytes[9];   /* [s] = bytes of one sample entering segment s; [n_stages] unused */
    int64_t out_bytes[8];
    float thr[8];              /* exit thresholds stored in the blob */
    int err;
} server;

typedef struct { int b; int32_t* ids; char* act; } batch;

static void log_event(server* S, int kind, int stage, int b, int aux)
{
    if (S->events && S->stats->n_events < S->max_events) {
        orc_event* e = &S->events[S->stats->n_events];
        e->t_ns = S->now; e->kind = kind; e->stage = stage; e->b = b; e->aux = aux;
    }
    S->stats->n_events++;
}

static int64_t lut(const server* S, int stage, int b) { return S->opts->lut_ns[(int64_t)stage * S->b_max + (b - 1)]; }

/* all requests that have arrived by `now` join the queue; N_Q = next_arrival - q_head */
static void admit(server* S)
{
    while (S->next_arrival < S->n && S->arrival[S->next_arrival] <= S->now) S->next_arrival++;
}
static int64_t queue_size(const server* S) { return S->next_arrival - S->q_head; }

/* pop `count` requests from the head of the queue into slots [0,count) of `bt` */
static void pop_into(server* S, batch* bt, int count)
{
    bt->b = count;
    for (int k = 0; k < count; ++k) {
        const int64_t id = S->q_head++;
        bt->ids[k] = (int32_t)id;
        if (!S->forced) memcpy(bt->act + (int64_t)k * S->sample_bytes[0], S->pool + id * S->sample_bytes[0], (size_t)S->sample_bytes[0]);
    }
}

/* Process segment `stage` and its exit on the whole batch; exited samples complete at the new
 * `now`.  On return the batch holds the survivors, compacted in order, with the segment's output. */
static void proc_until_exit(server* S, batch* bt, int stage, int catchup, char* scratch, int32_t* scratch_ids)
{
    const int b = bt->b, last = stage == S->n_stages - 1;
    uint8_t flag[1024]; int32_t label[1024]; float conf[1024]; int64_t score[1024];
    log_event(S, catchup ? ORC_EV_PROC_CATCHUP : ORC_EV_PROC, stage, b, 0);
    S->stats->seg_runs[stage]++; S->stats->seg_samples[stage] += b;
    if (S->forced) {
        for (int k = 0; k < b; ++k) { flag[k] = (uint8_t)(last || S->forced[bt->ids[k]] == stage); label[k] = -1; conf[k] = 0.f; score[k] = 0; }
    } else {
        int rc = orc_stage_forward(S->blob, S->bytes, stage, b, bt->act, scratch);
        if (!rc) rc = orc_exit_head(S->blob, S->bytes, stage, b, scratch, S->thr[stage], label, conf, score, flag, NULL);
        if (rc) { S->err = rc; return; }
    }
    S->now += lut(S, stage, b);                       /* virtual clock: segment time incl. its exit head */
    for (int k = 0; k < b; ++k)
        if (flag[k]) {
            orc_result* r = &S->results[bt->ids[k]];
            r->exit_idx = stage; r->label = label[k]; r->conf = conf[k]; r->pad_ = 0; r->score = score[k];
            r->latency_ns = S->now - S->arrival[bt->ids[k]];
            S->done++;
        }
    int b_rem = 0;
    if (S->forced) {
        for (int k = 0; k < b; ++k) if (!flag[k]) bt->ids[b_rem++] = bt->ids[k];
    } else {
        orc_compact_refill(S->out_bytes[stage], b, flag, scratch, bt->act, bt->ids, scratch_ids, NULL, NULL, 0, &b_rem, NULL);
        memcpy(bt->ids, scratch_ids, sizeof(int32_t) * (size_t)b_rem);
    }
    bt->b = b_rem;
}

/* ---- stage pools (extension) ---------------------------------------------------------------------
 * Level 0 is the arrival queue; level i >= 1 holds, in order of arrival at the level, the samples
 * that survived exit i-1 (with segment i-1's output).  n_i = size of level i, b_i = min(n_i, B_max).
 * The server has `lanes` lanes (1..4); a lane is idle or runs one step: segment L on the b_L samples
 * that have waited longest at level L, started at t0 and finished at t0 + T[L][b_L].  At most one step
 * per level is in flight.  At time `now`:
 *   1. every step whose finish time has come ends, earliest first (equal times: lowest lane first): its
 *      samples that exit complete at the step's finish time, its survivors join level L+1 in slot order;
 *   2. the arrivals up to `now` join level 0;
 *   3. every idle lane, lowest first, may start a step.  A level is eligible when no step of it is in
 *      flight, n_i > 0 and its successor has room (i is the last level or n_{i+1} < B_max).  While
 *      some step is in flight only full batches are eligible (n_i >= B_max): a lane rather waits for the
 *      running steps than launch an under-filled segment beside them.  The preferred level P is the
 *      deepest eligible level with n_i >= B_max; if there is none, the deepest eligible level i >= 1; if
 *      there is none, level 0 if eligible; if there is none the lane stays idle;
 *      with an SLO (T_SLO >= 0) a level i >= 1, i != P, n_i > 0, no step of it in flight, whose successor
 *      has room overrides P when its oldest sample still meets the SLO if its remaining segments run now but
 *      not if P's step runs first: with
 *      T_slack = T_SLO - (now - arrival of that sample)   (Eq. 3) and
 *      T_rest = sum_{s >= i} T[s][b_i]                     (table of Sec. III-B, entering batch size as the bound),
 *      T_rest < T_slack  and not  T[P][b_P] + T_rest < T_slack; deepest such level first;
 *   4. the clock moves to the next event: the earliest finish time of a running step, or, when a lane is
 *      idle, the next arrival if that comes first; with nothing running and nothing waiting, the next arrival.
 * With one lane this is: choose, run, advance the clock by T[L][b_L], repeat.
 */
static int64_t serve_pooled_rest(const server* S, int level, int b)
{
    int64_t t = 0;
    for (int s = level; s < S->n_stages; ++s) t += lut(S, s, b);
    return t;
}

typedef struct {
    int busy, level, b_in, b_rem;          /* b_in samples entered, b_rem survive */
    int64_t t_finish;
    int32_t* ids;                          /* [b_in] on entry; the first b_rem are the survivors afterwards */
    char* act;                             /* the batch's input, then the survivors' output */
    uint8_t flag[1024]; int32_t label[1024]; float conf[1024]; int64_t score[1024];
    int32_t all_ids[1024];                 /* the ids that entered, in slot order (flag / label / ... are indexed alike) */
} lane_t;

static int serve_pooled(server* S)
{
    const int E = S->n_stages, B = S->b_max, cap = 2 * B;
    const int NL = S->opts->lanes > 1 ? S->opts->lanes : 1;
    if (NL > 4) return ORC_ERR_ARG;
    int cnt[8] = {0}, inflight[8] = {0};
    int32_t* ids[8] = {0}; char* act[8] = {0};
    int64_t max_bytes = 1;
    for (int s = 0; s < E; ++s) {
        if (S->sample_bytes[s] > max_bytes) max_bytes = S->sample_bytes[s];
        if (S->out_bytes[s] > max_bytes) max_bytes = S->out_bytes[s];
    }
    const size_t buf = S->forced ? 1 : (size_t)max_bytes * (size_t)B;
    lane_t* lane = (lane_t*)calloc((size_t)NL, sizeof(lane_t));
    for (int j = 0; j < NL; ++j) { lane[j].ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)B); lane[j].act = (char*)malloc(buf); }
    char* scratch = (char*)malloc(buf);
    int32_t* scratch_ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)B);
    for (int i = 1; i < E; ++i) {
        ids[i] = (int32_t*)malloc(sizeof(int32_t) * (size_t)cap);
        act[i] = (char*)malloc(S->forced ? 1 : (size_t)S->sample_bytes[i] * (size_t)cap);
    }
    S->now = S->arrival[0];
    while (S->done < S->n && !S->err) {
        /* 1. steps whose time has come end, earliest first */
        for (;;) {
            int j = -1;
            for (int k = 0; k < NL; ++k)
                if (lane[k].busy && lane[k].t_finish <= S->now && (j < 0 || lane[k].t_finish < lane[j].t_finish)) j = k;
            if (j < 0) break;
            lane_t* ln = &lane[j];
            const int L = ln->level;
            for (int k = 0; k < ln->b_in; ++k)
                if (ln->flag[k]) {
                    orc_result* r = &S->results[ln->all_ids[k]];
                    r->exit_idx = L; r->label = ln->label[k]; r->conf = ln->conf[k]; r->pad_ = 0; r->score = ln->score[k];
                    r->latency_ns = ln->t_finish - S->arrival[ln->all_ids[k]];
                    S->done++;
                }
            if (L + 1 < E && ln->b_rem > 0) {                                /* survivors wait for segment L+1 */
                if (cnt[L + 1] + ln->b_rem > cap) { S->err = ORC_ERR_OVERFLOW; break; }   /* cannot happen: the successor had room */
                memcpy(ids[L + 1] + cnt[L + 1], ln->ids, sizeof(int32_t) * (size_t)ln->b_rem);
                if (!S->forced) memcpy(act[L + 1] + S->sample_bytes[L + 1] * cnt[L + 1], ln->act, (size_t)(S->sample_bytes[L + 1] * ln->b_rem));
                cnt[L + 1] += ln->b_rem;
            }
            ln->busy = 0; inflight[L] = 0;
        }
        if (S->err || S->done >= S->n) break;
        /* 2. arrivals */
        admit(S);
        /* 3. idle lanes start steps */
        int running = 0;
        for (int k = 0; k < NL; ++k) running += lane[k].busy;
        for (int j = 0; j < NL && !S->err; ++j) {
            if (lane[j].busy) continue;
            const int64_t n0 = queue_size(S);
            int size[8], ok[8];
            for (int i = 0; i < E; ++i) {
                size[i] = i ? cnt[i] : (int)(n0 < 2 * (int64_t)B ? n0 : 2 * (int64_t)B);
                ok[i] = !inflight[i] && size[i] > 0 && (i == E - 1 || cnt[i + 1] < B) && (!running || size[i] >= B);
            }
            int P = -1;
            for (int i = E - 1; i >= 0 && P < 0; --i) if (ok[i] && size[i] >= B) P = i;
            for (int i = E - 1; i >= 1 && P < 0; --i) if (ok[i]) P = i;
            if (P < 0 && ok[0]) P = 0;
            if (P < 0) continue;
            int L = P;
            if (S->opts->t_slo_ns >= 0) {
                const int64_t t_first = lut(S, P, size[P] < B ? size[P] : B);
                for (int i = E - 1; i >= 1; --i) {
                    if (i == P || cnt[i] == 0 || inflight[i] || (i + 1 < E && cnt[i + 1] >= B)) continue;
                    int64_t oldest = S->arrival[ids[i][0]];
                    for (int k = 1; k < cnt[i]; ++k) if (S->arrival[ids[i][k]] < oldest) oldest = S->arrival[ids[i][k]];
                    const int64_t t_slack = S->opts->t_slo_ns - (S->now - oldest);
                    const int64_t t_rest = serve_pooled_rest(S, i, cnt[i] < B ? cnt[i] : B);
                    const int urgent = t_rest < t_slack && !(t_first + t_rest < t_slack);
                    S->stats->criterion_evals++;
                    log_event(S, ORC_EV_CRITERION, i, cnt[i] < B ? cnt[i] : B, urgent);
                    if (urgent) { L = i; S->stats->preemptions++; break; }
                }
            }
            /* take the batch from the front of level L */
            lane_t* ln = &lane[j];
            batch bt; bt.ids = ln->ids; bt.act = ln->act; bt.b = 0;
            if (L == 0) {
                pop_into(S, &bt, (int)(n0 < B ? n0 : B));
                S->stats->rounds++;
            } else {
                const int b = cnt[L] < B ? cnt[L] : B;
                const int64_t sb = S->sample_bytes[L];
                memcpy(bt.ids, ids[L], sizeof(int32_t) * (size_t)b);
                memmove(ids[L], ids[L] + b, sizeof(int32_t) * (size_t)(cnt[L] - b));
                if (!S->forced) {
                    memcpy(bt.act, act[L], (size_t)(sb * b));
                    memmove(act[L], act[L] + sb * b, (size_t)(sb * (cnt[L] - b)));
                }
                cnt[L] -= b; bt.b = b;
            }
            /* the step is computed now and takes effect at its finish time */
            const int b = bt.b, last = L == E - 1;
            ln->busy = 1; ln->level = L; ln->b_in = b; ln->t_finish = S->now + lut(S, L, b);
            inflight[L] = 1; ++running;
            memcpy(ln->all_ids, bt.ids, sizeof(int32_t) * (size_t)b);
            log_event(S, ORC_EV_PROC, L, b, j);
            S->stats->seg_runs[L]++; S->stats->seg_samples[L] += b;
            if (S->forced) {
                for (int k = 0; k < b; ++k) { ln->flag[k] = (uint8_t)(last || S->forced[bt.ids[k]] == L); ln->label[k] = -1; ln->conf[k] = 0.f; ln->score[k] = 0; }
                int b_rem = 0;
                for (int k = 0; k < b; ++k) if (!ln->flag[k]) bt.ids[b_rem++] = bt.ids[k];
                ln->b_rem = b_rem;
            } else {
                int rc = orc_stage_forward(S->blob, S->bytes, L, b, bt.act, scratch);
                if (!rc) rc = orc_exit_head(S->blob, S->bytes, L, b, scratch, S->thr[L], ln->label, ln->conf, ln->score, ln->flag, NULL);
                if (rc) { S->err = rc; break; }
                int b_rem = 0;
                orc_compact_refill(S->out_bytes[L], b, ln->flag, scratch, bt.act, bt.ids, scratch_ids, NULL, NULL, 0, &b_rem, NULL);
                memcpy(bt.ids, scratch_ids, sizeof(int32_t) * (size_t)b_rem);
                ln->b_rem = b_rem;
            }
        }
        if (S->err) break;
        /* 4. the next event */
        int64_t t_next = INT64_MAX;
        int idle = 0;
        for (int k = 0; k < NL; ++k) {
            if (lane[k].busy) { if (lane[k].t_finish < t_next) t_next = lane[k].t_finish; }
            else ++idle;
        }
        if (idle && S->next_arrival < S->n && S->arrival[S->next_arrival] < t_next) t_next = S->arrival[S->next_arrival];
        if (t_next == INT64_MAX) { S->err = ORC_ERR_ARG; break; }             /* cannot happen: something is running or yet to arrive */
        if (t_next > S->now) S->now = t_next;
    }
    S->stats->end_time_ns = S->now;
    for (int i = 1; i < E; ++i) { free(ids[i]); free(act[i]); }
    for (int j = 0; j < NL; ++j) { free(lane[j].ids); free(lane[j].act); }
    free(lane); free(scratch); free(scratch_ids);
    return S->err;
}

int orc_serve_stream(const void* blob, size_t bytes, int64_t n, const int64_t* arrival_ns, const void* input_pool,
                     const orc_serve_opts* opts, const int32_t* forced_exit, int n_stages_forced,
                     orc_result* results, orc_serve_stats* stats, orc_event* events, int64_t max_events)
{
    if (!opts || !stats || n < 0 || (n && (!arrival_ns || !results))) return ORC_ERR_ARG;
    if (opts->b_max < 1 || opts->b_max > 1024 || !opts->lut_ns || opts->clock != 1) return ORC_ERR_ARG;
    for (int64_t k = 1; k < n; ++k) if (arrival_ns[k] < arrival_ns[k - 1]) return ORC_ERR_ARG;
    server S; memset(&S, 0, sizeof S);
    memset(stats, 0, sizeof *stats);
    S.blob = blob; S.bytes = bytes; S.b_max = opts->b_max; S.n = n; S.arrival = arrival_ns; S.pool = (const char*)input_pool;
    S.opts = opts; S.forced = forced_exit; S.results = results; S.stats = stats; S.events = events; S.max_events = max_events;
    int64_t max_bytes = 1;
    if (forced_exit) {
        if (n_stages_forced < 1 || n_stages_forced > 8) return ORC_ERR_ARG;
        S.n_stages = n_stages_forced;
    } else {
        int rc = orc_blob_check(blob, bytes);
        if (rc) return rc;
        if (!input_pool && n) return ORC_ERR_ARG;
        int64_t in_b[8];
        rc = orc_query(blob, bytes, &S.n_stages, in_b, S.out_bytes, S.thr);
        if (rc) return rc;
        for (int s = 0; s < S.n_stages; ++s) {
            S.sample_bytes[s] = in_b[s];
            if (in_b[s] > max_bytes) max_bytes = in_b[s];
            if (S.out_bytes[s] > max_bytes) max_bytes = S.out_bytes[s];
        }
    }
    if (n == 0) return ORC_OK;
    if (opts->refill == 2) return serve_pooled(&S);

    batch active, fresh;
    const size_t buf = forced_exit ? 1 : (size_t)max_bytes * (size_t)S.b_max;
    active.ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)S.b_max); active.act = (char*)malloc(buf);
    fresh.ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)S.b_max); fresh.act = (char*)malloc(buf);
    char* scratch = (char*)malloc(buf); char* merged = (char*)malloc(buf);
    int32_t* scratch_ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)S.b_max);
    int32_t* merged_ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)S.b_max);
    const int E = S.n_stages;
    const int min_incr = opts->min_incr > 1 ? opts->min_incr : 1;

    S.now = arrival_ns[0];                               /* execution starts with the first request */
    while (S.done < n && !S.err) {
        admit(&S);
        if (queue_size(&S) == 0) { S.now = arrival_ns[S.next_arrival]; admit(&S); }   /* idle until the next arrival */
        if (opts->refill == 0 && opts->t_timeout_ns > 0) {
            /* adaptive batching <B_max, T_timeout> (Sec. II-D): a full batch is issued at once, an incomplete one
               when the batch-forming window, counted from the arrival of the oldest queued request, has passed */
            while (queue_size(&S) < S.b_max) {
                const int64_t deadline = arrival_ns[S.q_head] + opts->t_timeout_ns;
                if (S.now >= deadline) break;
                if (S.next_arrival < n && arrival_ns[S.next_arrival] <= deadline) {
                    if (arrival_ns[S.next_arrival] > S.now) S.now = arrival_ns[S.next_arrival];
                    admit(&S);
                } else {
                    S.now = deadline;
                    break;
                }
            }
        }
        int64_t nq = queue_size(&S);
        pop_into(&S, &active, (int)(nq < S.b_max ? nq : S.b_max));      /* B_act <- min(N_Q, B_max) */
        stats->rounds++;
        log_event(&S, ORC_EV_ROUND, 0, active.b, 0);
        for (int i = 0; i < E && !S.err; ++i) {
            proc_until_exit(&S, &active, i, 0, scratch, scratch_ids);   /* ProcUntilExit; leaves B_rem survivors */
            if (i == E - 1) break;
            int b_rem = active.b;
            if (b_rem == 0) break;
            while (opts->refill && b_rem < S.b_max && !S.err) {
                admit(&S);
                const int b_slack = S.b_max - b_rem;
                nq = queue_size(&S);
                const int b_incr = (int)(nq < b_slack ? nq : b_slack);
                if (b_incr < min_incr) break;
                /* Eq. 3: slack of the oldest sample of the active batch */
                int64_t oldest = arrival_ns[active.ids[0]];
                for (int k = 1; k < b_rem; ++k) if (arrival_ns[active.ids[k]] < oldest) oldest = arrival_ns[active.ids[k]];
                /* Eq. 4: new batch up to exit i, then the merged batch to the end */
                int64_t t_overhead = 0;
                for (int s = 0; s <= i; ++s) t_overhead += lut(&S, s, b_incr);
                for (int s = i + 1; s < E; ++s) t_overhead += lut(&S, s, b_rem + b_incr);
                int accept = 1;
                if (opts->t_slo_ns >= 0) {
                    const int64_t t_slack = opts->t_slo_ns - (S.now - oldest);
                    accept = t_overhead < t_slack;
                }
                stats->criterion_evals++;
                log_event(&S, ORC_EV_CRITERION, i, b_incr, accept);
                if (!accept) break;
                stats->preemptions++;                                   /* PreemptActiveBatch: survivors stay parked */
                pop_into(&S, &fresh, b_incr);
                for (int s = 0; s <= i && fresh.b > 0 && !S.err; ++s)   /* ProcFromStartUntilExit, no nested refill */
                    proc_until_exit(&S, &fresh, s, 1, scratch, scratch_ids);
                if (S.err) break;
                if (!forced_exit) {                                     /* merge: survivors first, newcomers appended */
                    uint8_t keep[1024]; memset(keep, 0, sizeof keep);
                    int br = 0, bm = 0;
                    orc_compact_refill(S.out_bytes[i], b_rem, keep, active.act, merged, active.ids, merged_ids,
                                       fresh.act, fresh.ids, fresh.b, &br, &bm);
                    char* t = active.act; active.act = merged; merged = t;
                    int32_t* ti = active.ids; active.ids = merged_ids; merged_ids = ti;
                    active.b = bm;
                } else {
                    for (int k = 0; k < fresh.b; ++k) active.ids[b_rem + k] = fresh.ids[k];
                    active.b = b_rem + fresh.b;
                }
                b_rem = active.b;                                       /* B_rem, B_act <- B_merged */
                log_event(&S, ORC_EV_MERGE, i, b_rem, fresh.b);
            }
        }
    }
    stats->end_time_ns = S.now;
    free(active.ids); free(active.act); free(fresh.ids); free(fresh.act); free(scratch); free(merged); free(scratch_ids); free(merged_ids);
    return S.err;
}
