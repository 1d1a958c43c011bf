// Stream serving: the exit-aware preemptive scheduler (Algorithm 1) as a plain host-side
// driver over the three device steps (segment, exit head, compaction / refill).
//
// The scheduler is written once against an executor interface; the GPU executor enqueues the
// kernels and reads the per-slot exit decisions back once per exit boundary (the only
// device-to-host crossing, as in the paper where B_exit is reported at each exit), the table
// executor replaces the network by a list of forced exits so that the policy can be tested on
// its own.
//
// Readings of Algorithm 1 where it is silent (kept identical to the documented policy):
//   - the last segment is processed after the printed loop ends and everyone left exits there;
//   - B_incr below max(1, min_incr) ends the refill loop; B_rem = 0 ends the round;
//   - Eq. 4 uses the latency table by segment and entering batch size, with the upper bound
//     B_rem + B_incr for the merged batch;
//   - the server idles until the next arrival when the queue is empty; FIFO admission.
//
// A second policy, stage pools (refill = 2), is an extension that is not in the paper: the survivors of
// exit i wait in a pool in front of segment i+1 and a segment is launched on a full batch of B_max
// whenever a pool (or the arrival queue) holds one.  See PoolScheduler below.
#include <chrono>
#include <cstring>
#include <thread>

#include "ee_ctx.hpp"

using namespace ee;

namespace {

struct SlotOutcome { uint8_t flag; int32_t label; float conf; int64_t score; };

// ---- clocks -----------------------------------------------------------------------------------
struct VirtualClock {
    const int64_t* lut; int b_max; int64_t t;
    void start(int64_t t0) { t = t0; }
    int64_t now() { return t; }
    void segment_done(int stage, int b) { t += lut[(int64_t)stage * b_max + b - 1]; }
    void idle_until(int64_t when) { if (when > t) t = when; }
};

struct WallClock {
    std::chrono::steady_clock::time_point origin; int64_t t0;
    void start(int64_t first_arrival) { origin = std::chrono::steady_clock::now(); t0 = first_arrival; }
    int64_t now() { return t0 + std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - origin).count(); }
    void segment_done(int, int) {}
    void idle_until(int64_t when)
    {
        while (now() < when) {
            const int64_t left = when - now();
            if (left > 200000) std::this_thread::sleep_for(std::chrono::nanoseconds(left - 100000));
        }
    }
};

// ---- executors ------------------------------------------------------------------------------------
// An executor owns the activations of the two batches Algorithm 1 juggles: the active batch and
// the catch-up batch.  Slots are implicit: batch slot k of the batch entering segment s lives in
// row k of that segment's packed input buffer.
struct TableExec {
    const int32_t* forced; int n_stages;
    int admit(const int32_t*, int) { return EE_OK; }
    int segment(int stage, const int32_t* ids, int b, SlotOutcome* out, int, int, int)
    {
        for (int k = 0; k < b; ++k) out[k] = SlotOutcome{(uint8_t)(stage == n_stages - 1 || forced[ids[k]] == stage), -1, 0.f, 0};
        return EE_OK;
    }
};

struct GpuExec {
    ee_ctx* ctx; const unsigned char* pool;

    explicit GpuExec(ee_ctx* c, const void* input_pool) : ctx(c), pool((const unsigned char*)input_pool) {}
    // A0: copy the queued inputs into slots [0, b) of segment 0's input buffer.  The kernel reads the
    // request ids straight from pinned host memory; two id blocks are used in turn, and an exit-head wait
    // lies between two admissions, so a block is never rewritten while a kernel may still read it.
    int admit(const int32_t* ids, int b)
    {
        int32_t* h_ids = ctx->h_ids[ctx->ids_turn];
        ctx->ids_turn ^= 1;
        std::memcpy(h_ids, ids, sizeof(int32_t) * (size_t)b);
        const int64_t sb = ctx->stage_in_bytes(0);
        hipError_t e;
        if (const OpPlan* p = ctx->admission_fold()) {
            // the first layer reads a zero-padded, folded copy of its input: admission writes that copy directly
            const OpDesc& d = p->d;
            const int es = ctx->net.elem_bytes();
            e = ctx->timed(EE_K_ADMIT, 0.0, (double)b * (sb + (double)p->Hp * p->Wp * 16 * es), [&] {
                return launch_space_to_depth(pool, ctx->pad_bufs[p->pad_buf], h_ids, b, d.h_in, d.w_in, d.c_in, p->Hp, p->Wp, d.pad, ctx->net.dtype, ctx->stream);
            });
        } else {
            e = ctx->timed(EE_K_ADMIT, 0.0, 2.0 * sb * b, [&] { return launch_admit(pool, ctx->in_buf[0], h_ids, b, sb, ctx->stream); });
        }
        return e == hipSuccess ? EE_OK : EE_ERR_DEVICE;
    }
    // A1 + A2 (+ A3 / A4): segment and exit head on the b samples in input slots [src_off, src_off + b); the
    // survivors (flags stay on the device) are packed into the next segment's input slots
    // [dst_off, dst_off + B_rem) right behind the head, dst_off > 0 merging a catch-up batch behind the parked
    // survivors; with ring_rows > 0 those slots form a ring and the destination wraps around its end.
    // Then the one device-to-host crossing of the boundary: the head kernel has written the per-slot outcomes
    // into pinned host memory and stores a sequence word when they are complete; the host polls that word.
    int segment(int stage, const int32_t*, int b, SlotOutcome* out, int src_off, int dst_off, int ring_rows)
    {
        const unsigned char* in = (const unsigned char*)ctx->in_buf[stage] + (int64_t)src_off * ctx->stage_in_bytes(stage);
        int rc = ctx->run_stage(stage, b, in, ctx->out_buf[stage], stage == 0 && ctx->admission_fold() != nullptr);
        if (!rc) rc = ctx->run_head(stage, b, ctx->out_buf[stage], ctx->net.exits[stage].thr, ctx->d_label, ctx->d_conf, ctx->d_score, ctx->d_flag, true);
        if (rc) return rc;
        long long compact_rec = -1;                     // index of the compaction launch's timing record, if one is kept
        if (stage + 1 < (int)ctx->in_buf.size()) {
            const int64_t sb = ctx->stage_out_bytes(stage);
            if (ctx->profiling) compact_rec = (long long)ctx->prof_used;
            hipError_t e = ctx->timed(EE_K_COMPACT, 0.0, 2.0 * sb * b, [&] {
                return launch_compact(ctx->d_flag, ctx->out_buf[stage], ctx->in_buf[stage + 1], nullptr, nullptr, b, sb, dst_off, ring_rows, nullptr, nullptr, ctx->stream);
            });
            if (e != hipSuccess) return EE_ERR_DEVICE;
        }
        if ((rc = wait_outcomes())) return rc;
        int kept = 0;
        for (int k = 0; k < b; ++k) {
            const HostOutcome& h = ctx->h_out[k];
            out[k] = SlotOutcome{(uint8_t)h.flag, h.label, h.conf, h.score};
            kept += h.flag == 0;
        }
        // the compaction launch was booked before B_rem was known: only the survivors are read and written
        if (compact_rec >= 0) ctx->prof[(size_t)compact_rec].bytes = 2.0 * (double)ctx->stage_out_bytes(stage) * kept;
        return EE_OK;
    }
    int wait_outcomes()
    {
        const unsigned want = ctx->seq;
        const auto t0 = std::chrono::steady_clock::now();
        for (unsigned spins = 0; __atomic_load_n(ctx->h_seq, __ATOMIC_ACQUIRE) != want; ++spins) {
            if ((spins & 0xFFFF) == 0xFFFF && std::chrono::steady_clock::now() - t0 > std::chrono::seconds(2)) {
                // no word after two seconds: let the runtime say what happened to the stream
                if (hipStreamSynchronize(ctx->stream) != hipSuccess) return EE_ERR_DEVICE;
                return __atomic_load_n(ctx->h_seq, __ATOMIC_ACQUIRE) == want ? EE_OK : EE_ERR_DEVICE;
            }
        }
        return EE_OK;
    }
};

// ---- what both policies share: the arrival queue, the books, one segment run --------------------------
template <class Exec, class Clock>
class ServeBase {
protected:
    ServeBase(Exec& ex, Clock& ck, int n_stages, const ee_trace* tr, const ee_serve_opts* o, ee_result* res,
              ee_serve_stats* st, ee_event* ev, int64_t max_ev)
        : exec(ex), clock(ck), E(n_stages), n(tr->n), arrival(tr->arrival_ns), opts(*o), results(res), stats(st), events(ev), max_events(max_ev),
          outcome(o->b_max) {}

    Exec& exec; Clock& clock;
    const int E; const int64_t n; const int64_t* arrival; const ee_serve_opts opts;
    ee_result* results; ee_serve_stats* stats; ee_event* events; const int64_t max_events;
    std::vector<SlotOutcome> outcome;
    int64_t arrived = 0, popped = 0, completed = 0;

    int64_t queued() const { return arrived - popped; }                       // N_Q
    void admit_arrivals() { const int64_t t = clock.now(); while (arrived < n && arrival[arrived] <= t) ++arrived; }
    int64_t lut(int s, int b) const { return opts.lut_ns[(int64_t)s * opts.b_max + b - 1]; }
    void log(int kind, int stage, int b, int aux)
    {
        if (events && stats->n_events < max_events) events[stats->n_events] = ee_event{clock.now(), kind, stage, b, aux};
        stats->n_events++;
    }
    void pop(int32_t* ids, int count) { for (int k = 0; k < count; ++k) ids[k] = (int32_t)popped++; }

    // ProcUntilExit for one segment: run it (the executor also packs the survivors for the next segment),
    // book the samples that leave, keep the survivors' ids in order.
    // `b` is updated to the number of survivors.
    int proc_until_exit(int32_t* ids, int& b, int stage, bool catchup, int src_off, int dst_off, int ring_rows)
    {
        log(catchup ? EE_EV_PROC_CATCHUP : EE_EV_PROC, stage, b, 0);
        stats->seg_runs[stage]++;
        stats->seg_samples[stage] += b;
        int rc = exec.segment(stage, ids, b, outcome.data(), src_off, dst_off, ring_rows);
        if (rc) return rc;
        clock.segment_done(stage, b);
        const int64_t t = clock.now();
        int kept = 0;
        for (int k = 0; k < b; ++k) {
            const SlotOutcome& o = outcome[k];
            if (o.flag) {
                ee_result& r = results[ids[k]];
                r.exit_idx = stage; r.label = o.label; r.conf = o.conf; r.pad_ = 0; r.score = o.score;
                r.latency_ns = t - arrival[ids[k]];
                ++completed;
            } else {
                ids[kept++] = ids[k];
            }
        }
        b = kept;
        return rc;
    }
};

// ---- Algorithm 1 ---------------------------------------------------------------------------------------
template <class Exec, class Clock>
class FluidScheduler : ServeBase<Exec, Clock> {
    using Base = ServeBase<Exec, Clock>;
    using Base::exec; using Base::clock; using Base::E; using Base::n; using Base::arrival; using Base::opts; using Base::stats;
    using Base::arrived; using Base::completed; using Base::queued; using Base::admit_arrivals; using Base::lut; using Base::log;
    using Base::pop; using Base::proc_until_exit;

public:
    FluidScheduler(Exec& ex, Clock& ck, int n_stages, const ee_trace* tr, const ee_serve_opts* o, ee_result* res,
                   ee_serve_stats* st, ee_event* ev, int64_t max_ev)
        : Base(ex, ck, n_stages, tr, o, res, st, ev, max_ev), active(o->b_max), fresh(o->b_max) {}

    int run()
    {
        clock.start(arrival[0]);
        int rc = EE_OK;
        while (completed < n && !rc) {
            admit_arrivals();
            if (queued() == 0) { clock.idle_until(arrival[arrived]); admit_arrivals(); }
            rc = start_round();
            for (int i = 0; i < E && !rc && b_act > 0; ++i) {
                rc = proc_until_exit(active.data(), b_act, i, /*catchup=*/false, 0, /*merge_at=*/0, 0);
                if (rc || i == E - 1 || b_act == 0) break;
                if (opts.refill) rc = refill_at_exit(i);
            }
        }
        stats->end_time_ns = clock.now();
        return rc;
    }

private:
    std::vector<int32_t> active, fresh;      // request ids per slot
    int b_act = 0;

    int start_round()
    {
        b_act = (int)std::min<int64_t>(queued(), opts.b_max);                 // B_act <- min(N_Q, B_max)
        pop(active.data(), b_act);
        stats->rounds++;
        log(EE_EV_ROUND, 0, b_act, 0);
        return exec.admit(active.data(), b_act);
    }

    // The inner loop of Algorithm 1 at exit i: while there is room, take B_incr requests, check the
    // SLO criterion, let them catch up to exit i and merge them behind the parked survivors.
    int refill_at_exit(int i)
    {
        int b_rem = b_act;
        const int min_incr = std::max(1, (int)opts.min_incr);
        while (b_rem < opts.b_max) {
            admit_arrivals();
            const int b_slack = opts.b_max - b_rem;
            const int b_incr = (int)std::min<int64_t>(queued(), b_slack);
            if (b_incr < min_incr) break;
            int64_t t_overhead = 0;                                               // Eq. 4
            for (int s = 0; s <= i; ++s) t_overhead += lut(s, b_incr);
            for (int s = i + 1; s < E; ++s) t_overhead += lut(s, b_rem + b_incr);
            bool accept = true;
            if (opts.t_slo_ns >= 0) {                                             // Eq. 3
                int64_t oldest = arrival[active[0]];
                for (int k = 1; k < b_rem; ++k) oldest = std::min(oldest, arrival[active[k]]);
                const int64_t t_slack = opts.t_slo_ns - (clock.now() - oldest);
                accept = t_overhead < t_slack;
            }
            stats->criterion_evals++;
            log(EE_EV_CRITERION, i, b_incr, accept ? 1 : 0);
            if (!accept) break;
            stats->preemptions++;                                                 // the survivors stay parked in their slots
            int b_new = b_incr;
            pop(fresh.data(), b_new);
            int rc = exec.admit(fresh.data(), b_new);
            for (int s = 0; s <= i && !rc && b_new > 0; ++s)                      // catch-up run, no nested refill
                rc = proc_until_exit(fresh.data(), b_new, s, true, 0, s == i ? b_rem : 0, 0);
            if (rc) return rc;
            for (int k = 0; k < b_new; ++k) active[b_rem + k] = fresh[k];
            b_rem += b_new;                                                       // B_merged
            log(EE_EV_MERGE, i, b_rem, b_new);
        }
        b_act = b_rem;
        return EE_OK;
    }
};

// ---- stage pools (extension) ------------------------------------------------------------------------------
// Level 0 is the arrival queue; level i >= 1 is a first-in first-out pool of the samples that survived
// exit i-1, parked in segment i's input slots, which form a ring of 2 B_max rows.  A batch is the front
// min(n_i, B_max) samples of one level.  Which level runs next:
//   the preferred level is the deepest one that holds a full batch; failing that the deepest non-empty pool
//   (samples in flight finish before new ones start); failing that the queue; failing that the server idles;
//   with an SLO, a pool whose oldest sample still meets it if the pool's remaining segments run now
//   (T_rest < T_slack, Eq. 3 with the latency table) but not if the preferred step runs first
//   (not T_first + T_rest < T_slack) goes first instead, the deepest such pool whose successor is not full.
// A segment never runs while the pool behind it holds a full batch, so a pool never exceeds 2 B_max - 1
// samples; batches start at ring row 0 or B_max and never wrap (a pool that is emptied restarts at row 0).
template <class Exec, class Clock>
class PoolScheduler : ServeBase<Exec, Clock> {
    using Base = ServeBase<Exec, Clock>;
    using Base::exec; using Base::clock; using Base::E; using Base::n; using Base::arrival; using Base::opts; using Base::stats;
    using Base::arrived; using Base::completed; using Base::queued; using Base::admit_arrivals; using Base::lut; using Base::log;
    using Base::pop; using Base::proc_until_exit;

public:
    PoolScheduler(Exec& ex, Clock& ck, int n_stages, const ee_trace* tr, const ee_serve_opts* o, ee_result* res,
                  ee_serve_stats* st, ee_event* ev, int64_t max_ev)
        : Base(ex, ck, n_stages, tr, o, res, st, ev, max_ev), B(o->b_max), ring(2 * o->b_max), batch(o->b_max)
    {
        for (int i = 0; i < E; ++i) { ids[i].assign(i ? ring : 0, -1); head[i] = cnt[i] = 0; }
    }

    int run()
    {
        clock.start(arrival[0]);
        int rc = EE_OK;
        while (completed < n && !rc) {
            admit_arrivals();
            const int level = choose();
            if (level < 0) { clock.idle_until(arrival[arrived]); continue; }
            rc = run_level(level);
        }
        stats->end_time_ns = clock.now();
        return rc;
    }

private:
    const int B, ring;
    std::vector<int32_t> ids[8];             // request ids of the pools, same ring geometry as the activations
    int head[8], cnt[8];
    std::vector<int32_t> batch;

    int size_of(int level) const { return level ? cnt[level] : (int)std::min<int64_t>(queued(), INT32_MAX); }
    int batch_of(int level) const { return std::min(size_of(level), B); }

    int choose()
    {
        int pref = -1;
        for (int i = E - 1; i >= 0 && pref < 0; --i) if (size_of(i) >= B) pref = i;
        for (int i = E - 1; i >= 1 && pref < 0; --i) if (cnt[i] > 0) pref = i;
        if (pref < 0 && queued() > 0) pref = 0;
        if (pref < 0 || opts.t_slo_ns < 0) return pref;
        const int64_t t_first = lut(pref, batch_of(pref));
        for (int i = E - 1; i >= 1; --i) {
            if (i == pref || cnt[i] == 0 || (i + 1 < E && cnt[i + 1] >= B)) continue;
            const int b = batch_of(i);
            const int64_t t_slack = opts.t_slo_ns - (clock.now() - arrival[ids[i][head[i]]]);   // the front is the oldest
            int64_t t_rest = 0;
            for (int s = i; s < E; ++s) t_rest += lut(s, b);
            const bool urgent = t_rest < t_slack && !(t_first + t_rest < t_slack);
            stats->criterion_evals++;
            log(EE_EV_CRITERION, i, b, urgent ? 1 : 0);
            if (urgent) { stats->preemptions++; return i; }
        }
        return pref;
    }

    int run_level(int level)
    {
        int b = batch_of(level), src = 0, rc = EE_OK;
        if (level == 0) {
            pop(batch.data(), b);
            stats->rounds++;
            rc = exec.admit(batch.data(), b);
        } else {
            src = head[level];
            for (int k = 0; k < b; ++k) batch[k] = ids[level][src + k];
            cnt[level] -= b;
            head[level] = cnt[level] ? (src + b) % ring : 0;
        }
        if (rc) return rc;
        const bool last = level == E - 1;
        const int tail = last ? 0 : (head[level + 1] + cnt[level + 1]) % ring;
        rc = proc_until_exit(batch.data(), b, level, false, src, tail, ring);
        if (rc || last) return rc;
        if (cnt[level + 1] + b > ring - 1) return EE_ERR_OVERFLOW;                     // cannot happen, see above
        for (int k = 0; k < b; ++k) ids[level + 1][(tail + k) % ring] = batch[k];
        cnt[level + 1] += b;
        return EE_OK;
    }
};

int check_serve_args(const ee_trace* tr, const ee_serve_opts* o, const ee_result* res, int n_stages)
{
    if (!tr || !o || tr->n < 0 || (tr->n > 0 && (!tr->arrival_ns || !res))) return EE_ERR_ARG;
    if (o->b_max < 1 || o->b_max > 1024 || !o->lut_ns || n_stages < 1 || n_stages > 8) return EE_ERR_ARG;
    if ((o->clock != 0 && o->clock != 1) || o->refill < 0 || o->refill > 2) return EE_ERR_ARG;
    if (tr->n > INT32_MAX) return EE_ERR_OVERFLOW;
    for (int64_t k = 1; k < tr->n; ++k)
        if (tr->arrival_ns[k] < tr->arrival_ns[k - 1]) return EE_ERR_ARG;
    return EE_OK;
}

}  // namespace

extern "C" int ee_serve_stream(ee_ctx* ctx, const ee_trace* trace, const void* input_pool, const ee_serve_opts* opts,
                               ee_result* results, ee_serve_stats* stats, ee_event* events, int64_t max_events)
{
    if (!ctx) return EE_ERR_ARG;
    const int n_stages = (int)ctx->net.stages.size();
    int rc = check_serve_args(trace, opts, results, n_stages);
    if (rc) return rc;
    if (opts->b_max > ctx->b_max) return EE_ERR_ARG;
    ee_serve_stats local;
    if (!stats) stats = &local;
    std::memset(stats, 0, sizeof *stats);
    if (trace->n == 0) return EE_OK;
    if (!input_pool || (reinterpret_cast<uintptr_t>(input_pool) & 15u)) return EE_ERR_ARG;
    GpuExec exec(ctx, input_pool);
    if (opts->clock == 1) {
        VirtualClock ck{opts->lut_ns, opts->b_max, 0};
        rc = opts->refill == 2 ? PoolScheduler<GpuExec, VirtualClock>(exec, ck, n_stages, trace, opts, results, stats, events, max_events).run()
                               : FluidScheduler<GpuExec, VirtualClock>(exec, ck, n_stages, trace, opts, results, stats, events, max_events).run();
    } else {
        WallClock ck{};
        rc = opts->refill == 2 ? PoolScheduler<GpuExec, WallClock>(exec, ck, n_stages, trace, opts, results, stats, events, max_events).run()
                               : FluidScheduler<GpuExec, WallClock>(exec, ck, n_stages, trace, opts, results, stats, events, max_events).run();
    }
    if (hipStreamSynchronize(ctx->stream) != hipSuccess && !rc) rc = EE_ERR_DEVICE;    // the call is synchronous
    return rc;
}

extern "C" int ee_schedule_sim(int n_stages, const ee_trace* trace, const int32_t* forced_exit, const ee_serve_opts* opts,
                               ee_result* results, ee_serve_stats* stats, ee_event* events, int64_t max_events)
{
    int rc = check_serve_args(trace, opts, results, n_stages);
    if (rc) return rc;
    if (opts->clock != 1 || (trace->n > 0 && !forced_exit)) return EE_ERR_ARG;
    ee_serve_stats local;
    if (!stats) stats = &local;
    std::memset(stats, 0, sizeof *stats);
    if (trace->n == 0) return EE_OK;
    TableExec exec{forced_exit, n_stages};
    VirtualClock ck{opts->lut_ns, opts->b_max, 0};
    if (opts->refill == 2) return PoolScheduler<TableExec, VirtualClock>(exec, ck, n_stages, trace, opts, results, stats, events, max_events).run();
    return FluidScheduler<TableExec, VirtualClock>(exec, ck, n_stages, trace, opts, results, stats, events, max_events).run();
}
