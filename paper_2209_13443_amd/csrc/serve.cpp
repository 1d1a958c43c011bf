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
    static constexpr bool is_virtual = true;
    const int64_t* lut; int b_max; int64_t t;
    void start(int64_t t0) { t = t0; }
    int64_t now() { return t; }
    void segment_done(int stage, int b) { t += lut[(int64_t)stage * b_max + b - 1]; }
    void idle_until(int64_t when) { if (when > t) t = when; }
};

struct WallClock {
    static constexpr bool is_virtual = false;
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
    std::vector<SlotOutcome> held[4];            // lanes: the outcomes of the step a lane is running
    int lanes() const { return 4; }
    int admit(int, const int32_t*, int) { return EE_OK; }
    int segment(int stage, const int32_t* ids, int b, SlotOutcome* out, int, int, int)
    {
        for (int k = 0; k < b; ++k) out[k] = SlotOutcome{(uint8_t)(stage == n_stages - 1 || forced[ids[k]] == stage), -1, 0.f, 0};
        return EE_OK;
    }
    int launch(int lane, int stage, const int32_t* ids, int b, int, int, int)
    {
        held[lane].resize((size_t)b);
        return segment(stage, ids, b, held[lane].data(), 0, 0, 0);
    }
    bool done(int) { return true; }
    int collect(int lane, int b, SlotOutcome* out)
    {
        for (int k = 0; k < b; ++k) out[k] = held[lane][(size_t)k];
        return EE_OK;
    }
    int pack(int, int, int, int, int, int) { return EE_OK; }
    void book_pack(int, int, int) {}
};

// Zero-copy compaction (zc): a sample that survives an exit stays where the segment wrote it.  Every level behind the
// first owns a set of sample slots; a step takes free slots of the next level for its outputs, the segment's last layer
// scatters into them, and "compaction" is the host writing the survivors' slot numbers into the row -> slot map of the
// next level while the slots of the samples that left, and the input slots the step consumed, return to the free list.
// The schedulers keep addressing batch rows exactly as with the copying kernel; only this executor translates.
struct GpuExec {
    ee_ctx* ctx; const unsigned char* pool;
    bool zc;
    std::vector<uint16_t> row2slot[8], free_slots[8];
    struct Step { SlotTab in, out; int b = 0, stage = -1, dst = -1, ring = 0; bool has_out = false; } step_of[4];

    explicit GpuExec(ee_ctx* c, const void* input_pool, bool zero_copy = false) : ctx(c), pool((const unsigned char*)input_pool), zc(zero_copy)
    {
        if (!zc) return;
        for (size_t s = 1; s < ctx->in_buf.size() && s < 8; ++s) {
            row2slot[s].assign((size_t)ctx->zc_slots, 0);
            free_slots[s].resize((size_t)ctx->zc_slots);
            for (int k = 0; k < ctx->zc_slots; ++k) free_slots[s][(size_t)k] = (uint16_t)(ctx->zc_slots - 1 - k);
        }
    }
    // the step's tables: input rows [src_off, src_off + b) of `stage` through the map, fresh slots of the next level
    int zc_begin(int lane, int stage, int b, int src_off, int ring_rows)
    {
        Step& st = step_of[lane];
        st.b = b; st.stage = stage; st.dst = -1; st.ring = ring_rows;
        const int E = (int)ctx->in_buf.size();
        if (stage > 0) {
            const int rows = (int)row2slot[stage].size();
            for (int k = 0; k < b; ++k) st.in.s[k] = row2slot[stage][(size_t)((src_off + k) % rows)];
        }
        st.has_out = stage + 1 < E;
        if (st.has_out) {
            std::vector<uint16_t>& fr = free_slots[stage + 1];
            if ((int)fr.size() < b) return EE_ERR_OVERFLOW;            // cannot happen: five blocks cover what can be held
            for (int k = 0; k < b; ++k) { st.out.s[k] = fr.back(); fr.pop_back(); }
        }
        // both tables go to the lane's device buffer in one tiny launch ahead of the step's kernels
        if (launch_upload_slots(st.in, st.out, ctx->d_slots, ctx->stream) != hipSuccess) return EE_ERR_DEVICE;
        ctx->zc_in = stage > 0 ? ctx->d_slots : nullptr;
        ctx->zc_out = st.has_out ? ctx->d_slots + EE_ZC_MAX_B : nullptr;
        return EE_OK;
    }
    // the step has ended (its exit head has reported): the input slots it read are free again
    void zc_release_inputs(int lane)
    {
        Step& st = step_of[lane];
        if (st.stage > 0)
            for (int k = 0; k < st.b; ++k) free_slots[st.stage].push_back(st.in.s[k]);
    }
    // "compaction": survivors keep their slots, which become rows dst_off.. of the next level in slot order
    void zc_pack(int lane, int dst_off, int ring_rows)
    {
        Step& st = step_of[lane];
        if (!st.has_out) return;
        const HostOutcome* h = ctx->lanes[(size_t)lane].h_out;
        std::vector<uint16_t>& map = row2slot[st.stage + 1];
        const int rows = ring_rows > 0 ? ring_rows : (int)map.size();
        int j = 0;
        for (int k = 0; k < st.b; ++k) {
            if (outcome_exits(h[k])) free_slots[st.stage + 1].push_back(st.out.s[k]);
            else map[(size_t)((dst_off + j++) % rows)] = st.out.s[k];
        }
        st.has_out = false;
    }
    // where the step's kernels read and write
    const void* step_in(int stage, int src_off) const
    {
        return (const unsigned char*)ctx->in_buf[stage] + (zc && stage > 0 ? 0 : (int64_t)src_off * ctx->stage_in_bytes(stage));
    }
    void* step_out(int stage) const { return zc && stage + 1 < (int)ctx->in_buf.size() ? ctx->in_buf[stage + 1] : ctx->out_buf[stage]; }
    int run_step(int lane, int stage, int b, int src_off, int ring_rows)
    {
        if (zc) { const int rc = zc_begin(lane, stage, b, src_off, ring_rows); if (rc) return rc; }
        ctx->gap_fuse_dst = ctx->sums;                   // the segment's last layer pools for the exit head where it can
        int rc = ctx->run_stage(stage, b, step_in(stage, src_off), step_out(stage), stage == 0 && ctx->admission_fold() != nullptr);
        ctx->gap_fuse_dst = nullptr;
        if (!rc) rc = ctx->run_head(stage, b, step_out(stage), ctx->net.exits[stage].thr, ctx->d_label, ctx->d_conf, ctx->d_score, ctx->d_flag, true, nullptr, ctx->zc_out, ctx->gap_fused);
        ctx->zc_in = ctx->zc_out = nullptr;
        return rc;
    }
    // A0: copy the queued inputs into slots [0, b) of segment 0's input buffer.  The kernel reads the
    // request ids straight from pinned host memory; two id blocks are used in turn, and an exit-head wait
    // lies between two admissions, so a block is never rewritten while a kernel may still read it.
    int lanes() const { return (int)ctx->lanes.size(); }
    int admit(int lane, const int32_t* ids, int b)
    {
        ctx->bind_lane(lane);
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
                return launch_space_to_depth(pool, ctx->pad_bufs[p->pad_buf], h_ids, b, d.h_in, d.w_in, d.c_in, p->Hp, p->Wp, d.pad, ctx->net.dtype, ctx->stream, true);
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
    // Then the one device-to-host crossing of the boundary: the head kernel writes the per-slot outcomes into pinned
    // host memory, every record with the launch's tag; the host polls the records until all of them carry it.
    int segment(int stage, const int32_t*, int b, SlotOutcome* out, int src_off, int dst_off, int ring_rows)
    {
        ctx->bind_lane(0);
        int rc = run_step(0, stage, b, src_off, ring_rows);
        if (rc) return rc;
        long long compact_rec = -1;                     // index of the compaction launch's timing record, if one is kept
        if (!zc && stage + 1 < (int)ctx->in_buf.size()) {
            const int64_t sb = ctx->stage_out_bytes(stage);
            if (ctx->profiling) compact_rec = (long long)ctx->prof_used;
            hipError_t e = ctx->timed(EE_K_COMPACT, 0.0, 2.0 * sb * b, [&] {
                return launch_compact(ctx->d_flag, ctx->out_buf[stage], ctx->in_buf[stage + 1], nullptr, nullptr, b, sb, dst_off, ring_rows, nullptr, nullptr, ctx->stream);
            });
            if (e != hipSuccess) return EE_ERR_DEVICE;
        }
        if ((rc = ctx->wait_head())) return rc;
        int kept = 0;
        for (int k = 0; k < b; ++k) {
            const Outcome h = ctx->head_outcome(k);
            out[k] = SlotOutcome{h.flag, h.label, h.conf, h.score};
            kept += h.flag == 0;
        }
        if (zc) { zc_release_inputs(0); zc_pack(0, dst_off, ring_rows); }
        // the compaction launch was booked before B_rem was known: only the survivors are read and written
        if (compact_rec >= 0) ctx->prof[(size_t)compact_rec].bytes = 2.0 * (double)ctx->stage_out_bytes(stage) * kept;
        return EE_OK;
    }
    // ---- several steps in flight: the same device work in three parts -----------------------------------------
    // launch: segment and exit head of the b samples in input slots [src_off, src_off + b) on the lane's stream.  Rows that
    // another lane's compaction kernel wrote are waited for with that lane's event.  eager_dst >= 0: the compaction into
    // the next segment's ring at that row follows right behind the head (single-lane serving: nothing can change the
    // ring before this step ends).
    int launch(int lane, int stage, const int32_t*, int b, int src_off, int eager_dst, int ring_rows)
    {
        ctx->bind_lane(lane);
        // (zero-copy: the rows were written by segment kernels that had ended before the host learned of the survivors)
        if (stage > 0 && !zc)
            for (size_t j = 0; j < ctx->lanes.size(); ++j)
                if ((int)j != lane && ctx->lanes[j].packed_set[stage] && hipStreamWaitEvent(ctx->stream, ctx->lanes[j].packed[stage], 0) != hipSuccess)
                    return EE_ERR_DEVICE;
        int rc = run_step(lane, stage, b, src_off, ring_rows);
        if (zc) step_of[lane].dst = eager_dst;
        else if (!rc && eager_dst >= 0) rc = pack(lane, stage, b, -1, eager_dst, ring_rows);
        return rc;
    }
    bool done(int lane)
    {
        if (lane == ctx->lane) return ctx->head_reported();              // the bound lane's counters are the context's
        const LaneState& L = ctx->lanes[(size_t)lane];
        return outcomes_ready(L.h_out, L.head_b, outcome_tag(L.seq));
    }
    int collect(int lane, int b, SlotOutcome* out)
    {
        ctx->bind_lane(lane);
        const int rc = ctx->wait_head();
        if (rc) return rc;
        for (int k = 0; k < b; ++k) {
            const Outcome h = ctx->head_outcome(k);
            out[k] = SlotOutcome{h.flag, h.label, h.conf, h.score};
        }
        if (zc) zc_release_inputs(lane);
        return EE_OK;
    }
    // compaction of the lane's step into the next segment's ring at row dst_off; kept: the survivors, when known (timing books)
    int pack(int lane, int stage, int b, int kept, int dst_off, int ring_rows)
    {
        if (stage + 1 >= (int)ctx->in_buf.size()) return EE_OK;
        if (zc) { zc_pack(lane, dst_off, ring_rows); return EE_OK; }
        ctx->bind_lane(lane);
        const int64_t sb = ctx->stage_out_bytes(stage);
        hipError_t e = ctx->timed(EE_K_COMPACT, 0.0, 2.0 * sb * (kept >= 0 ? kept : b), [&] {
            return launch_compact(ctx->d_flag, ctx->out_buf[stage], ctx->in_buf[stage + 1], nullptr, nullptr, b, sb, dst_off, ring_rows, nullptr, nullptr, ctx->stream);
        });
        if (e != hipSuccess) return EE_ERR_DEVICE;
        pack_rec[lane] = ctx->profiling ? (long long)ctx->prof_used - 1 : -1;
        LaneState& L = ctx->lanes[(size_t)lane];
        if (ctx->lanes.size() > 1) {
            if (hipEventRecord(L.packed[stage + 1], ctx->stream) != hipSuccess) return EE_ERR_DEVICE;
            L.packed_set[stage + 1] = true;
        }
        return EE_OK;
    }
    long long pack_rec[4] = {-1, -1, -1, -1};     // timing record of each lane's latest compaction launch
    // a compaction that was launched before its step's outcome was known is booked with the survivors that really moved
    void book_pack(int lane, int stage, int kept)
    {
        if (zc) { zc_pack(lane, step_of[lane].dst, step_of[lane].ring); return; }
        if (pack_rec[lane] >= 0 && ctx->profiling) ctx->prof[(size_t)pack_rec[lane]].bytes = 2.0 * (double)ctx->stage_out_bytes(stage) * kept;
        pack_rec[lane] = -1;
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
            if (opts.refill == 0 && opts.t_timeout_ns > 0) wait_for_batch();
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

    // Adaptive batching <B_max, T_timeout> (Sec. II-D): a full batch is issued at once, an incomplete one when the
    // batch-forming window, counted from the arrival of the oldest queued request, has passed.
    void wait_for_batch()
    {
        while (queued() < opts.b_max) {
            const int64_t deadline = arrival[Base::popped] + opts.t_timeout_ns;
            if (clock.now() >= deadline) break;
            if (arrived < n && arrival[arrived] <= deadline) {
                clock.idle_until(arrival[arrived]);
                admit_arrivals();
            } else {
                clock.idle_until(deadline);
                break;
            }
        }
    }

    int start_round()
    {
        b_act = (int)std::min<int64_t>(queued(), opts.b_max);                 // B_act <- min(N_Q, B_max)
        pop(active.data(), b_act);
        stats->rounds++;
        log(EE_EV_ROUND, 0, b_act, 0);
        return exec.admit(0, active.data(), b_act);
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
            int rc = exec.admit(0, fresh.data(), b_new);
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
// exit i-1, parked in segment i's input slots.  A batch is the front min(n_i, B_max) samples of one level.
// The server has 1..4 lanes; a lane is idle or runs one step (one segment on one batch), and at most one step
// per level is in flight.  Whenever the clock reaches an event:
//   1. the steps that have ended are booked, earliest first: samples that exit complete at the step's end, the
//      survivors join the next level in slot order;
//   2. arrivals join the queue;
//   3. every idle lane, lowest first, may start a step.  A level is eligible when no step of it is in flight, it
//      is not empty and its successor has room (fewer than B_max waiting); while a step is in flight only full
//      batches are eligible.  Preferred: the deepest eligible level holding a full batch; failing that the deepest
//      eligible pool (samples in flight finish before new ones start); failing that the queue; else the lane idles.
//      With an SLO, a pool whose oldest sample still meets it if the pool's remaining segments run now
//      (T_rest < T_slack, Eq. 3 with the latency table) but not if the preferred step runs first
//      (not T_first + T_rest < T_slack) goes first instead, the deepest such pool whose successor has room;
//   4. the clock moves on to the next end of a step, or to the next arrival when a lane is idle.
// Memory: segment i's input slots form a ring of three blocks of B_max rows.  A pool's content starts on a block
// boundary and is shorter than two blocks, a batch never crosses a boundary, and the content always starts in the
// block behind the batch that was taken last, so the rows a running step still reads are never written.
template <class Exec, class Clock>
class PoolScheduler : ServeBase<Exec, Clock> {
    using Base = ServeBase<Exec, Clock>;
    using Base::exec; using Base::clock; using Base::E; using Base::n; using Base::arrival; using Base::opts; using Base::stats;
    using Base::arrived; using Base::completed; using Base::queued; using Base::admit_arrivals; using Base::lut; using Base::log;
    using Base::pop; using Base::results; using Base::outcome;

public:
    PoolScheduler(Exec& ex, Clock& ck, int n_stages, const ee_trace* tr, const ee_serve_opts* o, ee_result* res,
                  ee_serve_stats* st, ee_event* ev, int64_t max_ev)
        : Base(ex, ck, n_stages, tr, o, res, st, ev, max_ev), B(o->b_max), ring(3 * o->b_max), NL(std::max(1, (int)o->lanes))
    {
        for (int i = 0; i < E; ++i) { ids[i].assign(i ? ring : 0, -1); head[i] = cnt[i] = 0; inflight[i] = false; }
        for (int j = 0; j < NL; ++j) run_of[j].ids.assign((size_t)B, -1);
    }

    int run()
    {
        clock.start(arrival[0]);
        int rc = EE_OK;
        while (completed < n && !rc) {
            for (int j; !rc && (j = ended_lane()) >= 0;) rc = finish(j);
            if (rc || completed >= n) break;
            admit_arrivals();
            int running = 0;
            for (int j = 0; j < NL; ++j) running += run_of[j].busy;
            for (int j = 0; j < NL && !rc; ++j) {
                if (run_of[j].busy) continue;
                const int level = choose(running > 0);
                if (level < 0) continue;
                rc = start(j, level);
                ++running;
            }
            if (rc) break;
            if (running == 0) { clock.idle_until(arrival[arrived]); continue; }       // nothing in flight, nothing waiting
            if constexpr (Clock::is_virtual) {
                int64_t t_next = INT64_MAX;
                for (int j = 0; j < NL; ++j) if (run_of[j].busy) t_next = std::min(t_next, run_of[j].t_finish);
                if (running < NL && arrived < n) t_next = std::min(t_next, arrival[arrived]);
                clock.idle_until(t_next);
            }
        }
        stats->end_time_ns = clock.now();
        return rc;
    }

private:
    struct Run { bool busy = false; int level = 0, b = 0, tail = 0; int64_t t_finish = 0; std::vector<int32_t> ids; };
    const int B, ring, NL;
    std::vector<int32_t> ids[8];             // request ids of the pools, same ring geometry as the activations
    int head[8], cnt[8];
    bool inflight[8];
    Run run_of[4];

    int size_of(int level) const { return level ? cnt[level] : (int)std::min<int64_t>(queued(), INT32_MAX); }
    int batch_of(int level) const { return std::min(size_of(level), B); }
    bool has_room_behind(int level) const { return level == E - 1 || cnt[level + 1] < B; }
    bool eligible(int level, bool full_only) const
    {
        return !inflight[level] && size_of(level) > 0 && has_room_behind(level) && (!full_only || size_of(level) >= B);
    }

    // the lane whose step has ended: on the virtual clock the earliest finish time that has come (lowest lane first),
    // on the wall clock the first lane whose exit head has reported
    int ended_lane()
    {
        int best = -1;
        for (int j = 0; j < NL; ++j) {
            if (!run_of[j].busy) continue;
            if constexpr (Clock::is_virtual) {
                if (run_of[j].t_finish <= clock.now() && (best < 0 || run_of[j].t_finish < run_of[best].t_finish)) best = j;
            } else {
                if (exec.done(j)) return j;
            }
        }
        return best;
    }

    int choose(bool full_only)
    {
        int pref = -1;
        for (int i = E - 1; i >= 0 && pref < 0; --i) if (eligible(i, full_only) && size_of(i) >= B) pref = i;
        for (int i = E - 1; i >= 1 && pref < 0; --i) if (eligible(i, full_only)) pref = i;
        if (pref < 0 && eligible(0, full_only)) pref = 0;
        if (pref < 0 || opts.t_slo_ns < 0) return pref;
        const int64_t t_first = lut(pref, batch_of(pref));
        for (int i = E - 1; i >= 1; --i) {
            if (i == pref || cnt[i] == 0 || inflight[i] || !has_room_behind(i)) continue;
            const int b = batch_of(i);
            int64_t oldest = arrival[ids[i][head[i]]];
            for (int k = 1; k < cnt[i]; ++k) oldest = std::min(oldest, arrival[ids[i][(head[i] + k) % ring]]);
            const int64_t t_slack = opts.t_slo_ns - (clock.now() - oldest);
            int64_t t_rest = 0;
            for (int s = i; s < E; ++s) t_rest += lut(s, b);
            const bool urgent = t_rest < t_slack && !(t_first + t_rest < t_slack);
            stats->criterion_evals++;
            log(EE_EV_CRITERION, i, b, urgent ? 1 : 0);
            if (urgent) { stats->preemptions++; return i; }
        }
        return pref;
    }

    int start(int j, int level)
    {
        Run& r = run_of[j];
        const int b = batch_of(level);
        int src = 0, rc = EE_OK;
        if (level == 0) {
            pop(r.ids.data(), b);
            stats->rounds++;
            rc = exec.admit(j, r.ids.data(), b);
        } else {
            src = head[level];                                        // a block boundary: the batch does not wrap
            for (int k = 0; k < b; ++k) r.ids[k] = ids[level][src + k];
            cnt[level] -= b;
            head[level] = (src / B + 1) * B % ring;                   // what is left, or comes next, starts in the next block
            if (cnt[level] > 0 && b != B) return EE_ERR_OVERFLOW;     // cannot happen: a partial batch empties its pool
        }
        if (rc) return rc;
        log(EE_EV_PROC, level, b, j);
        stats->seg_runs[level]++;
        stats->seg_samples[level] += b;
        r.busy = true; r.level = level; r.b = b;
        r.t_finish = clock.now() + (Clock::is_virtual ? lut(level, b) : 0);
        inflight[level] = true;
        // one lane: nothing can touch the next level's ring before this step ends, so its compaction is queued right away
        r.tail = level + 1 < E ? (head[level + 1] + cnt[level + 1]) % ring : 0;
        return exec.launch(j, level, r.ids.data(), b, src, NL == 1 && level + 1 < E ? r.tail : -1, ring);
    }

    int finish(int j)
    {
        Run& r = run_of[j];
        int rc = exec.collect(j, r.b, outcome.data());
        if (rc) return rc;
        const int64_t t = Clock::is_virtual ? r.t_finish : clock.now();
        const int level = r.level;
        int kept = 0;
        for (int k = 0; k < r.b; ++k) {
            const SlotOutcome& o = outcome[k];
            if (o.flag) {
                ee_result& out = results[r.ids[k]];
                out.exit_idx = level; out.label = o.label; out.conf = o.conf; out.pad_ = 0; out.score = o.score;
                out.latency_ns = t - arrival[r.ids[k]];
                ++completed;
            } else {
                r.ids[kept++] = r.ids[k];
            }
        }
        r.busy = false;
        inflight[level] = false;
        if (level == E - 1) return kept == 0 ? EE_OK : EE_ERR_DEVICE;               // the last exit takes everyone
        if (cnt[level + 1] + kept > 2 * B - 1) return EE_ERR_OVERFLOW;               // cannot happen: the successor had room
        const int tail = (head[level + 1] + cnt[level + 1]) % ring;
        if (NL == 1) {
            if (tail != r.tail) return EE_ERR_DEVICE;                                  // the ring did not move under a single lane
            exec.book_pack(j, level, kept);
        } else if (kept > 0) {
            rc = exec.pack(j, level, r.b, kept, tail, ring);
        }
        for (int k = 0; k < kept; ++k) ids[level + 1][(tail + k) % ring] = r.ids[k];
        cnt[level + 1] += kept;
        return rc;
    }
};

int check_serve_args(const ee_trace* tr, const ee_serve_opts* o, const ee_result* res, int n_stages)
{
    if (!tr || !o || tr->n < 0 || (tr->n > 0 && (!tr->arrival_ns || !res))) return EE_ERR_ARG;
    if (o->b_max < 1 || o->b_max > 1024 || !o->lut_ns || n_stages < 1 || n_stages > 8) return EE_ERR_ARG;
    if ((o->clock != 0 && o->clock != 1) || o->refill < 0 || o->refill > 2 || o->lanes < 0 || o->lanes > 4) return EE_ERR_ARG;
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
    if (opts->refill == 2 && opts->lanes > (int)ctx->lanes.size()) return EE_ERR_ARG;      // ee_lanes makes them, ahead of time
    ee_serve_stats local;
    if (!stats) stats = &local;
    std::memset(stats, 0, sizeof *stats);
    if (trace->n == 0) return EE_OK;
    if (!input_pool || (reinterpret_cast<uintptr_t>(input_pool) & 15u)) return EE_ERR_ARG;
    if (opts->zero_copy != 0 && opts->zero_copy != 1) return EE_ERR_ARG;
    if (opts->zero_copy && !ctx->zero_copy_ok) return EE_ERR_UNSUPPORTED;
    if (opts->zero_copy && opts->refill == 2 && opts->lanes > 2) return EE_ERR_ARG;      // the slots cover two steps in flight
    GpuExec exec(ctx, input_pool, opts->zero_copy != 0);
    if (opts->clock == 1) {
        VirtualClock ck{opts->lut_ns, opts->b_max, 0};
        rc = opts->refill == 2 ? PoolScheduler<GpuExec, VirtualClock>(exec, ck, n_stages, trace, opts, results, stats, events, max_events).run()
                               : FluidScheduler<GpuExec, VirtualClock>(exec, ck, n_stages, trace, opts, results, stats, events, max_events).run();
    } else {
        WallClock ck{};
        rc = opts->refill == 2 ? PoolScheduler<GpuExec, WallClock>(exec, ck, n_stages, trace, opts, results, stats, events, max_events).run()
                               : FluidScheduler<GpuExec, WallClock>(exec, ck, n_stages, trace, opts, results, stats, events, max_events).run();
    }
    for (const LaneState& L : ctx->lanes)                                                  // the call is synchronous
        if (hipStreamSynchronize(L.stream) != hipSuccess && !rc) rc = EE_ERR_DEVICE;
    ctx->bind_lane(0);
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
