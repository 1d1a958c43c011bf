// The library context: device copies of the packed weights, the pre-allocated activation
// workspace and the per-segment launch plans.
#pragma once
#include <chrono>

#include "ee_internal.hpp"

namespace ee {

enum Impl { IMPL_MFMA = 0, IMPL_MFMA_C4 = 1, IMPL_DIRECT = 2, IMPL_DW = 3, IMPL_POOL = 4, IMPL_MFMA_CPAD = 5, IMPL_MFMA_S2D = 6, IMPL_AVGPOOL = 7, IMPL_THIN = 8 };
enum { BUF_EXT_IN = -1, BUF_EXT_OUT = -2 };

struct OpPlan {
    OpDesc d;
    int impl = IMPL_DIRECT;
    void* w_dev = nullptr;      // packed weights
    void* b_dev = nullptr;      // bias, padded to the weight rows
    void* w3_dev = nullptr;     // int8 3x3 depthwise: weights packed per kernel row for the dot-product kernel
    int Kp = 0, kwp = 0, Hp = 0, Wp = 0;
    int src_buf = 0, dst_buf = 0, res_buf = 0;   // BUF_EXT_* or an index into Ctx::pool
    int pad_buf = -1;           // padded copy of the input: 4 channels + spatial border (IMPL_MFMA_C4), channels to 16 bytes (IMPL_MFMA_CPAD)
    int ci_eff = 0;             // input channels the matrix-core kernel sees (c_in, or c_in padded to a 16-byte multiple)
    // IMPL_MFMA_S2D: stride-2 first layer over <= 4 channels, run as a stride-1 convolution with a ks2 x ks2 kernel over the
    // zero-padded image folded into Hp x Wp super-pixels of 2 x 2 pixels x 4 channels (Hp, Wp, ks2 reuse the fields above)
    std::vector<int> cfg;       // kernel configuration per batch bucket (see ee_autotune); empty = by shape
    bool pair = false;          // this layer and the next one (a 1x1 layer that alone reads it) can run as one fused launch
    std::vector<int> pair_cfg;  // per batch bucket: configuration of the fused launch, 0 = run the two layers separately; empty = not tuned
    // this layer (a 1x1 expansion), the 3x3 depthwise layer behind it and the 1x1 projection behind that can run as one fused launch
    bool ir = false;
    bool ir_noexp = false;      // the block has no expansion: this layer is the depthwise layer, the projection follows it (two layers)
    bool ir_bneck = false;      // the block is a bottleneck block (1x1 -> 3x3 -> 1x1): its own kernel, the same table and switches
    bool ir_sc = false;         // a bottleneck block with the 1x1 convolution on its shortcut in front: this layer is that convolution (four layers)
    void* ir_ws = nullptr; void* ir_bs = nullptr;
    bool ir_stem = false;       // this layer is a folded stride-2 first convolution and the 3x3 / 2 max-pool behind it can run in the same launch (two layers)
    int ir_last() const { return ir_noexp || ir_stem ? 1 : ir_sc ? 3 : 2; }   // the block's last layer, counted from its head
    std::vector<int> ir_cfg;    // per batch bucket: 1 = the fused launch, 0 = the three layers separately; empty = not tuned
    void* ir_we = nullptr; void* ir_be = nullptr; void* ir_wd = nullptr; void* ir_bd = nullptr; void* ir_wp = nullptr; void* ir_bp = nullptr;
    int ir_kx = 0, ir_ce32 = 0;
    double ops_per_sample = 0, bytes_per_sample = 0, weight_bytes = 0;
};

// What one lane of the stream driver owns: a HIP stream, the intermediate tensors of a segment, the raw segment
// outputs, the exit head's scratch and outputs, and its block of pinned host memory.  Steps on different lanes
// run concurrently on the GPU; the input rings of the segments behind the first are shared by all lanes.
struct LaneState {
    hipStream_t stream = nullptr;
    bool own_stream = false;
    std::vector<void*> pool, pad_bufs, out_buf;
    void* in0 = nullptr;                         // input slots of the first segment
    int32_t* sums = nullptr; int32_t* gap_partial = nullptr; void* logits = nullptr;
    int32_t* d_label = nullptr; float* d_conf = nullptr; int64_t* d_score = nullptr; uint8_t* d_flag = nullptr;
    uint16_t* d_slots = nullptr;                 // the lane's two slot tables (zero-copy compaction)
    void* h_pinned = nullptr; HostOutcome* h_out = nullptr; int32_t* h_ids[2] = {nullptr, nullptr};
    unsigned seq = 0;
    int head_b = 0;
    int ids_turn = 0;
    hipEvent_t packed[8] = {};                   // recorded behind this lane's latest compaction into segment s's input ring
    bool packed_set[8] = {};
};

struct HeadScratch { int32_t* sums; int32_t* gap_partial; void* logits; };

struct ProfRec { int cls; int op; hipEvent_t e0, e1; double ops, bytes; };

}  // namespace ee

struct ee_ctx {
    ee::NetDesc net;
    int b_max = 0;
    hipStream_t stream = nullptr;
    std::vector<ee::OpPlan> plans;               // same order as net.ops
    std::vector<void*> pool;                     // intermediate activations, b_max samples each
    std::vector<size_t> pool_sample_bytes;
    std::vector<void*> pad_bufs;                 // zero-padded 4-channel input copies (first layers)
    std::vector<void*> owned;                    // every device allocation, for ee_destroy
    std::vector<void*> wfc_dev, bfc_dev;         // exit heads
    int32_t* sums = nullptr;                     // [b_max][C_max]
    int32_t* gap_partial = nullptr;              // [(b_max + 1024)][C_max] partial rows of the pooling splits
    void* logits = nullptr;                      // [b_max][n_cls]
    void* zero_page = nullptr;                   // zero bytes read in place of padding taps
    int* d_count = nullptr;                      // device int scratch (B_rem)
    // stream serving workspace
    std::vector<void*> in_buf, out_buf;          // per segment: packed input slots, raw output slots
    int32_t* d_ids = nullptr;                    // admission ids
    int32_t* d_label = nullptr; float* d_conf = nullptr; int64_t* d_score = nullptr; uint8_t* d_flag = nullptr;
    void* h_pinned = nullptr;                    // pinned, device-visible host memory: the three blocks below
    ee::HostOutcome* h_out = nullptr;            // [b_max] per-slot outcomes written by the exit-head kernel
    int32_t* h_ids[2] = {nullptr, nullptr};      // admission ids read by the admission kernel, used in turn
    unsigned seq = 0;                            // number of exit heads that have reported to the host: the latest one's tag follows from it
    int head_b = 0;                              // batch of that exit head: records [0, head_b) of h_out
    uint16_t* d_slots = nullptr;                 // the bound lane's two slot tables (zero-copy compaction)
    int ids_turn = 0;
    // zero-copy compaction (stream serving): slot tables of the step being enqueued, or null.  With zc_in, sample n of a
    // segment's input is slot zc_in->s[n] of act_in; with zc_out, sample n of its output goes to slot zc_out->s[n] of act_out.
    // Exit-head pooling fused into the last layer of a segment (int8): gap_fuse_op[s] is that layer (an index into plans) when
    // it can carry the pooling, else -1.  run_stage adds the sums into gap_fuse_dst when that is set and says so in gap_fused;
    // run_head then skips its pooling kernel.
    std::vector<int> gap_fuse_op;
    int32_t* gap_fuse_dst = nullptr;
    bool gap_fused = false;
    const uint16_t* zc_in = nullptr;             // device memory
    const uint16_t* zc_out = nullptr;
    bool zero_copy_ok = false;                   // every segment boundary can be served that way (set by ee_create)
    int zc_slots = 0;                            // sample slots in every in_buf behind the first
    int pair_mode = 1;                           // fused layer pairs: 0 never, 1 as the table says, 2 wherever possible
    int ir_mode = 1;                             // fused inverted-residual blocks: likewise
    // lanes of the stream driver: lanes[lane] is a copy of the per-lane members above while that lane is bound
    std::vector<ee::LaneState> lanes;
    int lane = 0;
    std::vector<size_t> pad_buf_bytes;           // size of every padded / folded input copy, for further lanes
    size_t c_max = 0;                            // widest exit head
    void bind_lane(int j);                       // makes lane j's stream and buffers the ones the launchers use
    // kernel timing
    bool profiling = false;
    std::vector<ee::ProfRec> prof;
    size_t prof_used = 0;

    int64_t stage_in_bytes(int s) const
    {
        const ee::StageDesc& st = net.stages[s];
        return (int64_t)st.in_h * st.in_w * st.in_c * net.elem_bytes();
    }
    int64_t stage_out_bytes(int s) const
    {
        const ee::StageDesc& st = net.stages[s];
        return (int64_t)st.out_h * st.out_w * st.out_c * net.elem_bytes();
    }

    // internal entry points shared by the C ABI and the stream driver (no argument checks)
    // first_packed: the first layer's folded input copy already holds these samples (admission wrote it)
    // only_op >= 0: just that layer (an index into plans; fused pairs run as separate layers then); only_op <= -2: just the
    // inverted-residual block headed by layer -2 - only_op (one launch or three, as ir_mode and the table say);
    // cfg_force > 0: that kernel configuration for every matrix-core layer instead of the table's
    int run_stage(int stage, int b_act, const void* act_in, void* act_out, bool first_packed = false, int only_op = -1, int cfg_force = 0);
    // the plan of segment 0's first layer when that layer reads a folded copy admission can write directly, else null
    const ee::OpPlan* admission_fold() const
    {
        const ee::StageDesc& st = net.stages[0];
        const ee::OpPlan& p = plans[st.first_op];
        if (p.impl != ee::IMPL_MFMA_S2D || p.src_buf != ee::BUF_EXT_IN) return nullptr;
        for (int k = 1; k < st.n_ops; ++k)           // nobody else may read the segment input: it is never written then
            if (plans[st.first_op + k].src_buf == ee::BUF_EXT_IN || plans[st.first_op + k].res_buf == ee::BUF_EXT_IN) return nullptr;
        return &p;
    }
    // launches layer `op` (an index into plans) on b samples with the given kernel configuration (0 = by shape)
    hipError_t launch_conv(int op, int b, const void* src, void* dst, const void* res, int cfg, const uint16_t* xs = nullptr, const uint16_t* ys = nullptr, int32_t* gap_sums = nullptr);
    // layers op and op + 1 as one fused launch: src feeds layer op, res and dst belong to layer op + 1
    hipError_t launch_pair(int op, int b, const void* src, void* dst, const void* res, int cfg);
    void fill_ir_args(int op, int b, ee::IrArgs& a) const;      // the block headed by layer `op`; x, res and y are left to the caller
    void fill_conv_args(int op, int b, ee::ConvArgs& a) const;
    static int bucket_of(int b) { int k = 0; while ((1 << k) < b) ++k; return k; }     // smallest k with 2^k >= b
    // to_host: the outcomes also go to h_out, every record with the tag of ++seq (the records are cleared first)
    // own: scratch memory to use instead of the context's (sums, gap_partial, logits)
    int run_head(int stage, int b_act, const void* act, float thr, int32_t* label, float* conf, int64_t* score, uint8_t* flag,
                 bool to_host = false, const ee::HeadScratch* own = nullptr, const uint16_t* slots = nullptr, bool pooled = false);
    // the bound lane's latest exit head with to_host has written all its records; wait_head spins until it has (EE_ERR_DEVICE
    // when the stream has failed or nothing has come after two seconds)
    bool head_reported() const { return ee::outcomes_ready(h_out, head_b, ee::outcome_tag(seq)); }
    int wait_head();
    ee::Outcome head_outcome(int k) const { return ee::decode_outcome(h_out[k], net.dtype == EE_I8); }
    // times `launch` with a pair of events attached to its dispatch when profiling
    template <typename F>
    hipError_t timed(int cls, double ops, double bytes, F&& launch, int op = -1);
};

template <typename F>
hipError_t ee_ctx::timed(int cls, double ops, double bytes, F&& launch, int op)
{
    if (!profiling) return launch();
    if (prof_used == prof.size()) {
        ee::ProfRec r{};
        if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) return hipErrorOutOfMemory;
        prof.push_back(r);
    }
    ee::ProfRec& r = prof[prof_used++];
    r.cls = cls; r.op = op; r.ops = ops; r.bytes = bytes;
    ee::g_launch_start = r.e0;                    // attached to the dispatch (of the last kernel, if `launch` issues several)
    ee::g_launch_stop = r.e1;
    hipError_t e = launch();
    ee::g_launch_start = ee::g_launch_stop = nullptr;
    return e;
}
