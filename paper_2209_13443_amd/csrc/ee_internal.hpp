// Internal declarations of the early-exit serving library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <cstring>
#include <hip/hip_ext.h>

#include <cstdint>
#include <string>
#include <vector>

#include "../../include/ee.h"

namespace ee {

// ---- network description parsed from the blob ------------------------------------------------
enum OpKind { OP_CONV = 0, OP_DWCONV = 1, OP_MAXPOOL = 2, OP_AVGPOOL = 3 };

struct OpDesc {
    int kind, src, dst, res;
    int h_in, w_in, c_in, h_out, w_out, c_out;
    int kh, kw, stride, pad;      // pad: rows of zero padding above and below
    int shift, res_shift, lo, hi;
    float f_lo, f_hi;
    int64_t w_off, b_off;
    int pad_w;                    // columns of zero padding left and right
    int c_off, c_tot;             // the op writes channels [c_off, c_off + c_out) of a tensor of c_tot channels (concatenation)
};

struct ExitDesc {
    int h, w, c, n_cls, gap_shift, frac_bits;
    float logit_scale, thr;
    int64_t w_off, b_off;
};

struct StageDesc {
    int first_op, n_ops, n_tensors, out_tensor;
    int in_h, in_w, in_c, out_h, out_w, out_c;
};

struct NetDesc {
    int dtype = 0, n_classes = 0, in_h = 0, in_w = 0, in_c = 0;
    std::vector<StageDesc> stages;
    std::vector<OpDesc> ops;
    std::vector<ExitDesc> exits;
    int elem_bytes() const { return dtype == EE_I8 ? 1 : 2; }
};

// Validates and decodes a blob.  Returns an ee_status.
int parse_blob(const void* blob, size_t bytes, NetDesc* out);

// ---- slot tables (zero-copy compaction) ----------------------------------------------------------
// Survivors of an exit are never moved: the samples of a batch live in arbitrary slots of the next segment's
// input memory and a table names the slot of every batch row (the GPU analogue of changing only the DMA
// addressing, Sec. III-A / III-B "Overhead").  The host hands a step's two tables (input rows, output rows) to one
// tiny kernel by value, which stores them in device memory; the convolution and pooling kernels read them there.
enum { EE_ZC_MAX_B = 256 };
struct SlotTab { uint16_t s[EE_ZC_MAX_B]; };
// dst[0..255] = in, dst[256..511] = out
hipError_t launch_upload_slots(const SlotTab& in, const SlotTab& out, uint16_t* dst, hipStream_t s);

// ---- kernel argument blocks --------------------------------------------------------------------
// Implicit-GEMM convolution: rows = output pixels m = (n, oy, ox), columns = output channels,
// reduction over (r, s, c).  Weights are pre-packed [Co_pad][Kp] with the reduction index the
// loader uses (see pack_weights in ee_api.cpp), zero padded.
struct ConvArgs {
    const void* x; const void* w; const void* bias; const void* res; void* y;
    const void* zeros;   // >= 16 readable zero bytes: what padding taps and rows past the batch read
    int M, H, W, Ci, Ho, Wo, Co;
    int kh, kw, stride, pad;   // pad: rows
    int pad_w;           // columns of padding
    int ldc, c_off;      // the output pixel has ldc channels, of which this layer writes [c_off, c_off + Co)
    int Kp;              // weight row pitch in elements (reduction length, zero padded)
    unsigned magic_howo, magic_wo;   // floor(2^32 / (Ho*Wo)), floor(2^32 / Wo): division by multiply-high
    unsigned tap_rows;   // bit r*kw set for every kernel row r (kh*kw <= 31)
    int plain_step;      // set by the launcher: bytes the source of a row advances per reduction step when no tap needs a check
    int mode;            // 0: Ci % 16 == 0 loader with bounds checks; 1: 4-channel zero-padded input
    int Hp, Wp, kwp;     // mode 1: padded input dims and padded kernel width
    int shift, res_shift, lo, hi;
    float f_lo, f_hi;
    int* gap_sums;       // not null (int8, conv_igemm_kernel, last layer of a segment): also add the per-sample channel sums of the output into gap_sums[n][Co]
    const uint16_t* xs;  // not null: sample n of the input is slot xs[n] of x (device memory; conv_igemm_kernel only)
    const uint16_t* ys;  // not null: sample n of the output is slot ys[n] of y (device memory; conv_igemm_kernel only)
};

// Two chained convolutions in one launch (kernels_pair.hip): c2 is the first layer (its y and res are unused, its
// output stays on chip), the rest describes the 1x1 layer that reads it.
struct PairArgs {
    ConvArgs c2;
    const void* w3; const void* bias3; const void* res; void* y;
    int Co3, Kp3;        // second layer: output channels, weight row pitch in elements
    int shift, res_shift, lo, hi;
    float f_lo, f_hi;
};

// An inverted-residual block in one launch (kernels_ir.hip): 1x1 expansion -> 3x3 depthwise -> 1x1 projection (+ residual).
// Weights and biases are packed for it when the context is created: expansion rows of Kx bytes (c_in padded with zeros
// to a multiple of 32) for Ce32 channels (the expanded channels padded to a multiple of 32, padding rows zero), the
// depthwise weights as ready matrix-instruction operands [Ce32 / 32][tap][lane][16] (diagonal matrices), projection rows
// of Ce32 bytes for NCO * 32 output channels; be and bd include the rounding constants of their shifts.
struct IrArgs {
    const void* x; const void* res; void* y;
    const void* we; const int* be;
    const void* wd; const int* bd;
    const void* wp; const int* bp;
    int B, H, W, Cin, Kx, Ce32, Cout, Ho, Wo, stride, pad;
    int sh_e, lo_e, hi_e, sh_d, lo_d, hi_d, sh_p, lo_p, hi_p, res_shift;
    const uint16_t* ys;  // bottleneck block only; not null: sample n of the output goes to slot ys[n] of y (device memory; B <= EE_ZC_MAX_B)
    int* gap_sums;       // bottleneck block only; not null: also add the per-sample channel sums of the output into gap_sums[n][Cout]
    const void* ws; const int* bs;   // bottleneck block only; not null: the residual is the 1x1 convolution of x with these operands and biases
    int sh_s, lo_s, hi_s;            // (res is null then), requantised with these
};

struct DirectConvArgs {   // one thread per output element; any shape (correctness fallback)
    const void* x; const void* w; const void* bias; const void* res; void* y;
    int M, H, W, Ci, Ho, Wo, Co, kh, kw, stride, pad, shift, res_shift, lo, hi;
    float f_lo, f_hi;
    int pad_w, ldc, c_off;
};

struct PoolArgs {         // depthwise 3x3 and max-pool share the shape block
    const void* x; const void* w; const void* bias; void* y;
    const void* w3;      // int8 3x3 depthwise: weights packed for the dot-product kernel, [C/16][column][4-channel group][channel] dwords (or null)
    int B, H, W, C, Ho, Wo, k, stride, pad, shift, lo, hi;
    float f_lo, f_hi;
    int ldc, c_off;      // pooling: the output pixel has ldc channels, of which this layer writes [c_off, c_off + C)
};

// ---- kernel launches ---------------------------------------------------------------------------------
// Every kernel goes out through EE_LAUNCH.  While a launch is being timed, the pair of events named here is attached
// to the dispatch itself (its own begin and end time stamps, what a kernel trace shows), instead of event records in
// front of and behind it, which would also count the dispatch latency of a stream whose back-to-back launches they break.
extern thread_local hipEvent_t g_launch_start, g_launch_stop;     // null: an ordinary launch
#define EE_LAUNCH(kernel, grid, block, lds_bytes, stream, ...) \
    hipExtLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, ee::g_launch_start, ee::g_launch_stop, 0, __VA_ARGS__)

// ---- launchers (defined in the .hip files) -------------------------------------------------------
hipError_t launch_conv_mfma_i8(const ConvArgs& a, hipStream_t s);
hipError_t launch_conv_mfma_bf16(const ConvArgs& a, hipStream_t s);
// asynchronous-copy implicit GEMM (ES = element bytes); tile 0 = chosen by shape, 1..4 forced
template <int ES> hipError_t launch_conv_igemm(const ConvArgs& a, int tile, hipStream_t s);
// the fused pair (ES = element bytes); cfg 0 = chosen by shape
template <int ES> hipError_t launch_conv_pair(const PairArgs& p, int cfg, hipStream_t s);
bool conv_pair_supported(int es, int co2, int kh, int kw, int ci, int co3);
// stride-1 "same" convolutions with the activation slab of a tile resident in LDS (kernels_slab.hip); cfg as documented there
bool conv_slab_supported(const ConvArgs& a, int es);
template <int ES> hipError_t launch_conv_slab(const ConvArgs& a, int cfg, hipStream_t s);
enum { EE_CFG_SLAB = 0x10000 };     // configuration words with this bit name the slab kernel
enum { EE_CFG_IR_BLOCK = 0x20000 }; // ee_time_layer: the fused inverted-residual block headed by the layer
// streaming kernel for large, thin int8 layers (es = element bytes); hipErrorInvalidValue for a layer it does not cover
bool conv_stream_supported(const ConvArgs& a, int es);
hipError_t launch_conv_stream(const ConvArgs& a, hipStream_t s);
// 1x1 int8 layers with at most 32 input channels: activations and weights straight from global memory into one
// matrix instruction per 32 x 32 outputs (w: packed rows of 32 bytes, zero padded; bias with the rounding constant)
struct ThinConvArgs {
    const void* x; const void* w; const void* bias; void* y;
    long long M;                 // output pixels of the batch
    int Ci, Co, ldc, c_off, shift, lo, hi;
};
hipError_t launch_conv_thin(const ThinConvArgs& a, hipStream_t s);
bool conv_thin_supported(int es, int kh, int kw, int stride, int pad, int pad_w, int ci, int co, int c_tot, int c_off, bool has_res);
int forced_conv_tile();
hipError_t launch_conv_direct(const DirectConvArgs& a, int dtype, hipStream_t s);
hipError_t launch_pad_input(const void* x, void* y, int B, int H, int W, int C, int Hp, int Wp, int pad, int dtype, hipStream_t s);
// [B][H][W][C<=4] -> [B][Hs][Ws][2][2][4]: zero padding `pad`, then 2 x 2 pixel blocks folded into channels;
// with gather (device-visible) sample n is read from row gather[n] of x
// gather_on_host: gather points to host memory the caller may read now (then up to 256 ids travel in the kernel arguments)
hipError_t launch_space_to_depth(const void* x, void* y, const int32_t* gather, int B, int H, int W, int C, int Hs, int Ws, int pad, int dtype, hipStream_t s,
                                 bool gather_on_host = false);
// [rows][c_bytes] -> [rows][cp_bytes] (both multiples of 4), the tail of every row zero
hipError_t launch_pad_channels(const void* x, void* y, long long rows, int c_bytes, int cp_bytes, hipStream_t s);
hipError_t launch_depthwise(const PoolArgs& a, int dtype, hipStream_t s);
// the fused inverted-residual block (int8); pointers may be null for ir_block_supported
bool ir_block_supported(const IrArgs& a);
int ir_block_out_blocks(int c_out);            // blocks of 32 output channels the kernel is instantiated with (weights are padded to it)
hipError_t launch_ir_block(const IrArgs& a, hipStream_t s);
// bottleneck block (1x1 -> 3x3 -> 1x1 + residual) in one launch; the same argument block: we / be, wd / bd, wp / bp are the three
// layers' operands and biases, Kx = Cin, Ce32 = the middle channels
// first convolution (folded stride-2 layer, 4 x 4 taps over 16-channel super-pixels, 64 output channels: a as for the streaming
// kernel, a.y unused) and the 3x3 / 2 max-pool with padding 1 behind it in one launch; yq: the pooled output [B][Hq][Wq][64]
bool stem_pool_supported(const ConvArgs& a, int Hq, int Wq);
hipError_t launch_stem_pool(const ConvArgs& a, void* yq, int Hq, int Wq, hipStream_t s);
bool bneck_block_supported(const IrArgs& a);
bool bneck_block_pools(const IrArgs& a);     // with a.gap_sums the launch also pools: only where its rows of sums fit into LDS
hipError_t launch_bneck_block(const IrArgs& a, hipStream_t s);
hipError_t launch_maxpool(const PoolArgs& a, int dtype, hipStream_t s);
hipError_t launch_avgpool(const PoolArgs& a, int dtype, hipStream_t s);

struct HeadArgs {
    const void* act; int B, HW, C, n_cls;
    int gap_shift, frac_bits; float logit_scale;
    const void* wfc; const void* bfc;
    int32_t* sums;       // [B][C] int32 sums (i8) or float means (bf16)
    int32_t* gap_partial;   // bf16: [(B + 1024)][C] partial rows of the pooling splits
    void* logits;        // [B][n_cls] int32 / float scratch
    int64_t s_thr; float thr; int last;
    int32_t* label; float* conf; int64_t* score; uint8_t* flag;
    // stream serving: per-slot outcomes written straight into pinned host memory, each with the launch's tag (null otherwise)
    struct HostOutcome* host_out; unsigned tag;
    const uint16_t* slots;   // pooling: not null: sample b of the batch is slot slots[b] of act (device memory)
};
// w0: bits 0-43 the score S (int8: S <= n_cls * 2^30 < 2^44; the host derives the confidence 2^30 / S) or the confidence's
// float bits (bf16); w1: bits 0-31 the label, bit 32 the exit flag; bits 44-63 of both: the launch's tag (never 0: a record the
// host has cleared matches no launch)
struct alignas(16) HostOutcome { uint64_t w0, w1; };
constexpr int EE_OUTCOME_TAG_SHIFT = 44;
inline unsigned outcome_tag(unsigned seq) { return seq % 0xFFFFFu + 1u; }
// host side: records [0, b) all carry the tag in both words
inline bool outcomes_ready(const HostOutcome* h, int b, unsigned tag)
{
    for (int k = b - 1; k >= 0; --k)
        if ((unsigned)(__atomic_load_n(&h[k].w0, __ATOMIC_ACQUIRE) >> EE_OUTCOME_TAG_SHIFT) != tag ||
            (unsigned)(__atomic_load_n(&h[k].w1, __ATOMIC_ACQUIRE) >> EE_OUTCOME_TAG_SHIFT) != tag) return false;
    return true;
}
struct Outcome { int64_t score; int32_t label; float conf; uint8_t flag; };
inline bool outcome_exits(const HostOutcome& h) { return (__atomic_load_n(&h.w1, __ATOMIC_RELAXED) >> 32) & 1u; }
inline Outcome decode_outcome(const HostOutcome& h, bool int8)
{
    const uint64_t w0 = __atomic_load_n(&h.w0, __ATOMIC_RELAXED), w1 = __atomic_load_n(&h.w1, __ATOMIC_RELAXED);
    const uint64_t payload = w0 & ((1ull << EE_OUTCOME_TAG_SHIFT) - 1);
    Outcome o;
    o.label = (int32_t)(uint32_t)w1;
    o.flag = (uint8_t)((w1 >> 32) & 1u);
    if (int8) {
        o.score = (int64_t)payload;
        o.conf = (float)(1073741824.0 / (double)o.score);       // as the kernel computes it for the device-side array
    } else {
        o.score = 0;
        const uint32_t bits = (uint32_t)payload;
        std::memcpy(&o.conf, &bits, 4);
    }
    return o;
}
// device address, on the current GPU, of the scratch array that is part of the library image (EE_STATIC_SCRATCH_BYTES bytes)
hipError_t static_scratch(void** out);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
// workgroups the pooling kernel splits a sample's pixels over (bf16 keeps one partial row per split)
int head_gap_splits(int B, int HW);
hipError_t launch_head_gap(const HeadArgs& a, int dtype, hipStream_t s);
hipError_t launch_head_fc(const HeadArgs& a, int dtype, hipStream_t s);
hipError_t launch_head_softmax(const HeadArgs& a, int dtype, hipStream_t s);

// Stable compaction + append.  dst_off: first destination slot of the survivors; ring_rows > 0: dst is a ring of that
// many slots and destination slots wrap around its end.
hipError_t launch_compact(const uint8_t* flag, const void* src, void* dst, const int32_t* ids_src, int32_t* ids_dst,
                          int b_act, int64_t sample_bytes, int dst_off, int ring_rows, int* b_rem_out, int* b_rem_out2, hipStream_t s);
hipError_t launch_append(const void* refill, void* dst, const int32_t* refill_ids, int32_t* ids_dst, const int* b_rem_dev,
                         int b_rem_host, int b_incr, int64_t sample_bytes, int* b_merged_out, hipStream_t s);
// Admission: pool rows ids[k] -> slots [0, b)
hipError_t launch_admit(const void* pool, void* dst, const int32_t* ids, int b, int64_t sample_bytes, hipStream_t s);

}  // namespace ee
