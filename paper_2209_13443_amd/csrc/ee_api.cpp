// C ABI entry points: context creation (weight packing, workspace planning), one backbone
// segment, one exit head, compaction / refill, latency-table measurement and kernel timing.
#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstring>

#include "ee_ctx.hpp"

namespace ee {
const uint32_t* exp2_table_host();
int set_conv_tile(int tile);
}

using namespace ee;

thread_local hipEvent_t ee::g_launch_start = nullptr, ee::g_launch_stop = nullptr;

namespace {

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <typename T>
int dev_alloc(ee_ctx* ctx, T** out, size_t bytes)
{
    void* p = nullptr;
    if (bytes == 0) bytes = 16;
    if (hipMalloc(&p, bytes) != hipSuccess) return EE_ERR_DEVICE;
    if (hipMemset(p, 0, bytes) != hipSuccess) { hipFree(p); return EE_ERR_DEVICE; }
    ctx->owned.push_back(p);
    *out = static_cast<T*>(p);
    return EE_OK;
}

int upload(ee_ctx* ctx, void** out, const std::vector<unsigned char>& host)
{
    unsigned char* p = nullptr;
    int rc = dev_alloc(ctx, &p, host.size());
    if (rc) return rc;
    if (!host.empty() && hipMemcpy(p, host.data(), host.size(), hipMemcpyHostToDevice) != hipSuccess) return EE_ERR_DEVICE;
    *out = p;
    return EE_OK;
}

// Packs one layer's weights for its kernel and uploads them with the (padded) bias.
int pack_op(ee_ctx* ctx, const unsigned char* blob, OpPlan& p)
{
    const OpDesc& d = p.d;
    const int es = ctx->net.elem_bytes();
    if (d.kind == OP_MAXPOOL || d.kind == OP_AVGPOOL) {
        // whole 16-byte chunks per pixel, also inside a concatenated output pixel
        if ((d.c_in * es) % 16 != 0 || (d.c_tot * es) % 16 != 0 || (d.c_off * es) % 16 != 0) return EE_ERR_UNSUPPORTED;
        p.impl = d.kind == OP_MAXPOOL ? IMPL_POOL : IMPL_AVGPOOL;
        return EE_OK;
    }
    const unsigned char* w = blob + d.w_off;
    const unsigned char* b = blob + d.b_off;
    if (d.kind == OP_DWCONV) {
        if ((d.c_in * es) % 16 != 0 || d.kh != d.kw || d.c_tot != d.c_out) return EE_ERR_UNSUPPORTED;
        p.impl = IMPL_DW;
        const int taps = d.kh * d.kw, C = d.c_in;
        std::vector<unsigned char> wp((size_t)taps * C * es);
        for (int c = 0; c < C; ++c)                       // [C][k][k] -> [k*k][C]
            for (int t = 0; t < taps; ++t) std::memcpy(&wp[((size_t)t * C + c) * es], w + ((size_t)c * taps + t) * es, es);
        std::vector<unsigned char> bp(b, b + 4 * (size_t)C);
        int rc = upload(ctx, &p.w_dev, wp);
        if (!rc) rc = upload(ctx, &p.b_dev, bp);
        if (!rc && es == 1 && d.kh == 3) {            // [C/16][column s][4-channel group][channel] dwords (w[0][s], w[1][s], w[2][s], 0)
            std::vector<unsigned char> w3((size_t)C * 12, 0);
            for (int ch = 0; ch < C; ++ch)
                for (int r = 0; r < 3; ++r)
                    for (int s2 = 0; s2 < 3; ++s2)
                        w3[((((size_t)(ch / 16) * 3 + s2) * 4 + (ch % 16) / 4) * 4 + ch % 4) * 4 + r] = w[(size_t)ch * 9 + r * 3 + s2];
            rc = upload(ctx, &p.w3_dev, w3);
        }
        p.weight_bytes = (double)wp.size() + bp.size();
        return rc;
    }
    const int Co = d.c_out, Ci = d.c_in, Co_pad = round_up(Co, 128);
    std::vector<unsigned char> bp(4 * (size_t)(Co_pad + 256), 0);     // the kernels copy 256 entries from the tile's first channel
    std::memcpy(bp.data(), b, 4 * (size_t)Co);
    std::vector<unsigned char> wp;
    if (conv_thin_supported(es, d.kh, d.kw, d.stride, d.pad, d.pad_w, Ci, Co, d.c_tot, d.c_off, d.res >= 0)) {
        p.impl = IMPL_THIN;                  // weight rows of 32 bytes, zero padded
        p.Kp = 32;
        wp.assign((size_t)Co_pad * p.Kp * es, 0);
        for (int o = 0; o < Co; ++o) std::memcpy(&wp[(size_t)o * p.Kp * es], w + (size_t)o * Ci * es, (size_t)Ci * es);
    } else if ((Ci * es) % 16 == 0 && Co % 4 == 0 && d.kh * d.kw <= 31) {
        p.impl = IMPL_MFMA;
        const int K = d.kh * d.kw * Ci;
        p.Kp = round_up(K * es, 256) / es;
        wp.assign((size_t)Co_pad * p.Kp * es, 0);
        for (int o = 0; o < Co; ++o) std::memcpy(&wp[(size_t)o * p.Kp * es], w + (size_t)o * K * es, (size_t)K * es);
    } else if (Ci > 4 && (Ci * es) % 4 == 0 && Co % 4 == 0 && d.kh * d.kw <= 31) {
        // pixels that are not 16-byte multiples: the layer reads a copy whose channels are zero padded to the
        // next multiple (made by a small kernel in front of it); the weights get the same per-tap padding
        p.impl = IMPL_MFMA_CPAD;
        const int cip = round_up(Ci * es, 16) / es, taps = d.kh * d.kw;
        p.ci_eff = cip;
        p.Kp = round_up(taps * cip * es, 256) / es;
        wp.assign((size_t)Co_pad * p.Kp * es, 0);
        for (int o = 0; o < Co; ++o)
            for (int t = 0; t < taps; ++t)
                std::memcpy(&wp[((size_t)o * p.Kp + (size_t)t * cip) * es], w + ((size_t)o * taps + t) * Ci * es, (size_t)Ci * es);
    } else if (Ci <= 4 && Co % 4 == 0 && d.stride == 2 && d.kh == d.kw && d.pad == d.pad_w && d.c_tot == Co && (d.kh + 1) / 2 * ((d.kh + 1) / 2) <= 31) {
        // stride-2 first layer: stride-1 convolution with a ceil(k/2)^2 kernel over the padded image folded into
        // super-pixels (dy, dx, c) of 2 x 2 pixels x 4 channels; weights W'[o][r'][s'][dy][dx][c] = W[o][2r'+dy][2s'+dx][c]
        p.impl = IMPL_MFMA_S2D;
        const int k2 = (d.kh + 1) / 2;
        p.kwp = k2;
        p.ci_eff = 16;
        p.Hp = std::max((d.h_in + 2 * d.pad + 1) / 2, d.h_out - 1 + k2);
        p.Wp = std::max((d.w_in + 2 * d.pad + 1) / 2, d.w_out - 1 + k2);
        p.Kp = round_up(k2 * k2 * 16 * es, 256) / es;
        wp.assign((size_t)Co_pad * p.Kp * es, 0);
        for (int o = 0; o < Co; ++o)
            for (int r = 0; r < d.kh; ++r)
                for (int s = 0; s < d.kw; ++s)
                    for (int ch = 0; ch < Ci; ++ch) {
                        const size_t kidx = ((size_t)((r >> 1) * k2 + (s >> 1)) * 4 + (r & 1) * 2 + (s & 1)) * 4 + ch;
                        std::memcpy(&wp[((size_t)o * p.Kp + kidx) * es], w + ((((size_t)o * d.kh + r) * d.kw + s) * Ci + ch) * es, es);
                    }
    } else if (Ci <= 4 && Co % 4 == 0 && d.pad == d.pad_w && d.c_tot == Co) {
        // first layer: the input is copied into a zero-padded 4-channel image, a kernel row of kwp taps is
        // then kwp*4 contiguous elements; k index = (r * kwp + s) * 4 + c
        p.impl = IMPL_MFMA_C4;
        p.kwp = round_up(d.kw, 16 / (4 * es));
        p.Kp = round_up(d.kh * p.kwp * 4 * es, 64) / es;
        p.Hp = d.h_in + 2 * d.pad;
        p.Wp = round_up(std::max(d.w_in + 2 * d.pad, (d.w_out - 1) * d.stride + p.kwp), 4);
        wp.assign((size_t)Co_pad * p.Kp * es, 0);
        for (int o = 0; o < Co; ++o)
            for (int r = 0; r < d.kh; ++r)
                for (int s = 0; s < d.kw; ++s)
                    for (int c = 0; c < Ci; ++c)
                        std::memcpy(&wp[((size_t)o * p.Kp + (size_t)(r * p.kwp + s) * 4 + c) * es],
                                    w + ((((size_t)o * d.kh + r) * d.kw + s) * Ci + c) * es, es);
    } else {
        p.impl = IMPL_DIRECT;
        wp.assign(w, w + (size_t)Co * d.kh * d.kw * Ci * es);
    }
    if ((p.impl == IMPL_MFMA || p.impl == IMPL_MFMA_CPAD || p.impl == IMPL_MFMA_S2D || p.impl == IMPL_THIN) && es == 1 && d.shift > 0) {
        // that kernel requantises with a bare arithmetic shift: the rounding constant 2^(shift-1) goes
        // into the bias (the sum fits int32: the network's calibration guarantees t + 2^(shift-1) does)
        for (int o = 0; o < Co; ++o) {
            int32_t v;
            std::memcpy(&v, &bp[4 * (size_t)o], 4);
            v += 1 << (d.shift - 1);
            std::memcpy(&bp[4 * (size_t)o], &v, 4);
        }
    }
    int rc = upload(ctx, &p.w_dev, wp);
    if (!rc) rc = upload(ctx, &p.b_dev, bp);
    p.weight_bytes = (double)Co * d.kh * d.kw * Ci * es + 4.0 * Co;
    return rc;
}

std::vector<unsigned char> ir_rounded_bias(const unsigned char* blob, const OpDesc& d, int n, int n_pad)
{
    std::vector<unsigned char> out(4 * (size_t)n_pad, 0);
    for (int o = 0; o < n; ++o) {
        int32_t v;
        std::memcpy(&v, blob + d.b_off + 4 * (size_t)o, 4);
        if (d.shift > 0) v += 1 << (d.shift - 1);
        std::memcpy(&out[4 * (size_t)o], &v, 4);
    }
    return out;
}

// depthwise weights [C][3][3] as ready matrix-instruction operands [group][tap][lane][16]: row m = lane % 32 of diag(w) lies
// in the lane whose 16 reduction bytes hold byte m
std::vector<unsigned char> ir_diag_operands(const unsigned char* w, int C, int C32)
{
    std::vector<unsigned char> wd((size_t)(C32 / 32) * 9 * 64 * 16, 0);
    for (int c = 0; c < C; ++c)
        for (int t = 0; t < 9; ++t) {
            const int g = c / 32, m = c % 32, lane = m + 32 * (m / 16);
            wd[(((size_t)g * 9 + t) * 64 + lane) * 16 + m % 16] = w[(size_t)c * 9 + t];
        }
    return wd;
}

// A depthwise 3x3 layer that no fused block in front of it covers, followed by the 1x1 convolution that alone reads it:
// the fused kernel without its expansion (two layers in one launch).
int pack_ir_noexp(ee_ctx* ctx, const unsigned char* blob, const StageDesc& st, int k)
{
    OpPlan& p = ctx->plans[st.first_op + k];
    if (k + 1 >= st.n_ops || (k >= 1 && ctx->plans[st.first_op + k - 1].ir && !ctx->plans[st.first_op + k - 1].ir_noexp)) return EE_OK;
    const OpDesc& dw = p.d;
    const OpDesc& pr = ctx->plans[st.first_op + k + 1].d;
    if (pr.kind != OP_CONV || dw.kh != 3 || dw.kw != 3 || dw.pad != 1 || dw.pad_w != 1 || dw.c_tot != dw.c_out) return EE_OK;
    if (pr.kh != 1 || pr.kw != 1 || pr.stride != 1 || pr.pad != 0 || pr.pad_w != 0 || pr.src != dw.dst || pr.c_tot != pr.c_out) return EE_OK;
    if (dw.dst == st.out_tensor || pr.res == dw.dst) return EE_OK;
    int readers = 0;
    for (int j = 0; j < st.n_ops; ++j) {
        const OpDesc& o = ctx->plans[st.first_op + j].d;
        readers += (o.src == dw.dst) + (o.res == dw.dst);
    }
    if (readers != 1) return EE_OK;
    const int C = dw.c_in, C32 = round_up(C, 32), Co = pr.c_out, Co32 = 32 * ir_block_out_blocks(Co);
    IrArgs probe{};
    probe.B = ctx->b_max; probe.H = dw.h_in; probe.W = dw.w_in; probe.Cin = C; probe.Kx = 0; probe.Ce32 = C32; probe.Cout = Co;
    probe.Ho = dw.h_out; probe.Wo = dw.w_out; probe.stride = dw.stride; probe.pad = dw.pad;
    if (!ir_block_supported(probe)) return EE_OK;
    std::vector<unsigned char> wp((size_t)Co32 * C32, 0);
    for (int o = 0; o < Co; ++o) std::memcpy(&wp[(size_t)o * C32], blob + pr.w_off + (size_t)o * C, (size_t)C);
    int rc = upload(ctx, &p.ir_wd, ir_diag_operands(blob + dw.w_off, C, C32));
    if (!rc) rc = upload(ctx, &p.ir_bd, ir_rounded_bias(blob, dw, C, C32));
    if (!rc) rc = upload(ctx, &p.ir_wp, wp);
    if (!rc) rc = upload(ctx, &p.ir_bp, ir_rounded_bias(blob, pr, Co, Co32));
    if (rc) return rc;
    p.ir_kx = 0; p.ir_ce32 = C32;
    p.ir = true;
    p.ir_noexp = true;
    return EE_OK;
}

// Marks layer k of the segment as the head of an inverted-residual block when the fused kernel covers it and packs the
// block's weights for that kernel (see IrArgs).
int pack_ir(ee_ctx* ctx, const unsigned char* blob, const StageDesc& st, int k)
{
    OpPlan& p = ctx->plans[st.first_op + k];
    if (p.d.kind == OP_DWCONV) return pack_ir_noexp(ctx, blob, st, k);
    if (k + 2 >= st.n_ops) return EE_OK;
    const OpDesc& e = p.d;
    const OpDesc& dw = ctx->plans[st.first_op + k + 1].d;
    const OpDesc& pr = ctx->plans[st.first_op + k + 2].d;
    if (e.kind != OP_CONV || dw.kind != OP_DWCONV || pr.kind != OP_CONV) return EE_OK;
    if (e.kh != 1 || e.kw != 1 || e.stride != 1 || e.pad != 0 || e.pad_w != 0 || e.res >= 0 || e.c_tot != e.c_out) return EE_OK;
    if (dw.kh != 3 || dw.kw != 3 || dw.pad != 1 || dw.pad_w != 1 || dw.src != e.dst || dw.c_tot != dw.c_out || dw.c_in != e.c_out) return EE_OK;
    if (pr.kh != 1 || pr.kw != 1 || pr.stride != 1 || pr.pad != 0 || pr.pad_w != 0 || pr.src != dw.dst || pr.c_tot != pr.c_out) return EE_OK;
    if (e.dst == st.out_tensor || dw.dst == st.out_tensor || pr.res == e.dst || pr.res == dw.dst) return EE_OK;
    int readers_e = 0, readers_d = 0;
    for (int j = 0; j < st.n_ops; ++j) {
        const OpDesc& o = ctx->plans[st.first_op + j].d;
        readers_e += (o.src == e.dst) + (o.res == e.dst);
        readers_d += (o.src == dw.dst) + (o.res == dw.dst);
    }
    if (readers_e != 1 || readers_d != 1) return EE_OK;
    const int Ci = e.c_in, Ce = e.c_out, Co = pr.c_out, Kx = round_up(Ci, 32), Ce32 = round_up(Ce, 32), Co32 = 32 * ir_block_out_blocks(Co);
    IrArgs probe{};
    probe.B = 1; probe.H = e.h_in; probe.W = e.w_in; probe.Cin = Ci; probe.Kx = Kx; probe.Ce32 = Ce32; probe.Cout = Co;
    probe.Ho = dw.h_out; probe.Wo = dw.w_out; probe.stride = dw.stride; probe.pad = dw.pad;
    probe.B = ctx->b_max;
    if (!ir_block_supported(probe)) return EE_OK;
    std::vector<unsigned char> we((size_t)Ce32 * Kx, 0), wp((size_t)Co32 * Ce32, 0);
    for (int c = 0; c < Ce; ++c) std::memcpy(&we[(size_t)c * Kx], blob + e.w_off + (size_t)c * Ci, (size_t)Ci);
    for (int o = 0; o < Co; ++o) std::memcpy(&wp[(size_t)o * Ce32], blob + pr.w_off + (size_t)o * Ce, (size_t)Ce);
    int rc = upload(ctx, &p.ir_we, we);
    if (!rc) rc = upload(ctx, &p.ir_be, ir_rounded_bias(blob, e, Ce, Ce32));
    if (!rc) rc = upload(ctx, &p.ir_wd, ir_diag_operands(blob + dw.w_off, Ce, Ce32));
    if (!rc) rc = upload(ctx, &p.ir_bd, ir_rounded_bias(blob, dw, Ce, Ce32));
    if (!rc) rc = upload(ctx, &p.ir_wp, wp);
    if (!rc) rc = upload(ctx, &p.ir_bp, ir_rounded_bias(blob, pr, Co, Co32));
    if (rc) return rc;
    p.ir_kx = Kx; p.ir_ce32 = Ce32;
    p.ir = true;
    return EE_OK;
}

// rows [rows][row_bytes] of a weight matrix as ready matrix-instruction operands [row block of 32][step of 32 bytes][lane][16]:
// lane m + 32 hi holds bytes 16 hi .. 16 hi + 15 of the step of row m
std::vector<unsigned char> bn_operands(const unsigned char* w, int rows, int row_bytes)
{
    std::vector<unsigned char> out((size_t)rows * row_bytes);
    const int steps = row_bytes / 32;
    for (int r = 0; r < rows; ++r)
        for (int k = 0; k < steps; ++k)
            for (int hi = 0; hi < 2; ++hi)
                std::memcpy(&out[((((size_t)(r / 32) * steps + k) * 64) + (r % 32) + 32 * hi) * 16], w + (size_t)r * row_bytes + 32 * k + 16 * hi, 16);
    return out;
}

// Marks layer k of the segment as the head of a bottleneck block (1x1 -> 3x3 -> 1x1 + residual) when the fused kernel covers
// it and packs the block's weights for that kernel.
int pack_bneck(ee_ctx* ctx, const unsigned char* blob, const StageDesc& st, int k)
{
    OpPlan& p = ctx->plans[st.first_op + k];
    if (k + 2 >= st.n_ops) return EE_OK;
    const OpDesc& c1 = p.d;
    const OpDesc& c2 = ctx->plans[st.first_op + k + 1].d;
    const OpDesc& c3 = ctx->plans[st.first_op + k + 2].d;
    if (c1.kind != OP_CONV || c2.kind != OP_CONV || c3.kind != OP_CONV) return EE_OK;
    if (c1.kh != 1 || c1.kw != 1 || c1.stride != 1 || c1.pad != 0 || c1.pad_w != 0 || c1.res >= 0 || c1.c_tot != c1.c_out) return EE_OK;
    if (c2.kh != 3 || c2.kw != 3 || c2.stride != 1 || c2.pad != 1 || c2.pad_w != 1 || c2.res >= 0 || c2.src != c1.dst || c2.c_tot != c2.c_out) return EE_OK;
    if (c3.kh != 1 || c3.kw != 1 || c3.stride != 1 || c3.pad != 0 || c3.pad_w != 0 || c3.src != c2.dst || c3.c_tot != c3.c_out) return EE_OK;
    if (c1.dst == st.out_tensor || c2.dst == st.out_tensor || c3.res == c1.dst || c3.res == c2.dst) return EE_OK;
    int readers_1 = 0, readers_2 = 0;
    for (int j = 0; j < st.n_ops; ++j) {
        const OpDesc& o = ctx->plans[st.first_op + j].d;
        readers_1 += (o.src == c1.dst) + (o.res == c1.dst);
        readers_2 += (o.src == c2.dst) + (o.res == c2.dst);
    }
    if (readers_1 != 1 || readers_2 != 1) return EE_OK;
    IrArgs probe{};
    probe.B = ctx->b_max; probe.H = c1.h_in; probe.W = c1.w_in; probe.Cin = c1.c_in; probe.Kx = c1.c_in; probe.Ce32 = c1.c_out; probe.Cout = c3.c_out;
    probe.Ho = c2.h_out; probe.Wo = c2.w_out; probe.stride = 1; probe.pad = 1;
    if (c2.c_in != c1.c_out || c2.c_out != c1.c_out || !bneck_block_supported(probe)) return EE_OK;
    int rc = upload(ctx, &p.ir_we, bn_operands(blob + c1.w_off, c1.c_out, c1.c_in));
    if (!rc) rc = upload(ctx, &p.ir_be, ir_rounded_bias(blob, c1, c1.c_out, c1.c_out));
    if (!rc) rc = upload(ctx, &p.ir_wd, bn_operands(blob + c2.w_off, c2.c_out, 9 * c2.c_in));
    if (!rc) rc = upload(ctx, &p.ir_bd, ir_rounded_bias(blob, c2, c2.c_out, c2.c_out));
    if (!rc) rc = upload(ctx, &p.ir_wp, bn_operands(blob + c3.w_off, c3.c_out, c3.c_in));
    if (!rc) rc = upload(ctx, &p.ir_bp, ir_rounded_bias(blob, c3, c3.c_out, c3.c_out));
    if (rc) return rc;
    p.ir_kx = c1.c_in; p.ir_ce32 = c1.c_out;
    p.ir = true;
    p.ir_bneck = true;
    return EE_OK;
}

// A bottleneck block whose residual is a 1x1 convolution of the block's own input, that convolution being the layer right in front
// of the block (the first block of a group): the convolution becomes the head of a block of four layers, run by the same kernel.
int pack_bneck_shortcut(ee_ctx* ctx, const unsigned char* blob, const StageDesc& st, int k)
{
    if (k + 3 >= st.n_ops) return EE_OK;
    OpPlan& p = ctx->plans[st.first_op + k];
    const OpPlan& h = ctx->plans[st.first_op + k + 1];
    const OpDesc& sc = p.d;
    const OpDesc& c1 = h.d;
    const OpDesc& c3 = ctx->plans[st.first_op + k + 3].d;
    if (p.ir || !h.ir_bneck || h.ir_sc || sc.kind != OP_CONV) return EE_OK;
    if (sc.kh != 1 || sc.kw != 1 || sc.stride != 1 || sc.pad != 0 || sc.pad_w != 0 || sc.res >= 0 || sc.c_tot != sc.c_out) return EE_OK;
    if (sc.src != c1.src || sc.c_in != 64 || sc.c_out != c3.c_out || c3.res != sc.dst || sc.dst == st.out_tensor) return EE_OK;
    int readers = 0;
    for (int j = 0; j < st.n_ops; ++j) {
        const OpDesc& o = ctx->plans[st.first_op + j].d;
        readers += (o.src == sc.dst) + (o.res == sc.dst);
    }
    if (readers != 1) return EE_OK;
    int rc = upload(ctx, &p.ir_ws, bn_operands(blob + sc.w_off, sc.c_out, sc.c_in));
    if (!rc) rc = upload(ctx, &p.ir_bs, ir_rounded_bias(blob, sc, sc.c_out, sc.c_out));
    if (rc) return rc;
    p.ir_we = h.ir_we; p.ir_be = h.ir_be; p.ir_wd = h.ir_wd; p.ir_bd = h.ir_bd; p.ir_wp = h.ir_wp; p.ir_bp = h.ir_bp;
    p.ir_kx = h.ir_kx; p.ir_ce32 = h.ir_ce32;
    p.ir = true;
    p.ir_bneck = true;
    p.ir_sc = true;
    return EE_OK;
}

// Assigns the intermediate tensors of every segment to a small pool of reusable buffers
// (greedy by liveness); the segment input and output stay with the caller.
void plan_buffers(ee_ctx* ctx)
{
    const int es = ctx->net.elem_bytes();
    for (const StageDesc& st : ctx->net.stages) {
        std::vector<int> last_use(st.n_tensors, -1), buf(st.n_tensors, -3);
        for (int k = 0; k < st.n_ops; ++k) {
            const OpDesc& d = ctx->plans[st.first_op + k].d;
            last_use[d.src] = k;
            if (d.res >= 0) last_use[d.res] = k;
            // the head of a fused pair: the one launch reads this layer's input while it writes the next layer's
            // output, so the input's buffer must stay reserved over both
            if (k > 0 && ctx->plans[st.first_op + k - 1].pair) last_use[ctx->plans[st.first_op + k - 1].d.src] = k;
            // likewise the head of a fused inverted-residual block, over its three layers
            if (k > 1 && ctx->plans[st.first_op + k - 2].ir && ctx->plans[st.first_op + k - 2].ir_last() == 2) last_use[ctx->plans[st.first_op + k - 2].d.src] = k;
            if (k > 2 && ctx->plans[st.first_op + k - 3].ir_sc) last_use[ctx->plans[st.first_op + k - 3].d.src] = k;
            if (k > 0 && (ctx->plans[st.first_op + k - 1].ir_noexp || ctx->plans[st.first_op + k - 1].ir_stem)) last_use[ctx->plans[st.first_op + k - 1].d.src] = k;
        }
        buf[0] = BUF_EXT_IN;
        buf[st.out_tensor] = BUF_EXT_OUT;
        std::vector<int> free_list;
        std::vector<char> in_use(ctx->pool_sample_bytes.size(), 0);
        for (int k = 0; k < st.n_ops; ++k) {
            OpPlan& p = ctx->plans[st.first_op + k];
            const OpDesc& d = p.d;
            if (buf[d.dst] == -3) {
                const size_t need = (size_t)d.h_out * d.w_out * d.c_tot * es;      // the whole tensor, also when this op writes a slice of it
                int pick = -1;
                for (size_t i = 0; i < in_use.size(); ++i)
                    if (!in_use[i]) { pick = (int)i; break; }
                if (pick < 0) {
                    pick = (int)ctx->pool_sample_bytes.size();
                    ctx->pool_sample_bytes.push_back(0);
                    in_use.push_back(0);
                }
                in_use[pick] = 1;
                ctx->pool_sample_bytes[pick] = std::max(ctx->pool_sample_bytes[pick], need);
                buf[d.dst] = pick;
            }
            p.src_buf = buf[d.src];
            p.dst_buf = buf[d.dst];
            p.res_buf = d.res >= 0 ? buf[d.res] : -3;
            // release tensors whose last reader was this op (the destination is never released here)
            for (int t = 1; t < st.n_tensors; ++t)
                if (t != d.dst && buf[t] >= 0 && last_use[t] == k) in_use[buf[t]] = 0;
        }
    }
}

// The per-lane part of the workspace (the lane's stream, intermediate tensors and padded input copies are set by the
// caller when they exist already).
int alloc_lane(ee_ctx* ctx, LaneState& L)
{
    int rc = EE_OK;
    const int n_st = (int)ctx->net.stages.size(), b_max = ctx->b_max;
    if (L.pool.empty()) {
        L.pool.resize(ctx->pool_sample_bytes.size(), nullptr);
        for (size_t i = 0; i < L.pool.size(); ++i)
            if ((rc = dev_alloc(ctx, &L.pool[i], ctx->pool_sample_bytes[i] * (size_t)b_max))) return rc;
    }
    if (L.pad_bufs.empty()) {
        L.pad_bufs.resize(ctx->pad_buf_bytes.size(), nullptr);
        for (size_t i = 0; i < L.pad_bufs.size(); ++i)
            if ((rc = dev_alloc(ctx, &L.pad_bufs[i], ctx->pad_buf_bytes[i]))) return rc;
    }
    L.out_buf.assign(n_st, nullptr);
    for (int s = 0; s < n_st; ++s)
        if ((rc = dev_alloc(ctx, &L.out_buf[s], (size_t)ctx->stage_out_bytes(s) * b_max))) return rc;
    if ((rc = dev_alloc(ctx, &L.in0, (size_t)ctx->stage_in_bytes(0) * b_max))) return rc;
    if ((rc = dev_alloc(ctx, &L.sums, sizeof(int32_t) * (size_t)b_max * ctx->c_max))) return rc;
    if ((rc = dev_alloc(ctx, &L.gap_partial, sizeof(int32_t) * ((size_t)b_max + 1024) * ctx->c_max))) return rc;
    if ((rc = dev_alloc(ctx, &L.logits, 4 * (size_t)b_max * ctx->net.n_classes))) return rc;
    if ((rc = dev_alloc(ctx, &L.d_label, sizeof(int32_t) * (size_t)b_max))) return rc;
    if ((rc = dev_alloc(ctx, &L.d_conf, sizeof(float) * (size_t)b_max))) return rc;
    if ((rc = dev_alloc(ctx, &L.d_score, sizeof(int64_t) * (size_t)b_max))) return rc;
    if ((rc = dev_alloc(ctx, &L.d_flag, (size_t)b_max + 16))) return rc;
    if ((rc = dev_alloc(ctx, &L.d_slots, 2 * sizeof(uint16_t) * EE_ZC_MAX_B))) return rc;
    const size_t out_bytes = round_up((int)(sizeof(HostOutcome) * (size_t)b_max), 256), ids_bytes = round_up(4 * b_max, 256);
    if (hipHostMalloc(&L.h_pinned, out_bytes + 2 * ids_bytes, hipHostMallocCoherent) != hipSuccess) return EE_ERR_DEVICE;
    std::memset(L.h_pinned, 0, out_bytes + 2 * ids_bytes);
    unsigned char* hp = static_cast<unsigned char*>(L.h_pinned);
    L.h_out = reinterpret_cast<HostOutcome*>(hp);
    L.h_ids[0] = reinterpret_cast<int32_t*>(hp + out_bytes);
    L.h_ids[1] = reinterpret_cast<int32_t*>(hp + out_bytes + ids_bytes);
    for (int s = 0; s < 8; ++s)
        if (hipEventCreateWithFlags(&L.packed[s], hipEventDisableTiming) != hipSuccess) return EE_ERR_DEVICE;
    return EE_OK;
}

void* resolve(ee_ctx* ctx, int buf, const void* ext_in, void* ext_out)
{
    if (buf == BUF_EXT_IN) return const_cast<void*>(ext_in);
    if (buf == BUF_EXT_OUT) return ext_out;
    return buf >= 0 ? ctx->pool[buf] : nullptr;
}

}  // namespace

// ---------------------------------------------------------------------------------------------
extern "C" const char* ee_strerror(int status)
{
    switch (status) {
        case EE_OK: return "ok";
        case EE_ERR_ARG: return "invalid argument";
        case EE_ERR_SHAPE: return "tensor shapes of the network do not chain";
        case EE_ERR_UNSUPPORTED: return "unsupported dtype or layer";
        case EE_ERR_DEVICE: return "HIP device error";
        case EE_ERR_OVERFLOW: return "size exceeds the library's limits";
        default: return "unknown status";
    }
}

extern "C" const char* ee_kernel_name(int k)
{
    static const char* names[EE_K_COUNT] = {"conv_mfma", "conv_first", "conv_direct", "depthwise", "maxpool", "pad_input",
                                            "gap", "fc", "softmax", "compact", "admit", "conv_stream"};
    return k >= 0 && k < EE_K_COUNT ? names[k] : "?";
}

extern "C" const uint32_t* ee_exp2_table(void) { return exp2_table_host(); }

extern "C" int ee_tune_conv_tile(int cfg)
{
    const int tile = cfg & 15, ksel = (cfg >> 4) & 15, ns = (cfg >> 8) & 15, kspl = (cfg >> 12) & 15;
    if (cfg < 0 || (cfg >> 17) || ksel > 3 || (ns != 0 && (ns < 2 || ns > 4)) || (kspl != 0 && kspl != 2 && kspl != 4)) return EE_ERR_ARG;
    if (cfg & EE_CFG_SLAB) {
        if (tile < 1 || tile > 4 || ksel == 1 || kspl != 0) return EE_ERR_ARG;
    } else if (tile > 4 && cfg != 7) return EE_ERR_ARG;
    return set_conv_tile(cfg);
}

extern "C" int ee_blob_check(const void* blob, size_t bytes) { return parse_blob(blob, bytes, nullptr); }

extern "C" int ee_create(const void* blob, size_t bytes, int b_max, int dtype, void* hip_stream, ee_ctx** out)
{
    if (!out) return EE_ERR_ARG;
    *out = nullptr;
    if (b_max < 1 || b_max > 1024) return EE_ERR_ARG;
    NetDesc net;
    int rc = parse_blob(blob, bytes, &net);
    if (rc) return rc;
    if (dtype != net.dtype) return EE_ERR_UNSUPPORTED;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return EE_ERR_DEVICE;
    ee_ctx* ctx = new (std::nothrow) ee_ctx();
    if (!ctx) return EE_ERR_DEVICE;
    ctx->net = std::move(net);
    ctx->b_max = b_max;
    ctx->stream = static_cast<hipStream_t>(hip_stream);
    const int es = ctx->net.elem_bytes();
    const unsigned char* base = static_cast<const unsigned char*>(blob);
    auto fail = [&](int code) { ee_destroy(ctx); return code; };

    ctx->plans.resize(ctx->net.ops.size());
    for (size_t i = 0; i < ctx->plans.size(); ++i) {
        OpPlan& p = ctx->plans[i];
        p.d = ctx->net.ops[i];
        if ((rc = pack_op(ctx, base, p))) return fail(rc);
        const OpDesc& d = p.d;
        // the kernels address a batch tensor with 32-bit byte offsets
        const double in_rows = (double)d.h_in * d.w_in * std::max(d.c_in, 16), out_rows = (double)d.h_out * d.w_out * d.c_tot;
        if (std::max(in_rows, out_rows) * es * b_max >= 2147483648.0) return fail(EE_ERR_OVERFLOW);
        const double out_e = (double)d.h_out * d.w_out * d.c_out, in_e = (double)d.h_in * d.w_in * d.c_in;
        const double kred = d.kind == OP_CONV ? (double)d.kh * d.kw * d.c_in : (double)d.kh * d.kw;
        p.ops_per_sample = d.kind == OP_MAXPOOL || d.kind == OP_AVGPOOL ? 0.0 : 2.0 * out_e * kred;
        p.bytes_per_sample = (in_e + out_e + (d.res >= 0 ? out_e : 0.0)) * es;
        if (p.impl == IMPL_MFMA_C4 || p.impl == IMPL_MFMA_CPAD || p.impl == IMPL_MFMA_S2D) {
            void* pb = nullptr;
            const size_t bytes = p.impl == IMPL_MFMA_C4    ? (size_t)b_max * p.Hp * p.Wp * 4 * es
                                 : p.impl == IMPL_MFMA_S2D ? (size_t)b_max * p.Hp * p.Wp * 16 * es
                                                           : (size_t)b_max * d.h_in * d.w_in * p.ci_eff * es;
            if ((rc = dev_alloc(ctx, &pb, bytes + 256))) return fail(rc);
            p.pad_buf = (int)ctx->pad_bufs.size();
            ctx->pad_bufs.push_back(pb);
            ctx->pad_buf_bytes.push_back(bytes + 256);
        }
        if (p.ci_eff == 0) p.ci_eff = d.c_in;
    }
    // layer pairs one fused launch can take: a matrix-core convolution without residual whose output is read by
    // exactly one layer, the next one, and that one is a 1x1 stride-1 matrix-core convolution
    for (const StageDesc& st : ctx->net.stages)
        for (int k = 0; k + 1 < st.n_ops; ++k) {
            OpPlan& p = ctx->plans[st.first_op + k];
            const OpPlan& q = ctx->plans[st.first_op + k + 1];
            if (p.impl != IMPL_MFMA || q.impl != IMPL_MFMA || p.d.res >= 0 || p.d.dst == st.out_tensor) continue;
            if (p.d.c_tot != p.d.c_out || q.d.c_tot != q.d.c_out) continue;           // no channel slices
            if (q.d.src != p.d.dst || q.d.res == p.d.dst || q.d.kh != 1 || q.d.kw != 1 || q.d.stride != 1 || q.d.pad != 0) continue;
            int readers = 0;
            for (int j = 0; j < st.n_ops; ++j) {
                const OpDesc& o = ctx->plans[st.first_op + j].d;
                readers += (o.src == p.d.dst) + (o.res == p.d.dst);
            }
            p.pair = readers == 1 && conv_pair_supported(es, p.d.c_out, p.d.kh, p.d.kw, p.ci_eff, q.d.c_out);
        }
    // inverted-residual blocks one fused launch can take (int8): a 1x1 stride-1 convolution without residual whose output
    // is read only by the next layer, a 3x3 depthwise layer with padding 1, whose output is read only by the layer after
    // it, a 1x1 stride-1 convolution (with or without residual); none of the three writes a channel slice
    if (es == 1)
        for (const StageDesc& st : ctx->net.stages)
            for (int k = 0; k + 1 < st.n_ops; ++k) {
                if ((rc = pack_ir(ctx, (const unsigned char*)blob, st, k))) return fail(rc);
                // likewise bottleneck blocks: 1x1 -> 3x3 (stride 1, padding 1) -> 1x1 (+ residual), each read only by the next
                if (!ctx->plans[st.first_op + k].ir && (rc = pack_bneck(ctx, (const unsigned char*)blob, st, k))) return fail(rc);
            }
    if (es == 1)
        for (const StageDesc& st : ctx->net.stages)
            for (int k = 0; k + 3 < st.n_ops; ++k)
                if ((rc = pack_bneck_shortcut(ctx, (const unsigned char*)blob, st, k))) return fail(rc);
    // the folded first convolution with the max-pool that alone reads it (nothing to pack: the kernel takes the layer's own weights)
    if (es == 1)
        for (const StageDesc& st : ctx->net.stages)
            for (int k = 0; k + 1 < st.n_ops; ++k) {
                OpPlan& p = ctx->plans[st.first_op + k];
                const OpDesc& c = p.d;
                const OpDesc& q = ctx->plans[st.first_op + k + 1].d;
                if (p.ir || p.impl != IMPL_MFMA_S2D || c.res >= 0 || c.dst == st.out_tensor || q.kind != OP_MAXPOOL || q.src != c.dst) continue;
                if (q.kh != 3 || q.kw != 3 || q.stride != 2 || q.pad != 1 || q.pad_w != 1 || q.c_tot != q.c_out || q.c_off != 0 || q.dst == st.out_tensor) continue;
                int readers = 0;
                for (int j = 0; j < st.n_ops; ++j) {
                    const OpDesc& o = ctx->plans[st.first_op + j].d;
                    readers += (o.src == c.dst) + (o.res == c.dst);
                }
                ConvArgs probe{};
                ctx->fill_conv_args(st.first_op + k, b_max, probe);
                if (readers != 1 || !stem_pool_supported(probe, q.h_out, q.w_out)) continue;
                p.ir = true;
                p.ir_stem = true;
            }
    plan_buffers(ctx);
    ctx->pool.resize(ctx->pool_sample_bytes.size(), nullptr);
    for (size_t i = 0; i < ctx->pool.size(); ++i)
        if ((rc = dev_alloc(ctx, &ctx->pool[i], ctx->pool_sample_bytes[i] * (size_t)b_max))) return fail(rc);

    // exit heads
    int c_max = 0;
    const int n_st = (int)ctx->net.stages.size();
    ctx->wfc_dev.resize(n_st);
    ctx->bfc_dev.resize(n_st);
    for (int s = 0; s < n_st; ++s) {
        const ExitDesc& e = ctx->net.exits[s];
        if ((e.c * es) % 16 != 0 || e.c * es / 16 > 256 || e.n_cls > 2048) return fail(EE_ERR_UNSUPPORTED);
        c_max = std::max(c_max, e.c);
        std::vector<unsigned char> w(base + e.w_off, base + e.w_off + (size_t)e.n_cls * e.c * es);
        std::vector<unsigned char> b(base + e.b_off, base + e.b_off + 4 * (size_t)e.n_cls);
        if ((rc = upload(ctx, &ctx->wfc_dev[s], w)) || (rc = upload(ctx, &ctx->bfc_dev[s], b))) return fail(rc);
        if (ctx->stage_out_bytes(s) % 16 != 0 || ctx->stage_in_bytes(s) % 16 != 0) return fail(EE_ERR_UNSUPPORTED);
    }
    ctx->c_max = (size_t)c_max;
    if ((rc = dev_alloc(ctx, &ctx->d_count, 64))) return fail(rc);
    if ((rc = dev_alloc(ctx, &ctx->zero_page, 256))) return fail(rc);
    if ((rc = dev_alloc(ctx, &ctx->d_ids, sizeof(int32_t) * (size_t)b_max))) return fail(rc);

    // stream-serving workspace.  Shared by all lanes: the packed input slots of every segment behind the first, a ring of
    // 3 b_max samples (the stage-pool policy keeps up to 2 b_max - 1 waiting samples there while a batch of up to b_max
    // is being read).  Per lane: everything alloc_lane makes; lane 0 is made here on the caller's stream.
    // the layer of each segment that can carry the exit head's pooling in its epilogue: int8, the only writer of the segment's
    // output, a whole (not sliced) tensor of 16-byte pixels, a general matrix-core layer with a residual (its tile is staged
    // behind the ring, which the sums then use), and at most 8 samples per 128-row tile
    ctx->gap_fuse_op.assign((size_t)n_st, -1);
    for (int s = 0; s < n_st && dtype == EE_I8; ++s) {
        const StageDesc& st = ctx->net.stages[s];
        int writer = -1, writers = 0;
        for (int k = 0; k < st.n_ops; ++k)
            if (ctx->plans[st.first_op + k].dst_buf == BUF_EXT_OUT) { writer = st.first_op + k; ++writers; }
        if (writers != 1) continue;
        const OpPlan& p = ctx->plans[(size_t)writer];
        const OpDesc& d = p.d;
        const ExitDesc& e = ctx->net.exits[s];
        if (p.impl == IMPL_MFMA && d.res >= 0 && d.c_tot == d.c_out && d.c_off == 0 && d.c_out % 16 == 0 && d.c_out == e.c &&
            d.h_out * d.w_out == e.h * e.w && 127 / (d.h_out * d.w_out) + 2 <= 8)
            ctx->gap_fuse_op[(size_t)s] = writer;
    }
    // Zero-copy compaction needs five blocks: up to 2 b_max - 1 waiting samples, the batch that is being read, and the
    // outputs of two steps in flight.  It is offered when every tensor that crosses a segment boundary is read and
    // written by the general matrix-core kernel only (the kernel that takes slot tables), b_max fits a table, and the
    // slots stay below 2 GiB (32-bit byte offsets).
    ctx->zero_copy_ok = b_max <= EE_ZC_MAX_B && n_st > 1;
    for (int s = 0; s < n_st && ctx->zero_copy_ok; ++s) {
        const StageDesc& st = ctx->net.stages[s];
        for (int k = 0; k < st.n_ops; ++k) {
            const OpPlan& p = ctx->plans[st.first_op + k];
            if (s > 0 && (p.src_buf == BUF_EXT_IN || (p.d.res >= 0 && p.res_buf == BUF_EXT_IN)) && (p.impl != IMPL_MFMA || (p.d.res >= 0 && p.res_buf == BUF_EXT_IN))) ctx->zero_copy_ok = false;
            if (s + 1 < n_st && p.dst_buf == BUF_EXT_OUT && p.impl != IMPL_MFMA) ctx->zero_copy_ok = false;
            if (p.src_buf == BUF_EXT_OUT || (p.d.res >= 0 && p.res_buf == BUF_EXT_OUT)) ctx->zero_copy_ok = false;   // the scattered output is not read back
        }
        if (s > 0 && (double)ctx->stage_in_bytes(s) * b_max * 5 >= 2147483648.0) ctx->zero_copy_ok = false;
    }
    ctx->zc_slots = (ctx->zero_copy_ok ? 5 : 3) * b_max;
    ctx->in_buf.assign(n_st, nullptr);
    for (int s = 1; s < n_st; ++s)
        if ((rc = dev_alloc(ctx, &ctx->in_buf[s], (size_t)ctx->stage_in_bytes(s) * ctx->zc_slots))) return fail(rc);
    ctx->lanes.resize(1);
    {
        LaneState& L0 = ctx->lanes[0];
        L0.stream = ctx->stream;
        L0.pool = ctx->pool;
        L0.pad_bufs = ctx->pad_bufs;
        if ((rc = alloc_lane(ctx, L0))) return fail(rc);
        ctx->lane = -1;
        ctx->bind_lane(0);
    }
    if (hipDeviceSynchronize() != hipSuccess) return fail(EE_ERR_DEVICE);
    *out = ctx;
    return EE_OK;
}

void ee_ctx::bind_lane(int j)
{
    if (j == lane) return;
    if (lane >= 0) {                              // the counters of the lane that was bound travel back
        lanes[(size_t)lane].seq = seq;
        lanes[(size_t)lane].head_b = head_b;
        lanes[(size_t)lane].ids_turn = ids_turn;
    }
    const ee::LaneState& L = lanes[(size_t)j];
    stream = L.stream; pool = L.pool; pad_bufs = L.pad_bufs; out_buf = L.out_buf; in_buf[0] = L.in0;
    sums = L.sums; gap_partial = L.gap_partial; logits = L.logits;
    d_label = L.d_label; d_conf = L.d_conf; d_score = L.d_score; d_flag = L.d_flag; d_slots = L.d_slots;
    h_out = L.h_out; h_ids[0] = L.h_ids[0]; h_ids[1] = L.h_ids[1]; seq = L.seq; head_b = L.head_b; ids_turn = L.ids_turn;
    lane = j;
}

// Further lanes for the stream driver (a set-up call, like ee_autotune: it allocates their workspace and streams).
extern "C" int ee_lanes(ee_ctx* ctx, int n)
{
    if (!ctx || n < 1 || n > 4) return EE_ERR_ARG;
    ctx->bind_lane(0);
    while ((int)ctx->lanes.size() < n) {
        LaneState L;
        if (hipStreamCreateWithFlags(&L.stream, hipStreamNonBlocking) != hipSuccess) return EE_ERR_DEVICE;   // default priority
        L.own_stream = true;
        const int rc = alloc_lane(ctx, L);
        ctx->lanes.push_back(L);                  // kept also on failure: ee_destroy releases what it holds
        if (rc) return rc;
    }
    if (hipDeviceSynchronize() != hipSuccess) return EE_ERR_DEVICE;
    return (int)ctx->lanes.size();
}

extern "C" int ee_destroy(ee_ctx* ctx)
{
    if (!ctx) return EE_OK;
    hipDeviceSynchronize();
    for (void* p : ctx->owned) hipFree(p);
    for (ee::LaneState& L : ctx->lanes) {
        if (L.h_pinned) hipHostFree(L.h_pinned);
        for (int s = 0; s < 8; ++s) if (L.packed[s]) hipEventDestroy(L.packed[s]);
        if (L.own_stream && L.stream) hipStreamDestroy(L.stream);
    }
    ctx->h_pinned = nullptr;
    for (ProfRec& r : ctx->prof) { hipEventDestroy(r.e0); hipEventDestroy(r.e1); }
    delete ctx;
    return EE_OK;
}

extern "C" int ee_query(const ee_ctx* ctx, int* n_stages, int64_t* in_bytes, int64_t* out_bytes)
{
    if (!ctx) return EE_ERR_ARG;
    const int n = (int)ctx->net.stages.size();
    if (n_stages) *n_stages = n;
    for (int s = 0; s < n; ++s) {
        if (in_bytes) in_bytes[s] = ctx->stage_in_bytes(s);
        if (out_bytes) out_bytes[s] = ctx->stage_out_bytes(s);
    }
    return EE_OK;
}

// ---- one convolution on the matrix cores -----------------------------------------------------------
void ee_ctx::fill_conv_args(int op, int b, ConvArgs& a) const
{
    const OpPlan& p = plans[op];
    const OpDesc& d = p.d;
    a.w = p.w_dev; a.bias = p.b_dev; a.zeros = zero_page;
    a.magic_howo = (unsigned)(0x100000000ull / (unsigned)(d.h_out * d.w_out) - (d.h_out * d.w_out == 1));
    a.magic_wo = (unsigned)(0x100000000ull / (unsigned)d.w_out - (d.w_out == 1));
    a.M = b * d.h_out * d.w_out; a.H = d.h_in; a.W = d.w_in; a.Ci = p.ci_eff; a.Ho = d.h_out; a.Wo = d.w_out; a.Co = d.c_out;
    a.kh = d.kh; a.kw = d.kw; a.stride = d.stride; a.pad = d.pad; a.pad_w = d.pad_w; a.Kp = p.Kp;
    a.ldc = d.c_tot; a.c_off = d.c_off;
    if (p.impl == IMPL_MFMA_S2D) {      // the folded tensor: ks2 x ks2 kernel, stride 1, padding already inside
        a.H = p.Hp; a.W = p.Wp; a.kh = a.kw = p.kwp; a.stride = 1; a.pad = a.pad_w = 0;
    }
    for (int r = 0; r < a.kh && r * a.kw < 32; ++r) a.tap_rows |= 1u << (r * a.kw);
    a.shift = d.shift; a.res_shift = d.res_shift; a.lo = d.lo; a.hi = d.hi; a.f_lo = d.f_lo; a.f_hi = d.f_hi;
}

hipError_t ee_ctx::launch_conv(int op, int b, const void* src, void* dst, const void* res, int cfg, const uint16_t* xs, const uint16_t* ys, int32_t* gap_sums)
{
    const OpPlan& p = plans[op];
    const int dt = net.dtype;
    ConvArgs a{};
    fill_conv_args(op, b, a);
    a.res = res; a.y = dst;
    if (p.impl == IMPL_MFMA_S2D || p.impl == IMPL_MFMA_CPAD) src = pad_bufs[p.pad_buf];
    if (p.impl == IMPL_MFMA_C4) {
        a.x = pad_bufs[p.pad_buf]; a.mode = 1; a.Hp = p.Hp; a.Wp = p.Wp; a.kwp = p.kwp;
        return dt == EE_I8 ? launch_conv_mfma_i8(a, stream) : launch_conv_mfma_bf16(a, stream);
    }
    a.x = src; a.mode = 0;
    if (xs || ys || gap_sums) {                          // slot tables, fused pooling: the general kernel only
        if (p.impl != IMPL_MFMA || ((xs || ys) && b > EE_ZC_MAX_B)) return hipErrorInvalidValue;
        a.xs = xs; a.ys = ys;
        a.gap_sums = gap_sums;
        if ((cfg & EE_CFG_SLAB) || (cfg & 15) == 7) cfg = 0;
        return dt == EE_I8 ? launch_conv_igemm<1>(a, cfg, stream) : launch_conv_igemm<2>(a, cfg, stream);
    }
    const bool streamable = conv_stream_supported(a, dt == EE_I8 ? 1 : 2);
    if ((cfg & 15) == 7) {
        if (streamable) return launch_conv_stream(a, stream);
        if (forced_conv_tile() != 7) return hipErrorInvalidValue;
        cfg = 0;                                         // forced for the whole process: layers it does not cover keep the default
    }
    if (cfg & EE_CFG_SLAB) {
        hipError_t e = hipErrorInvalidValue;             // a layer that is not of its kind, or a tile whose slab does not fit LDS
        if (conv_slab_supported(a, dt == EE_I8 ? 1 : 2)) e = dt == EE_I8 ? launch_conv_slab<1>(a, cfg & 0xFFFF, stream) : launch_conv_slab<2>(a, cfg & 0xFFFF, stream);
        if (e != hipErrorInvalidValue || forced_conv_tile() != cfg) return e;
        (void)hipGetLastError();
        cfg = 0;                                         // forced for the whole process: layers it does not cover keep the default
    }
    if (cfg == 0 && streamable && a.M >= 32768) return launch_conv_stream(a, stream);   // untuned: it wins on every large layer it covers
    return dt == EE_I8 ? launch_conv_igemm<1>(a, cfg, stream) : launch_conv_igemm<2>(a, cfg, stream);
}

void ee_ctx::fill_ir_args(int op, int b, IrArgs& a) const
{
    const OpPlan& p = plans[(size_t)op];
    const int o1 = p.ir_sc ? 1 : 0;                                     // the shortcut convolution in front: the block proper starts one layer on
    const OpDesc& e = plans[(size_t)op + o1].d;                         // without expansion: the depthwise layer itself
    const OpDesc& dw = plans[(size_t)op + o1 + (p.ir_noexp ? 0 : 1)].d;
    const OpDesc& pr = plans[(size_t)op + o1 + (p.ir_noexp ? 1 : 2)].d;
    a.we = p.ir_we; a.be = (const int*)p.ir_be; a.wd = p.ir_wd; a.bd = (const int*)p.ir_bd; a.wp = p.ir_wp; a.bp = (const int*)p.ir_bp;
    a.B = b; a.H = e.h_in; a.W = e.w_in; a.Cin = e.c_in; a.Kx = p.ir_kx; a.Ce32 = p.ir_ce32; a.Cout = pr.c_out;
    a.ys = nullptr; a.gap_sums = nullptr;
    a.ws = nullptr; a.bs = nullptr;
    if (p.ir_sc) { a.ws = p.ir_ws; a.bs = (const int*)p.ir_bs; a.sh_s = p.d.shift; a.lo_s = p.d.lo; a.hi_s = p.d.hi; }
    a.Ho = dw.h_out; a.Wo = dw.w_out; a.stride = dw.stride; a.pad = dw.pad;
    a.sh_e = e.shift; a.lo_e = e.lo; a.hi_e = e.hi;
    a.sh_d = dw.shift; a.lo_d = dw.lo; a.hi_d = dw.hi;
    a.sh_p = pr.shift; a.lo_p = pr.lo; a.hi_p = pr.hi; a.res_shift = pr.res_shift;
}

hipError_t ee_ctx::launch_pair(int op, int b, const void* src, void* dst, const void* res, int cfg)
{
    const OpPlan& q = plans[op + 1];
    PairArgs pa{};
    fill_conv_args(op, b, pa.c2);
    pa.c2.x = src; pa.c2.mode = 0;
    pa.w3 = q.w_dev; pa.bias3 = q.b_dev; pa.res = res; pa.y = dst;
    pa.Co3 = q.d.c_out; pa.Kp3 = q.Kp;
    pa.shift = q.d.shift; pa.res_shift = q.d.res_shift; pa.lo = q.d.lo; pa.hi = q.d.hi; pa.f_lo = q.d.f_lo; pa.f_hi = q.d.f_hi;
    return net.dtype == EE_I8 ? launch_conv_pair<1>(pa, cfg, stream) : launch_conv_pair<2>(pa, cfg, stream);
}

// ---- per-(layer, B_act) kernel configuration table ----------------------------------------------------
// The GPU face of the paper's run-time configuration look-up (Sec. III-A: one entry per layer and active
// batch size, fetched at run time): for every matrix-core convolution and every batch bucket 2^k the
// candidate tilings / reduction steps / ring depths are timed on the workspace buffers and the fastest
// is kept.  Results never depend on the choice.
extern "C" int ee_autotune(ee_ctx* ctx, int reps)
{
    if (!ctx || reps < 1 || reps > 1000) return EE_ERR_ARG;
    ctx->bind_lane(0);
    const bool was = ctx->profiling;
    ctx->profiling = false;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return EE_ERR_DEVICE;
    const int es = ctx->net.elem_bytes();
    int rc = EE_OK;
    std::vector<int> buckets;
    for (int k = 0; (1 << k) < 2 * ctx->b_max; ++k) buckets.push_back(std::min(1 << k, ctx->b_max));
    std::vector<std::vector<float>> best_time(ctx->plans.size());       // per layer and bucket: ms of `reps` launches of the best configuration
    for (size_t s = 0; s < ctx->net.stages.size() && !rc; ++s) {
        const StageDesc& st = ctx->net.stages[s];
        for (int k = 0; k < st.n_ops && !rc; ++k) {
            OpPlan& p = ctx->plans[st.first_op + k];
            if (p.impl != IMPL_MFMA && p.impl != IMPL_MFMA_CPAD && p.impl != IMPL_MFMA_S2D) continue;
            const OpDesc& d = p.d;
            const void* src = resolve(ctx, p.src_buf, ctx->in_buf[s], ctx->out_buf[s]);
            void* dst = resolve(ctx, p.dst_buf, ctx->in_buf[s], ctx->out_buf[s]);
            const void* res = d.res >= 0 ? resolve(ctx, p.res_buf, ctx->in_buf[s], ctx->out_buf[s]) : nullptr;
            const int kbytes = (p.impl == IMPL_MFMA_S2D ? p.kwp * p.kwp : d.kh * d.kw) * p.ci_eff * es;
            std::vector<int> best(buckets.size(), 0);
            best_time[st.first_op + k].assign(buckets.size(), 1e30f);
            for (size_t bi = 0; bi < buckets.size() && !rc; ++bi) {
                float& best_ms = best_time[st.first_op + k][bi];
                std::vector<int> cands;
                for (int tile = 1; tile <= 5; ++tile)
                    for (int ksel = 1; ksel <= 3; ++ksel)
                        for (int ns = 2; ns <= 4; ++ns)
                            for (int kspl = 1; kspl <= 4; kspl *= 2) {
                                if (tile == 5 && (ksel > 1 || ns > 2 || kspl > 1)) continue;  // the streaming kernel has one configuration
                                if (ksel > 1 && kbytes <= 64 * (ksel - 1)) continue;        // a longer step than the whole reduction
                                if (kspl > 1 && (ksel != 3 || tile < 3 || (kspl == 4 && tile != 3) || kbytes < 1024)) continue;   // combinations that exist
                                cands.push_back(tile == 5 ? 7 : tile | (ksel << 4) | (ns << 8) | ((kspl > 1 ? kspl : 0) << 12));
                            }
                for (int tile = 1; tile <= 4; ++tile)                                   // the slab kernel, where the layer is of its kind
                    for (int ksel = 2; ksel <= 3; ++ksel)
                        for (int ns = 2; ns <= 4; ++ns) cands.push_back(EE_CFG_SLAB | tile | (ksel << 4) | (ns << 8));
                for (const int cfg : cands) {
                    if (ctx->launch_conv(st.first_op + k, buckets[bi], src, dst, res, cfg) != hipSuccess) {
                        (void)hipGetLastError();                       // this configuration does not exist or fit here: skip it
                        continue;
                    }
                    hipEventRecord(e0, ctx->stream);
                    for (int r = 0; r < reps; ++r) ctx->launch_conv(st.first_op + k, buckets[bi], src, dst, res, cfg);
                    hipEventRecord(e1, ctx->stream);
                    if (hipEventSynchronize(e1) != hipSuccess) { rc = EE_ERR_DEVICE; break; }
                    float ms = 0.f;
                    hipEventElapsedTime(&ms, e0, e1);
                    if (ms < best_ms) { best_ms = ms; best[bi] = cfg; }
                }
            }
            if (!rc) p.cfg = best;
        }
        // fused pairs: every configuration of the fused kernel against the two best separate kernels
        for (int k = 0; k + 1 < st.n_ops && !rc; ++k) {
            OpPlan& p = ctx->plans[st.first_op + k];
            if (!p.pair) continue;
            const OpPlan& q = ctx->plans[st.first_op + k + 1];
            const void* src = resolve(ctx, p.src_buf, ctx->in_buf[s], ctx->out_buf[s]);
            void* dst = resolve(ctx, q.dst_buf, ctx->in_buf[s], ctx->out_buf[s]);
            const void* res = q.d.res >= 0 ? resolve(ctx, q.res_buf, ctx->in_buf[s], ctx->out_buf[s]) : nullptr;
            std::vector<int> best(buckets.size(), 0);
            for (size_t bi = 0; bi < buckets.size() && !rc; ++bi) {
                float best_ms = best_time[st.first_op + k][bi] + best_time[st.first_op + k + 1][bi];
                for (int tile = 1; tile <= 2; ++tile)
                    for (int ksel = 1; ksel <= 2; ++ksel)
                        for (int ns = 2; ns <= 4; ++ns) {
                            const int cfg = tile | (ksel << 4) | (ns << 8);
                            if (ctx->launch_pair(st.first_op + k, buckets[bi], src, dst, res, cfg) != hipSuccess) {
                                (void)hipGetLastError();
                                continue;
                            }
                            hipEventRecord(e0, ctx->stream);
                            for (int r = 0; r < reps; ++r) ctx->launch_pair(st.first_op + k, buckets[bi], src, dst, res, cfg);
                            hipEventRecord(e1, ctx->stream);
                            if (hipEventSynchronize(e1) != hipSuccess) { rc = EE_ERR_DEVICE; break; }
                            float ms = 0.f;
                            hipEventElapsedTime(&ms, e0, e1);
                            if (ms < best_ms) { best_ms = ms; best[bi] = cfg; }
                        }
            }
            if (!rc) p.pair_cfg = best;
        }
    }
    // fused blocks: the one launch against the block's layers with their tuned configurations.  A block of four layers (a
    // convolution on the shortcut in front of a bottleneck block) is tuned after the others, against that convolution followed
    // by whatever the table says for the block of three behind it.
    const int ir_was = ctx->ir_mode;
    for (int pass = 0; pass < 2 && !rc; ++pass)
        for (size_t s = 0; s < ctx->net.stages.size() && !rc; ++s) {
            const StageDesc& st = ctx->net.stages[s];
            for (int k = 0; k + 1 < st.n_ops && !rc; ++k) {
                OpPlan& p = ctx->plans[st.first_op + k];
                if (!p.ir || (pass == 1) != p.ir_sc) continue;
                std::vector<int> best(buckets.size(), 0);
                for (size_t bi = 0; bi < buckets.size() && !rc; ++bi) {
                    float ms[2] = {0.f, 0.f};
                    for (int fused = 0; fused < 2 && !rc; ++fused) {
                        ctx->ir_mode = fused ? 2 : (p.ir_sc ? 1 : 0);
                        p.ir_cfg.assign(buckets.size(), 0);                  // table mode: this head stays separate, the block behind it as tuned
                        if (fused || !p.ir_sc) p.ir_cfg.clear();
                        auto block = [&]() -> int {                          // the block alone: its head runs all its layers when fused
                            return ctx->run_stage((int)s, buckets[bi], ctx->in_buf[s], ctx->out_buf[s], false, -2 - (st.first_op + k));
                        };
                        if ((rc = block())) break;
                        hipEventRecord(e0, ctx->stream);
                        for (int r = 0; r < reps && !rc; ++r) rc = block();
                        hipEventRecord(e1, ctx->stream);
                        if (hipEventSynchronize(e1) != hipSuccess) rc = EE_ERR_DEVICE;
                        hipEventElapsedTime(&ms[fused], e0, e1);
                    }
                    best[bi] = ms[1] < ms[0] ? 1 : 0;
                }
                ctx->ir_mode = ir_was;
                if (!rc) p.ir_cfg = best;
            }
        }
    ctx->ir_mode = ir_was;
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    ctx->profiling = was;
    return rc;
}

/* copies the table of layer `op` (one entry per batch bucket 2^k, 0 = not tuned) to cfg_out[n]; returns the entry count */
extern "C" int ee_config_table(const ee_ctx* ctx, int op, int* cfg_out, int n)
{
    if (!ctx || op < 0 || op >= (int)ctx->plans.size() || n < 0 || (n > 0 && !cfg_out)) return EE_ERR_ARG;
    const std::vector<int>& c = ctx->plans[op].cfg;
    for (int i = 0; i < n && i < (int)c.size(); ++i) cfg_out[i] = c[i];
    return (int)c.size();
}

/* the fused-pair table of layer `op` (one entry per batch bucket, 0 = the two layers run separately); returns the entry
   count, 0 when the layer heads no pair or nothing was tuned */
extern "C" int ee_pair_table(const ee_ctx* ctx, int op, int* cfg_out, int n)
{
    if (!ctx || op < 0 || op >= (int)ctx->plans.size() || n < 0 || (n > 0 && !cfg_out)) return EE_ERR_ARG;
    const std::vector<int>& c = ctx->plans[op].pair_cfg;
    for (int i = 0; i < n && i < (int)c.size(); ++i) cfg_out[i] = c[i];
    return (int)c.size();
}

// Loading a stored table (the paper builds its look-up tables once, at design time, and loads them at run time).
extern "C" int ee_config_set(ee_ctx* ctx, int op, const int* cfg, int n)
{
    if (!ctx || op < 0 || op >= (int)ctx->plans.size() || n < 0 || n > 16 || (n > 0 && !cfg)) return EE_ERR_ARG;
    OpPlan& p = ctx->plans[op];
    if (p.impl != IMPL_MFMA && p.impl != IMPL_MFMA_CPAD && p.impl != IMPL_MFMA_S2D) return EE_ERR_ARG;
    for (int i = 0; i < n; ++i) {
        const int tile = cfg[i] & 15, ksel = (cfg[i] >> 4) & 15, ns = (cfg[i] >> 8) & 15, kspl = (cfg[i] >> 12) & 15;
        if (cfg[i] == 7) {                                                   // the streaming kernel, for the layers it covers
            ConvArgs a{};
            ctx->fill_conv_args(op, 1, a);
            a.res = p.d.res >= 0 ? (const void*)ctx : nullptr;               // only whether there is one matters here
            if (!conv_stream_supported(a, ctx->net.elem_bytes())) return EE_ERR_ARG;
            continue;
        }
        if (cfg[i] > 0 && (cfg[i] & EE_CFG_SLAB)) {                          // the slab kernel, for the layers it covers
            ConvArgs a{};
            ctx->fill_conv_args(op, 1, a);
            if (p.impl != IMPL_MFMA || !conv_slab_supported(a, ctx->net.elem_bytes())) return EE_ERR_ARG;
            if ((cfg[i] >> 17) || tile < 1 || tile > 4 || (ksel != 0 && ksel != 2 && ksel != 3) || (ns != 0 && (ns < 2 || ns > 4)) || kspl != 0) return EE_ERR_ARG;
            continue;
        }
        if (cfg[i] < 0 || (cfg[i] >> 16) || tile > 4 || ksel > 3 || (ns != 0 && (ns < 2 || ns > 4)) || (kspl != 0 && kspl != 2 && kspl != 4)) return EE_ERR_ARG;
    }
    p.cfg.assign(cfg, cfg + n);
    return EE_OK;
}

extern "C" int ee_pair_set(ee_ctx* ctx, int op, const int* cfg, int n)
{
    if (!ctx || op < 0 || op >= (int)ctx->plans.size() || n < 0 || n > 16 || (n > 0 && !cfg)) return EE_ERR_ARG;
    OpPlan& p = ctx->plans[op];
    if (!p.pair) return EE_ERR_ARG;
    for (int i = 0; i < n; ++i) {
        const int tile = cfg[i] & 15, ksel = (cfg[i] >> 4) & 15, ns = (cfg[i] >> 8) & 15;
        if (cfg[i] < 0 || (cfg[i] >> 12) || tile > 2 || ksel > 2 || (ns != 0 && (ns < 2 || ns > 4))) return EE_ERR_ARG;
    }
    p.pair_cfg.assign(cfg, cfg + n);
    return EE_OK;
}

extern "C" int ee_ir_count(const ee_ctx* ctx)
{
    if (!ctx) return EE_ERR_ARG;
    int n = 0;
    for (const OpPlan& p : ctx->plans) n += p.ir;
    return n;
}

extern "C" int ee_ir_layers(const ee_ctx* ctx, int layer)
{
    if (!ctx || layer < 0 || layer >= (int)ctx->plans.size()) return EE_ERR_ARG;
    const OpPlan& p = ctx->plans[(size_t)layer];
    return p.ir ? p.ir_last() + 1 : 0;
}

extern "C" int ee_ir_mode(ee_ctx* ctx, int mode)
{
    if (!ctx || mode < 0 || mode > 2) return EE_ERR_ARG;
    ctx->ir_mode = mode;
    return EE_OK;
}

extern "C" int ee_ir_table(const ee_ctx* ctx, int op, int* cfg_out, int n)
{
    if (!ctx || op < 0 || op >= (int)ctx->plans.size() || n < 0 || (n > 0 && !cfg_out)) return EE_ERR_ARG;
    const std::vector<int>& c = ctx->plans[op].ir_cfg;
    for (int i = 0; i < n && i < (int)c.size(); ++i) cfg_out[i] = c[i];
    return (int)c.size();
}

extern "C" int ee_ir_set(ee_ctx* ctx, int op, const int* cfg, int n)
{
    if (!ctx || op < 0 || op >= (int)ctx->plans.size() || n < 0 || n > 16 || (n > 0 && !cfg)) return EE_ERR_ARG;
    OpPlan& p = ctx->plans[op];
    if (!p.ir) return EE_ERR_ARG;
    for (int i = 0; i < n; ++i)
        if (cfg[i] != 0 && cfg[i] != 1) return EE_ERR_ARG;
    p.ir_cfg.assign(cfg, cfg + n);
    return EE_OK;
}

extern "C" int ee_pair_mode(ee_ctx* ctx, int mode)
{
    if (!ctx || mode < 0 || mode > 2) return EE_ERR_ARG;
    ctx->pair_mode = mode;
    return EE_OK;
}

extern "C" int ee_zero_copy_supported(const ee_ctx* ctx) { return ctx ? (ctx->zero_copy_ok ? 1 : 0) : EE_ERR_ARG; }

extern "C" int ee_pair_count(const ee_ctx* ctx)
{
    if (!ctx) return EE_ERR_ARG;
    int n = 0;
    for (const OpPlan& p : ctx->plans) n += p.pair;
    return n;
}

// ---- one backbone segment ------------------------------------------------------------------------
int ee_ctx::run_stage(int stage, int b, const void* act_in, void* act_out, bool first_packed, int only_op, int cfg_force)
{
    const int only_block = only_op <= -2 ? -2 - only_op : -1;      // <= -2: just the three layers of the block headed by layer -2 - only_op
    gap_fused = false;
    const StageDesc& st = net.stages[stage];
    const int dt = net.dtype, es = net.elem_bytes();
    for (int k = 0; k < st.n_ops; ++k) {
        if (only_op >= 0 && st.first_op + k != only_op) continue;
        if (only_block >= 0 && (st.first_op + k < only_block || st.first_op + k > only_block + plans[(size_t)only_block].ir_last())) continue;
        OpPlan& p = plans[st.first_op + k];
        const OpDesc& d = p.d;
        const void* src = resolve(this, p.src_buf, act_in, act_out);
        void* dst = resolve(this, p.dst_buf, act_in, act_out);
        const void* res = d.res >= 0 ? resolve(this, p.res_buf, act_in, act_out) : nullptr;
        const double ops = p.ops_per_sample * b, bytes = p.bytes_per_sample * b + p.weight_bytes;
        hipError_t e = hipSuccess;
        int32_t* gap_dst = gap_fuse_dst && only_op < 0 && st.first_op + k == gap_fuse_op[(size_t)stage] ? gap_fuse_dst : nullptr;
        const uint16_t* xs = p.src_buf == BUF_EXT_IN ? zc_in : nullptr;
        const uint16_t* ys = p.dst_buf == BUF_EXT_OUT ? zc_out : nullptr;
        if ((xs || ys) && p.impl != IMPL_MFMA) return EE_ERR_UNSUPPORTED;
        if (zc_in && d.res >= 0 && p.res_buf == BUF_EXT_IN) return EE_ERR_UNSUPPORTED;
        const int ir_last = p.ir_last();                                    // the block's last layer, counted from this one
        // a bottleneck block may sit in a segment whose last layer writes slots, and may be that layer (its kernel takes the slot table)
        // (the fused first convolution + pool writes inside the segment: slots do not concern it)
        const bool ir_slots_ok = p.ir_bneck ? !(zc_in && plans[st.first_op + k + ir_last].res_buf == BUF_EXT_IN) : p.ir_stem || !zc_out;
        // the exit head's pooling rides on the segment's last layer: a bottleneck block's kernel carries it (with a residual), the others do not
        const bool ir_pools = gap_fuse_dst && only_op < 0 && st.first_op + k + ir_last == gap_fuse_op[(size_t)stage];
        if (p.ir && ir_mode > 0 && cfg_force == 0 && forced_conv_tile() == 0 && only_op < 0 && !xs && ir_slots_ok &&
            !(ir_pools && !(p.ir_bneck && plans[st.first_op + k + ir_last].d.res >= 0))) {
            // this layer, the depthwise layer and the projection as one launch, where the table says it is faster
            const int ic = p.ir_cfg.empty() ? 0 : p.ir_cfg[std::min<size_t>(bucket_of(b), p.ir_cfg.size() - 1)];
            if ((ic != 0 || ir_mode == 2) && p.ir_stem) {
                const OpPlan& q2 = plans[st.first_op + k + 1];
                if (!(first_packed && k == 0)) {                                 // the folded copy of the input, as in front of the layer alone
                    const double pb = (double)b * ((double)d.h_in * d.w_in * d.c_in + (double)p.Hp * p.Wp * 16) * es;
                    e = timed(EE_K_PAD_INPUT, 0.0, pb, [&] { return launch_space_to_depth(src, pad_bufs[p.pad_buf], nullptr, b, d.h_in, d.w_in, d.c_in, p.Hp, p.Wp, d.pad, dt, stream); });
                    if (e != hipSuccess) return EE_ERR_DEVICE;
                }
                ConvArgs ca{};
                fill_conv_args(st.first_op + k, b, ca);
                ca.x = pad_bufs[p.pad_buf]; ca.mode = 0;
                void* yq = resolve(this, q2.dst_buf, act_in, act_out);
                const double mid = 2.0 * b * (double)d.h_out * d.w_out * d.c_out;      // the tensor that stays on chip
                e = timed(EE_K_CONV_STREAM, ops + q2.ops_per_sample * b, bytes + q2.bytes_per_sample * b + q2.weight_bytes - mid,
                          [&] { return launch_stem_pool(ca, yq, q2.d.h_out, q2.d.w_out, stream); }, st.first_op + k);
                if (e != hipSuccess) return EE_ERR_DEVICE;
                ++k;                                                             // the pool is done
                continue;
            }
            if (ic != 0 || ir_mode == 2) {
                const OpPlan& q2 = plans[st.first_op + k + ir_last];
                IrArgs ia{};
                fill_ir_args(st.first_op + k, b, ia);
                ia.x = src;
                ia.y = resolve(this, q2.dst_buf, act_in, act_out);
                ia.res = q2.d.res >= 0 && !p.ir_sc ? resolve(this, q2.res_buf, act_in, act_out) : nullptr;   // the kernel computes the shortcut itself
                ia.ys = q2.dst_buf == BUF_EXT_OUT ? zc_out : nullptr;
                ia.gap_sums = ir_pools && bneck_block_pools(ia) ? gap_fuse_dst : nullptr;       // else the head pools the output itself
                double f_ops = ops, f_bytes = bytes;                             // the block's layers; the tensors between them stay on chip
                for (int j = 1; j <= ir_last; ++j) {
                    const OpPlan& q = plans[st.first_op + k + j];
                    const OpDesc& prev = plans[st.first_op + k + j - 1].d;
                    f_ops += q.ops_per_sample * b;
                    f_bytes += q.bytes_per_sample * b + q.weight_bytes - 2.0 * b * (double)prev.h_out * prev.w_out * prev.c_out;
                }
                e = timed(EE_K_CONV_MFMA, f_ops, f_bytes, [&] { return p.ir_bneck ? launch_bneck_block(ia, stream) : launch_ir_block(ia, stream); }, st.first_op + k);
                if (e != hipSuccess) return EE_ERR_DEVICE;
                if (ia.gap_sums) gap_fused = true;
                k += ir_last;                                                    // the block's other layers are done
                continue;
            }
        }
        if (p.impl == IMPL_MFMA || p.impl == IMPL_MFMA_C4 || p.impl == IMPL_MFMA_CPAD || p.impl == IMPL_MFMA_S2D) {
            if (p.impl == IMPL_MFMA_S2D && !(first_packed && k == 0)) {
                const double pb = (double)b * ((double)d.h_in * d.w_in * d.c_in + (double)p.Hp * p.Wp * 16) * es;
                e = timed(EE_K_PAD_INPUT, 0.0, pb, [&] { return launch_space_to_depth(src, pad_bufs[p.pad_buf], nullptr, b, d.h_in, d.w_in, d.c_in, p.Hp, p.Wp, d.pad, dt, stream); });
                if (e != hipSuccess) return EE_ERR_DEVICE;
            }
            if (p.impl == IMPL_MFMA_CPAD) {
                const double pb = (double)b * d.h_in * d.w_in * (d.c_in + p.ci_eff) * es;
                e = timed(EE_K_PAD_INPUT, 0.0, pb, [&] {
                    return launch_pad_channels(src, pad_bufs[p.pad_buf], (long long)b * d.h_in * d.w_in, d.c_in * es, p.ci_eff * es, stream);
                });
                if (e != hipSuccess) return EE_ERR_DEVICE;
            }
            if (p.impl == IMPL_MFMA_C4) {
                const double pb = (double)b * ((double)d.h_in * d.w_in * d.c_in + (double)p.Hp * p.Wp * 4) * es;
                e = timed(EE_K_PAD_INPUT, 0.0, pb, [&] { return launch_pad_input(src, pad_bufs[p.pad_buf], b, d.h_in, d.w_in, d.c_in, p.Hp, p.Wp, d.pad, dt, stream); });
                if (e != hipSuccess) return EE_ERR_DEVICE;
            }
            int cfg = cfg_force > 0 ? cfg_force : forced_conv_tile();
            const bool q_scatter = k + 1 < st.n_ops && ((zc_out && plans[st.first_op + k + 1].dst_buf == BUF_EXT_OUT) ||
                                                        (gap_fuse_dst && only_op < 0 && st.first_op + k + 1 == gap_fuse_op[(size_t)stage]));
            if (p.pair && pair_mode > 0 && cfg == 0 && only_op < 0 && !xs && !ys && !q_scatter) {
                // this layer and the next as one launch, unless the table says the two separate kernels are faster here
                const int pc = p.pair_cfg.empty() ? 0 : p.pair_cfg[std::min<size_t>(bucket_of(b), p.pair_cfg.size() - 1)];
                // untuned: fused below 32 samples, where it was measured to win (one launch fewer counts most there)
                if ((p.pair_cfg.empty() && b < 32) || pc != 0 || pair_mode == 2) {
                    const OpPlan& q = plans[st.first_op + k + 1];
                    void* dst2 = resolve(this, q.dst_buf, act_in, act_out);
                    const void* res2 = q.d.res >= 0 ? resolve(this, q.res_buf, act_in, act_out) : nullptr;
                    const double mid = 2.0 * d.h_out * d.w_out * d.c_out * es * b;      // the tensor that stays on chip
                    e = timed(EE_K_CONV_MFMA, ops + q.ops_per_sample * b, bytes + q.bytes_per_sample * b + q.weight_bytes - mid,
                              [&] { return launch_pair(st.first_op + k, b, src, dst2, res2, pc); }, st.first_op + k);
                    if (e != hipSuccess) return EE_ERR_DEVICE;
                    ++k;                                                             // the next layer is done
                    continue;
                }
            }
            if (cfg == 0 && !p.cfg.empty()) cfg = p.cfg[std::min<size_t>(bucket_of(b), p.cfg.size() - 1)];
            int cls = p.impl == IMPL_MFMA_C4 ? EE_K_CONV_FIRST : EE_K_CONV_MFMA;
            if (p.impl != IMPL_MFMA_C4 && ((cfg & 15) == 7 || cfg == 0)) {             // the streaming kernel is booked in its own class
                ConvArgs probe{};
                fill_conv_args(st.first_op + k, b, probe);
                probe.res = res;
                if (conv_stream_supported(probe, es) && ((cfg & 15) == 7 || probe.M >= 32768)) cls = EE_K_CONV_STREAM;
            }
            e = timed(cls, ops, bytes, [&] { return launch_conv(st.first_op + k, b, src, dst, res, cfg, xs, ys, gap_dst); }, st.first_op + k);
            if (gap_dst && e == hipSuccess) gap_fused = true;
        } else if (p.impl == IMPL_THIN) {
            ThinConvArgs a{src, p.w_dev, p.b_dev, dst, (long long)b * d.h_out * d.w_out, d.c_in, d.c_out, d.c_tot, d.c_off, d.shift, d.lo, d.hi};
            e = timed(EE_K_CONV_STREAM, ops, bytes, [&] { return launch_conv_thin(a, stream); }, st.first_op + k);
        } else if (p.impl == IMPL_DIRECT) {
            DirectConvArgs a{src, p.w_dev, p.b_dev, res, dst, b * d.h_out * d.w_out, d.h_in, d.w_in, d.c_in, d.h_out, d.w_out, d.c_out,
                             d.kh, d.kw, d.stride, d.pad, d.shift, d.res_shift, d.lo, d.hi, d.f_lo, d.f_hi, d.pad_w, d.c_tot, d.c_off};
            e = timed(EE_K_CONV_DIRECT, ops, bytes, [&] { return launch_conv_direct(a, dt, stream); }, st.first_op + k);
        } else {
            PoolArgs a{src, p.w_dev, p.b_dev, dst, p.w3_dev, b, d.h_in, d.w_in, d.c_in, d.h_out, d.w_out, d.kh, d.stride, d.pad, d.shift, d.lo, d.hi, d.f_lo, d.f_hi,
                       d.c_tot, d.c_off};
            if (p.impl == IMPL_DW) e = timed(EE_K_DEPTHWISE, ops, bytes, [&] { return launch_depthwise(a, dt, stream); }, st.first_op + k);
            else if (p.impl == IMPL_AVGPOOL) e = timed(EE_K_MAXPOOL, 0.0, bytes, [&] { return launch_avgpool(a, dt, stream); }, st.first_op + k);   // timed with the pooling class
            else e = timed(EE_K_MAXPOOL, 0.0, bytes, [&] { return launch_maxpool(a, dt, stream); }, st.first_op + k);
        }
        if (e != hipSuccess) return EE_ERR_DEVICE;
    }
    return EE_OK;
}

extern "C" int ee_stage_forward(ee_ctx* ctx, int stage, int b_act, const void* act_in, void* act_out)
{
    if (!ctx || stage < 0 || stage >= (int)ctx->net.stages.size() || b_act < 0 || b_act > ctx->b_max) return EE_ERR_ARG;
    ctx->bind_lane(0);
    if (b_act == 0) return EE_OK;
    if (!act_in || !act_out || act_in == act_out || !aligned16(act_in) || !aligned16(act_out)) return EE_ERR_ARG;
    return ctx->run_stage(stage, b_act, act_in, act_out);
}

// ---- one exit head ------------------------------------------------------------------------------------
int ee_ctx::run_head(int stage, int b, const void* act, float thr, int32_t* label, float* conf, int64_t* score, uint8_t* flag, bool to_host,
                     const ee::HeadScratch* own, const uint16_t* slots, bool pooled)
{
    const ExitDesc& e = net.exits[stage];
    const int dt = net.dtype, es = net.elem_bytes();
    HeadArgs a{};
    a.act = act; a.B = b; a.HW = e.h * e.w; a.C = e.c; a.n_cls = e.n_cls;
    a.gap_shift = e.gap_shift; a.frac_bits = e.frac_bits; a.logit_scale = e.logit_scale;
    a.wfc = wfc_dev[stage]; a.bfc = bfc_dev[stage];
    a.sums = own ? own->sums : sums; a.gap_partial = own ? own->gap_partial : gap_partial; a.logits = own ? own->logits : logits;
    a.thr = thr;
    a.s_thr = !(thr > 0.0f) ? INT64_MAX : (thr > 1.0f ? 0 : (int64_t)std::floor(1073741824.0 / (double)thr));
    a.last = stage == (int)net.stages.size() - 1;
    a.label = label; a.conf = conf; a.score = score; a.flag = flag;
    a.slots = slots;
    if (to_host) {
        // cleared records match no tag: the host takes none of an earlier launch for one of this
        for (int k = 0; k < b; ++k) {
            __atomic_store_n(&h_out[k].w0, 0ull, __ATOMIC_RELAXED);
            __atomic_store_n(&h_out[k].w1, 0ull, __ATOMIC_RELAXED);
        }
        a.host_out = h_out; a.tag = ee::outcome_tag(++seq); head_b = b;
    }
    const double act_bytes = (double)b * a.HW * a.C * es;
    if (!pooled && timed(EE_K_GAP, 0.0, act_bytes + 4.0 * b * a.C, [&] { return launch_head_gap(a, dt, stream); }) != hipSuccess) return EE_ERR_DEVICE;
    if (timed(EE_K_FC, 2.0 * b * a.C * a.n_cls, (double)a.C * a.n_cls * es + 4.0 * b * (a.C + a.n_cls),
              [&] { return launch_head_fc(a, dt, stream); }) != hipSuccess) return EE_ERR_DEVICE;
    if (timed(EE_K_SOFTMAX, 0.0, 4.0 * b * a.n_cls + 17.0 * b, [&] { return launch_head_softmax(a, dt, stream); }) != hipSuccess) return EE_ERR_DEVICE;
    return EE_OK;
}

int ee_ctx::wait_head()
{
    const auto t0 = std::chrono::steady_clock::now();
    for (unsigned spins = 0; !head_reported(); ++spins)
        if ((spins & 0xFFF) == 0xFFF && std::chrono::steady_clock::now() - t0 > std::chrono::seconds(2)) {
            // no records after two seconds: let the runtime say what happened to the stream
            if (hipStreamSynchronize(stream) != hipSuccess) return EE_ERR_DEVICE;
            return head_reported() ? EE_OK : EE_ERR_DEVICE;
        }
    return EE_OK;
}

extern "C" int ee_exit_head(ee_ctx* ctx, int stage, int b_act, const void* act, float thr,
                            int32_t* label, float* conf, int64_t* score, uint8_t* exit_flag)
{
    if (!ctx || stage < 0 || stage >= (int)ctx->net.stages.size() || b_act < 0 || b_act > ctx->b_max) return EE_ERR_ARG;
    ctx->bind_lane(0);
    if (b_act == 0) return EE_OK;
    if (!act || !label || !conf || !score || !exit_flag || !aligned16(act)) return EE_ERR_ARG;
    return ctx->run_head(stage, b_act, act, thr, label, conf, score, exit_flag);
}

// The same head with its scratch memory (pooled sums, partial rows of the float pooling, logits) in the array that is
// part of the library image instead of the context's workspace: the call allocates nothing.
extern "C" int ee_exit_head_static(ee_ctx* ctx, int stage, int b_act, const void* act, float thr,
                                   int32_t* label, float* conf, int64_t* score, uint8_t* exit_flag)
{
    if (!ctx || stage < 0 || stage >= (int)ctx->net.stages.size() || b_act < 0 || b_act > ctx->b_max) return EE_ERR_ARG;
    ctx->bind_lane(0);
    if (b_act == 0) return EE_OK;
    if (!act || !label || !conf || !score || !exit_flag || !aligned16(act)) return EE_ERR_ARG;
    const ExitDesc& e = ctx->net.exits[stage];
    auto up256 = [](size_t v) { return (v + 255) / 256 * 256; };
    const size_t sums_bytes = up256(4 * (size_t)b_act * e.c);
    const size_t logit_bytes = up256(4 * (size_t)b_act * e.n_cls);
    const int splits = ctx->net.dtype == EE_BF16 ? head_gap_splits(b_act, e.h * e.w) : 0;
    const size_t partial_bytes = splits > 1 ? up256(4 * (size_t)b_act * splits * e.c) : 0;
    if (sums_bytes + logit_bytes + partial_bytes > (size_t)EE_STATIC_SCRATCH_BYTES) return EE_ERR_OVERFLOW;
    void* base = nullptr;
    if (static_scratch(&base) != hipSuccess) return EE_ERR_DEVICE;
    unsigned char* p = static_cast<unsigned char*>(base);
    HeadScratch own{reinterpret_cast<int32_t*>(p), reinterpret_cast<int32_t*>(p + sums_bytes + logit_bytes), p + sums_bytes};
    // the array keeps what the last call on this GPU left: the integer pooling adds into sums that start at zero
    if (ctx->net.dtype == EE_I8 && launch_fill_zero(own.sums, sums_bytes, ctx->stream) != hipSuccess) return EE_ERR_DEVICE;
    return ctx->run_head(stage, b_act, act, thr, label, conf, score, exit_flag, false, &own);
}

extern "C" int ee_static_scratch_bytes(void) { return EE_STATIC_SCRATCH_BYTES; }

extern "C" int ee_last_logits(ee_ctx* ctx, int b_act, void* host_out)
{
    if (!ctx || !host_out || b_act < 0 || b_act > ctx->b_max) return EE_ERR_ARG;
    ctx->bind_lane(0);
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return EE_ERR_DEVICE;
    if (b_act && hipMemcpy(host_out, ctx->logits, 4 * (size_t)b_act * ctx->net.n_classes, hipMemcpyDeviceToHost) != hipSuccess) return EE_ERR_DEVICE;
    return EE_OK;
}

// ---- compaction and refill ------------------------------------------------------------------------------
extern "C" int ee_compact_refill(ee_ctx* ctx, int stage, int b_act, const uint8_t* exit_flag,
                                 const void* act_src, void* act_dst, const int32_t* ids_src, int32_t* ids_dst,
                                 const void* refill_act, const int32_t* refill_ids, int b_incr,
                                 int* b_rem_out, int* b_merged_out)
{
    if (!ctx || stage < 0 || stage >= (int)ctx->net.stages.size() || b_act < 0 || b_incr < 0 || b_act + b_incr > ctx->b_max) return EE_ERR_ARG;
    ctx->bind_lane(0);
    if (b_act > 0 && (!exit_flag || !act_src || !aligned16(act_src))) return EE_ERR_ARG;
    if (b_incr > 0 && (!refill_act || !aligned16(refill_act))) return EE_ERR_ARG;
    if ((b_act > 0 || b_incr > 0) && (!act_dst || !aligned16(act_dst) || act_dst == act_src || act_dst == refill_act)) return EE_ERR_ARG;
    const int64_t sb = ctx->stage_out_bytes(stage);
    hipStream_t s = ctx->stream;
    if (b_act > 0) {
        // only the survivors move: B_rem samples read and written.  The host does not know B_rem here, so a timed run
        // (and only a timed run) reads the flags back to count them.
        double bytes = 2.0 * sb * b_act;
        if (ctx->profiling) {
            std::vector<uint8_t> hf((size_t)b_act);
            if (hipStreamSynchronize(s) != hipSuccess || hipMemcpy(hf.data(), exit_flag, (size_t)b_act, hipMemcpyDeviceToHost) != hipSuccess) return EE_ERR_DEVICE;
            bytes = 2.0 * sb * (double)std::count(hf.begin(), hf.end(), (uint8_t)0);
        }
        if (ctx->timed(EE_K_COMPACT, 0.0, bytes, [&] {
                return launch_compact(exit_flag, act_src, act_dst, ids_src, ids_dst, b_act, sb, 0, 0, ctx->d_count, b_rem_out, s);
            }) != hipSuccess)
            return EE_ERR_DEVICE;
    } else {
        if (hipMemsetAsync(ctx->d_count, 0, sizeof(int), s) != hipSuccess) return EE_ERR_DEVICE;
        if (b_rem_out && hipMemsetAsync(b_rem_out, 0, sizeof(int), s) != hipSuccess) return EE_ERR_DEVICE;
    }
    if (b_incr > 0) {
        if (ctx->timed(EE_K_COMPACT, 0.0, 2.0 * sb * b_incr, [&] {
                return launch_append(refill_act, act_dst, refill_ids, ids_dst, ctx->d_count, 0, b_incr, sb, b_merged_out, s);
            }) != hipSuccess)
            return EE_ERR_DEVICE;
    } else if (b_merged_out) {
        if (hipMemcpyAsync(b_merged_out, ctx->d_count, sizeof(int), hipMemcpyDefault, s) != hipSuccess) return EE_ERR_DEVICE;
    }
    return EE_OK;
}

// ---- design-time latency table ---------------------------------------------------------------------------
// The design-time exit-level latency table (Sec. III-B, "Exit-Level Latency Prediction").  An entry is what a step of the
// stream driver costs on the wall clock, measured the way the driver runs it: the segment (the first one reads its input
// through the admission copy, as when requests are admitted), the exit head writing its outcomes to host memory, the
// compaction of all b samples behind it (nobody exits: the upper bound), and the host waiting for the head's records.
// Eq. 4 relies on the table not under-estimating (a preemption it accepts must not cause a violation).
extern "C" int ee_measure_lut(ee_ctx* ctx, int reps, int64_t* lut_ns)
{
    if (!ctx || !lut_ns || reps < 1) return EE_ERR_ARG;
    ctx->bind_lane(0);
    const int n_st = (int)ctx->net.stages.size(), bm = ctx->b_max;
    const bool was = ctx->profiling;
    ctx->profiling = false;
    const int step = std::max(1, bm / 64);
    int rc = EE_OK;
    for (int k = 0; k < bm; ++k) ctx->h_ids[0][k] = ctx->h_ids[1][k] = k;      // admission of rows 0..b-1 of segment 0's own input slots
    const OpPlan* fold = ctx->admission_fold();
    for (int s = 0; s < n_st && !rc; ++s) {
        std::vector<int> measured;
        for (int b = 1; b <= bm; b += step) measured.push_back(b);
        if (measured.back() != bm) measured.push_back(bm);
        std::vector<double> t(measured.size());
        const int64_t sb_out = ctx->stage_out_bytes(s);
        for (size_t i = 0; i < measured.size() && !rc; ++i) {
            const int b = measured[i];
            for (int pass = 0; pass < 2 && !rc; ++pass) {               // pass 0 warms caches and code objects
                const int n = pass == 0 ? 1 : reps;
                if (hipStreamSynchronize(ctx->stream) != hipSuccess) rc = EE_ERR_DEVICE;
                const auto t0 = std::chrono::steady_clock::now();
                for (int r = 0; r < n && !rc; ++r) {
                    if (s == 0 && fold) {
                        const OpDesc& d = fold->d;
                        if (launch_space_to_depth(ctx->in_buf[0], ctx->pad_bufs[fold->pad_buf], ctx->h_ids[0], b, d.h_in, d.w_in, d.c_in, fold->Hp, fold->Wp, d.pad, ctx->net.dtype, ctx->stream, true) != hipSuccess) rc = EE_ERR_DEVICE;
                    }
                    ctx->gap_fuse_dst = ctx->sums;
                    if (!rc) rc = ctx->run_stage(s, b, ctx->in_buf[s], ctx->out_buf[s], s == 0 && fold != nullptr);
                    ctx->gap_fuse_dst = nullptr;
                    if (!rc) rc = ctx->run_head(s, b, ctx->out_buf[s], 2.0f, ctx->d_label, ctx->d_conf, ctx->d_score, ctx->d_flag, true, nullptr, nullptr, ctx->gap_fused);
                    if (!rc && s + 1 < n_st && launch_compact(ctx->d_flag, ctx->out_buf[s], ctx->in_buf[s + 1], nullptr, nullptr, b, sb_out, 0, 0, nullptr, nullptr, ctx->stream) != hipSuccess) rc = EE_ERR_DEVICE;
                    if (!rc) rc = ctx->wait_head();
                }
                if (hipStreamSynchronize(ctx->stream) != hipSuccess) rc = EE_ERR_DEVICE;
                t[i] = std::chrono::duration<double, std::nano>(std::chrono::steady_clock::now() - t0).count() / n;
            }
        }
        for (int b = 1; b <= bm && !rc; ++b) {                          // linear interpolation between measured sizes
            size_t hi = 0;
            while (measured[hi] < b) ++hi;
            double v = t[hi];
            if (measured[hi] != b) {
                const double w = (double)(b - measured[hi - 1]) / (measured[hi] - measured[hi - 1]);
                v = t[hi - 1] * (1 - w) + t[hi] * w;
            }
            lut_ns[(size_t)s * bm + b - 1] = (int64_t)std::llround(v);
        }
    }
    ctx->profiling = was;
    return rc;
}

// One layer alone, `reps` launches back to back on the workspace buffers (design-time measurement, like the tables above).
extern "C" int ee_time_layer(ee_ctx* ctx, int layer, int b, int cfg, int reps, double* us_out, double* ops_out, double* bytes_out)
{
    if (!ctx || layer < 0 || layer >= (int)ctx->plans.size() || b < 1 || b > ctx->b_max || reps < 1 || reps > 100000 || cfg < 0 || !us_out) return EE_ERR_ARG;
    ctx->bind_lane(0);
    int stage = -1;
    for (size_t s = 0; s < ctx->net.stages.size(); ++s)
        if (layer >= ctx->net.stages[s].first_op && layer < ctx->net.stages[s].first_op + ctx->net.stages[s].n_ops) stage = (int)s;
    if (stage < 0) return EE_ERR_ARG;
    const bool fused_block = cfg == EE_CFG_IR_BLOCK;               // the inverted-residual block headed by `layer` as one launch
    if (fused_block && !ctx->plans[layer].ir) return EE_ERR_ARG;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return EE_ERR_DEVICE;
    const int ir_was = ctx->ir_mode;
    if (fused_block) ctx->ir_mode = 2;
    const bool was = ctx->profiling;
    ctx->profiling = false;
    int rc = EE_OK;
    for (int pass = 0; pass < 2 && !rc; ++pass) {                   // pass 0 warms caches and code objects
        const int n = pass == 0 ? 2 : reps;
        hipEventRecord(e0, ctx->stream);
        for (int r = 0; r < n && !rc; ++r)
            rc = fused_block ? ctx->run_stage(stage, b, ctx->in_buf[stage], ctx->out_buf[stage], false, -2 - layer)
                             : ctx->run_stage(stage, b, ctx->in_buf[stage], ctx->out_buf[stage], false, layer, cfg);
        hipEventRecord(e1, ctx->stream);
        if (hipEventSynchronize(e1) != hipSuccess) rc = EE_ERR_DEVICE;
        float ms = 0.f;
        hipEventElapsedTime(&ms, e0, e1);
        *us_out = (double)ms * 1e3 / n;
    }
    (void)hipGetLastError();
    ctx->ir_mode = ir_was;
    const OpPlan& p = ctx->plans[layer];
    if (ops_out) *ops_out = p.ops_per_sample * b;
    if (bytes_out) *bytes_out = p.bytes_per_sample * b + p.weight_bytes;
    if (fused_block)                                                 // the block's layers; the tensors between them stay on chip
        for (int j = 1; j <= p.ir_last(); ++j) {
            const OpPlan& q = ctx->plans[layer + j];
            const OpDesc& prev = ctx->plans[layer + j - 1].d;
            if (ops_out) *ops_out += q.ops_per_sample * b;
            if (bytes_out) *bytes_out += q.bytes_per_sample * b + q.weight_bytes - 2.0 * b * (double)prev.h_out * prev.w_out * prev.c_out;
        }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    ctx->profiling = was;
    return rc;
}

// ---- kernel timing ------------------------------------------------------------------------------------------
extern "C" int ee_profile_enable(ee_ctx* ctx, int enable)
{
    if (!ctx) return EE_ERR_ARG;
    ctx->profiling = enable != 0;
    return EE_OK;
}

extern "C" int ee_profile_reserve(ee_ctx* ctx, int64_t n_pairs)
{
    if (!ctx || n_pairs < 0 || n_pairs > (1 << 22)) return EE_ERR_ARG;
    while ((int64_t)ctx->prof.size() < n_pairs) {
        ProfRec r{};
        if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) return EE_ERR_DEVICE;
        ctx->prof.push_back(r);
    }
    return EE_OK;
}

extern "C" int ee_profile_read(ee_ctx* ctx, ee_kernel_stat* stats, ee_kernel_stat* per_layer)
{
    if (!ctx || !stats) return EE_ERR_ARG;
    for (const LaneState& L : ctx->lanes)
        if (hipStreamSynchronize(L.stream) != hipSuccess) return EE_ERR_DEVICE;
    for (int k = 0; k < EE_K_COUNT; ++k) stats[k] = ee_kernel_stat{0, 0.0, 0.0, 0.0};
    if (per_layer)
        for (size_t k = 0; k < ctx->plans.size(); ++k) per_layer[k] = ee_kernel_stat{0, 0.0, 0.0, 0.0};
    for (size_t i = 0; i < ctx->prof_used; ++i) {
        const ProfRec& r = ctx->prof[i];
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) continue;
        stats[r.cls].launches++;
        stats[r.cls].ms += ms;
        stats[r.cls].ops += r.ops;
        stats[r.cls].bytes += r.bytes;
        if (per_layer && r.op >= 0) {
            per_layer[r.op].launches++;
            per_layer[r.op].ms += ms;
            per_layer[r.op].ops += r.ops;
            per_layer[r.op].bytes += r.bytes;
        }
    }
    ctx->prof_used = 0;
    return EE_OK;
}
