// Decoding and validation of the network blob (host only).
//
// Layout (little endian): 128-byte header, stage records (32 B), op records (112 B), exit records
// (64 B), then the weight / bias tensors.  Tensor ids are local to a stage: 0 is the stage input; an op
// writes a new tensor, or a channel slice of a concatenation tensor that other ops fill as well.
#include <cstring>
#include <utility>

#include "ee_internal.hpp"

namespace ee {
namespace {

template <typename T>
T rd(const unsigned char* p) { T v; std::memcpy(&v, p, sizeof(T)); return v; }

struct Cursor {
    const unsigned char* p;
    template <typename T> T next() { T v = rd<T>(p); p += sizeof(T); return v; }
};

}  // namespace

int parse_blob(const void* blob, size_t bytes, NetDesc* out)
{
    if (!blob || bytes < 128) return EE_ERR_ARG;
    const unsigned char* base = static_cast<const unsigned char*>(blob);
    if (std::memcmp(base, "EENETv2\0", 8) != 0) return EE_ERR_ARG;
    Cursor h{base + 8};
    const int version = h.next<int32_t>();
    NetDesc net;
    net.dtype = h.next<int32_t>();
    const int n_stages = h.next<int32_t>(), n_ops = h.next<int32_t>();
    net.in_h = h.next<int32_t>(); net.in_w = h.next<int32_t>(); net.in_c = h.next<int32_t>();
    net.n_classes = h.next<int32_t>();
    const int64_t stages_off = h.next<int64_t>(), ops_off = h.next<int64_t>(), exits_off = h.next<int64_t>();
    const int64_t data_off = h.next<int64_t>(), total = h.next<int64_t>();
    if (version != 2) return EE_ERR_ARG;
    if (net.dtype != EE_I8 && net.dtype != EE_BF16) return EE_ERR_UNSUPPORTED;
    if (n_stages < 1 || n_stages > 8 || n_ops < 0 || n_ops > 4096 || total < 0 || (size_t)total > bytes) return EE_ERR_ARG;
    if (stages_off < 128 || ops_off < stages_off + 32ll * n_stages || exits_off < ops_off + 112ll * n_ops ||
        data_off < exits_off + 64ll * n_stages || (size_t)data_off > bytes)
        return EE_ERR_ARG;
    if (net.in_h <= 0 || net.in_w <= 0 || net.in_c <= 0 || net.n_classes <= 0) return EE_ERR_SHAPE;
    const int es = net.elem_bytes();

    net.ops.resize(n_ops);
    for (int i = 0; i < n_ops; ++i) {
        Cursor c{base + ops_off + 112ll * i};
        OpDesc& o = net.ops[i];
        o.kind = c.next<int32_t>(); o.src = c.next<int32_t>(); o.dst = c.next<int32_t>(); o.res = c.next<int32_t>();
        o.h_in = c.next<int32_t>(); o.w_in = c.next<int32_t>(); o.c_in = c.next<int32_t>();
        o.h_out = c.next<int32_t>(); o.w_out = c.next<int32_t>(); o.c_out = c.next<int32_t>();
        o.kh = c.next<int32_t>(); o.kw = c.next<int32_t>(); o.stride = c.next<int32_t>(); o.pad = c.next<int32_t>();
        o.shift = c.next<int32_t>(); o.res_shift = c.next<int32_t>(); o.lo = c.next<int32_t>(); o.hi = c.next<int32_t>();
        o.f_lo = c.next<float>(); o.f_hi = c.next<float>();
        o.w_off = c.next<int64_t>(); o.b_off = c.next<int64_t>();
        o.pad_w = c.next<int32_t>(); o.c_off = c.next<int32_t>(); o.c_tot = c.next<int32_t>();
    }
    net.stages.resize(n_stages);
    net.exits.resize(n_stages);
    int prev_h = net.in_h, prev_w = net.in_w, prev_c = net.in_c;
    for (int s = 0; s < n_stages; ++s) {
        Cursor c{base + stages_off + 32ll * s};
        StageDesc& st = net.stages[s];
        st.first_op = c.next<int32_t>(); st.n_ops = c.next<int32_t>(); st.n_tensors = c.next<int32_t>();
        st.out_tensor = c.next<int32_t>();
        st.out_h = c.next<int32_t>(); st.out_w = c.next<int32_t>(); st.out_c = c.next<int32_t>();
        st.in_h = prev_h; st.in_w = prev_w; st.in_c = prev_c;
        if (st.first_op < 0 || st.n_ops < 0 || st.first_op + st.n_ops > n_ops || st.n_tensors < 1 || st.n_tensors > 256)
            return EE_ERR_SHAPE;
        // walk the ops and make sure every tensor shape chains: a tensor is read only after it has been written
        // completely, and is written once, or slice by slice along its channels
        std::vector<int> th(st.n_tensors), tw(st.n_tensors), tc(st.n_tensors), filled(st.n_tensors, 0);
        std::vector<std::vector<std::pair<int, int>>> slices(st.n_tensors);      // (first channel, count) written so far
        th[0] = prev_h; tw[0] = prev_w; tc[0] = prev_c; filled[0] = prev_c;
        for (int k = 0; k < st.n_ops; ++k) {
            const OpDesc& o = net.ops[st.first_op + k];
            if (o.kind < OP_CONV || o.kind > OP_AVGPOOL) return EE_ERR_UNSUPPORTED;
            if (o.src < 0 || o.src >= st.n_tensors || o.dst < 1 || o.dst >= st.n_tensors || o.dst == o.src) return EE_ERR_SHAPE;
            if (filled[o.src] == 0 || filled[o.src] != tc[o.src]) return EE_ERR_SHAPE;
            if (o.h_in != th[o.src] || o.w_in != tw[o.src] || o.c_in != tc[o.src]) return EE_ERR_SHAPE;
            if (o.kh < 1 || o.kw < 1 || o.stride < 1 || o.pad < 0 || o.pad_w < 0 || o.kh > 15 || o.kw > 15) return EE_ERR_SHAPE;
            const int ho = (o.h_in + 2 * o.pad - o.kh) / o.stride + 1, wo = (o.w_in + 2 * o.pad_w - o.kw) / o.stride + 1;
            if (ho < 1 || wo < 1 || o.h_out != ho || o.w_out != wo || o.c_out < 1) return EE_ERR_SHAPE;
            if (o.kind != OP_CONV && (o.c_out != o.c_in || o.pad != o.pad_w || o.kh != o.kw)) return EE_ERR_SHAPE;
            if ((o.kind == OP_MAXPOOL || o.kind == OP_AVGPOOL) && o.pad >= o.kh) return EE_ERR_SHAPE;
            if (o.c_off < 0 || o.c_tot < o.c_off + o.c_out) return EE_ERR_SHAPE;
            if (filled[o.dst] == 0) { th[o.dst] = ho; tw[o.dst] = wo; tc[o.dst] = o.c_tot; }
            else if (th[o.dst] != ho || tw[o.dst] != wo || tc[o.dst] != o.c_tot || o.c_tot == o.c_out) return EE_ERR_SHAPE;
            for (const auto& sl : slices[o.dst])                                     // slices of one tensor must not overlap
                if (o.c_off < sl.first + sl.second && sl.first < o.c_off + o.c_out) return EE_ERR_SHAPE;
            slices[o.dst].emplace_back(o.c_off, o.c_out);
            filled[o.dst] += o.c_out;
            if (filled[o.dst] > o.c_tot) return EE_ERR_SHAPE;
            if (o.res >= 0) {
                if (o.kind != OP_CONV || o.res >= st.n_tensors || o.c_tot != o.c_out || filled[o.res] == 0 || filled[o.res] != tc[o.res]) return EE_ERR_SHAPE;
                if (th[o.res] != ho || tw[o.res] != wo || tc[o.res] != o.c_out) return EE_ERR_SHAPE;
            }
            if (net.dtype == EE_I8 && (o.shift < 0 || o.shift > 30 || o.res_shift < 0 || o.res_shift > 23 || o.lo < -128 || o.hi > 127 || o.lo > o.hi))
                return EE_ERR_SHAPE;
            if (o.kind == OP_CONV || o.kind == OP_DWCONV) {
                const int64_t nw = (int64_t)o.c_out * o.kh * o.kw * (o.kind == OP_DWCONV ? 1 : o.c_in);
                if (o.w_off < data_off || (size_t)(o.w_off + nw * es) > bytes) return EE_ERR_SHAPE;
                if (o.b_off < data_off || (size_t)(o.b_off + 4ll * o.c_out) > bytes) return EE_ERR_SHAPE;
            }
        }
        for (int t = 0; t < st.n_tensors; ++t)                       // every tensor of the stage is written completely
            if (filled[t] == 0 || filled[t] != tc[t]) return EE_ERR_SHAPE;
        if (st.out_tensor < 0 || st.out_tensor >= st.n_tensors) return EE_ERR_SHAPE;
        if (th[st.out_tensor] != st.out_h || tw[st.out_tensor] != st.out_w || tc[st.out_tensor] != st.out_c) return EE_ERR_SHAPE;
        Cursor e{base + exits_off + 64ll * s};
        ExitDesc& ex = net.exits[s];
        ex.h = e.next<int32_t>(); ex.w = e.next<int32_t>(); ex.c = e.next<int32_t>(); ex.n_cls = e.next<int32_t>();
        ex.gap_shift = e.next<int32_t>(); ex.frac_bits = e.next<int32_t>();
        ex.logit_scale = e.next<float>(); ex.thr = e.next<float>();
        ex.w_off = e.next<int64_t>(); ex.b_off = e.next<int64_t>();
        if (ex.h != st.out_h || ex.w != st.out_w || ex.c != st.out_c || ex.n_cls != net.n_classes) return EE_ERR_SHAPE;
        if (ex.gap_shift < 0 || ex.gap_shift > 30 || ex.frac_bits < 0 || ex.frac_bits > 30) return EE_ERR_SHAPE;
        if (ex.w_off < data_off || (size_t)(ex.w_off + (int64_t)ex.n_cls * ex.c * es) > bytes) return EE_ERR_SHAPE;
        if (ex.b_off < data_off || (size_t)(ex.b_off + 4ll * ex.n_cls) > bytes) return EE_ERR_SHAPE;
        prev_h = st.out_h; prev_w = st.out_w; prev_c = st.out_c;
    }
    if (out) *out = std::move(net);
    return EE_OK;
}

}  // namespace ee
