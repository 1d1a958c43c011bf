// Bottleneck block (int8) of the 56 x 56 group of ResNet-50-style networks in one launch, for gfx950:
// 1x1 reduction (64 or 256 -> 64 channels) -> 3x3 convolution (64 -> 64, stride 1) -> 1x1 expansion (64 -> 256) + residual.
// Layer by layer the block moves its 256-channel input twice (as the first layer's input and as the residual) and the two
// 64-channel tensors in between twice each; here the input is read once for the convolutions, the residual comes out of the
// cache the input just went through, and the tensors in between only ever exist in LDS.
//
// One workgroup of eight wavefronts per CU walks over tiles of 8 x 8 output pixels (persistent: the weights of all three
// layers, 68 KB, are loaded once per wavefront and stay in registers as ready matrix-instruction operands).  The wavefronts
// have two roles, and every SIMD holds one of each, so that the matrix cores of a SIMD see the sum of both.  Per tile there
// are two halves with a workgroup barrier behind each:
//   first half   front (wavefronts 0-3), one tile ahead: the 10 x 10 input pixels under tile i + 1 (staged in LDS one
//                iteration before) go through the first layer, 32 pixels per wavefront, both blocks of 32 output channels
//                per staged operand; results are requantised and written to LDS as the second layer's input (pixels outside
//                the image as zeros: the second layer pads its input).  Before that the wavefront writes the pixels of tile
//                i + 2, which it requested one iteration ago, to LDS and requests those of tile i + 3.
//                back (wavefronts 4-7), on tile i: (pixel block of 8 x 4, half of the 64 middle channels) per wavefront: nine
//                taps x two reduction steps of the 3x3 layer, requantisation, the result to LDS;
//   second half  all eight wavefronts: the last layer of tile i, (pixel block, two of the eight blocks of 32 output channels)
//                each: bias, residual (requested in the first half), requantisation, 16-byte stores.
// All sums are int32 and exact, rounding points are those of the three separate layers: results are equal bit for bit.
#include "ee_internal.hpp"
#include "ir_device.hpp"

namespace ee {

struct BnTile {
    int tiles_x, tiles_y;      // tiles of 8 x 8 output pixels per image
    int total;                 // tiles in all
    int per_xcd, nslots;       // tiles per XCD (a contiguous run), workgroups per XCD
    int xp, x_bytes;           // bytes per staged input pixel, per buffer of staged pixels
    int gap_rows;              // pooling: rows of 256 channel sums in LDS, one per tile of a workgroup
};

constexpr int BN_M1_PX = 80;                     // second layer's input in LDS: 64 bytes per pixel + 16
constexpr int BN_M1_ROW = 10 * BN_M1_PX + 96;    // ten pixels per row; rows half a bank cycle apart
constexpr int BN_M1_BYTES = 10 * BN_M1_ROW;
constexpr int BN_BIAS_BYTES = 4 * (64 + 64 + 256);
constexpr int BN_M2_BYTES = 4 * 1024;            // requantised second-layer outputs [pixel block][channel half][lane][16]
constexpr int BN_SLOT_BYTES = 2 * EE_ZC_MAX_B;   // the output slot of every sample

// K1: reduction steps of the first layer, c_in / 32; RES: the last layer adds a residual; GAP: the per-sample channel sums of the
// output are also added into a.gap_sums (the exit head's pooling); SC: the residual is a 1x1 convolution of the block's input
// (64 -> 256 channels, the shortcut of a group's first block), computed here from the staged pixels and requantised as that layer
// would have written it (a third buffer keeps a tile's pixels until its last layer has run)
template <int K1, bool RES, bool GAP, bool SC>
__global__ __launch_bounds__(512, 1) __attribute__((amdgpu_waves_per_eu(2, 2))) void bneck_block_i8_kernel(IrArgs a, BnTile t)
{
    constexpr int CIN = 32 * K1, CPP = 2 * K1;                         // 16-byte chunks per input pixel
    constexpr int NCH = 100 * CPP, NL = (NCH + 511) / 512;             // chunks per tile, loads per lane (all eight wavefronts stage)
    constexpr int NXB = SC ? 3 : 2;                                    // buffers of staged pixels
    static_assert(!SC || (K1 == 2 && RES), "the shortcut convolution reads 64 channels and is the residual");
    extern __shared__ __attribute__((aligned(16))) unsigned char bn_lds[];
    const int tid = threadIdx.x, lane = tid & 63, m = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool front = wave < 4;
    const int xcd = (int)(blockIdx.x & 7), slot = (int)(blockIdx.x >> 3);
    const int cnt = min(t.per_xcd, t.total - xcd * t.per_xcd);         // tiles of this XCD
    if (cnt <= slot) return;                                           // whole workgroup: no barrier is skipped by a part of it
    const int T = (cnt - slot + t.nslots - 1) / t.nslots;              // tiles of this workgroup: u0, u0 + nslots, ...
    const int u0 = xcd * t.per_xcd + slot;
    const int tpi = t.tiles_x * t.tiles_y;
    int* const l_b1 = (int*)bn_lds;
    int* const l_b2 = l_b1 + 64;
    int* const l_b3 = l_b1 + 128;
    unsigned char* const l_x = bn_lds + BN_BIAS_BYTES;                  // two buffers of staged input pixels
    unsigned char* const l_m1 = l_x + NXB * t.x_bytes;                  // two buffers of second-layer input
    unsigned char* const l_m2 = l_m1 + 2 * BN_M1_BYTES;
    const unsigned short* const l_slot = (const unsigned short*)(l_m2 + BN_M2_BYTES);
    int* const l_bs = (int*)(l_m2 + BN_M2_BYTES + BN_SLOT_BYTES);       // shortcut bias (SC)
    const IrClamp cl_s = ir_clamp(a.sh_s, a.lo_s, a.hi_s);
    const IrClamp cl1 = ir_clamp(a.sh_e, a.lo_e, a.hi_e), cl2 = ir_clamp(a.sh_d, a.lo_d, a.hi_d), cl3 = ir_clamp(a.sh_p, a.lo_p, a.hi_p);

    if (tid < 64) { l_b1[tid] = a.be[tid]; l_b2[tid] = a.bd[tid]; }
    if (tid < 256) l_b3[tid] = a.bp[tid];
    if constexpr (SC) { if (tid < 256) l_bs[tid] = a.bs[tid]; }
    if (a.ys && tid < a.B) ((unsigned short*)l_slot)[tid] = a.ys[tid];   // B <= EE_ZC_MAX_B <= 512 with a slot table: checked by the launcher
    // pooling (GAP): a tile's channel sums are gathered in LDS, a row of 256 per tile of this workgroup, and added to a.gap_sums
    // when the last tile is through: the global atomics then sit behind the loop, where no wait of the loop (for staged pixels
    // or residuals) has them in front of it
    int* const l_gap = l_bs + (SC ? 256 : 0);
    int* const l_gap_n = l_gap + 256 * t.gap_rows;                      // the sample of every row
    if constexpr (GAP) {
        for (int i = tid; i < 256 * t.gap_rows; i += 512) l_gap[i] = 0;
    }

    // A workgroup's tiles are nslots apart: a tile's (sample, tile row, tile column) follows from the one before by additions
    // (the divisions are done once).
    struct Cursor { int n, ty, tx; };
    const int step_n = t.nslots / tpi, step_r = t.nslots - step_n * tpi, step_ty = step_r / t.tiles_x, step_tx = step_r - step_ty * t.tiles_x;
    auto advance = [&](Cursor& c) {
        c.tx += step_tx;
        if (c.tx >= t.tiles_x) { c.tx -= t.tiles_x; ++c.ty; }
        c.ty += step_ty;
        if (c.ty >= t.tiles_y) { c.ty -= t.tiles_y; ++c.n; }
        c.n += step_n;
    };
    Cursor first;
    first.n = u0 / tpi;
    first.ty = (u0 - first.n * tpi) / t.tiles_x;
    first.tx = u0 - first.n * tpi - first.ty * t.tiles_x;
    auto bias16 = [&](const int* lb, int blk) {                         // a block's bias in the accumulator layout
        v16i_r acc;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const v4i_r b4 = *(const v4i_r*)(lb + blk * 32 + 8 * q + 4 * hi);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[4 * q + e] = b4[e];
        }
        return acc;
    };

    // ---- the last layer, shared out: a wavefront of either role takes (pixel block, half of the output channels), the back
    //      role blocks 0-1 of the half's four blocks of 32 channels, the front role blocks 2-3 ------------------------------
    const int pb = wave & 1, half = (wave >> 1) & 1;
    const int cb0 = 4 * half + (front ? 2 : 0);                         // first of this wavefront's two output blocks
    const int ty = m >> 3, tx = m & 7;
    v4i_r w3[2][2], rr[2];                                              // operands [block][step]; the residual of the lane's pixel, 16 channels per block
    v4i_r wsc[SC ? 2 : 1][2];                                           // the shortcut's operands [block][step]
    if constexpr (SC) {
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int k = 0; k < 2; ++k) wsc[c][k] = *(const v4i_r*)((const unsigned char*)a.ws + ((size_t)((cb0 + c) * 2 + k) * 64 + lane) * 16);
    }
    const int xc_off = ((4 * pb + ty + 1) * 10 + tx + 1) * t.xp + 16 * hi;   // the lane's output pixel among the staged ones
    int xb_out = NXB - 1, xb_l1 = 0, xb_st = 1;                         // buffers of tile it, it + 1, it + 2 (it = -1 at first)
    auto next_buffers = [&] {
        xb_out = xb_out + 1 == NXB ? 0 : xb_out + 1;
        xb_l1 = xb_l1 + 1 == NXB ? 0 : xb_l1 + 1;
        xb_st = xb_st + 1 == NXB ? 0 : xb_st + 1;
    };
    unsigned pix_y = 0;
    bool px_ok = false;
    int gap_n = 0, gap_row = -1;                                        // the sample of the tile in hand, its row of sums
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int k = 0; k < 2; ++k) w3[c][k] = *(const v4i_r*)((const unsigned char*)a.wp + ((size_t)((cb0 + c) * 2 + k) * 64 + lane) * 16);
    auto out_pixel = [&](const Cursor& cu) {                            // where the lane's pixel of that tile goes; its residual is requested
        const int n = cu.n;
        gap_n = n;
        ++gap_row;
        const int oy = 8 * cu.ty + 4 * pb + ty, ox = 8 * cu.tx + tx;
        px_ok = oy < a.H && ox < a.W;
        const int sp = px_ok ? (oy * a.W + ox) * 256 + cb0 * 32 + 16 * hi : 0;                  // < 2^31 with the sample: checked by the launcher
        const int slot_n = a.ys ? (int)l_slot[n] : n;                   // from LDS: a global load here would sit in front of every later wait
        pix_y = (unsigned)(slot_n * a.H * a.W * 256 + sp);
        if constexpr (RES && !SC) {
            const unsigned char* rp = (const unsigned char*)a.res + (unsigned)(n * a.H * a.W * 256 + sp);
            rr[0] = *(const v4i_r*)rp;                                  // unconditional and in range
            rr[1] = *(const v4i_r*)(rp + 32);
        }
        __builtin_amdgcn_sched_barrier(0);                              // requested here, not where the compiler finds its first use
    };
    // pooling: one more matrix instruction with the packed outputs as the A operand (rows = pixels, reduction = channels) and
    // the identity as B transposes the block: lane (channel, hi) then holds that channel's values of 16 pixels as integers
    v4i_r ident = v4i_r{0, 0, 0, 0};
    if constexpr (GAP) {
#pragma unroll
        for (int j = 0; j < 4; ++j) ident[j] = (m >> 2) == 4 * hi + j ? 1 << (8 * (m & 3)) : 0;
    }
    auto last_layer = [&](const v4i_r& d0, const v4i_r& d1) {           // the two reduction steps: channels 0-31 and 32-63 of the lane's pixel block
        __builtin_amdgcn_sched_barrier(0);                              // nothing of this moves into the first half
        if constexpr (SC) {
            const unsigned char* xc = l_x + xb_out * t.x_bytes + xc_off;
            const v4i_r x0 = *(const v4i_r*)xc, x1 = *(const v4i_r*)(xc + 32);
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                v16i_r acc = bias16(l_bs, cb0 + c);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wsc[c][0], x0, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wsc[c][1], x1, acc, 0, 0, 0);
                rr[c] = ir_requant_pack(acc, cl_s);                     // 16 channels per lane in pixel order: what the layer would have stored
            }
        }
        v4i_r out[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            v16i_r acc = bias16(l_b3, cb0 + c);
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w3[c][0], d0, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(w3[c][1], d1, acc, 0, 0, 0);
            if constexpr (RES) {
                // the residual in the store layout, then back into the accumulator layout
                const auto s02 = __builtin_amdgcn_permlane32_swap((unsigned)rr[c][0], (unsigned)rr[c][1], false, false);
                const auto s13 = __builtin_amdgcn_permlane32_swap((unsigned)rr[c][2], (unsigned)rr[c][3], false, false);
                const unsigned rq[4] = {s02[0], s13[0], s02[1], s13[1]};
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[4 * q + e] += __builtin_amdgcn_sbfe((int)rq[q], 8 * e, 8) << a.res_shift;
                out[c] = ir_requant_pack<false>(acc, cl3);              // every accumulator has been through an addition
            } else {
                out[c] = ir_requant_pack(acc, cl3);
            }
        }
        if (px_ok) {
            *(v4i_r*)((unsigned char*)a.y + pix_y) = out[0];
            *(v4i_r*)((unsigned char*)a.y + pix_y + 32) = out[1];
        }
        if constexpr (GAP) {
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const v4i_r o = px_ok ? out[c] : v4i_r{0, 0, 0, 0};     // pixels outside the image count nothing
                v16i_r tr;
#pragma unroll
                for (int i = 0; i < 16; ++i) tr[i] = 0;
                tr = __builtin_amdgcn_mfma_i32_32x32x32_i8(o, ident, tr, 0, 0, 0);
                int sum = 0;
#pragma unroll
                for (int i = 0; i < 16; ++i) sum += tr[i];
                const auto both = __builtin_amdgcn_permlane32_swap((unsigned)sum, (unsigned)sum, false, false);   // the other 16 pixels
                sum = (int)(both[0] + both[1]);
                // integer sums: exact in any order
                if (hi == 0) __hip_atomic_fetch_add((__attribute__((address_space(3))) int*)l_gap + gap_row * 256 + (cb0 + c) * 32 + m, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            if (tid == 0) l_gap_n[gap_row] = gap_n;
        }
    };

    // ---- this lane's chunks of a staged tile: offsets from the tile's first pixel, -------------------------------------
    v4i_r st[NL];                                                   // the loaded chunks
    int lrel[NL], lpyx[NL];                                         // global byte offset from the tile's pixel (0, 0); staged row | column << 8
    unsigned ldst[NL];                                              // LDS byte offset of the chunk, ~0u: none
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int e0 = 512 * i + tid, e = min(e0, NCH - 1), q = e / CPP, ch = e - q * CPP, py = q / 10, px = q - 10 * py;
        lrel[i] = ((py - 1) * a.W + (px - 1)) * CIN + 16 * ch;
        lpyx[i] = py | px << 8;
        ldst[i] = e0 < NCH ? (unsigned)(q * t.xp + 16 * ch) : ~0u;
    }
    auto x_load = [&](const Cursor& cu) {                           // unconditional and in range: a pixel outside the image reads the image's first one
        const int n = cu.n, oy0 = 8 * cu.ty, ox0 = 8 * cu.tx;
        const unsigned char* x = (const unsigned char*)a.x + (size_t)n * a.H * a.W * CIN;
        const int base = (oy0 * a.W + ox0) * CIN;
        // staged rows y_first .. y_last and columns x_first .. x_last lie inside the image
        const int y_first = oy0 == 0 ? 1 : 0, y_last = min(9, a.H - oy0), x_first = ox0 == 0 ? 1 : 0, x_last = min(9, a.W - ox0);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int py = lpyx[i] & 255, px = lpyx[i] >> 8;
            const bool ok = (unsigned)(py - y_first) <= (unsigned)(y_last - y_first) && (unsigned)(px - x_first) <= (unsigned)(x_last - x_first);
            st[i] = *(const v4i_r*)(x + (ok ? (unsigned)(base + lrel[i]) : 0u));
        }
    };
    auto x_store = [&](unsigned char* xb) {
#pragma unroll
        for (int i = 0; i < NL; ++i)
            if (512 * (i + 1) <= NCH || ldst[i] != ~0u) *(v4i_r*)(xb + ldst[i]) = st[i];     // only the last chunk may be missing
    };
    // ---- prologue: the role's weights (front: the first layer's operands [block][step]; back: [tap][step] of the 3x3 layer for
    //      this half's 32 middle channels), requested in front of the first tile's pixels so that one wait covers both ---------
    constexpr int NWR = 2 * K1 > 18 ? 2 * K1 : 18;
    v4i_r wr[NWR];
    if (front) {
#pragma unroll
        for (int k = 0; k < 2 * K1; ++k) wr[k] = *(const v4i_r*)((const unsigned char*)a.we + ((size_t)k * 64 + lane) * 16);
    } else {
#pragma unroll
        for (int k = 0; k < 18; ++k) wr[k] = *(const v4i_r*)((const unsigned char*)a.wd + ((size_t)(half * 18 + k) * 64 + lane) * 16);
    }
    Cursor c_ld = first;                                                // the tile whose pixels are requested next
    x_load(c_ld);
    advance(c_ld);
    x_store(l_x);
    // every weight has arrived before the loops, so that nothing inside them waits for a weight by count
#pragma unroll
    for (int k = 0; k < NWR; ++k)
        if (k < 18 || front) asm volatile("" : "+v"(wr[k]));
#pragma unroll
    for (int k = 0; k < 4; ++k) asm volatile("" : "+v"(w3[k >> 1][k & 1]));
    if constexpr (SC) {
#pragma unroll
        for (int k = 0; k < 4; ++k) asm volatile("" : "+v"(wsc[k >> 1][k & 1]));
    }
    if (1 < T) x_load(c_ld);                                            // in flight over the first iteration
    advance(c_ld);
    // per iteration: tile it + 2, requested one iteration ago, goes into the buffer the first layer read one iteration ago
    // (tile it's); then the next request, in flight over a whole iteration
    // (the requests go out behind the wavefront's matrix instructions of the first half, whose results take a while anyway:
    // at the top of the half all eight wavefronts would queue up at the memory pipeline with nothing else to issue)
    auto stage_write = [&](int it) {
        if (it + 2 < T) x_store(l_x + xb_st * t.x_bytes);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto stage_request = [&](int it) {
        __builtin_amdgcn_sched_barrier(0);
        if (it + 3 < T) x_load(c_ld);
        advance(c_ld);
        __builtin_amdgcn_sched_barrier(0);
    };

    // Each role has its own loop (a wavefront has one role for good, and the registers that live over a loop are the role's
    // own); both loops run the same iterations with the same two barriers, so the workgroup's barriers pair up.
    if (front) {
        const int hp = 32 * wave + m, hpc = min(hp, 99), hy = hpc / 10, hx = hpc - 10 * hy;
        const int xoff = hpc * t.xp + 16 * hi, m1off = hy * BN_M1_ROW + hx * BN_M1_PX + 16 * hi;
        Cursor c_out = first, c_l1 = first;                             // the tiles of the last layer, of the first layer
        __syncthreads();                                                // biases and the first tile's pixels are in LDS
        for (int it = -1; it < T; ++it) {
            stage_write(it);
            if (it >= 0) { out_pixel(c_out); advance(c_out); }
            if (it + 1 < T) {
                const int oy0 = 8 * c_l1.ty, ox0 = 8 * c_l1.tx;
                advance(c_l1);
                const bool in_img = hp < 100 && (unsigned)(oy0 - 1 + hy) < (unsigned)a.H && (unsigned)(ox0 - 1 + hx) < (unsigned)a.W;
                const unsigned char* xb = l_x + xb_l1 * t.x_bytes + xoff;
                unsigned char* m1 = l_m1 + ((it + 1) & 1) * BN_M1_BYTES + m1off;
                v16i_r acc0 = bias16(l_b1, 0), acc1 = bias16(l_b1, 1);
                v4i_r b[K1];                                            // every operand requested before the first is used
#pragma unroll
                for (int k = 0; k < K1; ++k) b[k] = *(const v4i_r*)(xb + 32 * k);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int k = 0; k < K1; ++k) {
                    acc0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(wr[k], b[k], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(wr[K1 + k], b[k], acc1, 0, 0, 0);
                }
                stage_request(it);
                v4i_r o0 = ir_requant_pack(acc0, cl1), o1 = ir_requant_pack(acc1, cl1);
                if (!in_img) { o0 = v4i_r{0, 0, 0, 0}; o1 = v4i_r{0, 0, 0, 0}; }
                if (hp < 100) {
                    *(v4i_r*)m1 = o0;
                    *(v4i_r*)(m1 + 32) = o1;
                }
            }
            __syncthreads();                                            // the halves of the second layer's output are in LDS
            if (it >= 0) last_layer(*(const v4i_r*)(l_m2 + ((pb * 2 + 0) * 64 + lane) * 16), *(const v4i_r*)(l_m2 + ((pb * 2 + 1) * 64 + lane) * 16));
            next_buffers();
            __syncthreads();                                            // tile it + 1 is through the first layer, tile it + 2 is staged
        }
    } else {
        const int woff = (pb * 4 + ty) * BN_M1_ROW + tx * BN_M1_PX + 16 * hi;
        __syncthreads();                                                // biases and the first tile's pixels are in LDS
        Cursor c_out = first;
        for (int it = -1; it < T; ++it) {
            stage_write(it);
            v4i_r dq = v4i_r{0, 0, 0, 0};
            if (it < 0) stage_request(it);
            if (it >= 0) {
            out_pixel(c_out);
            advance(c_out);
            v16i_r acc = bias16(l_b2, half);
            const unsigned char* win = l_m1 + (it & 1) * BN_M1_BYTES + woff;
            // the eighteen operands in three batches of six through two sets of registers: the third batch is requested when the
            // first has been used, behind the matrix instructions of the second
            auto tap = [&](int k) { return *(const v4i_r*)(win + (k / 6) * BN_M1_ROW + ((k / 2) % 3) * BN_M1_PX + (k & 1) * 32); };
            v4i_r b0[6], b1[6];
#pragma unroll
            for (int k = 0; k < 6; ++k) b0[k] = tap(k);
#pragma unroll
            for (int k = 0; k < 6; ++k) b1[k] = tap(6 + k);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 6; ++k) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wr[k], b0[k], acc, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 6; ++k) b0[k] = tap(12 + k);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 6; ++k) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wr[6 + k], b1[k], acc, 0, 0, 0);
#pragma unroll
            for (int k = 0; k < 6; ++k) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wr[12 + k], b0[k], acc, 0, 0, 0);
            stage_request(it);
            dq = ir_requant_pack(acc, cl2);
            *(v4i_r*)(l_m2 + ((pb * 2 + half) * 64 + lane) * 16) = dq;
            }
            __syncthreads();                                            // the halves of the second layer's output are in LDS
            if (it >= 0) {
                const v4i_r other = *(const v4i_r*)(l_m2 + ((pb * 2 + (half ^ 1)) * 64 + lane) * 16);
                last_layer(half ? other : dq, half ? dq : other);
            }
            next_buffers();
            __syncthreads();
        }
    }
    if constexpr (GAP) {                                                // every row is complete behind the loop's last barrier
        for (int i = tid; i < 256 * T; i += 512) atomicAdd(a.gap_sums + (size_t)l_gap_n[i >> 8] * 256 + (i & 255), l_gap[i]);
    }
}

// Shapes the kernel covers, and its tiling.
static bool bneck_block_plan(const IrArgs& a, BnTile& t)
{
    if (a.stride != 1 || a.pad != 1 || a.B < 1 || a.Ho != a.H || a.Wo != a.W || a.H < 1 || a.W < 1) return false;
    if ((a.Cin != 64 && a.Cin != 256) || a.Kx != a.Cin || a.Ce32 != 64 || a.Cout != 256) return false;
    if ((double)a.B * a.H * a.W * 256 >= 2147483648.0 || (a.ys && a.B > EE_ZC_MAX_B)) return false;
    t.tiles_x = (a.W + 7) / 8;
    t.tiles_y = (a.H + 7) / 8;
    const long long total = (long long)a.B * t.tiles_x * t.tiles_y;
    if (total > 0x3fffffff) return false;
    t.total = (int)total;
    t.per_xcd = (t.total + 7) / 8;
    t.nslots = t.per_xcd < 32 ? t.per_xcd : 32;                         // one workgroup per CU at most: 32 CUs per XCD
    t.xp = a.Cin + 16;
    t.x_bytes = 100 * t.xp + 64;
    t.gap_rows = (t.per_xcd + t.nslots - 1) / t.nslots;                  // the most tiles a workgroup has
    return true;
}

// LDS of a launch; 0: the rows of channel sums of a pooling launch do not fit
static size_t bneck_lds_bytes(const BnTile& t, bool sc, bool gap)
{
    size_t lds = (size_t)BN_BIAS_BYTES + (sc ? 3 : 2) * (size_t)t.x_bytes + 2 * BN_M1_BYTES + BN_M2_BYTES + BN_SLOT_BYTES + (sc ? 1024 : 0);
    if (gap) lds += (size_t)t.gap_rows * (1024 + 4);
    return lds <= 160 * 1024 ? lds : 0;
}

bool bneck_block_supported(const IrArgs& a)
{
    BnTile t;
    return bneck_block_plan(a, t);
}

bool bneck_block_pools(const IrArgs& a)
{
    BnTile t;
    return bneck_block_plan(a, t) && (a.res || a.ws) && bneck_lds_bytes(t, a.ws != nullptr, true) != 0;
}

template <int K1, bool RES, bool GAP, bool SC = false>
static hipError_t bneck_launch(const IrArgs& a, const BnTile& t, hipStream_t s)
{
    static const hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void*>(&bneck_block_i8_kernel<K1, RES, GAP, SC>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (granted != hipSuccess) return granted;
    const size_t lds = bneck_lds_bytes(t, SC, GAP);
    if (lds == 0) return hipErrorInvalidValue;                          // bneck_block_pools says so beforehand
    EE_LAUNCH((bneck_block_i8_kernel<K1, RES, GAP, SC>), dim3((unsigned)(8 * t.nslots)), dim3(512), lds, s, a, t);
    return hipGetLastError();
}

hipError_t launch_bneck_block(const IrArgs& a, hipStream_t s)
{
    BnTile t;
    if (!bneck_block_plan(a, t)) return hipErrorInvalidValue;
    if (a.ws) {                                                         // the residual is the shortcut convolution of the block's input
        if (a.Cin != 64 || a.res) return hipErrorInvalidValue;
        return a.gap_sums ? bneck_launch<2, true, true, true>(a, t, s) : bneck_launch<2, true, false, true>(a, t, s);
    }
    if (a.gap_sums) {                                                   // the pooling variant is built with a residual only (the blocks that end a segment have one)
        if (!a.res) return hipErrorInvalidValue;
        return a.Cin == 64 ? bneck_launch<2, true, true>(a, t, s) : bneck_launch<8, true, true>(a, t, s);
    }
    if (a.res) return a.Cin == 64 ? bneck_launch<2, true, false>(a, t, s) : bneck_launch<8, true, false>(a, t, s);
    return a.Cin == 64 ? bneck_launch<2, false, false>(a, t, s) : bneck_launch<8, false, false>(a, t, s);
}

}  // namespace ee
