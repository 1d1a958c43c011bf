// Inverted-residual block (int8) in one launch, for gfx950: 1x1 expansion -> 3x3 depthwise -> 1x1 projection
// (+ residual), the block of MobileNetV2-style networks.  Run layer by layer, the expanded tensor (6 x the block's
// input) is written by the expansion, read and written by the depthwise layer and read by the projection; here it
// only ever exists in LDS, one group of 32 expanded channels at a time, and all three layers run on the matrix cores.
//
// A workgroup (4 wavefronts) owns a tile of output pixels of one image: blocks of 32 pixels (NBH rows x NBW columns,
// NBH * NBW <= 32), at most MAXB blocks per wavefront.
//   * The block's input pixels under the tile (with the one-pixel frame of the 3x3 window) are staged once in LDS,
//     8 bytes per lane and load, a pixel's channels followed by padding up to the reduction length (a multiple of 32)
//     plus 16 bytes (an odd number of 16-byte chunks per pixel spreads consecutive pixels over the banks).  Bytes behind
//     a pixel's channels are never written: the expansion weights are zero there.
//   * For every group g of 32 expanded channels:
//       expansion   E_g[pixel][32] = requant(W_e[g] . x[pixel] + b_e[g]) for the staged pixels inside the image
//                   (v_mfma_i32_32x32x32_i8, rows = channels, columns = 32 staged pixels, shared out over the
//                   wavefronts), written to one of two LDS buffers laid out like the tile (32 bytes per pixel, 16 bytes
//                   of padding per row); pixels outside the image are zero there from the start and stay zero: the
//                   depthwise layer pads its input, the *expanded* tensor, with zeros;
//       depthwise   per block of 32 output pixels nine matrix instructions, one per tap, whose A operand is the
//                   diagonal matrix diag(w_d[c][tap]) of the group's channels and whose B operand is the 32 channels of
//                   the tap's input pixels (one 16-byte LDS read per lane): a multiply-add per output and tap costs a
//                   thirty-second of the instruction, and it is still several times cheaper than byte transposes and
//                   dot products on the vector ALU;
//       projection  the requantised depthwise outputs of a block are, after one exchange between the two halves of
//                   the wavefront (v_permlane32_swap), exactly the B operand (32 reduction channels x 32 pixels) of
//                   the projection, whose accumulators (NCO blocks of 32 output channels per pixel block) stay in
//                   registers over all groups.
//     The expansion of group g + 1 runs behind the depthwise + projection of group g without a barrier in between
//     (other buffer); there is one workgroup barrier per group.
//   * Epilogue: projection bias, residual, requantisation, 16-byte stores.
// Small images (a tile is at most MAXB blocks and 96 staged pixels; few workgroups, many channel groups) run the second
// form, GP: the four or eight wavefronts of a workgroup share the tile's *channel groups* instead of its pixels.  Each wavefront
// expands, filters and projects every pixel of the tile for the groups g = wavefront, wavefront + 4 (or 8), ... through a buffer
// of its own, with no barrier inside the loop; the partial projection sums are added in LDS (integer adds,
// exact in any order) and the epilogue is shared out by (pixel block, output block).
// Every accumulation is int32 and exact, rounding points are those of the three separate layers: results are equal
// bit for bit.
#include "ee_internal.hpp"
#include "ir_device.hpp"

namespace ee {

struct IrTile {
    int nbw, nbh;          // a block of 32 output pixels: nbh rows x nbw columns
    int pbw, pbh;          // blocks per workgroup tile along x and y
    int tiles_x, tiles_y;
    int iw, ih;            // staged pixels under a tile
    int cpp;               // 8-byte chunks per input pixel
    unsigned magic_cpp, magic_iw;   // floor(2^32 / d) + 1: n / d for n < 2^16
    int xp;                // bytes per staged input pixel
    int x_bytes, e_bytes;  // LDS: staged input, one buffer of expanded pixels
    int per_xcd, total;    // workgroups per XCD, workgroups with work
    int gp;                // 4 or 8: that many wavefronts share the channel groups (small images), 0: four share the pixels
};

constexpr int IR_BATCH = 8, IR_BATCHES = 2;   // 8-byte loads per lane that stage a tile, in batches: ih * iw * cpp <= 4096
constexpr int IR_MAXCB = 3;                   // blocks of 32 staged pixels per wavefront in the expansion: ih * iw <= 384
constexpr int IR_FILL = 4;                    // 16-byte loads per lane that fill a buffer without expansion: ih * iw * 2 <= 1024
constexpr int IR_MAXK = 5;                    // reduction steps of 32 input channels: c_in <= 160 (template parameter MAXK: 1, 2 or 5)

// GP = 0: four wavefronts share the pixels; GP = 4 or 8: that many wavefronts share the channel groups.
// MAXK = 0: a block without expansion (depthwise -> projection): the buffers of "expanded" pixels are filled with the
// block's input itself, 32 channels at a time.
template <int STRIDE, int NCO, int MAXB, int MAXK, int GP>
__global__ __launch_bounds__(GP ? 64 * GP : 256, (NCO == 1 && !GP && MAXK <= 1) ? (MAXK == 1 ? 4 : 3) : 2) void ir_block_i8_kernel(IrArgs a, IrTile t)
{
    constexpr int NW = GP ? GP : 4, NT = 64 * NW;                      // wavefronts and lanes per workgroup
    constexpr bool EXP = MAXK > 0;
    extern __shared__ __attribute__((aligned(16))) unsigned char ir_lds[];
    const int tid = threadIdx.x, lane = tid & 63, m = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int u = (int)(blockIdx.x & 7) * t.per_xcd + (int)(blockIdx.x >> 3);
    if (u >= t.total) return;                                          // whole workgroup: no barrier is skipped by a part of it
    const int tx_i = u % t.tiles_x, ty_i = (u / t.tiles_x) % t.tiles_y, n = u / (t.tiles_x * t.tiles_y);
    const int ox0 = tx_i * t.pbw * t.nbw, oy0 = ty_i * t.pbh * t.nbh;
    const int ix0 = ox0 * STRIDE - a.pad, iy0 = oy0 * STRIDE - a.pad;
    unsigned char* const l_be = ir_lds;                                 // expansion bias, depthwise bias (int32 per expanded channel)
    unsigned char* const l_bd = ir_lds + 4 * a.Ce32;
    unsigned char* const l_x = ir_lds + 8 * a.Ce32;
    unsigned char* const l_e = l_x + t.x_bytes;
    const int e_row = t.iw * 32 + 16;                                   // bytes per row of expanded pixels
    const int kx32 = a.Kx >> 5;
    const IrClamp cl_e = ir_clamp(a.sh_e, a.lo_e, a.hi_e), cl_d = ir_clamp(a.sh_d, a.lo_d, a.hi_d), cl_p = ir_clamp(a.sh_p, a.lo_p, a.hi_p);

    // ---- stage the input pixels under the tile; clear the expanded-pixel buffers; biases to LDS ----------------------------
    {
        const unsigned char* x = (const unsigned char*)a.x + (size_t)n * a.H * a.W * a.Cin;
        const int nchunks = EXP ? t.ih * t.iw * t.cpp : 0;
        v2i_r stage[IR_BATCH];
        unsigned dst[IR_BATCH];                                         // LDS byte offset, ~0u: nothing to write
#pragma unroll
        for (int batch = 0; batch < IR_BATCHES; ++batch) {
            if (batch > 0 && NT * IR_BATCH * batch >= nchunks) break;   // wave-uniform
#pragma unroll
            for (int i = 0; i < IR_BATCH; ++i) {
                dst[i] = ~0u;
                stage[i] = v2i_r{0, 0};
                const int e0 = NT * (batch * IR_BATCH + i);
                if (e0 < nchunks) {                                     // wave-uniform
                    const int e = min(e0 + tid, nchunks - 1);
                    const int q = t.cpp == 1 ? e : (int)__umulhi((unsigned)e, t.magic_cpp), ch = e - q * t.cpp;   // 2^32 / 1 + 1 does not fit the magic number
                    const int py = (int)__umulhi((unsigned)q, t.magic_iw), px = q - py * t.iw;
                    const int iy = iy0 + py, ix = ix0 + px;
                    const bool ok = e0 + tid < nchunks && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
                    // the load is unconditional and in range (a chunk that is not wanted reads the image's first bytes)
                    stage[i] = *(const v2i_r*)(x + (ok ? (unsigned)((iy * a.W + ix) * a.Cin + 8 * ch) : 0u));
                    if (ok) dst[i] = (unsigned)(q * t.xp + 8 * ch);
                }
            }
            if (batch == 0) {
                // the buffers of expanded pixels (two, or one per wavefront) and, behind them, the projection sums (GP)
                for (int o = tid * 16; o < (GP ? NW * t.e_bytes + MAXB * NCO * 4096 : 2 * t.e_bytes); o += 16 * NT) *(v4i_r*)(l_e + o) = v4i_r{0, 0, 0, 0};
                for (int o = tid * 16; o < 4 * a.Ce32; o += 16 * NT) {
                    if constexpr (EXP) *(v4i_r*)(l_be + o) = *(const v4i_r*)((const unsigned char*)a.be + o);
                    *(v4i_r*)(l_bd + o) = *(const v4i_r*)((const unsigned char*)a.bd + o);
                }
            }
#pragma unroll
            for (int i = 0; i < IR_BATCH; ++i)
                if (dst[i] != ~0u) *(v2i_r*)(l_x + dst[i]) = stage[i];
        }
    }

    // ---- the staged pixels inside the image, in blocks of 32 for the expansion -----------------------------------------
    const int y0 = max(0, -iy0), y1 = min(t.ih, a.H - iy0), x0 = max(0, -ix0), x1 = min(t.iw, a.W - ix0);
    const int sw = max(x1 - x0, 1), npix = max(x1 - x0, 0) * max(y1 - y0, 0);
    const int ncb = (npix + 31) >> 5;
    int xoff[IR_MAXCB], eoff[IR_MAXCB];                                 // this lane's pixel in the wavefront's j-th block: byte offsets (eoff < 0: none)
#pragma unroll
    for (int j = 0; j < IR_MAXCB; ++j) {
        const int hp = (GP ? j : wave + 4 * j) * 32 + m, hpc = min(hp, max(npix - 1, 0));
        const int ry = hpc / sw, rx = hpc - ry * sw;
        xoff[j] = ((y0 + ry) * t.iw + x0 + rx) * t.xp + 16 * hi;
        eoff[j] = hp < npix ? (y0 + ry) * e_row + (x0 + rx) * 32 + 16 * hi : -1;
    }
    // ---- this lane's output pixel in the wavefront's s-th block ---------------------------------------------------------
    const int ty = m / t.nbw, tx = m - ty * t.nbw;
    const bool lane_px = ty < t.nbh;
    const int tyc = lane_px ? ty : 0, txc = lane_px ? tx : 0;
    const int nblocks = t.pbw * t.pbh;
    int woff[MAXB];                                                     // window origin of the lane's pixel in the expanded-pixel buffer
#pragma unroll
    for (int s = 0; s < MAXB; ++s) {
        const int b = min(GP ? s : wave + 4 * s, nblocks - 1), by = b / t.pbw, bx = b - by * t.pbw;
        woff[s] = (by * t.nbh + tyc) * STRIDE * e_row + (bx * t.nbw + txc) * STRIDE * 32 + 16 * hi;
    }

    const unsigned char* const we_lane = (const unsigned char*)a.we + (size_t)m * a.Kx + 16 * hi;       // + g * 32 * Kx + k * 32
    const unsigned char* const wd_lane = (const unsigned char*)a.wd + (size_t)lane * 16;               // + (g * 9 + tap) * 1024
    const unsigned char* const wp_lane = (const unsigned char*)a.wp + (size_t)m * a.Ce32 + 16 * hi;     // + cob * 32 * Ce32 + g * 32
    v4i_r we[EXP ? MAXK : 1], wd[9], wp[NCO];
    v16i_r accp[MAXB][NCO];
#pragma unroll
    for (int s = 0; s < MAXB; ++s)
#pragma unroll
        for (int c = 0; c < NCO; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) accp[s][c][i] = 0;

    auto load_we = [&](int g) {
#pragma unroll
        for (int k = 0; k < MAXK; ++k)
            if (k < kx32) we[k] = *(const v4i_r*)(we_lane + (size_t)g * 32 * a.Kx + k * 32);
    };
    auto load_wd_wp = [&](int g) {
#pragma unroll
        for (int k = 0; k < 9; ++k) wd[k] = *(const v4i_r*)(wd_lane + (size_t)(g * 9 + k) * 1024);
#pragma unroll
        for (int c = 0; c < NCO; ++c) wp[c] = *(const v4i_r*)(wp_lane + (size_t)c * 32 * a.Ce32 + g * 32);
    };
    auto bias16 = [&](const unsigned char* lb, int g) {                 // the group's bias in the accumulator layout
        v16i_r acc;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const v4i_r b4 = *(const v4i_r*)(lb + 4 * (g * 32 + 8 * q + 4 * hi));
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[4 * q + e] = b4[e];
        }
        return acc;
    };
    auto expand = [&](int g, unsigned char* ebuf) {
#pragma unroll
        for (int j = 0; j < IR_MAXCB; ++j)
            if ((GP ? j : wave + 4 * j) < ncb) {                        // wave-uniform
                v16i_r acc = bias16(l_be, g);
#pragma unroll
                for (int k = 0; k < MAXK; ++k)
                    if (k < kx32) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(we[k], *(const v4i_r*)(l_x + xoff[j] + k * 32), acc, 0, 0, 0);
                const v4i_r out = ir_requant_pack(acc, cl_e);
                if (eoff[j] >= 0) *(v4i_r*)(ebuf + eoff[j]) = out;
            }
    };
    // without expansion: the group's 32 channels of the tile's input pixels, 16 bytes per lane and load, zeros past the last
    // channel; pixels outside the image are never written and stay zero.  Loads and stores are separate so that the loads of
    // the next group can be in flight over the work on this one.
    constexpr int FT = GP ? 64 : NT;                                    // lanes that fill one buffer: a wavefront's own (GP) or the workgroup's
    v4i_r fl[EXP ? 1 : IR_FILL];
    unsigned fdst[EXP ? 1 : IR_FILL];
    auto fill_load = [&](int g) {
        if constexpr (!EXP) {
            const unsigned char* x = (const unsigned char*)a.x + (size_t)n * a.H * a.W * a.Cin;
            const int nch = t.ih * t.iw * 2, ft = GP ? lane : tid;
#pragma unroll
            for (int i = 0; i < IR_FILL; ++i) {
                fdst[i] = ~0u;
                fl[i] = v4i_r{0, 0, 0, 0};
                if (FT * i < nch) {                                     // wave-uniform
                    const int e = min(FT * i + ft, nch - 1), p = e >> 1, half = e & 1;
                    const int py = (int)__umulhi((unsigned)p, t.magic_iw), px = p - py * t.iw;
                    const int iy = iy0 + py, ix = ix0 + px;
                    const bool in_img = FT * i + ft < nch && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
                    const bool ok = in_img && g * 32 + 16 * half < a.Cin;
                    fl[i] = *(const v4i_r*)(x + (ok ? (unsigned)((iy * a.W + ix) * a.Cin + g * 32 + 16 * half) : 0u));      // unconditional, in range
                    if (!ok) fl[i] = v4i_r{0, 0, 0, 0};
                    if (in_img) fdst[i] = (unsigned)(py * e_row + px * 32 + 16 * half);
                }
            }
        }
    };
    auto fill_store = [&](unsigned char* ebuf) {
        if constexpr (!EXP) {
#pragma unroll
            for (int i = 0; i < IR_FILL; ++i)
                if (fdst[i] != ~0u) *(v4i_r*)(ebuf + fdst[i]) = fl[i];
        }
    };
    auto dw_project = [&](int g, const unsigned char* ebuf) {
#pragma unroll
        for (int s = 0; s < MAXB; ++s)
            if ((GP ? s : wave + 4 * s) < nblocks) {                    // wave-uniform
                v16i_r acc = bias16(l_bd, g);
                const unsigned char* win = ebuf + woff[s];
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int c = 0; c < 3; ++c) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wd[3 * r + c], *(const v4i_r*)(win + r * e_row + c * 32), acc, 0, 0, 0);
                const v4i_r dq = ir_requant_pack(acc, cl_d);
#pragma unroll
                for (int c = 0; c < NCO; ++c) accp[s][c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wp[c], dq, accp[s][c], 0, 0, 0);
            }
    };

    const int ngroups = a.Ce32 >> 5;
    int* const l_r = (int*)(l_e + NW * t.e_bytes);                       // GP: projection sums [block][output block][register][lane]
    if constexpr (GP) {
        unsigned char* const my_e = l_e + wave * t.e_bytes;
        __syncthreads();                                                // staged pixels, cleared buffers and biases are in LDS
        for (int g = wave; g < ngroups; g += NW) {
            if constexpr (EXP) load_we(g); else fill_load(g);
            load_wd_wp(g);
            if constexpr (EXP) expand(g, my_e); else fill_store(my_e);
            dw_project(g, my_e);                                        // same wavefront, same buffer: LDS keeps a wavefront's accesses in order
        }
#pragma unroll
        for (int s = 0; s < MAXB; ++s)
            if (s < nblocks)
#pragma unroll
                for (int c = 0; c < NCO; ++c)
#pragma unroll
                    for (int i = 0; i < 16; ++i) atomicAdd(l_r + ((s * NCO + c) * 16 + i) * 64 + lane, accp[s][c][i]);
        __syncthreads();                                                // all four partial sums are in
    } else {
        if constexpr (EXP) load_we(0); else fill_load(0);
        __syncthreads();                                                // staged pixels, cleared buffers and biases are in LDS
        load_wd_wp(0);
        if constexpr (EXP) expand(0, l_e); else fill_store(l_e);
        for (int g = 0; g < ngroups; ++g) {
            if (g + 1 < ngroups) {
                if constexpr (EXP) load_we(g + 1); else fill_load(g + 1);
            }
            __syncthreads();                                            // group g is in its buffer; nobody reads the other buffer any more
            dw_project(g, l_e + (g & 1) * t.e_bytes);
            if (g + 1 < ngroups) {
                load_wd_wp(g + 1);
                if constexpr (EXP) expand(g + 1, l_e + ((g + 1) & 1) * t.e_bytes); else fill_store(l_e + ((g + 1) & 1) * t.e_bytes);
            }
        }
    }

    // ---- epilogue: bias, residual, requantisation, stores ------------------------------------------------------------------
#pragma unroll
    for (int s = 0; s < MAXB; ++s)
        if ((GP ? s : wave + 4 * s) < nblocks) {                        // wave-uniform
            const int b = GP ? s : wave + 4 * s, by = b / t.pbw, bx = b - by * t.pbw;
            const int oy = oy0 + by * t.nbh + tyc, ox = ox0 + bx * t.nbw + txc;
            const bool px_ok = lane_px && oy < a.Ho && ox < a.Wo;
            const unsigned pix = px_ok ? (unsigned)(((n * a.Ho + oy) * a.Wo + ox) * a.Cout) : 0u;      // < 2^31: checked by the launcher
#pragma unroll
            for (int c = 0; c < NCO; ++c) {
                if (GP && ((s * NCO + c) & (NW - 1)) != wave) continue; // wave-uniform: the (pixel block, output block) pairs take turns
                const int ch = 32 * c + 16 * hi;                        // first of the 16 channels this lane stores
                const int left = a.Cout - ch;                           // channels from there on (a multiple of 8)
                v16i_r acc = accp[s][c];
                if constexpr (GP) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[i] = l_r[((s * NCO + c) * 16 + i) * 64 + lane];
                }
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const v4i_r b4 = *(const v4i_r*)(a.bp + 32 * c + 8 * q + 4 * hi);      // padded to whole blocks of 32, rounding constant included
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[4 * q + e] += b4[e];
                }
                if (a.res) {
                    // the residual in the store layout, unconditional and in range, then back into the accumulator layout
                    const unsigned char* rp = (const unsigned char*)a.res + pix + (left >= 8 ? ch : 0);
                    const v2i_r r01 = *(const v2i_r*)rp, r23 = *(const v2i_r*)(rp + (left >= 16 ? 8 : 0));
                    const auto s02 = __builtin_amdgcn_permlane32_swap((unsigned)r01[0], (unsigned)r01[1], false, false);
                    const auto s13 = __builtin_amdgcn_permlane32_swap((unsigned)r23[0], (unsigned)r23[1], false, false);
                    const unsigned rq[4] = {s02[0], s13[0], s02[1], s13[1]};
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[4 * q + e] += __builtin_amdgcn_sbfe((int)rq[q], 8 * e, 8) << a.res_shift;
                }
                const v4i_r out = ir_requant_pack(acc, cl_p);
                if (px_ok) {
                    unsigned char* yp = (unsigned char*)a.y + pix + ch;
                    if (left >= 16) *(v4i_r*)yp = out;
                    else if (left >= 8) *(v2i_r*)yp = v2i_r{out[0], out[1]};
                }
            }
        }
}

int ir_block_out_blocks(int c_out)
{
    const int nco = (c_out + 31) / 32;
    return nco == 4 ? 5 : nco;                                          // instantiated: 1, 2, 3, 5 blocks of 32 output channels
}

// Shapes the kernel covers, and the tile it takes them with.
bool ir_block_plan(const IrArgs& a, IrTile& t, int& nco, int& maxb)
{
    if ((a.stride != 1 && a.stride != 2) || a.pad != 1 || a.B < 1) return false;
    const bool expands = a.Kx > 0;                                      // Kx = 0: depthwise -> projection, no expansion in front
    if (a.Cout % 8 != 0 || a.Ce32 % 32 != 0 || a.Ce32 < 32) return false;
    if (expands ? (a.Cin % 8 != 0 || a.Cin > 32 * IR_MAXK || a.Kx % 32 != 0 || a.Kx < a.Cin) : (a.Cin % 16 != 0 || a.Ce32 < a.Cin || a.Ce32 - a.Cin >= 32)) return false;
    if ((double)a.B * a.H * a.W * a.Cin >= 2147483648.0 || (double)a.B * a.Ho * a.Wo * a.Cout >= 2147483648.0) return false;
    nco = ir_block_out_blocks(a.Cout);
    if (nco > 5) return false;
    maxb = nco == 1 ? 2 : nco <= 3 ? 2 : 1;
    t.nbw = a.Wo % 8 == 0 ? 8 : a.Wo % 14 == 0 ? 14 : a.Wo % 7 == 0 ? 7 : 8;
    t.nbh = 32 / t.nbw;
    const int bx_max = (a.Wo + t.nbw - 1) / t.nbw, by_max = (a.Ho + t.nbh - 1) / t.nbh;
    t.pbw = 1; t.pbh = 1;
    auto fits = [&] {
        t.iw = (t.pbw * t.nbw - 1) * a.stride + 3;
        t.ih = (t.pbh * t.nbh - 1) * a.stride + 3;
        t.cpp = expands ? a.Cin / 8 : 1;
        t.xp = a.Kx + 16;
        t.x_bytes = expands ? t.ih * t.iw * t.xp + 128 : 0;             // the last pixel's reduction bytes may be read past its channels
        t.e_bytes = t.ih * (t.iw * 32 + 16);
        if (t.pbw * t.pbh > 4 * maxb || 8 * a.Ce32 + t.x_bytes + 2 * t.e_bytes > 64 * 1024) return false;
        return expands ? t.ih * t.iw <= 128 * IR_MAXCB && t.ih * t.iw * t.cpp <= 256 * IR_BATCH * IR_BATCHES
                       : t.ih * t.iw * 2 <= 256 * IR_FILL;
    };
    if (!fits()) return false;
    for (;;) {                                                          // grow the shorter side in pixels while the tile fits
        const bool can_x = t.pbw < bx_max, can_y = t.pbh < by_max;
        const bool prefer_y = can_y && (!can_x || t.pbh * t.nbh <= t.pbw * t.nbw);
        bool grown = false;
        for (int pass = 0; pass < 2 && !grown; ++pass) {
            const bool grow_y = pass == 0 ? prefer_y : !prefer_y;
            if (grow_y ? !can_y : !can_x) continue;
            (grow_y ? t.pbh : t.pbw) += 1;
            const long long wgs = (long long)a.B * ((bx_max + t.pbw - 1) / t.pbw) * ((by_max + t.pbh - 1) / t.pbh);
            if (fits() && wgs >= 256) grown = true; else (grow_y ? t.pbh : t.pbw) -= 1;   // a larger tile only while every CU still gets a workgroup
        }
        if (!grown) break;
    }
    fits();
    t.tiles_x = (bx_max + t.pbw - 1) / t.pbw;
    t.tiles_y = (by_max + t.pbh - 1) / t.pbh;
    t.magic_cpp = t.cpp > 1 ? (unsigned)(4294967296.0 / t.cpp) + 1u : 0u;
    t.magic_iw = (unsigned)(4294967296.0 / t.iw) + 1u;
    const long long total = (long long)a.B * t.tiles_x * t.tiles_y;
    if (total > 0x3fffffff) return false;
    t.total = (int)total;
    t.per_xcd = (t.total + 7) / 8;
    // small images: the wavefronts share the channel groups (instantiated for 2 or more output blocks and 2 or more reduction steps)
    const int nw = a.Ce32 >= 320 ? 8 : 4;                               // ten or more groups: eight wavefronts
    t.gp = nco >= 2 && a.Ce32 >= 128 && t.pbw * t.pbh <= maxb && total <= 2048 && 8 * a.Ce32 + t.x_bytes + nw * t.e_bytes + maxb * nco * 4096 <= 64 * 1024 &&
                   (expands ? a.Kx >= 64 && t.ih * t.iw <= 32 * IR_MAXCB && t.ih * t.iw * t.cpp <= 64 * nw * IR_BATCH * IR_BATCHES
                            : t.ih * t.iw * 2 <= 64 * IR_FILL)
               ? nw : 0;
    return true;
}

bool ir_block_supported(const IrArgs& a)
{
    IrTile t;
    int nco, maxb;
    return ir_block_plan(a, t, nco, maxb);
}

template <int STRIDE, int NCO, int MAXB, int MAXK, int GP>
static void ir_launch5(const IrArgs& a, const IrTile& t, size_t lds, hipStream_t s)
{
    EE_LAUNCH((ir_block_i8_kernel<STRIDE, NCO, MAXB, MAXK, GP>), dim3((unsigned)(t.per_xcd * 8)), dim3(GP ? 64 * GP : 256), lds, s, a, t);
}

template <int STRIDE, int NCO, int MAXB>
static void ir_launch(const IrArgs& a, const IrTile& t, size_t lds, hipStream_t s)
{
    const int kx32 = a.Kx >> 5;                                         // registers for the expansion weights: 1, 2 or 5 steps
    if (kx32 == 0) {                                                    // no expansion
        if constexpr (NCO >= 2) {
            if (t.gp == 4) { ir_launch5<STRIDE, NCO, MAXB, 0, 4>(a, t, lds, s); return; }
            if (t.gp == 8) { ir_launch5<STRIDE, NCO, MAXB, 0, 8>(a, t, lds, s); return; }
        }
        ir_launch5<STRIDE, NCO, MAXB, 0, 0>(a, t, lds, s);
        return;
    }
    if constexpr (NCO >= 2) {
        if (t.gp == 4) {
            if (kx32 <= 2) ir_launch5<STRIDE, NCO, MAXB, 2, 4>(a, t, lds, s);
            else ir_launch5<STRIDE, NCO, MAXB, IR_MAXK, 4>(a, t, lds, s);
            return;
        }
        if (t.gp == 8) {
            if (kx32 <= 2) ir_launch5<STRIDE, NCO, MAXB, 2, 8>(a, t, lds, s);
            else ir_launch5<STRIDE, NCO, MAXB, IR_MAXK, 8>(a, t, lds, s);
            return;
        }
    }
    if (kx32 <= 1) ir_launch5<STRIDE, NCO, MAXB, 1, 0>(a, t, lds, s);
    else if (kx32 <= 2) ir_launch5<STRIDE, NCO, MAXB, 2, 0>(a, t, lds, s);
    else ir_launch5<STRIDE, NCO, MAXB, IR_MAXK, 0>(a, t, lds, s);
}

hipError_t launch_ir_block(const IrArgs& a, hipStream_t s)
{
    IrTile t;
    int nco, maxb;
    if (!ir_block_plan(a, t, nco, maxb)) return hipErrorInvalidValue;
    const size_t lds = (size_t)8 * a.Ce32 + t.x_bytes + (t.gp ? t.gp * (size_t)t.e_bytes + (size_t)maxb * nco * 4096 : 2 * (size_t)t.e_bytes);
    const int v = (a.stride - 1) * 4 + (nco == 1 ? 0 : nco == 2 ? 1 : nco == 3 ? 2 : 3);
    switch (v) {
    case 0: ir_launch<1, 1, 2>(a, t, lds, s); break;
    case 1: ir_launch<1, 2, 2>(a, t, lds, s); break;
    case 2: ir_launch<1, 3, 2>(a, t, lds, s); break;
    case 3: ir_launch<1, 5, 1>(a, t, lds, s); break;
    case 4: ir_launch<2, 1, 2>(a, t, lds, s); break;
    case 5: ir_launch<2, 2, 2>(a, t, lds, s); break;
    case 6: ir_launch<2, 3, 2>(a, t, lds, s); break;
    default: ir_launch<2, 5, 1>(a, t, lds, s); break;
    }
    return hipGetLastError();
}

}  // namespace ee
