// Bias / residual staging and the epilogue shared by the matrix-core convolution kernels whose four wavefronts
// (per wavefront group) own a BM x BN tile as 2 x 2: accumulator acc[j][i] of a wavefront covers channels
// wn0 + 32 j .. and pixel rows wm0 + 32 i ..; lane l holds column (pixel) l % 32, and register v row (channel)
// 8 (v / 4) + 4 (l / 32) + v % 4.
#pragma once
#include <type_traits>

#include "ee_internal.hpp"
#include "igemm_device.hpp"

namespace ee {
namespace {

// The output tile in LDS: rows of BN elements, chunk c of row r at c ^ oswz(r), oswz(r) = (r / rows per 256 bytes)
// & (chunks per row - 1): the 32 rows a wavefront touches with one 4- or 8-byte access per lane then spread over
// the banks as evenly as the row length allows.
template <int ES, int BN>
struct OutTile {
    static constexpr int CR = BN * ES / 16, OROW = BN * ES, OR256 = OROW >= 256 ? 1 : 256 / OROW;
    static __device__ __forceinline__ int oswz(int r) { return (r / OR256) & (CR - 1); }
};

// Copies the bias of the tile's channels (256 entries from the first one) and, for a layer with a residual whose pixels
// are whole 16-byte chunks, the residual tile into LDS.  Asynchronous: the copies are counted by vmcnt like the
// operand copies issued behind them and are complete when the first of those is.  NT: lanes of the workgroup.
template <int ES, int BM, int BN, int NT>
__device__ __forceinline__ void igemm_stage_bias_res(const ConvArgs& a, unsigned lds0, unsigned ro_off, unsigned bias_off, int m0, int n0,
                                                     int tid, int wave, int lane, bool res_tile)
{
    using T = OutTile<ES, BN>;
    constexpr int CR = T::CR, NO = (BM * CR + NT - 1) / NT;
    const unsigned char* zp = (const unsigned char*)a.zeros;
    if (wave == 0) dma16(lds0 + bias_off, (const unsigned char*)a.bias + (size_t)n0 * 4 + lane * 16);
    if (res_tile) {
#pragma unroll
        for (int j = 0; j < NO; ++j) {
            const int q = tid + NT * j, row = q / CR, chunk = (q % CR) ^ T::oswz(row);
            const int m = m0 + row, ch = n0 + chunk * (16 / ES);
            const unsigned char* p = (m < a.M && ch < a.Co) ? (const unsigned char*)a.res + ((size_t)m * a.Co + ch) * ES : zp;
            if (NT * j + 64 * wave < BM * CR) dma16(lds0 + ro_off + (NT * j + 64 * wave) * 16, p);      // wave-uniform
        }
    }
}

// Bias, residual, requantisation / clamp and packing in the accumulator layout, the tile through LDS (at ro_off; with a
// staged residual tile the results replace it in place), then 16-byte stores along the channels.  Every wavefront of the
// workgroup calls it (it contains a barrier); `active` says whether this wavefront holds accumulators to write.
// Layers whose pixels are not whole 16-byte chunks (wide == false) store straight from the registers.
template <int ES, int BM, int BN, int NT, typename ACC>
__device__ __forceinline__ void igemm_epilogue(const ConvArgs& a, ACC& acc, unsigned char* lds, unsigned ro_off, unsigned bias_off, int m0, int n0,
                                               int wm0, int wn0, int tid, bool has_res, bool wide, bool active)
{
    using T = OutTile<ES, BN>;
    constexpr int TM = BM / 64, TN = BN / 64, CR = T::CR, OROW = T::OROW, NO = (BM * CR + NT - 1) / NT;
    auto oswz = [](int r) { return T::oswz(r); };
    const int lane = tid & 63, frow = lane & 31, hi = lane >> 5;
    unsigned char* ro = lds + ro_off;
    const int* lbias = (const int*)(lds + bias_off);
    // Exit-head pooling fused into the segment's last layer (int8, a.gap_sums set by the launcher only for a layer with a
    // staged residual tile, so that the ring in front of the tile is free now): per-sample column sums of the finished
    // tile are added up in LDS, then one global atomic per (sample, channel) of the tile goes into sums[n][Co].  int32
    // addition is exact in any order, so the sums are those of the pooling kernel.
    constexpr int GAP_S = 8;                                  // samples a tile may touch (the launcher checks (BM - 1) / HW + 2 <= GAP_S)
    int* gacc = (int*)lds;                                    // [GAP_S][BN]
    const bool fuse_gap = ES == 1 && a.gap_sums != nullptr && wide && has_res && ro_off >= GAP_S * BN * 4;
    if (fuse_gap)
        for (int i = tid; i < GAP_S * BN; i += NT) gacc[i] = 0;
    // Cell of (pixel row r, channel cl) in the output tile: chunk (cl*ES/16) ^ oswz(r) of row r.  oswz has period
    // 16, so it is oswz(frow) for all of a lane's rows, and the chunk index splits into a wave-uniform part
    // and a compile-time part: one XOR and one add per cell remain.
    // zero-copy compaction: sample n of the output goes to slot ys[n] of y
    auto out_row = [&](int m) -> long long {
        if (!a.ys || m >= a.M) return m;
        const unsigned howo = (unsigned)(a.Ho * a.Wo), n = fast_div((unsigned)m, howo, a.magic_howo);
        return (long long)a.ys[n] * howo + ((unsigned)m - n * howo);
    };
    const int swz_l = oswz(frow);
    auto finish = [&](auto res_tag, auto wide_tag) {
        constexpr bool RES = decltype(res_tag)::value, WIDE = decltype(wide_tag)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int r = wm0 + 32 * i + frow;
            const int m = m0 + r;
            unsigned char* rowp = ro + r * OROW + 4 * hi * ES;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int cl = wn0 + 32 * j + 8 * g + 4 * hi;                     // first of this lane's 4 channels
                    const int chunk = (wn0 * ES >> 4) + ((32 * j + 8 * g) * ES >> 4);  // 4*hi*ES stays inside the chunk
                    unsigned char* cell = rowp + ((chunk ^ swz_l) << 4) + (((32 * j + 8 * g) * ES) & 15);
                    const long long o = (long long)m * a.Co + n0 + cl;                  // in the residual (never a slice)
                    const long long oy_ = (WIDE ? 0ll : out_row(m) * a.ldc) + a.c_off + n0 + cl;   // in the output (used by the direct stores only)
                    const bool inside = WIDE || (m < a.M && n0 + cl < a.Co);
                    const v4i b4 = *(const v4i*)(lbias + cl);
                    if constexpr (ES == 1) {
                        int packed = 0;
                        if (RES) packed = WIDE ? *(const int*)cell : (inside ? *(const int*)((const signed char*)a.res + o) : 0);
                        int q[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            int t = acc[j][i][4 * g + e] + b4[e];                     // the rounding constant is part of the bias
                            if (RES) t += __builtin_amdgcn_sbfe(packed, 8 * e, 8) << a.res_shift;
                            q[e] = clamp_i32(t >> a.shift, a.lo, a.hi);
                        }
                        const unsigned out = pack4_i8(q[0], q[1], q[2], q[3]);
                        if (WIDE) *(unsigned*)cell = out;
                        else if (inside) *(unsigned*)((signed char*)a.y + oy_) = out;
                    } else {
                        uint2 packed = {0u, 0u};
                        if (RES) packed = WIDE ? *(const uint2*)cell : (inside ? *(const uint2*)((const uint16_t*)a.res + o) : packed);
                        const float r0 = __uint_as_float(packed.x << 16), r1 = __uint_as_float(packed.x & 0xFFFF0000u);
                        const float r2 = __uint_as_float(packed.y << 16), r3 = __uint_as_float(packed.y & 0xFFFF0000u);
                        float t0 = acc[j][i][4 * g + 0] + __int_as_float(b4[0]), t1 = acc[j][i][4 * g + 1] + __int_as_float(b4[1]);
                        float t2 = acc[j][i][4 * g + 2] + __int_as_float(b4[2]), t3 = acc[j][i][4 * g + 3] + __int_as_float(b4[3]);
                        if (RES) { t0 += r0; t1 += r1; t2 += r2; t3 += r3; }
                        t0 = fminf(fmaxf(t0, a.f_lo), a.f_hi); t1 = fminf(fmaxf(t1, a.f_lo), a.f_hi);
                        t2 = fminf(fmaxf(t2, a.f_lo), a.f_hi); t3 = fminf(fmaxf(t3, a.f_lo), a.f_hi);
                        uint2 out;
                        out.x = to_bf16_rne(t0) | (to_bf16_rne(t1) << 16);
                        out.y = to_bf16_rne(t2) | (to_bf16_rne(t3) << 16);
                        if (WIDE) *(uint2*)cell = out;
                        else if (inside) *(uint2*)((uint16_t*)a.y + oy_) = out;
                    }
                }
        }
    };
    if (active) {
        if (wide) {
            if (has_res) finish(std::true_type{}, std::true_type{});
            else finish(std::false_type{}, std::true_type{});
        } else {
            if (has_res) finish(std::true_type{}, std::false_type{});
            else finish(std::false_type{}, std::false_type{});
        }
    }
    if (wide) {
        lds_barrier();
        if (fuse_gap) {
            constexpr int CG = BN / 4, NRG = NT / CG, RG = (BM + NRG - 1) / NRG;     // dword columns, row groups, rows per group
            const int cg = tid % CG, rg = tid / CG;
            const unsigned hw = (unsigned)(a.Ho * a.Wo);
            const int nfirst = (int)fast_div((unsigned)min(m0, a.M - 1), hw, a.magic_howo);
            int cur = -1, s0 = 0, s1 = 0, s2 = 0, s3 = 0;
            auto flush = [&]() {
                if (cur < 0) return;
                int* g = gacc + (cur - nfirst) * BN + cg * 4;
                atomicAdd(g, s0); atomicAdd(g + 1, s1); atomicAdd(g + 2, s2); atomicAdd(g + 3, s3);
            };
            for (int r = 0; r < RG; ++r) {
                const int row = rg * RG + r, m = m0 + row;
                if (row >= BM || m >= a.M) break;
                const int n = (int)fast_div((unsigned)m, hw, a.magic_howo);
                if (n != cur) { flush(); cur = n; s0 = s1 = s2 = s3 = 0; }
                const int v = *(const int*)(ro + row * OROW + ((((cg * 4) >> 4) ^ oswz(row)) << 4) + ((cg * 4) & 15));
                s0 += __builtin_amdgcn_sbfe(v, 0, 8); s1 += __builtin_amdgcn_sbfe(v, 8, 8);
                s2 += __builtin_amdgcn_sbfe(v, 16, 8); s3 += __builtin_amdgcn_sbfe(v, 24, 8);
            }
            flush();
        }
#pragma unroll
        for (int j = 0; j < NO; ++j) {
            const int q = tid + NT * j, row = q / CR, chunk = (q % CR) ^ oswz(row);
            const int m = m0 + row, ch = n0 + chunk * (16 / ES);
            if (q < BM * CR && m < a.M && ch < a.Co) *(v4i*)((unsigned char*)a.y + ((size_t)out_row(m) * a.ldc + a.c_off + ch) * ES) = *(const v4i*)(ro + q * 16);
        }
        if (fuse_gap) {
            lds_barrier();
            const unsigned hw = (unsigned)(a.Ho * a.Wo);
            const int mlast = min(m0 + BM, a.M) - 1;
            const int nfirst = (int)fast_div((unsigned)min(m0, a.M - 1), hw, a.magic_howo), nlast = (int)fast_div((unsigned)mlast, hw, a.magic_howo);
            const int cnt = (nlast - nfirst + 1) * BN;
            for (int i = tid; i < cnt; i += NT) {
                const int sl = i / BN, c = i - sl * BN;
                if (n0 + c < a.Co) atomicAdd(a.gap_sums + (long long)(nfirst + sl) * a.Co + n0 + c, gacc[i]);
            }
        }
    }
}

}  // namespace
}  // namespace ee
