// Stride-1 "same" convolutions (3x3 pad 1, 1x7 pad 0/3, ...) on the matrix cores with the activations resident in LDS.
//
// The layer is still the GEMM  R x P . P x C  of the paper's Sec. II-C with the batch along R (Sec. III-A), but when the
// stride is 1 and the output has the input's height and width, output row m = (n, y, x) and input pixel m of the
// flattened NHWC tensor coincide, and tap (r, s) of row m is input row  m + (r - pad) W + (s - pad_w)  whenever it lies
// inside the image.  The input rows a tile of BM output rows needs are therefore ONE contiguous run of
// BM + (kh - 1) W + (kw - 1) rows: the workgroup copies that slab into LDS once and reads every tap's fragments out
// of it at shifted row addresses, instead of copying the same pixels once per tap through the vector memory path
// (nine times for a 3x3 kernel).  Only the weights stream through a ring of stages.  The general kernel's launches
// are bound by exactly that path (global -> LDS bytes per matrix instruction), so this form moves 0.4 - 0.6 x the
// bytes and can afford tall tiles (256 rows), which halve the weight traffic again.
//
// Copies, swizzle, fragment layout, pipelining of a reduction step and epilogue are those of conv_igemm_kernel
// (kernels_igemm.hip, igemm_epilogue.hpp).  Taps outside the image read a block of zeros in LDS (selected per lane
// from a closed-form validity mask), so zero padding costs nothing and the matrix instruction count is uniform.
#include <type_traits>
#include <utility>

#include "ee_internal.hpp"
#include "igemm_device.hpp"
#include "igemm_epilogue.hpp"

namespace ee {

// ES: element bytes.  BM x BN: workgroup tile (pixels x channels), four wavefronts as 2 x 2.  KS: bytes of the
// reduction axis per weight stage (128 or 256; a pixel's bytes CiB = Ci * ES are a power of two >= 64, so a 32-byte
// sub-step never straddles two taps).  ns: weight stages in the ring (2..4).
template <int ES, int BM, int BN, int KS>
__global__ __launch_bounds__(256) void conv_slab_kernel(ConvArgs a, int gm, int gn, unsigned magic_gn, int per_xcd, int ns, int cib_log2)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    constexpr int NT = 256;
    constexpr int CPRW = KS / 16;                  // 16-byte chunks per staged weight row
    constexpr int RPP = NT / CPRW;                 // weight rows one copy pass of the workgroup covers
    constexpr int LPT = BN / RPP;                  // copies per wavefront and stage
    constexpr int STAGE = BN * KS;
    constexpr int R256 = KS >= 256 ? 1 : 256 / KS; // staged weight rows per 256 bytes of LDS
    constexpr int TILE_O = BM * BN * ES;
    constexpr int SPW = KS / 32;                   // matrix sub-steps per stage
    constexpr int FD = EE_FRAG_DISTANCE, NFB = 4;                 // fragments are read FD sub-steps ahead into NFB register sets used in turn
    constexpr int ZERO_BYTES = 1024;               // what taps outside the image read; at least one pixel long
    static_assert(LPT >= 1 && BN % RPP == 0 && SPW >= 4 && SPW % NFB == 0, "tile / step not supported");

    const int xcd = blockIdx.x & 7, wslot = blockIdx.x >> 3;
    const int mslot = (int)fast_div((unsigned)wslot, (unsigned)gn, magic_gn);
    const int mt = xcd * per_xcd + mslot, nt = wslot - mslot * gn;
    if (mt >= gm || mslot >= per_xcd) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN;
    const int m0 = mt * BM, n0 = nt * BN;
    const unsigned char* xb = (const unsigned char*)a.x;
    const unsigned char* zp = (const unsigned char*)a.zeros;
    const int KpB = a.Kp * ES;                     // weight row pitch in bytes
    const int CiB = 1 << cib_log2;                 // bytes of a pixel
    const int nk = (a.kh * a.kw * CiB + KS - 1) / KS;
    const bool wide = (a.Co * ES) % 16 == 0 && (a.ldc * ES) % 16 == 0 && (a.c_off * ES) % 16 == 0;
    const bool has_res = a.res != nullptr;
    const unsigned lds0 = lds_addr(lds);

    // LDS map: slab | zeros | weight ring, the output tile aliases them | residual tile | bias
    const int halo_lo = a.pad * a.W + a.pad_w, halo_hi = (a.kh - 1 - a.pad) * a.W + (a.kw - 1 - a.pad_w);
    const int srows = BM + halo_lo + halo_hi;                        // slab rows
    const int cpr_log2 = cib_log2 - 4;                               // log2 of the 16-byte chunks per slab row
    const unsigned slab_chunks = (unsigned)srows << cpr_log2;
    const unsigned slab_bytes = ((slab_chunks + 255u) & ~255u) * 16u;  // whole copy passes of the workgroup
    const unsigned zero_off = slab_bytes, ring_off = slab_bytes + ZERO_BYTES;
    const unsigned front = ring_off + (unsigned)((ns < nk ? ns : nk) * STAGE);
    const unsigned region0 = front > (unsigned)TILE_O ? front : (unsigned)TILE_O;
    const unsigned ro_off = has_res && wide ? region0 : 0;
    const unsigned bias_off = has_res && wide ? region0 + TILE_O : region0;

    igemm_stage_bias_res<ES, BM, BN, NT>(a, lds0, ro_off, bias_off, m0, n0, tid, wave, lane, has_res && wide);

    // ---- the slab: input rows m0 - halo_lo .. m0 + BM + halo_hi - 1, clamped into the tensor (a clamped row is only
    // ever the source of taps that the validity mask rejects).  Chunk c of slab row r sits at c ^ sswz(r).
    const int s256_log2 = cib_log2 >= 8 ? 0 : 8 - cib_log2;          // log2 of the slab rows per 256 bytes
    const unsigned smask = cib_log2 >= 8 ? 15u : (unsigned)((1 << cpr_log2) - 1);
    {
        const int passes = (int)((slab_chunks + 255u) >> 8);
        for (int pss = 0; pss < passes; ++pss) {
            const unsigned q = (unsigned)(pss * 256 + tid);
            const unsigned row = q >> cpr_log2, pos = q & ((1u << cpr_log2) - 1u);
            const unsigned chunk = pos ^ ((row >> s256_log2) & smask);
            int g = m0 - halo_lo + (int)row;
            g = g < 0 ? 0 : (g >= a.M ? a.M - 1 : g);
            const unsigned char* p = q < slab_chunks ? xb + (((size_t)(unsigned)g << cib_log2) + chunk * 16u) : zp;
            dma16(lds0 + (unsigned)(pss * 256 + wave * 64) * 16u, p);
        }
        if (tid < ZERO_BYTES / 16) *(v4i*)(lds + zero_off + tid * 16) = v4i{0, 0, 0, 0};
    }

    // ---- per-lane weight copy state ----------------------------------------------------------------------------
    const int lrow = tid / CPRW;
    const int cchunk = (tid % CPRW) ^ ((lrow / R256) & (CPRW - 1));
    unsigned voffB[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) voffB[j] = (unsigned)(n0 + lrow + j * RPP) * (unsigned)KpB + cchunk * 16;
    auto issue_piece = [&](auto piece, unsigned sbase) {
        constexpr int P = decltype(piece)::value;
        dma16(sbase + P * (NT * 16), a.w, voffB[P]);
        voffB[P] += KS;
    };
    auto issue_all = [&](int stage) {
        const unsigned sbase = lds0 + ring_off + stage * STAGE + wave * 1024;
        static_for<LPT>([&](auto piece) { issue_piece(piece, sbase); });
    };

    // ---- fragment addressing -----------------------------------------------------------------------------------
    const int frow = lane & 31, hi = lane >> 5;
    int fragoff[SPW];                              // weights: as in conv_igemm_kernel
#pragma unroll
    for (int u = 0; u < SPW; ++u) fragoff[u] = frow * KS + (((2 * u + hi) ^ ((frow / R256) & (CPRW - 1))) * 16);
    // activations: row block i of this wavefront is slab rows base[i] + tap offset; bit t of vmask[i] says whether tap t
    // of the lane's pixel lies inside the image
    int base[TM];
    unsigned vmask[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int r = wm0 + 32 * i + frow;
        int m = m0 + r;
        const bool live = m < a.M;
        m = live ? m : a.M - 1;
        const unsigned n = fast_div((unsigned)m, (unsigned)(a.Ho * a.Wo), a.magic_howo);
        const unsigned rem = (unsigned)m - n * (unsigned)(a.Ho * a.Wo);
        const unsigned oy = fast_div(rem, (unsigned)a.Wo, a.magic_wo), ox = rem - oy * a.Wo;
        const int iy0 = (int)oy - a.pad, ix0 = (int)ox - a.pad_w;
        const int s_lo = max(0, -ix0), s_hi = min(a.kw, a.W - ix0), r_lo = max(0, -iy0), r_hi = min(a.kh, a.H - iy0);
        const unsigned colmask = s_hi > s_lo ? ((1u << s_hi) - 1u) & ~((1u << s_lo) - 1u) : 0u;
        const unsigned rowsel = r_hi > r_lo ? a.tap_rows & ((1u << (r_hi * a.kw)) - 1u) & ~((1u << (r_lo * a.kw)) - 1u) : 0u;
        vmask[i] = live ? colmask * rowsel : 0u;
        base[i] = r + halo_lo;
    }
    // State of the fragment reader (wave-uniform): the tap it is in, the byte offset inside the pixel, and per row block
    // the lane's address parts for that tap:  address = pa[i] + (cb ^ px[i]),  because the chunk index (cb / 16 + hi)
    // ^ swizzle splits into a per-tap part and cb, whose lowest set bit is 32.
    int r_tap = 0, r_ts = 0, r_toff = -halo_lo, r_cb = 0;
    unsigned pa[TM], px[TM];
    auto set_tap = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const unsigned row = (unsigned)(base[i] + r_toff);
            const unsigned sw = (row >> s256_log2) & smask;
            const bool ok = r_tap < 32 && ((vmask[i] >> r_tap) & 1u);
            pa[i] = ok ? (row << cib_log2) + (((unsigned)hi ^ (sw & 1u)) << 4) : zero_off;
            px[i] = ok ? (sw & 14u) << 4 : 0u;
        }
    };
    set_tap();
    auto advance_reader = [&]() {                   // one sub-step (32 bytes) further along (r, s, c)
        r_cb += 32;
        if (r_cb == CiB) {
            r_cb = 0;
            ++r_tap;
            ++r_toff;
            if (++r_ts == a.kw) { r_ts = 0; r_toff += a.W - a.kw; }
            set_tap();
        }
    };

    using acc_t = typename std::conditional<ES == 1, v16i, v16f>::type;
    acc_t acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0;

    v4i gw[NFB][TN], gx[NFB][TM];
    auto read_x = [&](v4i* x) {                     // the reader's current sub-step, then one further
#pragma unroll
        for (int i = 0; i < TM; ++i) x[i] = *(const v4i*)(lds + pa[i] + ((unsigned)r_cb ^ px[i]));
    };

    // One reduction step (see the pipelined step of conv_igemm_kernel): every matrix instruction is followed by at most
    // one fragment read and one copy; the wait for the next weight stage and the barrier sit FD sub-steps before the end.
    auto step = [&](int sc, int sn, int si, auto issue_tag, auto last_tag) {
        constexpr bool ISSUE = decltype(issue_tag)::value, LAST = decltype(last_tag)::value;
        constexpr int NM = TN * TM, ISUBS = SPW - FD, PPS = (LPT + ISUBS - 1) / ISUBS;
        const unsigned char* sb = lds + ring_off + sc * STAGE + wn0 * KS;
        const unsigned char* nb = lds + ring_off + sn * STAGE + wn0 * KS;
        const unsigned sbase = lds0 + ring_off + si * STAGE + wave * 1024;
        static_for<SPW>([&](auto sub_tag) {
            constexpr int SUB = decltype(sub_tag)::value;
            if constexpr (SUB == SPW - FD && !LAST) {
                if (!ISSUE || ns == 2) wait_all_then_barrier<0>();
                else if (ns == 3) wait_all_then_barrier<LPT>();
                else wait_all_then_barrier<2 * LPT>();
            }
            constexpr int TSUB = SUB + FD;                        // the sub-step whose fragments are read now
            constexpr bool NEXT = TSUB >= SPW;
            constexpr int RS = NEXT ? TSUB - SPW : TSUB;
            constexpr bool DO_READ = !(NEXT && LAST);
            const unsigned char* rb = NEXT ? nb : sb;
            static_for<NM>([&](auto q_tag) {
                constexpr int Q = decltype(q_tag)::value, J = Q / TM, I = Q % TM;
                if constexpr (ES == 1)
                    acc[J][I] = __builtin_amdgcn_mfma_i32_32x32x32_i8(gw[SUB % NFB][J], gx[SUB % NFB][I], acc[J][I], 0, 0, 0);
                else
                    acc[J][I] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, gw[SUB % NFB][J]),
                                                                         __builtin_bit_cast(v8bf, gx[SUB % NFB][I]), acc[J][I], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                // fragment reads of sub-step TSUB spread over the matrix instructions: weights first, then activations
                static_for<(TN + TM + NM - 1) / NM>([&](auto r_tag) {
                    constexpr int R = Q + NM * decltype(r_tag)::value;
                    if constexpr (DO_READ && R < TN) gw[TSUB % NFB][R] = *(const v4i*)(rb + 32 * R * KS + fragoff[RS]);
                    if constexpr (DO_READ && R >= TN && R < TN + TM)
                        gx[TSUB % NFB][R - TN] = *(const v4i*)(lds + pa[R - TN] + ((unsigned)r_cb ^ px[R - TN]));
                });
                if constexpr (ISSUE && SUB < ISUBS)
                    static_for<(PPS + NM - 1) / NM>([&](auto d_tag) {
                        constexpr int D = Q + NM * decltype(d_tag)::value, P = SUB * PPS + D;
                        if constexpr (D < PPS && P < LPT) issue_piece(std::integral_constant<int, P>{}, sbase);
                    });
                __builtin_amdgcn_sched_barrier(0);
            });
            if constexpr (DO_READ) advance_reader();
        });
    };

    // ---- main loop ---------------------------------------------------------------------------------------------
    for (int s = 0; s < ns - 1; ++s)
        if (s < nk) issue_all(s);
    {
        const int ahead = (ns - 1 < nk ? ns - 1 : nk) - 1;      // weight stages issued behind the first one
        if (ahead <= 0) wait_all_then_barrier<0>();             // also the zero block written above
        else if (ahead == 1) wait_all_then_barrier<LPT>();
        else wait_all_then_barrier<2 * LPT>();
    }
    static_for<FD>([&](auto u_tag) {                // fragments of the first FD sub-steps
        constexpr int U = decltype(u_tag)::value;
#pragma unroll
        for (int j = 0; j < TN; ++j) gw[U][j] = *(const v4i*)(lds + ring_off + wn0 * KS + 32 * j * KS + fragoff[U]);
        read_x(gx[U]);
        advance_reader();
    });
    int st_c = 0, st_i = ns - 1, ks = 0;
    auto next_of = [&](int st) { return st + 1 == ns ? 0 : st + 1; };
    for (; ks + ns - 1 < nk; ++ks) {
        step(st_c, next_of(st_c), st_i, std::true_type{}, std::false_type{});
        st_c = next_of(st_c);
        st_i = next_of(st_i);
    }
    for (; ks + 1 < nk; ++ks) {                     // nothing left to copy
        step(st_c, next_of(st_c), st_c, std::false_type{}, std::false_type{});
        st_c = next_of(st_c);
    }
    step(st_c, st_c, st_c, std::false_type{}, std::true_type{});
    lds_barrier();                                  // every wavefront is done with the slab and the ring

    igemm_epilogue<ES, BM, BN, NT>(a, acc, lds, ro_off, bias_off, m0, n0, wm0, wn0, tid, has_res, wide, true);
}

// ---- launch ------------------------------------------------------------------------------------------------
static int log2_exact(int v)
{
    int k = 0;
    while ((1 << k) < v) ++k;
    return (1 << k) == v ? k : -1;
}

// Stride 1, output as large as the input, a pixel of 64 .. 1024 bytes that is a power of two, 2 .. 31 taps, and a tensor
// below 2 GiB.  The reduction need not be a whole number of steps: the packed weight rows are zero padded to a multiple
// of 256 bytes, and the taps past the last one are outside every lane's validity mask.
bool conv_slab_supported(const ConvArgs& a, int es)
{
    const int cib = a.Ci * es, k = log2_exact(cib);
    if (a.xs || a.ys || a.gap_sums || a.mode != 0 || a.stride != 1 || a.Ho != a.H || a.Wo != a.W) return false;
    if (k < 6 || k > 10 || a.kh * a.kw > 31 || a.kh * a.kw < 2) return false;
    if (a.H + 2 * a.pad - a.kh + 1 != a.Ho || a.W + 2 * a.pad_w - a.kw + 1 != a.Wo) return false;
    return (long long)a.M * cib < (1ll << 31);
}

template <int ES, int BM, int BN, int KS>
static hipError_t launch_slab_tile(const ConvArgs& a, int ns, hipStream_t s)
{
    const int gm = (a.M + BM - 1) / BM, gn = (a.Co + BN - 1) / BN, per_xcd = (gm + 7) / 8;
    const dim3 grid((unsigned)(8 * per_xcd * gn));
    const unsigned magic_gn = (unsigned)(0x100000000ull / (unsigned)gn - (gn == 1));
    const int cib = a.Ci * ES, cib_log2 = log2_exact(cib);
    const bool res_tile = a.res != nullptr && (a.Co * ES) % 16 == 0;
    const int nk = (a.kh * a.kw * cib + KS - 1) / KS;
    if (nk * KS > a.Kp * ES) return hipErrorInvalidValue;      // a step may not reach past the padded weight row
    ns = ns < 2 ? 2 : (ns > 4 ? 4 : ns);
    const int srows = BM + (a.kh - 1) * a.W + (a.kw - 1);
    const size_t slab = ((((size_t)srows << (cib_log2 - 4)) + 255) & ~(size_t)255) * 16 + 1024;
    constexpr int TILE_O = BM * BN * ES;
    auto lds_need = [&](int stages) {
        const size_t front = slab + (size_t)(stages < nk ? stages : nk) * BN * KS;
        return (front > (size_t)TILE_O ? front : (size_t)TILE_O) + (res_tile ? (size_t)TILE_O : 0) + 1024;
    };
    while (ns > 2 && lds_need(ns) > 160 * 1024) --ns;      // the deepest ring that fits
    const size_t lds_bytes = lds_need(ns);
    if (lds_bytes > 160 * 1024) return hipErrorInvalidValue;
    static const hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_slab_kernel<ES, BM, BN, KS>),
                                                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (granted != hipSuccess) return granted;
    EE_LAUNCH((conv_slab_kernel<ES, BM, BN, KS>), grid, dim3(256), lds_bytes, s, a, gm, gn, magic_gn, per_xcd, ns, cib_log2);
    return hipGetLastError();
}

// cfg: bits 0-3 tile (1: 128x128, 2: 128x64, 3: 256x64, 4: 256x128; 0 = by shape), bits 4-7 weight step (2: 128, 3: 256 bytes;
// 0 = 128), bits 8-11 weight stages (2..4; 0 = 3).  hipErrorInvalidValue for a layer or configuration it does not cover.
template <int ES>
hipError_t launch_conv_slab(const ConvArgs& a, int cfg, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    if (!conv_slab_supported(a, ES)) return hipErrorInvalidValue;
    int tile = cfg & 15, ksel = (cfg >> 4) & 15, ns = (cfg >> 8) & 15;
    if (ksel == 0) ksel = 2;
    if (ns == 0) ns = 3;
    if (ksel != 2 && ksel != 3) return hipErrorInvalidValue;
    const int co_pad = (a.Co + 127) / 128 * 128;        // rows of the packed weights
    if (tile == 0) tile = a.Co <= 64 ? 3 : 1;
    const int bn = (tile == 1 || tile == 4) ? 128 : 64;
    if (((a.Co + bn - 1) / bn) * bn > co_pad) return hipErrorInvalidValue;
#define EE_SLAB(T_, BM_, BN_) \
    if (tile == T_) return ksel == 3 ? launch_slab_tile<ES, BM_, BN_, 256>(a, ns, s) : launch_slab_tile<ES, BM_, BN_, 128>(a, ns, s);
    EE_SLAB(1, 128, 128) EE_SLAB(2, 128, 64) EE_SLAB(3, 256, 64) EE_SLAB(4, 256, 128)
#undef EE_SLAB
    return hipErrorInvalidValue;
}

template hipError_t launch_conv_slab<1>(const ConvArgs&, int, hipStream_t);
template hipError_t launch_conv_slab<2>(const ConvArgs&, int, hipStream_t);

}  // namespace ee
