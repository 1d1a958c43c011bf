// Implicit-GEMM convolution for gfx950 (CDNA4) with asynchronous global -> LDS staging.
//
// Every CONV layer is the GEMM  R x P . P x C -> R x C  of the paper's Sec. II-C with the batch
// appended along R (R-batching, Sec. III-A).  The Toeplitz matrix is never materialised: the
// rows (output pixels) are gathered from the NHWC activation tensor while the reduction walks
// over (r, s, c) in steps of KS bytes.
//
// Data movement.  Both operands go from global memory straight into LDS with
// global_load_lds_dwordx4 (16 bytes per lane, no VGPR staging): lane l of a wavefront names its
// own source address and its 16 bytes land at  M0 + 16*l, so one instruction fills 1 KiB of LDS.
// A ring of ns stages keeps ns-1 reduction steps in flight; the wavefronts count their own
// outstanding copies (s_waitcnt vmcnt) and meet at one barrier per step.  Padding taps and rows
// past the end of the batch read a small zero page instead of being skipped, so every wavefront
// issues the same number of copies per step and the counting stays uniform.
//
// LDS layout of a stage: BM activation rows then BN weight rows of KS bytes, no padding.  The 16-byte
// chunk c of row r is stored at chunk position  c ^ swz(r)  (the lane that copies it simply reads
// a permuted source address), with swz chosen such that the 16-lane phases of a ds_read_b128 of
// a matrix-core fragment (32 consecutive rows, same c) touch all 64 banks once.
//
// Compute.  4 wavefronts as 2 x 2, each owning (BM/2) x (BN/2) outputs in 32x32 accumulators of
// v_mfma_i32_32x32x32_i8 / v_mfma_f32_32x32x16_bf16 (16 operand bytes per lane and instruction).
// The weight fragment is the A operand, the activation fragment the B operand, so a lane holds
// 4 consecutive output channels of one pixel per accumulator quad.
//   A: row l%32, k-bytes [16*(l/32), +16)      B: column l%32, same k-bytes
//   D: column l%32, rows 8*(v/4) + 4*(l/32) + v%4 for accumulator register v = 0..15
//
// Epilogue.  Bias (copied to LDS at kernel start) and the residual tile (likewise, so that its
// latency hides behind the main loop) are added in the accumulator layout, the result is
// requantised / clamped, packed and written into an LDS tile from which the workgroup stores whole
// 16-byte chunks along the channel axis.
#include <type_traits>
#include <utility>

#include "ee_internal.hpp"
#include "igemm_device.hpp"
#include "igemm_epilogue.hpp"

namespace ee {

#ifndef EE_IGEMM_PIPELINED
#define EE_IGEMM_PIPELINED 1
#endif

// ES: element bytes (1 int8, 2 bf16).  BM x BN: workgroup tile (pixels x channels).  KS: bytes of
// the reduction axis per stage.  ns (2..4, not above the number of steps + 1): stages in the ring.  PLAIN: 1x1 kernel without padding whose
// reduction length is a multiple of KS -- the source address of a row then simply advances by KS.
// KSPL (1, 2, 4): groups of 4 wavefronts per workgroup.  Every group owns the whole tile but only
// every KSPL-th part of each stage's sub-steps; the groups' accumulators are added through LDS before
// the epilogue.  This is the re-shaping the paper does in hardware when the row dimension under-fills
// the array (Sec. III-A, Eq. 1: samples mapped along P instead of R): with few output pixels the
// reduction axis supplies the parallelism that keeps a CU's matrix cores and copy queue busy.
template <int ES, int BM, int BN, int KS, int KSPL, bool PLAIN>
__global__ __launch_bounds__(256 * KSPL) void conv_igemm_kernel(ConvArgs a, int gm, int gn, unsigned magic_gn, int per_xcd, int ns)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int WM = BM / 2, WN = BN / 2, TM = WM / 32, TN = WN / 32;
    constexpr int CPRW = KS / 16;                  // 16-byte chunks per staged row
    constexpr int NT = 256 * KSPL;                 // lanes per workgroup
    constexpr int RPP = NT / CPRW;                 // rows one copy pass of the workgroup covers
    constexpr int NA = BM / RPP, NB = BN / RPP, LPT = NA + NB;
    constexpr int STAGE = (BM + BN) * KS;
    constexpr int R256 = KS >= 256 ? 1 : 256 / KS; // staged rows per 256 bytes of LDS
    constexpr int TILE_O = BM * BN * ES;           // the output tile in LDS (igemm_epilogue.hpp)
    constexpr int NSUB = KS / 32, SPW = NSUB / KSPL;   // matrix sub-steps per stage, and per wavefront
    constexpr int PART = TM * TN * 4096;           // bytes of one wavefront's accumulators
    static_assert(NA >= 1 && NB >= 1 && BM % RPP == 0 && BN % RPP == 0, "tile too small for this many lanes");
    static_assert(SPW >= 1 && SPW * KSPL == NSUB, "more wavefront groups than sub-steps");

    const int xcd = blockIdx.x & 7, wslot = blockIdx.x >> 3;
    const int mslot = (int)fast_div((unsigned)wslot, (unsigned)gn, magic_gn);
    const int mt = xcd * per_xcd + mslot, nt = wslot - mslot * gn;
    if (mt >= gm || mslot >= per_xcd) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave & 1) * WM, wn0 = ((wave >> 1) & 1) * WN, kpart = wave >> 2;
    const int m0 = mt * BM, n0 = nt * BN;
    const unsigned char* xb = (const unsigned char*)a.x;
    const unsigned char* zp = (const unsigned char*)a.zeros;
    const int KpB = a.Kp * ES;                     // weight row pitch in bytes
    const int nk = (a.kh * a.kw * a.Ci * ES + KS - 1) / KS;
    const int CiB = a.Ci * ES;
    // whole 16-byte chunks along the channels, also when the layer writes a slice of a wider (concatenated) pixel
    const bool wide = (a.Co * ES) % 16 == 0 && (a.ldc * ES) % 16 == 0 && (a.c_off * ES) % 16 == 0;
    const bool has_res = a.res != nullptr;
    const unsigned lds0 = lds_addr(lds);
    // LDS map: ring | residual tile (without one the output tile aliases the ring) | bias
    const unsigned ring = igemm_ring_bytes(ns, nk, STAGE, TILE_O > (KSPL - 1) * 4 * PART ? TILE_O : (KSPL - 1) * 4 * PART);
    const unsigned ro_off = has_res && wide ? ring : 0;
    const unsigned bias_off = has_res && wide ? ring + TILE_O : ring;

    // ---- bias and residual tile: copied first, consumed last --------------------------------------
    igemm_stage_bias_res<ES, BM, BN, NT>(a, lds0, ro_off, bias_off, m0, n0, tid, wave, lane, has_res && wide);

    // ---- per-lane copy state ------------------------------------------------------------------------
    const int lrow = tid / CPRW;
    const int cchunk = (tid % CPRW) ^ ((lrow / R256) & (CPRW - 1));     // the source chunk this lane copies
    unsigned voffB[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) voffB[j] = (unsigned)(n0 + lrow + j * RPP) * (unsigned)KpB + cchunk * 16;
    unsigned voffA[NA];                            // PLAIN: byte offset of the chunk;  else: byte offset of the patch corner
    unsigned maskA[NA];                            // else: bit (r * kw + s) set iff that tap of the row is inside the image
    int tap = 0, ts = 0, tc = 0, toff = 0;         // else: this lane's position inside the patch
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        int m = m0 + lrow + j * RPP;
        const bool live = m < a.M;
        m = live ? m : a.M - 1;
        const unsigned n = fast_div((unsigned)m, (unsigned)(a.Ho * a.Wo), a.magic_howo);
        const unsigned rem = (unsigned)m - n * (unsigned)(a.Ho * a.Wo);
        const unsigned oy = fast_div(rem, (unsigned)a.Wo, a.magic_wo), ox = rem - oy * a.Wo;
        const int iy0 = (int)oy * a.stride - a.pad, ix0 = (int)ox * a.stride - a.pad_w;
        const unsigned nx = a.xs ? (unsigned)a.xs[n] : n;                    // zero-copy compaction: sample n is slot xs[n] of x
        voffA[j] = (unsigned)((((int)nx * a.H + iy0) * a.W + ix0) * CiB);
        if (PLAIN) {
            voffA[j] += cchunk * 16;
            maskA[j] = 0;
        } else {
            // taps s in [s_lo, s_hi) and r in [r_lo, r_hi) fall inside the image; bit r*kw + s of the mask says so
            const int s_lo = max(0, -ix0), s_hi = min(a.kw, a.W - ix0), r_lo = max(0, -iy0), r_hi = min(a.kh, a.H - iy0);
            const unsigned colmask = s_hi > s_lo ? ((1u << s_hi) - 1u) & ~((1u << s_lo) - 1u) : 0u;
            const unsigned rowsel = r_hi > r_lo ? a.tap_rows & ((1u << (r_hi * a.kw)) - 1u) & ~((1u << (r_lo * a.kw)) - 1u) : 0u;
            maskA[j] = live ? colmask * rowsel : 0u;
        }
    }
    const int ntaps = a.kh * a.kw;
    auto advance_tap = [&](int bytes) {             // moves this lane's chunk `bytes` further along the (r, s, c) axis
        tc += bytes;
        toff += bytes;                              // taps of one kernel row are contiguous in NHWC
        while (tc >= CiB) {
            tc -= CiB;
            ++tap;
            if (++ts == a.kw) { ts = 0; toff += (a.W - a.kw) * CiB; }
        }
    };
    if (!PLAIN) advance_tap(cchunk * 16);

    // One piece = one 16-byte-per-lane copy: pieces 0..NA-1 are activation rows, NA..LPT-1 weight rows.
    auto issue_piece = [&](auto piece, unsigned sbase, unsigned tapbit) {
        constexpr int P = decltype(piece)::value;
        if constexpr (P < NA) {
            if (PLAIN) {
                dma16(sbase + P * (NT * 16), xb, voffA[P]);
                voffA[P] += a.plain_step;
            } else {
                const unsigned char* p = (maskA[P] & tapbit) ? xb + (unsigned)(voffA[P] + toff) : zp;
                dma16(sbase + P * (NT * 16), p);
            }
        } else {
            dma16(sbase + BM * KS + (P - NA) * (NT * 16), a.w, voffB[P - NA]);
            voffB[P - NA] += KS;
        }
    };
    auto issue_all = [&](int stage) {
        const unsigned sbase = lds0 + stage * STAGE + wave * 1024;
        const unsigned tapbit = tap < ntaps ? 1u << tap : 0u;
        static_for<LPT>([&](auto piece) { issue_piece(piece, sbase, tapbit); });
        if (!PLAIN) advance_tap(KS);
    };

    // ---- fragment addressing ---------------------------------------------------------------------------
    const int frow = lane & 31, hi = lane >> 5;
    int fragoff[SPW];                              // this wavefront's sub-steps: kpart * SPW + u
#pragma unroll
    for (int u = 0; u < SPW; ++u) fragoff[u] = frow * KS + (((2 * (kpart * SPW + u) + hi) ^ ((frow / R256) & (CPRW - 1))) * 16);

    using acc_t = typename std::conditional<ES == 1, v16i, v16f>::type;
    acc_t acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0;

    // One reduction step out of stage `sc`; with ISSUE the copies of a later step into stage `si` are
    // spread between the matrix instructions so that the copy queue fills while the matrix cores work.
    // Fragments of sub-step u+1 are read while sub-step u multiplies.
    auto step = [&](int sc, int si, auto issue_tag) {
        constexpr bool ISSUE = decltype(issue_tag)::value;
        constexpr int PPS = (LPT + SPW - 1) / SPW;
        const unsigned char* sa = lds + sc * STAGE + wm0 * KS;
        const unsigned char* sb = lds + sc * STAGE + (BM + wn0) * KS;
        const unsigned sbase = lds0 + si * STAGE + wave * 1024;
        const unsigned tapbit = tap < ntaps ? 1u << tap : 0u;
        v4i fw[2][TN], fx[2][TM];
        auto read_frags = [&](int sub, v4i* w, v4i* x) {
#pragma unroll
            for (int j = 0; j < TN; ++j) w[j] = *(const v4i*)(sb + 32 * j * KS + fragoff[sub]);
#pragma unroll
            for (int i = 0; i < TM; ++i) x[i] = *(const v4i*)(sa + 32 * i * KS + fragoff[sub]);
        };
        read_frags(0, fw[0], fx[0]);
        static_for<SPW>([&](auto sub_tag) {
            constexpr int SUB = decltype(sub_tag)::value;
            // fixed order (the scheduler may not move anything across these fences): next fragments, copies,
            // then this sub-step's matrix instructions, which only wait for the fragments read one round earlier
            if constexpr (SUB + 1 < SPW) read_frags(SUB + 1, fw[(SUB + 1) & 1], fx[(SUB + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (ISSUE)
                static_for<PPS>([&](auto q_tag) {
                    constexpr int P = SUB * PPS + decltype(q_tag)::value;
                    if constexpr (P < LPT) issue_piece(std::integral_constant<int, P>{}, sbase, tapbit);
                });
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    if constexpr (ES == 1)
                        acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[SUB & 1][j], fx[SUB & 1][i], acc[j][i], 0, 0, 0);
                    else
                        acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, fw[SUB & 1][j]),
                                                                             __builtin_bit_cast(v8bf, fx[SUB & 1][i]), acc[j][i], 0, 0, 0);
                }
            __builtin_amdgcn_sched_barrier(0);
        });
        if (ISSUE && !PLAIN) advance_tap(KS);
    };

    // ---- the pipelined form of a step (steps of at least four sub-steps, one wavefront group) -----------------
    // A wavefront issues in order, so whatever stands between two matrix instructions delays the second one.
    // Here every matrix instruction is followed by at most one fragment read and one copy, fragments are read
    // FD sub-steps before they are used (into NFB register sets used in turn), and the wait for the next stage
    // plus the workgroup barrier sit FD sub-steps before the end of a step, so that the first fragments of the
    // next step are on their way while this step still multiplies.  Copies of a step are issued in its first
    // SPW - FD sub-steps, i.e. before that barrier: behind it only the ns - 2 later stages are outstanding.
    constexpr bool V2 = EE_IGEMM_PIPELINED && KSPL == 1 && SPW >= 4;
    constexpr int FD = EE_FRAG_DISTANCE, NFB = 4;
    v4i gw[V2 ? NFB : 1][TN], gx[V2 ? NFB : 1][TM];
    auto step2 = [&](int sc, int sn, int si, auto issue_tag, auto last_tag) {
        constexpr bool ISSUE = decltype(issue_tag)::value, LAST = decltype(last_tag)::value;
        constexpr int NM = TN * TM, NR = TN + TM, ISUBS = SPW > FD ? SPW - FD : 1, PPS = (LPT + ISUBS - 1) / ISUBS;
        const unsigned char* sa = lds + sc * STAGE + wm0 * KS;
        const unsigned char* sb = lds + sc * STAGE + (BM + wn0) * KS;
        const unsigned char* na = lds + sn * STAGE + wm0 * KS;
        const unsigned char* nb = lds + sn * STAGE + (BM + wn0) * KS;
        const unsigned sbase = lds0 + si * STAGE + wave * 1024;
        const unsigned tapbit = tap < ntaps ? 1u << tap : 0u;
        static_for<SPW>([&](auto sub_tag) {
            constexpr int SUB = decltype(sub_tag)::value;
            if constexpr (SUB == SPW - FD && !LAST) {
                // the next stage has landed for everybody, and everybody has read the last fragments of the stage
                // before this one (whose slot the next step's copies overwrite)
                if (!ISSUE || ns == 2) wait_all_then_barrier<0>();
                else if (ns == 3) wait_all_then_barrier<LPT>();
                else wait_all_then_barrier<2 * LPT>();
            }
            constexpr int TSUB = SUB + FD;                        // the sub-step whose fragments are read now
            constexpr bool NEXT = TSUB >= SPW;
            constexpr int RS = NEXT ? TSUB - SPW : TSUB;
            constexpr bool DO_READ = !(NEXT && LAST);
            const unsigned char* ra = NEXT ? na : sa;
            const unsigned char* rb = NEXT ? nb : sb;
            static_for<NM>([&](auto q_tag) {
                constexpr int Q = decltype(q_tag)::value, J = Q / TM, I = Q % TM;
                if constexpr (ES == 1)
                    acc[J][I] = __builtin_amdgcn_mfma_i32_32x32x32_i8(gw[SUB % NFB][J], gx[SUB % NFB][I], acc[J][I], 0, 0, 0);
                else
                    acc[J][I] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, gw[SUB % NFB][J]),
                                                                         __builtin_bit_cast(v8bf, gx[SUB % NFB][I]), acc[J][I], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                static_for<(NR + NM - 1) / NM>([&](auto r_tag) {
                    constexpr int R = Q + NM * decltype(r_tag)::value;
                    if constexpr (DO_READ && R < NR) {
                        if constexpr (R < TN) gw[TSUB % NFB][R] = *(const v4i*)(rb + 32 * R * KS + fragoff[RS]);
                        else gx[TSUB % NFB][R - TN] = *(const v4i*)(ra + 32 * (R - TN) * KS + fragoff[RS]);
                    }
                });
                if constexpr (ISSUE && SUB < ISUBS)
                    static_for<(PPS + NM - 1) / NM>([&](auto d_tag) {
                        constexpr int D = Q + NM * decltype(d_tag)::value, P = SUB * PPS + D;
                        if constexpr (D < PPS && P < LPT) issue_piece(std::integral_constant<int, P>{}, sbase, tapbit);
                    });
                __builtin_amdgcn_sched_barrier(0);
            });
        });
        if (ISSUE && !PLAIN) advance_tap(KS);
    };

    // ---- main loop: step ks computes out of stage ks % ns while steps ks+1 .. ks+ns-1 are in flight ----
    for (int s = 0; s < ns - 1; ++s)
        if (s < nk) issue_all(s);
    int st_c = 0, st_i = ns - 1, ks = 0;
    if constexpr (V2) {
        const int ahead = (ns - 1 < nk ? ns - 1 : nk) - 1;      // stages issued behind the first one
        if (ahead <= 0) wait_copies_then_barrier<0>();
        else if (ahead == 1) wait_copies_then_barrier<LPT>();
        else wait_copies_then_barrier<2 * LPT>();
        static_for<FD>([&](auto u_tag) {                // fragments of the first FD sub-steps
            constexpr int U = decltype(u_tag)::value;
#pragma unroll
            for (int j = 0; j < TN; ++j) gw[U][j] = *(const v4i*)(lds + (BM + wn0) * KS + 32 * j * KS + fragoff[U]);
#pragma unroll
            for (int i = 0; i < TM; ++i) gx[U][i] = *(const v4i*)(lds + wm0 * KS + 32 * i * KS + fragoff[U]);
        });
        auto next_of = [&](int st) { return st + 1 == ns ? 0 : st + 1; };
        for (; ks + ns - 1 < nk; ++ks) {
            step2(st_c, next_of(st_c), st_i, std::true_type{}, std::false_type{});
            st_c = next_of(st_c);
            st_i = next_of(st_i);
        }
        for (; ks + 1 < nk; ++ks) {                     // nothing left to copy
            step2(st_c, next_of(st_c), st_c, std::false_type{}, std::false_type{});
            st_c = next_of(st_c);
        }
        step2(st_c, st_c, st_c, std::false_type{}, std::true_type{});
    } else {
    for (; ks + ns - 1 < nk; ++ks) {
        // steps ks+1 .. ks+ns-2 may still be in flight, each LPT copies of this wavefront
        if (ns == 2) wait_copies_then_barrier<0>();
        else if (ns == 3) wait_copies_then_barrier<LPT>();
        else wait_copies_then_barrier<2 * LPT>();
        step(st_c, st_i, std::true_type{});
        st_c = st_c + 1 == ns ? 0 : st_c + 1;
        st_i = st_i + 1 == ns ? 0 : st_i + 1;
    }
    for (; ks < nk; ++ks) {                         // the last ns-1 steps: nothing left to copy
        wait_copies_then_barrier<0>();
        step(st_c, st_c, std::false_type{});
        st_c = st_c + 1 == ns ? 0 : st_c + 1;
    }
    }
    lds_barrier();                                  // every wavefront is done with the ring
    if constexpr (KSPL > 1) {
        // groups 1 .. KSPL-1 park their accumulators in LDS (16 bytes per lane and store: conflict free),
        // group 0 adds them up and alone carries on into the epilogue
        unsigned char* park = lds + ((kpart - 1) * 4 + (wave & 3)) * PART + lane * 16;
        if (kpart > 0) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        v4i v;
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = ES == 1 ? (int)acc[j][i][4 * g + e] : __float_as_int((float)acc[j][i][4 * g + e]);
                        *(v4i*)(park + ((j * TM + i) * 4 + g) * 1024) = v;
                    }
        }
        lds_barrier();
        if (kpart == 0) {
#pragma unroll
            for (int kp = 1; kp < KSPL; ++kp)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const v4i v = *(const v4i*)(lds + ((kp - 1) * 4 + (wave & 3)) * PART + lane * 16 + ((j * TM + i) * 4 + g) * 1024);
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                if constexpr (ES == 1) acc[j][i][4 * g + e] += v[e];
                                else acc[j][i][4 * g + e] += __int_as_float(v[e]);
                            }
                        }
        }
        lds_barrier();                              // the parking area is free again: the output tile may alias it
    }

    igemm_epilogue<ES, BM, BN, NT>(a, acc, lds, ro_off, bias_off, m0, n0, wm0, wn0, tid, has_res, wide, KSPL == 1 || kpart == 0);
}

// ---- launch ------------------------------------------------------------------------------------------------
template <int ES, int BM, int BN, int KS, int KSPL>
static hipError_t launch_igemm_tile(const ConvArgs& a, bool plain, int ns, hipStream_t s)
{
    const int gm = (a.M + BM - 1) / BM, gn = (a.Co + BN - 1) / BN, per_xcd = (gm + 7) / 8;
    const dim3 grid((unsigned)(8 * per_xcd * gn));
    const unsigned magic_gn = (unsigned)(0x100000000ull / (unsigned)gn - (gn == 1));
    const bool res_tile = a.res != nullptr && (a.Co * ES) % 16 == 0;
    const int nk = (a.kh * a.kw * a.Ci * ES + KS - 1) / KS;
    ns = ns < 2 ? 2 : (ns > 4 ? 4 : ns);
    constexpr int TILE_O = BM * BN * ES, PARK = (KSPL - 1) * 4 * (BM / 64) * (BN / 64) * 4096;
    auto lds_need = [&](int stages) { return igemm_ring_bytes(stages, nk, (BM + BN) * KS, TILE_O > PARK ? TILE_O : PARK) + (res_tile ? (size_t)TILE_O : 0) + 1024; };
    while (ns > 2 && lds_need(ns) > 160 * 1024) --ns;      // the deepest ring that fits
    const size_t lds_bytes = lds_need(ns);
    // more than 64 KiB of dynamic LDS has to be granted once per kernel
    static const hipError_t granted = [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_igemm_kernel<ES, BM, BN, KS, KSPL, true>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_igemm_kernel<ES, BM, BN, KS, KSPL, false>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        return e;
    }();
    if (granted != hipSuccess) return granted;
    if (lds_bytes > 160 * 1024) return hipErrorInvalidValue;
    if (plain)
        EE_LAUNCH((conv_igemm_kernel<ES, BM, BN, KS, KSPL, true>), grid, dim3(256 * KSPL), lds_bytes, s, a, gm, gn, magic_gn, per_xcd, ns);
    else
        EE_LAUNCH((conv_igemm_kernel<ES, BM, BN, KS, KSPL, false>), grid, dim3(256 * KSPL), lds_bytes, s, a, gm, gn, magic_gn, per_xcd, ns);
    return hipGetLastError();
}

// cfg: bits 0-3 tile (0 = by shape; 1: 128x128, 2: 128x64, 3: 64x64, 4: 64x128), bits 4-7 reduction step
// (0 = by shape, 1: 64, 2: 128, 3: 256 bytes), bits 8-11 ring stages (0 = by shape, else 2..4), bits 12-15
// wavefront groups splitting the reduction inside a workgroup (0 or 1: none, 2, 4).  Not every combination
// exists: hipErrorInvalidValue for one that does not (or does not fit LDS).
template <int ES>
hipError_t launch_conv_igemm(const ConvArgs& a_in, int cfg, hipStream_t s)
{
    if (a_in.M <= 0) return hipSuccess;
    int tile = cfg & 15, ksel = (cfg >> 4) & 15, ns = (cfg >> 8) & 15, kspl = (cfg >> 12) & 15;
    const int kbytes = a_in.kh * a_in.kw * a_in.Ci * ES;
    if (ksel == 0) ksel = kbytes % 128 == 0 ? 2 : 1;
    const int ks = ksel == 3 ? 256 : (ksel == 2 ? 128 : 64);
    // PLAIN: every reduction step of a row is one contiguous, always valid run of ks bytes: a 1x1 kernel whose
    // pixel is a multiple of the step (the address advances by the step), or an unpadded stride-1 kernel whose
    // kernel row is exactly one step (the address advances by one image row)
    ConvArgs a = a_in;
    const bool plain_1x1 = a.kh == 1 && a.kw == 1 && a.pad == 0 && a.pad_w == 0 && kbytes % ks == 0;
    const bool plain_rows = !plain_1x1 && a.pad == 0 && a.pad_w == 0 && a.stride == 1 && a.kw * a.Ci * ES == ks;
    const bool plain = plain_1x1 || plain_rows;
    a.plain_step = plain_rows ? a.W * a.Ci * ES : ks;
    if (tile == 0) {
        auto blocks = [&](int bm, int bn) { return (long long)((a.M + bm - 1) / bm) * ((a.Co + bn - 1) / bn); };
        const long long want = 2 * 256;
        if (a.Co > 64) tile = blocks(128, 128) >= want ? 1 : (blocks(64, 128) >= want ? 4 : 3);
        else tile = blocks(128, 64) >= want ? 2 : 3;
    }
    if (ns == 0) ns = 2;     // measured: more workgroups per CU beat a deeper ring at these problem sizes
    if (kspl >= 2) {          // measured to pay only for small tiles with the longest step
        if (kspl == 2 && ks == 256 && tile == 3) return launch_igemm_tile<ES, 64, 64, 256, 2>(a, plain, ns, s);
        if (kspl == 2 && ks == 256 && tile == 4) return launch_igemm_tile<ES, 64, 128, 256, 2>(a, plain, ns, s);
        if (kspl == 4 && ks == 256 && tile == 3) return launch_igemm_tile<ES, 64, 64, 256, 4>(a, plain, ns, s);
        return hipErrorInvalidValue;
    }
    if (ks == 256) {
        if (tile == 1) return launch_igemm_tile<ES, 128, 128, 256, 1>(a, plain, ns, s);
        if (tile == 2) return launch_igemm_tile<ES, 128, 64, 256, 1>(a, plain, ns, s);
        if (tile == 4) return launch_igemm_tile<ES, 64, 128, 256, 1>(a, plain, ns, s);
        return launch_igemm_tile<ES, 64, 64, 256, 1>(a, plain, ns, s);
    }
    if (ks == 128) {
        if (tile == 1) return launch_igemm_tile<ES, 128, 128, 128, 1>(a, plain, ns, s);
        if (tile == 2) return launch_igemm_tile<ES, 128, 64, 128, 1>(a, plain, ns, s);
        if (tile == 4) return launch_igemm_tile<ES, 64, 128, 128, 1>(a, plain, ns, s);
        return launch_igemm_tile<ES, 64, 64, 128, 1>(a, plain, ns, s);
    }
    if (tile == 1) return launch_igemm_tile<ES, 128, 128, 64, 1>(a, plain, ns, s);
    if (tile == 2) return launch_igemm_tile<ES, 128, 64, 64, 1>(a, plain, ns, s);
    if (tile == 4) return launch_igemm_tile<ES, 64, 128, 64, 1>(a, plain, ns, s);
    return launch_igemm_tile<ES, 64, 64, 64, 1>(a, plain, ns, s);
}

template hipError_t launch_conv_igemm<1>(const ConvArgs&, int, hipStream_t);
template hipError_t launch_conv_igemm<2>(const ConvArgs&, int, hipStream_t);

}  // namespace ee
