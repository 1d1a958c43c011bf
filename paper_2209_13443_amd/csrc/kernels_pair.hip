// Two convolutions of a bottleneck block in one kernel for gfx950 (CDNA4): a k x k convolution whose output
// channels fit one tile (conv2 of the block), followed by the 1x1 convolution that is its only reader (conv3,
// with the block's residual).  The first result never goes to memory: it is requantised into an LDS tile, which
// is exactly the staged-row layout the matrix cores read, and serves as the activation operand of the second GEMM.
//
// Why: at the batch sizes of the stream these layers are too small to hide their own fill and drain, and the
// 1x1 expansion is bound by memory traffic (it reads a narrow tensor and a wide residual, writes a wide tensor).
// Fusing removes one launch, one write and one read of the narrow tensor, and the expansion's activation
// operand costs no global -> LDS copy at all.  In the paper's terms (Sec. II-C) both layers are GEMMs over the
// same rows R; the tile of rows stays on chip between them.
//
// Phase 1 is the implicit GEMM of kernels_igemm.hip (same ring of asynchronous copies, same fragment layout)
// with BN1 = all output channels of the first layer.  Phase 2 walks the second layer's output channels in chunks
// of BN2: the chunk's weight rows are copied into a two-stage ring behind the tile, multiplied with the tile, and
// the results (bias, residual, requantisation) go into an LDS image of the whole BM x Co3 output block, into
// which the residual was copied at kernel start; the block is stored with 16-byte accesses at the end.  Keeping
// the whole block in LDS means that no global store is outstanding while copies are counted (s_waitcnt vmcnt
// counts both, and stores may complete out of order with loads).
#include "ee_internal.hpp"
#include "igemm_device.hpp"

namespace ee {

// ES: element bytes.  BM: pixel rows per workgroup.  BN1: output channels of the first layer (all of them).
// KS: bytes of the first reduction per ring stage.  BN2: output channels of the second layer per chunk.
template <int ES, int BM, int BN1, int KS, int BN2>
__global__ __launch_bounds__(256) void conv_pair_kernel(PairArgs p, int gm, int per_xcd, int ns)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    constexpr int WM = BM / 2, WN = BN1 / 2, TM = WM / 32, TN = WN / 32;
    constexpr int CPRW = KS / 16, NT = 256, RPP = NT / CPRW;
    constexpr int NA = BM / RPP, NB = BN1 / RPP, LPT = NA + NB;
    constexpr int STAGE = (BM + BN1) * KS;
    constexpr int R256 = KS >= 256 ? 1 : 256 / KS;
    constexpr int NSUB = KS / 32;
    // second GEMM: reduction over the first layer's channels
    constexpr int K2B = BN1 * ES;                          // bytes per row of the tile = reduction bytes
    constexpr int CPRW2 = K2B / 16, R256_2 = K2B >= 256 ? 1 : 256 / K2B;
    constexpr int T_BYTES = BM * K2B, WST2 = BN2 * K2B;
    constexpr int RPP2 = NT / CPRW2, NB2 = BN2 / RPP2;     // weight rows per copy pass, passes per chunk
    constexpr int NSUB2 = K2B / 32;
    constexpr int WN2 = BN2 / 2, TN2 = WN2 / 32;
    static_assert(NA >= 1 && NB >= 1 && BM % RPP == 0 && BN1 % RPP == 0, "tile too small for 256 lanes");
    static_assert(NB2 >= 1 && BN2 % RPP2 == 0 && NB2 <= 32, "second-layer chunk does not split into copy passes");
    static_assert(BN1 * 4 <= 1024, "first-layer bias is copied by one wavefront");

    const ConvArgs& a = p.c2;
    const int xcd = blockIdx.x & 7, mslot = blockIdx.x >> 3;
    const int mt = xcd * per_xcd + mslot;
    if (mt >= gm || mslot >= per_xcd) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave & 1) * WM, wn0 = (wave >> 1) * WN, wn0_2 = (wave >> 1) * WN2;
    const int m0 = mt * BM;
    const unsigned char* xb = (const unsigned char*)a.x;
    const unsigned char* zp = (const unsigned char*)a.zeros;
    const int KpB = a.Kp * ES, Kp3B = p.Kp3 * ES;
    const int nk = (a.kh * a.kw * a.Ci * ES + KS - 1) / KS;
    const int CiB = a.Ci * ES;
    const bool has_res = p.res != nullptr;
    const unsigned lds0 = lds_addr(lds);
    const int CR2 = p.Co3 * ES / 16;                       // 16-byte chunks per row of the output block (>= 16)
    const int OROW2 = p.Co3 * ES;
    const int NC = p.Co3 / BN2;
    // LDS map: [ring of phase 1 | tile + weight ring of phase 2] [output block] [bias 1] [bias 2]
    const unsigned ring1 = (unsigned)((ns < nk ? ns : nk) * STAGE);
    const unsigned region_a = ring1 > (unsigned)(T_BYTES + 2 * WST2) ? ring1 : (unsigned)(T_BYTES + 2 * WST2);
    const unsigned out_off = region_a;
    const unsigned bias1_off = out_off + (unsigned)BM * OROW2;
    const unsigned bias3_off = bias1_off + 1024;

    // ---- biases and the residual block: copied first, consumed last ----------------------------------------
    if (wave == 0) dma16(lds0 + bias1_off, (const unsigned char*)a.bias + lane * 16);
    for (int off = wave * 1024; off < p.Co3 * 4; off += 4096) dma16(lds0 + bias3_off + off, (const unsigned char*)p.bias3 + off + lane * 16);
    if (has_res) {
        // position q of the block (row q / CR2, slot q % CR2) holds chunk slot ^ (row & 15) of that row
        for (int base = 0; base < BM * CR2; base += NT) {
            const int q = base + tid, row = q / CR2, chunk = (q % CR2) ^ (row & 15);
            const int m = m0 + row;
            const unsigned char* src = m < a.M ? (const unsigned char*)p.res + ((size_t)m * p.Co3) * ES + chunk * 16 : zp;
            dma16(lds0 + out_off + (base + 64 * wave) * 16, src);
        }
    }

    // ---- phase 1: per-lane copy state (the general loader: any kernel, padding by masks) ---------------------
    const int lrow = tid / CPRW;
    const int cchunk = (tid % CPRW) ^ ((lrow / R256) & (CPRW - 1));
    unsigned voffB[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) voffB[j] = (unsigned)(lrow + j * RPP) * (unsigned)KpB + cchunk * 16;
    unsigned voffA[NA], maskA[NA];
    int tap = 0, ts = 0, tc = 0, toff = 0;
#pragma unroll
    for (int j = 0; j < NA; ++j) {
        int m = m0 + lrow + j * RPP;
        const bool live = m < a.M;
        m = live ? m : a.M - 1;
        const unsigned n = fast_div((unsigned)m, (unsigned)(a.Ho * a.Wo), a.magic_howo);
        const unsigned rem = (unsigned)m - n * (unsigned)(a.Ho * a.Wo);
        const unsigned oy = fast_div(rem, (unsigned)a.Wo, a.magic_wo), ox = rem - oy * a.Wo;
        const int iy0 = (int)oy * a.stride - a.pad, ix0 = (int)ox * a.stride - a.pad_w;
        voffA[j] = (unsigned)((((int)n * a.H + iy0) * a.W + ix0) * CiB);
        const int s_lo = max(0, -ix0), s_hi = min(a.kw, a.W - ix0), r_lo = max(0, -iy0), r_hi = min(a.kh, a.H - iy0);
        const unsigned colmask = s_hi > s_lo ? ((1u << s_hi) - 1u) & ~((1u << s_lo) - 1u) : 0u;
        const unsigned rowsel = r_hi > r_lo ? a.tap_rows & ((1u << (r_hi * a.kw)) - 1u) & ~((1u << (r_lo * a.kw)) - 1u) : 0u;
        maskA[j] = live ? colmask * rowsel : 0u;
    }
    const int ntaps = a.kh * a.kw;
    auto advance_tap = [&](int bytes) {
        tc += bytes;
        toff += bytes;
        while (tc >= CiB) {
            tc -= CiB;
            ++tap;
            if (++ts == a.kw) { ts = 0; toff += (a.W - a.kw) * CiB; }
        }
    };
    advance_tap(cchunk * 16);

    auto issue_piece = [&](auto piece, unsigned sbase, unsigned tapbit) {
        constexpr int P = decltype(piece)::value;
        if constexpr (P < NA) {
            const unsigned char* src = (maskA[P] & tapbit) ? xb + (unsigned)(voffA[P] + toff) : zp;
            dma16(sbase + P * (NT * 16), src);
        } else {
            dma16(sbase + BM * KS + (P - NA) * (NT * 16), a.w, voffB[P - NA]);
            voffB[P - NA] += KS;
        }
    };
    auto issue_all = [&](int stage) {
        const unsigned sbase = lds0 + stage * STAGE + wave * 1024;
        const unsigned tapbit = tap < ntaps ? 1u << tap : 0u;
        static_for<LPT>([&](auto piece) { issue_piece(piece, sbase, tapbit); });
        advance_tap(KS);
    };

    const int frow = lane & 31, hi = lane >> 5;
    int fragoff[NSUB];
#pragma unroll
    for (int u = 0; u < NSUB; ++u) fragoff[u] = frow * KS + (((2 * u + hi) ^ ((frow / R256) & (CPRW - 1))) * 16);

    // second-layer weight rows [c * BN2, +BN2) into stage c & 1 of the two-stage ring behind the tile; as in a ring
    // stage of phase 1, the lane that fills chunk position s of staged row r copies source chunk s ^ swizzle(r)
    const int lrow2 = tid / CPRW2;
    auto issue_w3 = [&](int c) {
        const unsigned sbase = lds0 + T_BYTES + (c & 1) * WST2 + wave * 1024;
#pragma unroll
        for (int j = 0; j < NB2; ++j) {
            const int row = lrow2 + j * RPP2;
            const int chunk = (tid % CPRW2) ^ ((row / R256_2) & (CPRW2 - 1));
            dma16(sbase + j * (NT * 16), p.w3, (unsigned)(c * BN2 + row) * (unsigned)Kp3B + chunk * 16);
        }
    };

    using acc_t = typename std::conditional<ES == 1, v16i, v16f>::type;
    auto mfma = [](const v4i& w, const v4i& x, acc_t c) -> acc_t {
        if constexpr (ES == 1) return __builtin_amdgcn_mfma_i32_32x32x32_i8(w, x, c, 0, 0, 0);
        else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, w), __builtin_bit_cast(v8bf, x), c, 0, 0, 0);
    };
    {
        acc_t acc[TN][TM];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[j][i][v] = 0;

        auto step = [&](int sc, int si, auto issue_tag) {
            constexpr bool ISSUE = decltype(issue_tag)::value;
            constexpr int PPS = (LPT + NSUB - 1) / NSUB;
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
            static_for<NSUB>([&](auto sub_tag) {
                constexpr int SUB = decltype(sub_tag)::value;
                if constexpr (SUB + 1 < NSUB) read_frags(SUB + 1, fw[(SUB + 1) & 1], fx[(SUB + 1) & 1]);
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
                    for (int i = 0; i < TM; ++i) acc[j][i] = mfma(fw[SUB & 1][j], fx[SUB & 1][i], acc[j][i]);
                __builtin_amdgcn_sched_barrier(0);
            });
            if (ISSUE) advance_tap(KS);
        };

        for (int s = 0; s < ns - 1; ++s)
            if (s < nk) issue_all(s);
        int st_c = 0, st_i = ns - 1, ks = 0;
        for (; ks + ns - 1 < nk; ++ks) {
            if (ns == 2) wait_copies_then_barrier<0>();
            else if (ns == 3) wait_copies_then_barrier<LPT>();
            else wait_copies_then_barrier<2 * LPT>();
            step(st_c, st_i, std::true_type{});
            st_c = st_c + 1 == ns ? 0 : st_c + 1;
            st_i = st_i + 1 == ns ? 0 : st_i + 1;
        }
        for (; ks < nk; ++ks) {
            wait_copies_then_barrier<0>();
            step(st_c, st_c, std::false_type{});
            st_c = st_c + 1 == ns ? 0 : st_c + 1;
        }
        lds_barrier();                              // every wavefront is done with the ring, no copy is outstanding

        // the first two weight chunks of the second layer travel while the tile is written (their stages lie behind it)
        issue_w3(0);
        if (NC > 1) issue_w3(1);

        // ---- phase 1 epilogue: bias, requantisation, into the tile in staged-row layout -------------------------
        // tile row r, 16-byte chunk c sits at chunk position c ^ ((r / R256_2) & (CPRW2 - 1)); the swizzle only
        // depends on r % 32, i.e. on the lane
        const int* lbias1 = (const int*)(lds + bias1_off);
        const int swz_t = (frow / R256_2) & (CPRW2 - 1);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            unsigned char* rowp = lds + (wm0 + 32 * i + frow) * K2B + 4 * hi * ES;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int cl = wn0 + 32 * j + 8 * g + 4 * hi;
                    const int chunk = (wn0 * ES >> 4) + ((32 * j + 8 * g) * ES >> 4);
                    unsigned char* cell = rowp + ((chunk ^ swz_t) << 4) + (((32 * j + 8 * g) * ES) & 15);
                    const v4i b4 = *(const v4i*)(lbias1 + cl);
                    if constexpr (ES == 1) {
                        int q[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) q[e] = clamp_i32((acc[j][i][4 * g + e] + b4[e]) >> a.shift, a.lo, a.hi);
                        *(unsigned*)cell = pack4_i8(q[0], q[1], q[2], q[3]);
                    } else {
                        float t[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) t[e] = fminf(fmaxf(acc[j][i][4 * g + e] + __int_as_float(b4[e]), a.f_lo), a.f_hi);
                        uint2 out;
                        out.x = to_bf16_rne(t[0]) | (to_bf16_rne(t[1]) << 16);
                        out.y = to_bf16_rne(t[2]) | (to_bf16_rne(t[3]) << 16);
                        *(uint2*)cell = out;
                    }
                }
        }
    }

    // ---- phase 2: tile x second-layer weights, chunk by chunk -------------------------------------------------
    const int swz2 = (frow / R256_2) & (CPRW2 - 1);
    const int* lbias3 = (const int*)(lds + bias3_off);
    unsigned char* ob = lds + out_off;
    const int swz_o = frow & 15;
    for (int c = 0; c < NC; ++c) {
        // chunk c's weights are there (the next chunk's copies may still fly); the first time round this is also
        // the barrier that publishes the tile
        if (c + 1 < NC) wait_all_then_barrier<NB2>();
        else wait_all_then_barrier<0>();
        acc_t acc2[TN2][TM];
#pragma unroll
        for (int j = 0; j < TN2; ++j)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc2[j][i][v] = 0;
        const unsigned char* sa = lds + wm0 * K2B + frow * K2B;
        const unsigned char* sb = lds + T_BYTES + (c & 1) * WST2 + wn0_2 * K2B + frow * K2B;
        v4i fw[2][TN2], fx[2][TM];
        auto read2 = [&](int sub, v4i* w, v4i* x) {
            const int o = ((2 * sub + hi) ^ swz2) << 4;
#pragma unroll
            for (int j = 0; j < TN2; ++j) w[j] = *(const v4i*)(sb + 32 * j * K2B + o);
#pragma unroll
            for (int i = 0; i < TM; ++i) x[i] = *(const v4i*)(sa + 32 * i * K2B + o);
        };
        read2(0, fw[0], fx[0]);
        static_for<NSUB2>([&](auto sub_tag) {
            constexpr int SUB = decltype(sub_tag)::value;
            if constexpr (SUB + 1 < NSUB2) read2(SUB + 1, fw[(SUB + 1) & 1], fx[(SUB + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < TN2; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i) acc2[j][i] = mfma(fw[SUB & 1][j], fx[SUB & 1][i], acc2[j][i]);
            __builtin_amdgcn_sched_barrier(0);
        });
        lds_barrier();                              // every wavefront is done with this weight stage
        if (c + 2 < NC) issue_w3(c + 2);

        // epilogue of the chunk: bias, residual (already in the cell), requantisation, back into the cell.
        // Output-block cell of (row r, channel ch): chunk (ch * ES / 16) ^ (r & 15) of row r.
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            unsigned char* rowp = ob + (size_t)(wm0 + 32 * i + frow) * OROW2 + 4 * hi * ES;
#pragma unroll
            for (int j = 0; j < TN2; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int ch0 = c * BN2 + wn0_2 + 32 * j + 8 * g;              // wave-uniform; the lane's 4 channels start at ch0 + 4 * hi
                    unsigned char* cell = rowp + ((((ch0 * ES) >> 4) ^ swz_o) << 4) + ((ch0 * ES) & 15);
                    const v4i b4 = *(const v4i*)(lbias3 + ch0 + 4 * hi);
                    if constexpr (ES == 1) {
                        const int packed = has_res ? *(const int*)cell : 0;
                        int q[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            int t = acc2[j][i][4 * g + e] + b4[e];
                            t += __builtin_amdgcn_sbfe(packed, 8 * e, 8) << p.res_shift;   // packed = 0 without a residual
                            q[e] = clamp_i32(t >> p.shift, p.lo, p.hi);
                        }
                        *(unsigned*)cell = pack4_i8(q[0], q[1], q[2], q[3]);
                    } else {
                        uint2 packed = {0u, 0u};
                        if (has_res) packed = *(const uint2*)cell;
                        const float r0 = __uint_as_float(packed.x << 16), r1 = __uint_as_float(packed.x & 0xFFFF0000u);
                        const float r2 = __uint_as_float(packed.y << 16), r3 = __uint_as_float(packed.y & 0xFFFF0000u);
                        float t0 = acc2[j][i][4 * g + 0] + __int_as_float(b4[0]), t1 = acc2[j][i][4 * g + 1] + __int_as_float(b4[1]);
                        float t2 = acc2[j][i][4 * g + 2] + __int_as_float(b4[2]), t3 = acc2[j][i][4 * g + 3] + __int_as_float(b4[3]);
                        if (has_res) { t0 += r0; t1 += r1; t2 += r2; t3 += r3; }
                        t0 = fminf(fmaxf(t0, p.f_lo), p.f_hi); t1 = fminf(fmaxf(t1, p.f_lo), p.f_hi);
                        t2 = fminf(fmaxf(t2, p.f_lo), p.f_hi); t3 = fminf(fmaxf(t3, p.f_lo), p.f_hi);
                        uint2 out;
                        out.x = to_bf16_rne(t0) | (to_bf16_rne(t1) << 16);
                        out.y = to_bf16_rne(t2) | (to_bf16_rne(t3) << 16);
                        *(uint2*)cell = out;
                    }
                }
        }
    }
    lds_barrier();
    for (int q = tid; q < BM * CR2; q += NT) {
        const int row = q / CR2, chunk = (q % CR2) ^ (row & 15);
        const int m = m0 + row;
        if (m < a.M) *(v4i*)((unsigned char*)p.y + ((size_t)m * p.Co3) * ES + chunk * 16) = *(const v4i*)(ob + (size_t)q * 16);
    }
}

// ---- launch ---------------------------------------------------------------------------------------------------
size_t conv_pair_lds_bytes(int es, int bm, int bn1, int ks, int bn2, int ns, int nk, int co3)
{
    const size_t ring1 = (size_t)(ns < nk ? ns : nk) * (bm + bn1) * ks;
    const size_t phase2 = (size_t)bm * bn1 * es + 2 * (size_t)bn2 * bn1 * es;
    return (ring1 > phase2 ? ring1 : phase2) + (size_t)bm * co3 * es + 1024 + (((size_t)co3 * 4 + 1023) / 1024) * 1024;
}

template <int ES, int BM, int BN1, int KS>
static hipError_t launch_pair_tile(const PairArgs& p, int ns, hipStream_t s)
{
    constexpr int BN2 = 128;
    const ConvArgs& a = p.c2;
    const int gm = (a.M + BM - 1) / BM, per_xcd = (gm + 7) / 8;
    const int nk = (a.kh * a.kw * a.Ci * ES + KS - 1) / KS;
    ns = ns < 2 ? 2 : (ns > 4 ? 4 : ns);
    const size_t lds_bytes = conv_pair_lds_bytes(ES, BM, BN1, KS, BN2, ns, nk, p.Co3);
    static const hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_pair_kernel<ES, BM, BN1, KS, BN2>),
                                                          hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (granted != hipSuccess) return granted;
    if (lds_bytes > 160 * 1024) return hipErrorInvalidValue;
    EE_LAUNCH((conv_pair_kernel<ES, BM, BN1, KS, BN2>), dim3((unsigned)(8 * per_xcd)), dim3(256), lds_bytes, s, p, gm, per_xcd, ns);
    return hipGetLastError();
}

// cfg: bits 0-3 rows per workgroup (1: 128, 2: 64; 0 = by shape), bits 4-7 reduction step of the first layer
// (1: 64, 2: 128 bytes; 0 = by shape), bits 8-11 ring stages (0 = 2).  hipErrorInvalidValue for a pair this kernel does
// not take (see conv_pair_supported) or a configuration that does not exist or does not fit LDS.
template <int ES>
hipError_t launch_conv_pair(const PairArgs& p, int cfg, hipStream_t s)
{
    const ConvArgs& a = p.c2;
    if (a.M <= 0) return hipSuccess;
    if (!conv_pair_supported(ES, a.Co, a.kh, a.kw, a.Ci, p.Co3)) return hipErrorInvalidValue;
    int tile = cfg & 15, ksel = (cfg >> 4) & 15, ns = (cfg >> 8) & 15;
    if (ksel == 0) ksel = 1;
    if (ns == 0) ns = 2;
    if (tile == 0) {        // 128 rows when that leaves two workgroups per CU and fits LDS, else 64
        const int nk = (a.kh * a.kw * a.Ci * ES + 63) / 64;
        const bool fits = conv_pair_lds_bytes(ES, 128, a.Co, 64, 128, ns, nk, p.Co3) <= 160 * 1024;
        tile = a.Co >= 256 || !fits || (a.M + 127) / 128 < 2 * 256 ? 2 : 1;
    }
    if (tile < 1 || tile > 2 || ksel < 1 || ksel > 2) return hipErrorInvalidValue;
    const int bm = tile == 1 ? 128 : 64, ks = ksel == 1 ? 64 : 128;
#define EE_PAIR(BM_, BN1_, KS_) if (bm == BM_ && a.Co == BN1_ && ks == KS_) return launch_pair_tile<ES, BM_, BN1_, KS_>(p, ns, s);
    EE_PAIR(128, 64, 64) EE_PAIR(128, 64, 128) EE_PAIR(64, 64, 64) EE_PAIR(64, 64, 128)
    EE_PAIR(128, 128, 64) EE_PAIR(128, 128, 128) EE_PAIR(64, 128, 64) EE_PAIR(64, 128, 128)
    EE_PAIR(64, 256, 64) EE_PAIR(64, 256, 128)
#undef EE_PAIR
    return hipErrorInvalidValue;
}

// A pair the fused kernel takes: the first layer's output channels are one tile (64, 128 or 256), its kernel fits the
// tap masks, rows are whole 16-byte chunks, and the second layer's output splits into chunks of 128 channels.
bool conv_pair_supported(int es, int co2, int kh, int kw, int ci, int co3)
{
    if (co2 != 64 && co2 != 128 && co2 != 256) return false;
    if (kh * kw > 31 || (ci * es) % 16 != 0) return false;
    if (co3 % 128 != 0 || (co3 * es) % 256 != 0) return false;      // chunks of 128 channels; rows of whole 256-byte groups
    return conv_pair_lds_bytes(es, 64, co2, 64, 128, 2, 2, co3) <= 160 * 1024;   // the smallest configuration must fit LDS
}

template hipError_t launch_conv_pair<1>(const PairArgs&, int, hipStream_t);
template hipError_t launch_conv_pair<2>(const PairArgs&, int, hipStream_t);

}  // namespace ee
