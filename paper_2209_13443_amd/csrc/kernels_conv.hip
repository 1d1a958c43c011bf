// Convolution kernels for gfx950 (CDNA4): implicit GEMM on the matrix cores.
//
// Every CONV layer is the GEMM  R x P . P x C -> R x C  of the paper's Sec. II-C with the batch
// appended along R (R-batching, Sec. III-A); here the Toeplitz matrix is never materialised:
// rows (output pixels) are gathered straight from the NHWC activation tensor while the K loop
// walks over (r, s, c).
//
// Tiling: a workgroup of 4 wavefronts (256 lanes) owns BM output pixels x BN output channels.
// Per 128-byte k-step both operands are staged in LDS (rows padded to 144 bytes so that the
// 16-lane phases of a ds_read_b128 hit 64 distinct banks); the next step's global loads are
// issued into registers before the current step's MFMAs, and several workgroups per CU overlap
// each other's barriers and memory latency.
// Each wavefront computes WM x WN outputs with v_mfma_i32_32x32x32_i8 (int8) or
// v_mfma_f32_32x32x16_bf16 (bf16).  The weight fragment is the A operand and the activation
// fragment the B operand, so that one lane ends up holding 4 consecutive output channels of
// one pixel per accumulator quad -- a packed store in NHWC.
//
// Operand layout assumed for the 32x32 MFMAs (lane l, 16 bytes per lane):
//   A: row l%32, k-bytes [16*(l/32), 16*(l/32)+16)      B: column l%32, same k-bytes
//   D: column l%32, rows 8*(v/4) + 4*(l/32) + v%4 for accumulator register v = 0..15
// (the k order inside an instruction is irrelevant as long as A and B agree).
#include <type_traits>

#include <cstring>

#include "ee_internal.hpp"

namespace ee {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kStep = 128;                 // bytes of the reduction axis staged per barrier
constexpr int kLdsRow = kStep + 16;        // staged row + 16 bytes of padding (conflict-free ds_read_b128)

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ __forceinline__ int requant_i8(int t, int shift, int lo, int hi)
{
    int q = shift > 0 ? (t + (1 << (shift - 1))) >> shift : t;
    return min(max(q, lo), hi);
}

// ES = element size in bytes (1: int8, 2: bf16).  MODE 0: generic NHWC input with C*ES % 16 == 0,
// bounds-checked taps.  MODE 1: 4-channel input already zero-padded in space ([Hp][Wp][4]); a kernel
// row of kwp taps is kwp*4*ES contiguous bytes, no bounds checks.
//
// Workgroup -> tile mapping: consecutive workgroup ids go round-robin to the 8 XCDs, each with its
// own L2.  Tile rows (pixel tiles) are split into 8 contiguous ranges, one per XCD, and all the
// channel tiles of a pixel tile run back to back on the same XCD, so the activation rows a tile
// reads (and the halo rows its neighbours share) stay in one L2.
template <int ES, int BM, int BN, int WM, int WN, int MODE>
__global__ __launch_bounds__(256) void conv_mfma_kernel(ConvArgs a, int gm, int gn, int per_xcd)
{
    constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
    static_assert(WAVES_M * WAVES_N == 4, "4 wavefronts per workgroup");
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int A_PER_T = BM / 32, B_PER_T = BN / 32;
    constexpr int OROW = BN * ES + 16;                    // epilogue tile row: BN outputs + padding
    constexpr int kMainBytes = (BM + BN) * kLdsRow, kEpiBytes = BM * OROW;
    __shared__ __attribute__((aligned(16))) unsigned char lds[kMainBytes > kEpiBytes ? kMainBytes : kEpiBytes];

    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int mt = xcd * per_xcd + slot / gn, nt = slot % gn;
    if (mt >= gm || slot / gn >= per_xcd) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
    const int m0 = mt * BM, n0 = nt * BN;
    const int cc = tid & 7, row_base = tid >> 3;
    const unsigned char* xb = (const unsigned char*)a.x;
    const unsigned char* wb = (const unsigned char*)a.w;
    const int KpB = a.Kp * ES;                            // padded reduction length in bytes (multiple of 64)
    const int nk = (KpB + kStep - 1) / kStep;
    const int HoWo = a.Ho * a.Wo;

    // ---- per-thread loader state -------------------------------------------------------------
    long long a_off[A_PER_T];     // MODE 0: byte offset of pixel (n, 0, 0); MODE 1: byte offset of the patch corner
    int a_iy0[A_PER_T], a_ix0[A_PER_T];
#pragma unroll
    for (int i = 0; i < A_PER_T; ++i) {
        int m = m0 + row_base + 32 * i;
        m = m < a.M ? m : a.M - 1;                       // rows past the end repeat the last pixel; never stored
        const int n = m / HoWo, rem = m - n * HoWo;
        const int oy = rem / a.Wo, ox = rem - oy * a.Wo;
        if (MODE == 0) {
            a_off[i] = (long long)n * a.H * a.W * a.Ci * ES;
            a_iy0[i] = oy * a.stride - a.pad;
            a_ix0[i] = ox * a.stride - a.pad;
        } else {
            a_off[i] = (((long long)n * a.Hp + oy * a.stride) * a.Wp + ox * a.stride) * 4 * ES;
            a_iy0[i] = a_ix0[i] = 0;
        }
    }
    const int CiB = a.Ci * ES;                           // bytes per input pixel (MODE 0)
    int tr, ts, tc;                                      // MODE 0: tap (r, s) and byte offset inside the pixel
    int prow, ppart;                                     // MODE 1: kernel row and 16-byte part inside it
    const int cpr = MODE == 1 ? a.kwp * 4 * ES / 16 : 1; // MODE 1: 16-byte chunks per kernel row
    if (MODE == 0) {
        const int kb = cc * 16;
        const int tap = kb / CiB;
        tc = kb - tap * CiB;
        tr = tap / a.kw;
        ts = tap - tr * a.kw;
        prow = ppart = 0;
    } else {
        prow = cc / cpr;
        ppart = cc - prow * cpr;
        tr = ts = tc = 0;
    }

    v4i ra[A_PER_T], rb[B_PER_T];
    auto load_global = [&](int ks) {
        const bool k_ok = ks * kStep + cc * 16 < KpB;     // the last step may be half empty
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) {
            v4i v = {0, 0, 0, 0};
            if (MODE == 0) {
                const int iy = a_iy0[i] + tr, ix = a_ix0[i] + ts;
                const bool ok = tr < a.kh && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
                if (ok) v = *(const v4i*)(xb + a_off[i] + ((long long)iy * a.W + ix) * CiB + tc);
            } else if (k_ok) {
                const int r = prow < a.kh ? prow : a.kh - 1;      // k padding: real bytes times zero weights
                const int* q = (const int*)(xb + a_off[i] + (long long)r * a.Wp * 4 * ES + ppart * 16);   // 4-byte aligned only
                v = v4i{q[0], q[1], q[2], q[3]};
            }
            ra[i] = v;
        }
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) {
            v4i v = {0, 0, 0, 0};
            if (k_ok) v = *(const v4i*)(wb + (long long)(n0 + row_base + 32 * i) * KpB + ks * kStep + cc * 16);
            rb[i] = v;
        }
        // advance the tap state by one k-step
        if (MODE == 0) {
            tc += kStep;
            while (tc >= CiB) {
                tc -= CiB;
                if (++ts == a.kw) { ts = 0; ++tr; }
            }
        } else {
            ppart += kStep / 16;
            while (ppart >= cpr) { ppart -= cpr; ++prow; }
        }
    };
    auto store_lds = [&]() {
#pragma unroll
        for (int i = 0; i < A_PER_T; ++i) *(v4i*)(&lds[(row_base + 32 * i) * kLdsRow + cc * 16]) = ra[i];
#pragma unroll
        for (int i = 0; i < B_PER_T; ++i) *(v4i*)(&lds[(BM + row_base + 32 * i) * kLdsRow + cc * 16]) = rb[i];
    };

    using acc_t = typename std::conditional<ES == 1, v16i, v16f>::type;
    acc_t acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0;

    // ---- main loop: registers hold step ks+1 while the matrix cores work on step ks out of LDS ----
    load_global(0);
    const int frag_row = lane & 31, frag_k = (lane >> 5) * 16;
    for (int ks = 0; ks < nk; ++ks) {
        store_lds();
        __syncthreads();
        if (ks + 1 < nk) load_global(ks + 1);
        const int nsub = min(4, (KpB - ks * kStep) / 32);
        for (int sub = 0; sub < nsub; ++sub) {
            v4i fw[TN], fx[TM];
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fw[j] = *(const v4i*)(&lds[(BM + wn0 + 32 * j + frag_row) * kLdsRow + sub * 32 + frag_k]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fx[i] = *(const v4i*)(&lds[(wm0 + 32 * i + frag_row) * kLdsRow + sub * 32 + frag_k]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    if constexpr (ES == 1)
                        acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[j], fx[i], acc[j][i], 0, 0, 0);
                    else
                        acc[j][i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, fw[j]),
                                                                             __builtin_bit_cast(v8bf, fx[i]), acc[j][i], 0, 0, 0);
                }
        }
        __syncthreads();
    }

    // ---- epilogue: bias, residual, requantise / clamp ---------------------------------------------
    // Fast path (rows of C_out are 16-byte multiples): the tile goes through LDS so that the residual
    // is read and the result written with 16 bytes per lane along the channel axis (whole cache
    // lines); each lane patches its own 4 outputs in place in between.
    const bool wide = (a.Co * ES) % 16 == 0;
    constexpr int CPR = BN * ES / 16;                     // 16-byte chunks per tile row
    if (wide && a.res) {
        for (int id = tid; id < BM * CPR; id += 256) {
            const int r = id / CPR, c16 = id - r * CPR;
            const int m = m0 + r, ch = n0 + c16 * (16 / ES);
            if (m < a.M && ch < a.Co)
                *(v4i*)(&lds[r * OROW + c16 * 16]) = *(const v4i*)((const unsigned char*)a.res + ((long long)m * a.Co + ch) * ES);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int r = wm0 + 32 * i + (lane & 31);
        const int m = m0 + r;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int cl = wn0 + 32 * j + 8 * g + 4 * (lane >> 5);
                const int c0 = n0 + cl;
                if (m >= a.M || c0 >= a.Co) continue;
                const long long o = (long long)m * a.Co + c0;
                unsigned char* tile = &lds[r * OROW + cl * ES];
                if constexpr (ES == 1) {
                    const v4i bias = *(const v4i*)((const int*)a.bias + c0);
                    int packed = 0;
                    if (a.res) packed = wide ? *(const int*)tile : *(const int*)((const signed char*)a.res + o);
                    unsigned out = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int rv = (int)(signed char)((packed >> (8 * e)) & 0xFF);
                        const int t = acc[j][i][4 * g + e] + bias[e] + (rv << a.res_shift);
                        out |= (unsigned)(requant_i8(t, a.shift, a.lo, a.hi) & 0xFF) << (8 * e);
                    }
                    if (wide) *(unsigned*)tile = out;
                    else *(unsigned*)((signed char*)a.y + o) = out;
                } else {
                    const float* bias = (const float*)a.bias + c0;
                    uint2 packed = {0u, 0u};
                    if (a.res) packed = wide ? *(const uint2*)tile : *(const uint2*)((const uint16_t*)a.res + o);
                    const uint16_t r4[4] = {(uint16_t)(packed.x & 0xFFFF), (uint16_t)(packed.x >> 16),
                                            (uint16_t)(packed.y & 0xFFFF), (uint16_t)(packed.y >> 16)};
                    uint16_t q[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float t = acc[j][i][4 * g + e] + bias[e];
                        if (a.res) t = t + bf16_to_f32(r4[e]);
                        t = fminf(fmaxf(t, a.f_lo), a.f_hi);
                        q[e] = f32_to_bf16_rne(t);
                    }
                    uint2 out;
                    out.x = (unsigned)q[0] | ((unsigned)q[1] << 16);
                    out.y = (unsigned)q[2] | ((unsigned)q[3] << 16);
                    if (wide) *(uint2*)tile = out;
                    else *(uint2*)((uint16_t*)a.y + o) = out;
                }
            }
    }
    if (wide) {
        __syncthreads();
        for (int id = tid; id < BM * CPR; id += 256) {
            const int r = id / CPR, c16 = id - r * CPR;
            const int m = m0 + r, ch = n0 + c16 * (16 / ES);
            if (m < a.M && ch < a.Co)
                *(v4i*)((unsigned char*)a.y + ((long long)m * a.Co + ch) * ES) = *(const v4i*)(&lds[r * OROW + c16 * 16]);
        }
    }
}

template <int ES, int BM, int BN, int WM, int WN>
static hipError_t launch_tile(const ConvArgs& a, hipStream_t s)
{
    const int gm = (a.M + BM - 1) / BM, gn = (a.Co + BN - 1) / BN, per_xcd = (gm + 7) / 8;
    dim3 grid((unsigned)(8 * per_xcd * gn));
    if (a.mode == 0)
        EE_LAUNCH((conv_mfma_kernel<ES, BM, BN, WM, WN, 0>), grid, dim3(256), 0, s, a, gm, gn, per_xcd);
    else
        EE_LAUNCH((conv_mfma_kernel<ES, BM, BN, WM, WN, 1>), grid, dim3(256), 0, s, a, gm, gn, per_xcd);
    return hipGetLastError();
}

// Tile choice per layer and active batch size: the widest tile that still gives every CU a few
// workgroups to overlap (the GPU face of the paper's per-layer, per-batch-size mapping problem,
// Sec. III-A).  Tiles are output pixels x output channels.
static int g_forced_tile = 0;    // 0 = by shape; 1: 128x128, 2: 128x64, 3: 64x64, 4: 64x128 (tuning / test control)
int set_conv_tile(int tile) { const int old = g_forced_tile; g_forced_tile = tile; return old; }
int forced_conv_tile() { return g_forced_tile; }

template <int ES>
static hipError_t launch_conv_mfma(const ConvArgs& a, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    int tile = g_forced_tile & 15;
    if (tile == 0 || tile > 4) {
        auto blocks = [&](int bm, int bn) { return (long long)((a.M + bm - 1) / bm) * ((a.Co + bn - 1) / bn); };
        const long long want = 3 * 256;
        if (a.Co > 64) tile = blocks(128, 128) >= want ? 1 : (blocks(64, 128) >= want ? 4 : 3);
        else tile = blocks(128, 64) >= want ? 2 : 3;
    }
    if (tile == 1) return launch_tile<ES, 128, 128, 64, 64>(a, s);
    if (tile == 2) return launch_tile<ES, 128, 64, 64, 32>(a, s);
    if (tile == 4) return launch_tile<ES, 64, 128, 32, 64>(a, s);
    return launch_tile<ES, 64, 64, 32, 32>(a, s);
}

hipError_t launch_conv_mfma_i8(const ConvArgs& a, hipStream_t s) { return launch_conv_mfma<1>(a, s); }
hipError_t launch_conv_mfma_bf16(const ConvArgs& a, hipStream_t s) { return launch_conv_mfma<2>(a, s); }

// ---- fallback: one thread per output element, any shape ----------------------------------------
template <int ES>
__global__ __launch_bounds__(256) void conv_direct_kernel(DirectConvArgs a)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)a.M * a.Co) return;
    const int co = (int)(idx % a.Co);
    const int m = (int)(idx / a.Co);
    const int HoWo = a.Ho * a.Wo;
    const int n = m / HoWo, rem = m - n * HoWo, oy = rem / a.Wo, ox = rem - oy * a.Wo;
    const long long odx = (long long)m * a.ldc + a.c_off + co;       // the output may be a channel slice of a wider pixel
    if constexpr (ES == 1) {
        const signed char* x = (const signed char*)a.x;
        const signed char* w = (const signed char*)a.w + (long long)co * a.kh * a.kw * a.Ci;
        int acc = ((const int*)a.bias)[co];
        for (int r = 0; r < a.kh; ++r) {
            const int iy = oy * a.stride + r - a.pad;
            if (iy < 0 || iy >= a.H) continue;
            for (int s = 0; s < a.kw; ++s) {
                const int ix = ox * a.stride + s - a.pad_w;
                if (ix < 0 || ix >= a.W) continue;
                const signed char* xp = x + (((long long)n * a.H + iy) * a.W + ix) * a.Ci;
                const signed char* wp = w + (r * a.kw + s) * a.Ci;
                for (int c = 0; c < a.Ci; ++c) acc += (int)xp[c] * (int)wp[c];
            }
        }
        if (a.res) acc += (int)((const signed char*)a.res)[idx] << a.res_shift;
        ((signed char*)a.y)[odx] = (signed char)requant_i8(acc, a.shift, a.lo, a.hi);
    } else {
        const uint16_t* x = (const uint16_t*)a.x;
        const uint16_t* w = (const uint16_t*)a.w + (long long)co * a.kh * a.kw * a.Ci;
        float acc = 0.f;
        for (int r = 0; r < a.kh; ++r) {
            const int iy = oy * a.stride + r - a.pad;
            if (iy < 0 || iy >= a.H) continue;
            for (int s = 0; s < a.kw; ++s) {
                const int ix = ox * a.stride + s - a.pad_w;
                if (ix < 0 || ix >= a.W) continue;
                const uint16_t* xp = x + (((long long)n * a.H + iy) * a.W + ix) * a.Ci;
                const uint16_t* wp = w + (r * a.kw + s) * a.Ci;
                for (int c = 0; c < a.Ci; ++c) acc = fmaf(bf16_to_f32(xp[c]), bf16_to_f32(wp[c]), acc);
            }
        }
        float t = acc + ((const float*)a.bias)[co];
        if (a.res) t = t + bf16_to_f32(((const uint16_t*)a.res)[idx]);
        t = fminf(fmaxf(t, a.f_lo), a.f_hi);
        ((uint16_t*)a.y)[odx] = f32_to_bf16_rne(t);
    }
}

hipError_t launch_conv_direct(const DirectConvArgs& a, int dtype, hipStream_t s)
{
    const long long total = (long long)a.M * a.Co;
    if (total <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dtype == EE_I8) EE_LAUNCH(conv_direct_kernel<1>, dim3(blocks), dim3(256), 0, s, a);
    else EE_LAUNCH(conv_direct_kernel<2>, dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ---- [B][H][W][C<=4] -> zero-padded [B][Hp][Wp][4] ------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void pad_input_kernel(const T* x, T* y, int B, int H, int W, int C, int Hp, int Wp, int pad)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)B * Hp * Wp) return;
    const int xp = (int)(idx % Wp);
    const int yp = (int)((idx / Wp) % Hp);
    const int n = (int)(idx / ((long long)Wp * Hp));
    const int iy = yp - pad, ix = xp - pad;
    T v[4] = {0, 0, 0, 0};
    if (iy >= 0 && iy < H && ix >= 0 && ix < W) {
        const T* p = x + (((long long)n * H + iy) * W + ix) * C;
        for (int c = 0; c < C; ++c) v[c] = p[c];
    }
    T* q = y + idx * 4;
    q[0] = v[0]; q[1] = v[1]; q[2] = v[2]; q[3] = v[3];
}

hipError_t launch_pad_input(const void* x, void* y, int B, int H, int W, int C, int Hp, int Wp, int pad, int dtype, hipStream_t s)
{
    const long long total = (long long)B * Hp * Wp;
    if (total <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dtype == EE_I8)
        EE_LAUNCH(pad_input_kernel<signed char>, dim3(blocks), dim3(256), 0, s, (const signed char*)x, (signed char*)y, B, H, W, C, Hp, Wp, pad);
    else
        EE_LAUNCH(pad_input_kernel<uint16_t>, dim3(blocks), dim3(256), 0, s, (const uint16_t*)x, (uint16_t*)y, B, H, W, C, Hp, Wp, pad);
    return hipGetLastError();
}

// ---- [B][H][W][C<=4] -> [B][Hs][Ws][(dy, dx, c)]: the image is zero padded by `pad`, then every 2 x 2 block of
// pixels becomes one 16-element super-pixel.  A stride-2 k x k convolution of the image is a stride-1
// ceil(k/2) x ceil(k/2) convolution of the folded tensor whose pixels are whole 16-byte chunks. --------------
template <typename T>
__global__ __launch_bounds__(256) void space_to_depth_kernel(const T* x, T* y, const int32_t* gather, int B, int H, int W, int C, int Hs, int Ws, int pad)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)B * Hs * Ws) return;
    const int xs = (int)(idx % Ws), ys = (int)((idx / Ws) % Hs), n = (int)(idx / ((long long)Ws * Hs));
    alignas(16) T v[16];
    const long long row = gather ? gather[n] : n;              // admission reads request gather[n] of a pool
    const T* img = x + row * H * W * C;
    // all loads first, from clamped (always valid) addresses; what lies in the padding becomes zero afterwards
#pragma unroll
    for (int dy = 0; dy < 2; ++dy)
#pragma unroll
        for (int dx = 0; dx < 2; ++dx) {
            const int iy = 2 * ys + dy - pad, ix = 2 * xs + dx - pad;
            const bool ok = iy >= 0 && iy < H && ix >= 0 && ix < W;
            const T* p = img + ((long long)min(max(iy, 0), H - 1) * W + min(max(ix, 0), W - 1)) * C;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const T t = c < C ? p[c < C ? c : 0] : (T)0;
                v[(dy * 2 + dx) * 4 + c] = ok ? t : (T)0;
            }
        }
    typedef int v4i_ __attribute__((ext_vector_type(4)));
    v4i_* q = (v4i_*)(y + idx * 16);
    const v4i_* src = (const v4i_*)v;
#pragma unroll
    for (int i = 0; i < (int)(sizeof(T) * 16 / 16); ++i) q[i] = src[i];
}

// The same folding for image rows that are whole dwords: one workgroup = RS rows of super-pixels of one sample.
// The 2 RS image rows it folds are copied into LDS with dword loads (a wavefront reads 256 contiguous bytes per
// instruction), and every lane gathers the 12 scalars of a super-pixel from LDS.  Loading them from global memory
// one byte at a time costs 12 vector-memory instructions per lane for 16 bytes of output.
// Admission: request ids[n] of a pool is read instead of row n.  For up to 256 samples the ids travel by value as the
// first kernel argument (IdTab) and are read from the kernel-argument segment; `gather` (device-visible memory, e.g.
// pinned host memory, where every read crosses the bus) serves larger batches.
struct IdTab { int32_t id[256]; };
template <typename T, int RS>
__global__ __launch_bounds__(256) void space_to_depth_rows_kernel(IdTab, const T* x, T* y, const int32_t* gather, int by_value, int H, int W, int C, int Hs, int Ws, int pad)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char s2d_lds[];
    const int ys0 = blockIdx.x * RS, n = blockIdx.y;
    const __attribute__((address_space(4))) int* tab = (const __attribute__((address_space(4))) int*)__builtin_amdgcn_kernarg_segment_ptr();
    const long long row = by_value ? tab[n] : (gather ? gather[n] : n);
    const int row_words = W * C * (int)sizeof(T) / 4;
    const int* img = (const int*)(x + row * H * W * C);
    int* l32 = (int*)s2d_lds;
    for (int i = threadIdx.x; i < 2 * RS * row_words; i += 256) {
        const int r = i / row_words, w = i - r * row_words;
        const int iy = 2 * ys0 + r - pad;
        l32[i] = (iy >= 0 && iy < H) ? img[(long long)iy * row_words + w] : 0;      // a row in the padding is all zero
    }
    __syncthreads();
    const T* lrow = (const T*)s2d_lds;
    for (int o = threadIdx.x; o < RS * Ws; o += 256) {
        const int rr = o / Ws, xs = o - rr * Ws, ys = ys0 + rr;
        if (ys >= Hs) break;
        alignas(16) T v[16];
#pragma unroll
        for (int dy = 0; dy < 2; ++dy)
#pragma unroll
            for (int dx = 0; dx < 2; ++dx) {
                const int ix = 2 * xs + dx - pad;
                const bool ok = ix >= 0 && ix < W;
                const T* p = lrow + ((2 * rr + dy) * W + min(max(ix, 0), W - 1)) * C;
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const T t = c < C ? p[c < C ? c : 0] : (T)0;
                    v[(dy * 2 + dx) * 4 + c] = ok ? t : (T)0;
                }
            }
        typedef int v4i_ __attribute__((ext_vector_type(4)));
        v4i_* q = (v4i_*)(y + (((long long)n * Hs + ys) * Ws + xs) * 16);
        const v4i_* src = (const v4i_*)v;
#pragma unroll
        for (int i = 0; i < (int)(sizeof(T) * 16 / 16); ++i) q[i] = src[i];
    }
}

// The same for int8 images of 3 channels whose rows are whole 16-byte chunks (the networks' input): the 2 RS image rows under RS folded
// rows are one contiguous piece of the image, copied with 16-byte loads into LDS rows that have 16 zero bytes in front and 48 behind
// (rows in the padding are zero), so that pixels left and right of the image read as zeros without a test.  A lane then builds two
// neighbouring super-pixels: four pixels are 12 contiguous bytes of an image row, read as four dwords around them, shifted into place
// and spread to 4 bytes per pixel with byte permutes.
template <int RS>
__global__ __launch_bounds__(256) void space_to_depth_rows_c3_kernel(IdTab, const signed char* x, signed char* y, const int32_t* gather, int by_value, int H, int W, int Hs, int Ws, int pad)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char s2d3_lds[];
    typedef int v4i_ __attribute__((ext_vector_type(4)));
    const int ys0 = blockIdx.x * RS, n = blockIdx.y, tid = threadIdx.x;
    const __attribute__((address_space(4))) int* tab = (const __attribute__((address_space(4))) int*)__builtin_amdgcn_kernarg_segment_ptr();
    const long long row = by_value ? tab[n] : (gather ? gather[n] : n);
    const int row_bytes = 3 * W, pitch = row_bytes + 64, row_chunks = row_bytes >> 4, pitch_chunks = pitch >> 4;
    const unsigned char* img = (const unsigned char*)x + row * H * row_bytes;
    // rows r of the 2 RS staged ones that lie inside the image: [ra, rb)
    const int iy_first = 2 * ys0 - pad;
    const int ra = min(max(-iy_first, 0), 2 * RS), rb = max(min(H - iy_first, 2 * RS), ra);
    // margins and padding rows: every chunk that the copy below does not write
    for (int c = tid; c < 2 * RS * pitch_chunks; c += 256) {
        const int r = c / pitch_chunks, w = c - r * pitch_chunks;
        if (r < ra || r >= rb || w == 0 || w > row_chunks) *(v4i_*)(s2d3_lds + c * 16) = v4i_{0, 0, 0, 0};
    }
    const unsigned char* first = img + (long long)(iy_first + ra) * row_bytes;
    for (int c = tid; c < (rb - ra) * row_chunks; c += 256) {
        const int r = c / row_chunks, w = c - r * row_chunks;
        *(v4i_*)(s2d3_lds + (ra + r) * pitch + 16 + 16 * w) = *(const v4i_*)(first + (long long)c * 16);
    }
    __syncthreads();
    const int pairs = (Ws + 1) >> 1;
    if (tid >= RS * pairs) return;
    const int rr = tid / pairs, xs = 2 * (tid - rr * pairs), ys = ys0 + rr;
    if (ys >= Hs) return;
    unsigned px[2][4];                                                  // [image row of the pair][pixel]: 3 channels and a zero byte
#pragma unroll
    for (int dy = 0; dy < 2; ++dy) {
        const int at = (2 * rr + dy) * pitch + 16 + 3 * (2 * xs - pad);   // first byte of the four pixels (>= 0: pad <= 5)
        const unsigned* wp = (const unsigned*)(s2d3_lds + (at & ~3));
        const unsigned w0 = wp[0], w1 = wp[1], w2 = wp[2], w3 = wp[3], sh = (unsigned)(at & 3) * 8;
        const unsigned d0 = __builtin_amdgcn_alignbit(w1, w0, sh), d1 = __builtin_amdgcn_alignbit(w2, w1, sh), d2 = __builtin_amdgcn_alignbit(w3, w2, sh);
        px[dy][0] = d0 & 0x00ffffffu;
        px[dy][1] = __builtin_amdgcn_perm(d1, d0, 0x0c050403u);         // bytes 3, 4, 5 of the twelve
        px[dy][2] = __builtin_amdgcn_perm(d2, d1, 0x0c040302u);         // bytes 6, 7, 8
        px[dy][3] = d2 >> 8;                                            // bytes 9, 10, 11
    }
    signed char* q = y + (((long long)n * Hs + ys) * Ws + xs) * 16;
    *(v4i_*)q = v4i_{(int)px[0][0], (int)px[0][1], (int)px[1][0], (int)px[1][1]};
    if (xs + 1 < Ws) *(v4i_*)(q + 16) = v4i_{(int)px[0][2], (int)px[0][3], (int)px[1][2], (int)px[1][3]};
}

hipError_t launch_space_to_depth(const void* x, void* y, const int32_t* gather, int B, int H, int W, int C, int Hs, int Ws, int pad, int dtype, hipStream_t s, bool gather_on_host)
{
    const long long total = (long long)B * Hs * Ws;
    if (total <= 0) return hipSuccess;
    const int es = dtype == EE_I8 ? 1 : 2;
    const size_t row_bytes = (size_t)W * C * es;
    constexpr int RS = 4;
    if (row_bytes % 4 == 0 && ((size_t)H * row_bytes) % 4 == 0 && 2 * RS * row_bytes <= 64 * 1024 && B <= 65535) {
        const dim3 grid((unsigned)((Hs + RS - 1) / RS), (unsigned)B);
        IdTab tab{};
        const bool host_ids = gather_on_host && gather && B <= 256;      // ids the host can read: by value
        if (host_ids) std::memcpy(tab.id, gather, sizeof(int32_t) * (size_t)B);
        if (dtype == EE_I8 && C == 3 && row_bytes % 16 == 0 && ((uintptr_t)x & 15) == 0 && pad >= 0 && pad <= 5 && RS * ((Ws + 1) / 2) <= 256 &&
            2 * RS * (row_bytes + 64) <= 64 * 1024 && Ws <= (W + 2 * pad + 1) / 2 + 1) {
            EE_LAUNCH((space_to_depth_rows_c3_kernel<RS>), grid, dim3(256), 2 * RS * (row_bytes + 64), s, tab, (const signed char*)x, (signed char*)y, gather, (int)host_ids, H, W, Hs, Ws, pad);
            return hipGetLastError();
        }
        if (dtype == EE_I8)
            EE_LAUNCH((space_to_depth_rows_kernel<signed char, RS>), grid, dim3(256), 2 * RS * row_bytes, s, tab, (const signed char*)x, (signed char*)y, gather, (int)host_ids, H, W, C, Hs, Ws, pad);
        else
            EE_LAUNCH((space_to_depth_rows_kernel<uint16_t, RS>), grid, dim3(256), 2 * RS * row_bytes, s, tab, (const uint16_t*)x, (uint16_t*)y, gather, (int)host_ids, H, W, C, Hs, Ws, pad);
        return hipGetLastError();
    }
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dtype == EE_I8)
        EE_LAUNCH(space_to_depth_kernel<signed char>, dim3(blocks), dim3(256), 0, s, (const signed char*)x, (signed char*)y, gather, B, H, W, C, Hs, Ws, pad);
    else
        EE_LAUNCH(space_to_depth_kernel<uint16_t>, dim3(blocks), dim3(256), 0, s, (const uint16_t*)x, (uint16_t*)y, gather, B, H, W, C, Hs, Ws, pad);
    return hipGetLastError();
}

// ---- [rows][c_bytes] -> [rows][cp_bytes], zero tail: gives layers whose pixels are not 16-byte multiples
// the row alignment the matrix-core loader needs ----------------------------------------------------------
__global__ __launch_bounds__(256) void pad_channels_kernel(const int* x, int* y, long long rows, int c_words, int cp_words)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * cp_words) return;
    const long long r = idx / cp_words;
    const int w = (int)(idx - r * cp_words);
    y[idx] = w < c_words ? x[r * c_words + w] : 0;
}

hipError_t launch_pad_channels(const void* x, void* y, long long rows, int c_bytes, int cp_bytes, hipStream_t s)
{
    const long long total = rows * (cp_bytes / 4);
    if (total <= 0) return hipSuccess;
    EE_LAUNCH(pad_channels_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const int*)x, (int*)y, rows, c_bytes / 4, cp_bytes / 4);
    return hipGetLastError();
}

}  // namespace ee
