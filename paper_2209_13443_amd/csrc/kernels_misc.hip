// Bandwidth-bound kernels for gfx950: depthwise 3x3, max-pool, the exit head (global average
// pool, FC, softmax top-1 and the exit decision), slot compaction / refill and admission.
// All of them move 16 bytes per lane per access along the channel (NHWC) or sample axis so
// that a wavefront touches whole cache lines.
#include "ee_internal.hpp"

namespace ee {

typedef int v4i __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint16_t f32_to_bf16_rne_m(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32_m(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ int med3_i32(int v, int lo, int hi)       // lo <= hi: v clamped to [lo, hi]
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}
__device__ __forceinline__ int byte_of(int word, int e) { return (int)(signed char)((word >> (8 * e)) & 0xFF); }

// ---- depthwise k x k: one lane = one output pixel x 16 bytes of channels ---------------------------
// weights repacked [k*k][C]; int8: int32 accumulate + bias, round-shift, clamp; bf16: float accumulate.
template <int ES>
__global__ __launch_bounds__(256) void depthwise_kernel(PoolArgs a)
{
    const int cchunks = a.C * ES / 16;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)a.B * a.Ho * a.Wo * cchunks) return;
    const int q = (int)(idx % cchunks);
    const long long pix = idx / cchunks;
    const int ox = (int)(pix % a.Wo), oy = (int)((pix / a.Wo) % a.Ho), n = (int)(pix / ((long long)a.Wo * a.Ho));
    const unsigned char* x = (const unsigned char*)a.x;
    if constexpr (ES == 1) {
        int acc[16];
        const int* bias = (const int*)a.bias + q * 16;
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[e] = bias[e];
        for (int r = 0; r < a.k; ++r) {
            const int iy = oy * a.stride + r - a.pad;
            if (iy < 0 || iy >= a.H) continue;
            for (int s = 0; s < a.k; ++s) {
                const int ix = ox * a.stride + s - a.pad;
                if (ix < 0 || ix >= a.W) continue;
                const v4i xv = *(const v4i*)(x + (((long long)n * a.H + iy) * a.W + ix) * a.C + q * 16);
                const v4i wv = *(const v4i*)((const unsigned char*)a.w + (long long)(r * a.k + s) * a.C + q * 16);
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[e] += byte_of(xv[e >> 2], e & 3) * byte_of(wv[e >> 2], e & 3);
            }
        }
        v4i out = {0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            int t = a.shift > 0 ? (acc[e] + (1 << (a.shift - 1))) >> a.shift : acc[e];
            t = min(max(t, a.lo), a.hi);
            out[e >> 2] |= (t & 0xFF) << (8 * (e & 3));
        }
        *(v4i*)((unsigned char*)a.y + pix * a.C + q * 16) = out;
    } else {
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        for (int r = 0; r < a.k; ++r) {
            const int iy = oy * a.stride + r - a.pad;
            if (iy < 0 || iy >= a.H) continue;
            for (int s = 0; s < a.k; ++s) {
                const int ix = ox * a.stride + s - a.pad;
                if (ix < 0 || ix >= a.W) continue;
                const v4i xv = *(const v4i*)(x + ((((long long)n * a.H + iy) * a.W + ix) * a.C) * 2 + q * 16);
                const v4i wv = *(const v4i*)((const unsigned char*)a.w + ((long long)(r * a.k + s) * a.C) * 2 + q * 16);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint16_t xe = (uint16_t)((unsigned)xv[e >> 1] >> (16 * (e & 1)));
                    const uint16_t we = (uint16_t)((unsigned)wv[e >> 1] >> (16 * (e & 1)));
                    acc[e] = fmaf(bf16_to_f32_m(xe), bf16_to_f32_m(we), acc[e]);
                }
            }
        }
        const float* bias = (const float*)a.bias + q * 8;
        v4i out = {0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float t = fminf(fmaxf(acc[e] + bias[e], a.f_lo), a.f_hi);
            out[e >> 1] |= (int)((unsigned)f32_to_bf16_rne_m(t) << (16 * (e & 1)));
        }
        *(v4i*)((unsigned char*)a.y + (pix * a.C) * 2 + q * 16) = out;
    }
}

// ---- depthwise 3x3, int8, on the 4-way dot product --------------------------------------------------------
// One lane = 4 output pixels along x times 16 channels.  v_dot4_i32_i8 wants the 4 bytes of a dword to be 4
// taps of one channel, NHWC delivers 4 channels of one tap: per input column the three row dwords (and a
// zero) of a 4-channel group are byte-transposed with 8 v_perm_b32, and one dot product per channel adds the
// column to every output pixel whose window holds it.  A column is transposed once for the up to three windows
// that share it, and the lane loads 18 (stride 1) or 27 (stride 2) times 16 bytes for 4 outputs instead of 36.
// Weights are packed per 16-channel chunk as [column s][4-channel group][channel] dwords
// (w[0][s], w[1][s], w[2][s], 0), 192 bytes per chunk.  Coordinates outside the image are clamped, so every
// load is in range; such taps become zero through the selectors of the first permute level (selector 0x0c
// yields a zero byte).  The rounding constant of the shift is added to the bias once.
template <int STRIDE, bool TABLE_IN_LDS>
__global__ __launch_bounds__(256) void depthwise3x3_i8_kernel(PoolArgs a, int groups_x)
{
    constexpr int PX = 4, COLS = (PX - 1) * STRIDE + 3;
    extern __shared__ __attribute__((aligned(16))) unsigned char dw_lds_raw[];
    v4i* dw_lds = (v4i*)dw_lds_raw;                    // per 16-channel chunk: 12 weight quads, then 4 bias quads
    const int cchunks = a.C / 16;
    const long long total = (long long)a.B * a.Ho * groups_x * cchunks;
    const long long idx = min((long long)blockIdx.x * 256 + threadIdx.x, total - 1);      // lanes past the end redo the last item
    const bool active = (long long)blockIdx.x * 256 + threadIdx.x < total;
    const int q = (int)(idx % cchunks);
    const int g = (int)(idx / cchunks);
    const int ox0 = (g % groups_x) * PX, oy = (g / groups_x) % a.Ho, n = g / (groups_x * a.Ho);
    const unsigned char* x = (const unsigned char*)a.x;
    const int iy0 = oy * STRIDE - a.pad, ix0 = ox0 * STRIDE - a.pad;
    // byte offsets inside the batch tensor fit 32 bits (checked when the context is created)
    unsigned rowoff[3], coloff[COLS];
    bool rowok[3], colok[COLS];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int iy = iy0 + r;
        rowok[r] = (unsigned)iy < (unsigned)a.H;
        rowoff[r] = (unsigned)((n * a.H + min(max(iy, 0), a.H - 1)) * a.W) * (unsigned)a.C + (unsigned)q * 16u;
    }
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
        const int ix = ix0 + c;
        colok[c] = (unsigned)ix < (unsigned)a.W;
        coloff[c] = (unsigned)(min(max(ix, 0), a.W - 1) * a.C);
    }
    v4i xv[3][COLS];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int c = 0; c < COLS; ++c) xv[r][c] = *(const v4i*)(x + (rowoff[r] + coloff[c]));
    // Weights and bias depend on the channel chunk only.  With few channels the workgroup copies the whole table
    // into LDS once (C * 16 bytes) instead of 16 loads of 16 bytes per lane through the vector memory path (the big
    // early layers: -10 %); with many channels and few pixels the copy is most of what a workgroup would read
    // anyway and only adds a step to a short launch, so those layers read the table per lane.
    if constexpr (TABLE_IN_LDS) {
        for (int i = threadIdx.x; i < cchunks * 16; i += 256) {
            const int qq = i >> 4, r = i & 15;
            dw_lds[i] = r < 12 ? ((const v4i*)a.w)[qq * 12 + r] : ((const v4i*)a.bias)[qq * 4 + (r - 12)];
        }
        __syncthreads();
    }
    if (!active) return;
    // first permute level of a column whose three rows are x0, x1, x2:
    //   (x0.b0, x1.b0, x0.b1, x1.b1), (x0.b2, x1.b2, x0.b3, x1.b3), (x2.b0, 0, x2.b1, 0), (x2.b2, 0, x2.b3, 0)
    const unsigned s_lo01 = (rowok[0] ? 0x00010000u : 0x000c000cu) | (rowok[1] ? 0x05000400u : 0x0c000c00u);
    const unsigned s_hi01 = (rowok[0] ? 0x00030002u : 0x000c000cu) | (rowok[1] ? 0x07000600u : 0x0c000c00u);
    const unsigned s_lo2 = rowok[2] ? 0x0c010c00u : 0x0c0c0c0cu, s_hi2 = rowok[2] ? 0x0c030c02u : 0x0c0c0c0cu;
    const int rnd = a.shift > 0 ? 1 << (a.shift - 1) : 0;
    v4i outv[PX];
#pragma unroll
    for (int cg = 0; cg < 4; ++cg) {
        v4i b4, w[3];
        if constexpr (TABLE_IN_LDS) {
            b4 = dw_lds[q * 16 + 12 + cg];
#pragma unroll
            for (int s = 0; s < 3; ++s) w[s] = dw_lds[q * 16 + s * 4 + cg];
        } else {
            b4 = *((const v4i*)a.bias + q * 4 + cg);
#pragma unroll
            for (int s = 0; s < 3; ++s) w[s] = *((const v4i*)a.w + q * 12 + s * 4 + cg);
        }
        int acc[PX][4];
#pragma unroll
        for (int p = 0; p < PX; ++p)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[p][e] = b4[e] + rnd;
#pragma unroll
        for (int c = 0; c < COLS; ++c) {
            const unsigned x0 = (unsigned)xv[0][c][cg], x1 = (unsigned)xv[1][c][cg], x2 = (unsigned)xv[2][c][cg];
            const unsigned lo01 = __builtin_amdgcn_perm(x1, x0, colok[c] ? s_lo01 : 0x0c0c0c0cu), hi01 = __builtin_amdgcn_perm(x1, x0, colok[c] ? s_hi01 : 0x0c0c0c0cu);
            const unsigned lo2 = __builtin_amdgcn_perm(0u, x2, colok[c] ? s_lo2 : 0x0c0c0c0cu), hi2 = __builtin_amdgcn_perm(0u, x2, colok[c] ? s_hi2 : 0x0c0c0c0cu);
            // bytes (x0.c, x1.c, x2.c, 0) for the group's channels c = 0..3
            const unsigned t[4] = {__builtin_amdgcn_perm(lo2, lo01, 0x05040100u), __builtin_amdgcn_perm(lo2, lo01, 0x07060302u),
                                   __builtin_amdgcn_perm(hi2, hi01, 0x05040100u), __builtin_amdgcn_perm(hi2, hi01, 0x07060302u)};
#pragma unroll
            for (int s = 0; s < 3; ++s)
                if ((c - s) >= 0 && (c - s) % STRIDE == 0 && (c - s) / STRIDE < PX) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[(c - s) / STRIDE][e] = __builtin_amdgcn_sdot4((int)t[e], w[s][e], acc[(c - s) / STRIDE][e], false);
                }
        }
#pragma unroll
        for (int p = 0; p < PX; ++p) {
            int t[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = med3_i32(acc[p][e] >> a.shift, a.lo, a.hi);
            const unsigned lo = __builtin_amdgcn_perm((unsigned)t[1], (unsigned)t[0], 0x0c0c0400u), hi = __builtin_amdgcn_perm((unsigned)t[3], (unsigned)t[2], 0x0c0c0400u);
            outv[p][cg] = (int)__builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
    }
#pragma unroll
    for (int p = 0; p < PX; ++p)
        if (ox0 + p < a.Wo) *(v4i*)((unsigned char*)a.y + ((((long long)n * a.Ho + oy) * a.Wo + ox0 + p) * a.C) + q * 16) = outv[p];
}

hipError_t launch_depthwise(const PoolArgs& a, int dtype, hipStream_t s)
{
    const int es = dtype == EE_I8 ? 1 : 2;
    if (dtype == EE_I8 && a.k == 3 && a.w3 && (a.stride == 1 || a.stride == 2)) {
        const int groups_x = (a.Wo + 3) / 4;
        const long long total = (long long)a.B * a.Ho * groups_x * (a.C / 16);
        if (total <= 0) return hipSuccess;
        PoolArgs b = a;
        b.w = a.w3;
        const dim3 grid((unsigned)((total + 255) / 256));
        if (a.C <= 192) {                   // the table in LDS: measured to pay up to 192 channels (see the kernel)
            const size_t lds_bytes = (size_t)a.C * 16;
            if (a.stride == 1) EE_LAUNCH((depthwise3x3_i8_kernel<1, true>), grid, dim3(256), lds_bytes, s, b, groups_x);
            else EE_LAUNCH((depthwise3x3_i8_kernel<2, true>), grid, dim3(256), lds_bytes, s, b, groups_x);
        } else {
            if (a.stride == 1) EE_LAUNCH((depthwise3x3_i8_kernel<1, false>), grid, dim3(256), 0, s, b, groups_x);
            else EE_LAUNCH((depthwise3x3_i8_kernel<2, false>), grid, dim3(256), 0, s, b, groups_x);
        }
        return hipGetLastError();
    }
    const long long total = (long long)a.B * a.Ho * a.Wo * (a.C * es / 16);
    if (total <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dtype == EE_I8) EE_LAUNCH(depthwise_kernel<1>, dim3(blocks), dim3(256), 0, s, a);
    else EE_LAUNCH(depthwise_kernel<2>, dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ---- max-pool k x k over the in-range taps ---------------------------------------------------------
template <int ES>
__global__ __launch_bounds__(256) void maxpool_kernel(PoolArgs a)
{
    const int cchunks = a.C * ES / 16;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)a.B * a.Ho * a.Wo * cchunks) return;
    const int q = (int)(idx % cchunks);
    const long long pix = idx / cchunks;
    const int ox = (int)(pix % a.Wo), oy = (int)((pix / a.Wo) % a.Ho), n = (int)(pix / ((long long)a.Wo * a.Ho));
    const unsigned char* x = (const unsigned char*)a.x;
    constexpr int NE = 16 / ES;
    float bestf[NE];
    int besti[NE];
    bool have = false;
    v4i bits = {0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < NE; ++e) { besti[e] = -129; bestf[e] = 0.f; }
    for (int r = 0; r < a.k; ++r) {
        const int iy = oy * a.stride + r - a.pad;
        if (iy < 0 || iy >= a.H) continue;
        for (int s = 0; s < a.k; ++s) {
            const int ix = ox * a.stride + s - a.pad;
            if (ix < 0 || ix >= a.W) continue;
            const v4i xv = *(const v4i*)(x + ((((long long)n * a.H + iy) * a.W + ix) * a.C) * ES + q * 16);
            if constexpr (ES == 1) {
#pragma unroll
                for (int e = 0; e < 16; ++e) besti[e] = max(besti[e], byte_of(xv[e >> 2], e & 3));
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint16_t xe = (uint16_t)((unsigned)xv[e >> 1] >> (16 * (e & 1)));
                    const float v = bf16_to_f32_m(xe);
                    if (!have || v > bestf[e]) {
                        bestf[e] = v;
                        bits[e >> 1] = (bits[e >> 1] & ~(0xFFFF << (16 * (e & 1)))) | ((int)xe << (16 * (e & 1)));
                    }
                }
            }
            have = true;
        }
    }
    if constexpr (ES == 1) {
#pragma unroll
        for (int e = 0; e < 16; ++e) bits[e >> 2] |= (besti[e] & 0xFF) << (8 * (e & 3));
    }
    *(v4i*)((unsigned char*)a.y + (pix * a.ldc + a.c_off) * ES + q * 16) = bits;     // a channel slice when ldc > C
}

// ---- average pool k x k: all k*k taps, padding counts as zero, divisor k*k ---------------------------------
// int8: y = floor((2 * sum + k*k) / (2 * k*k)) (round half up); the numerator is made non-negative by adding
// 128 * k*k to the sum (and 128 is taken off the quotient), the division is a multiply-high with
// floor(2^32 / (2 k*k)) and one correction step.  bf16: float sum in tap order / (k*k), rounded to bf16.
template <int ES>
__global__ __launch_bounds__(256) void avgpool_kernel(PoolArgs a, unsigned magic)
{
    const int cchunks = a.C * ES / 16;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)a.B * a.Ho * a.Wo * cchunks) return;
    const int q = (int)(idx % cchunks);
    const long long pix = idx / cchunks;
    const int ox = (int)(pix % a.Wo), oy = (int)((pix / a.Wo) % a.Ho), n = (int)(pix / ((long long)a.Wo * a.Ho));
    const unsigned char* x = (const unsigned char*)a.x;
    constexpr int NE = 16 / ES;
    int sumi[NE];
    float sumf[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) { sumi[e] = 0; sumf[e] = 0.f; }
    for (int r = 0; r < a.k; ++r) {
        const int iy = oy * a.stride + r - a.pad;
        if (iy < 0 || iy >= a.H) continue;
        for (int s = 0; s < a.k; ++s) {
            const int ix = ox * a.stride + s - a.pad;
            if (ix < 0 || ix >= a.W) continue;
            const v4i xv = *(const v4i*)(x + ((((long long)n * a.H + iy) * a.W + ix) * a.C) * ES + q * 16);
            if constexpr (ES == 1) {
#pragma unroll
                for (int e = 0; e < 16; ++e) sumi[e] += byte_of(xv[e >> 2], e & 3);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) sumf[e] += bf16_to_f32_m((uint16_t)((unsigned)xv[e >> 1] >> (16 * (e & 1))));
            }
        }
    }
    v4i bits = {0, 0, 0, 0};
    const int kk = a.k * a.k;
    if constexpr (ES == 1) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const unsigned num = (unsigned)(2 * (sumi[e] + 128 * kk) + kk);        // < 2 * 255 * 225 + 225 < 2^17
            unsigned qv = __umulhi(num, magic);                                        // floor(num / (2 kk)), corrected below
            if ((qv + 1) * (unsigned)(2 * kk) <= num) ++qv;
            if (qv * (unsigned)(2 * kk) > num) --qv;
            bits[e >> 2] |= (((int)qv - 128) & 0xFF) << (8 * (e & 3));
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) bits[e >> 1] |= (int)((unsigned)f32_to_bf16_rne_m(sumf[e] / (float)kk) << (16 * (e & 1)));
    }
    *(v4i*)((unsigned char*)a.y + (pix * a.ldc + a.c_off) * ES + q * 16) = bits;
}

// ---- int8 3x3 max / average pool on 16-bit halves ---------------------------------------------------------------
// One lane = 4 output pixels along x times 16 channels; the three rows of every input column are reduced
// first and shared by the windows that overlap it, so a lane issues 18 (stride 1) or 27 (stride 2) 16-byte
// loads for 4 outputs instead of 36, and works on two channels per instruction.  Coordinates outside the
// image are clamped to the nearest pixel inside, so every load is in range and needs no select.
//  max: the clamped pixel belongs to the window (pad < 3), so it changes nothing.  A 16-bit signed max of the
//       halves (b1:b0), (b3:b2) of a dword is decided by the high byte: the raw dword yields channels 1 and 3,
//       the dword shifted left by 8 channels 0 and 2 (the low bytes are don't-cares).
//  avg: v_perm_b32 sign-extends bytes 1 and 3 of a dword into 16-bit lanes (again of the dword and of the
//       dword shifted left by 8); a tap outside the image uses the selector that yields zero instead.  The
//       lanes add with v_pk_add_i16 (|sum| <= 1152).  With S = sum + 1152 >= 0,
//       floor((2 S + 9) / 18) = ((2 S + 9) * 3641) >> 16 exactly for all S <= 2295 (3641 * 18 = 2^16 + 2 and
//       4599 * 2 < 2^16); the product stays below 2^24, so the quotient is byte 2 of it, and it carries the
//       bias 128 = 1152 / 9 that the last xor removes.
typedef short v2s __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pk_max_i16(unsigned a, unsigned b)
{
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(v2s, a), __builtin_bit_cast(v2s, b)));
}
__device__ __forceinline__ unsigned pk_add_i16(unsigned a, unsigned b)
{
    return __builtin_bit_cast(unsigned, __builtin_bit_cast(v2s, a) + __builtin_bit_cast(v2s, b));
}

template <int STRIDE, bool AVG>
__global__ __launch_bounds__(256) void pool3x3_i8_kernel(PoolArgs a, int groups_x)
{
    constexpr int PX = 4, COLS = (PX - 1) * STRIDE + 3;
    const int cchunks = a.C / 16;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)a.B * a.Ho * groups_x * cchunks) return;
    const int q = (int)(idx % cchunks);
    const int g = (int)(idx / cchunks);
    const int ox0 = (g % groups_x) * PX, oy = (g / groups_x) % a.Ho, n = g / (groups_x * a.Ho);
    const unsigned char* x = (const unsigned char*)a.x;
    const int iy0 = oy * STRIDE - a.pad, ix0 = ox0 * STRIDE - a.pad;
    // byte offsets inside the batch tensor fit 32 bits (checked when the context is created)
    unsigned rowoff[3], coloff[COLS];
    bool rowok[3], colok[COLS];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int iy = iy0 + r;
        rowok[r] = (unsigned)iy < (unsigned)a.H;
        rowoff[r] = (unsigned)((n * a.H + min(max(iy, 0), a.H - 1)) * a.W) * (unsigned)a.C + (unsigned)q * 16u;
    }
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
        const int ix = ix0 + c;
        colok[c] = (unsigned)ix < (unsigned)a.W;
        coloff[c] = (unsigned)(min(max(ix, 0), a.W - 1) * a.C);
    }
    v4i xv[3][COLS];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int c = 0; c < COLS; ++c) xv[r][c] = *(const v4i*)(x + (rowoff[r] + coloff[c]));
    unsigned co[COLS][4], ce[COLS][4];         // per column and dword: channels 1, 3 and channels 0, 2 as 16-bit lanes
#pragma unroll
    for (int c = 0; c < COLS; ++c) {
        unsigned sel[3];                       // avg: bytes (b1, sign b1, b3, sign b3) of the second operand, or four zero bytes
#pragma unroll
        for (int r = 0; r < 3; ++r) sel[r] = rowok[r] && colok[c] ? 0x09030801u : 0x0c0c0c0cu;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const unsigned x0 = (unsigned)xv[0][c][d], x1 = (unsigned)xv[1][c][d], x2 = (unsigned)xv[2][c][d];
            if constexpr (AVG) {
                co[c][d] = pk_add_i16(pk_add_i16(__builtin_amdgcn_perm(0u, x0, sel[0]), __builtin_amdgcn_perm(0u, x1, sel[1])), __builtin_amdgcn_perm(0u, x2, sel[2]));
                ce[c][d] = pk_add_i16(pk_add_i16(__builtin_amdgcn_perm(0u, x0 << 8, sel[0]), __builtin_amdgcn_perm(0u, x1 << 8, sel[1])),
                                      __builtin_amdgcn_perm(0u, x2 << 8, sel[2]));
            } else {
                co[c][d] = pk_max_i16(pk_max_i16(x0, x1), x2);
                ce[c][d] = pk_max_i16(pk_max_i16(x0 << 8, x1 << 8), x2 << 8);
            }
        }
    }
#pragma unroll
    for (int p = 0; p < PX; ++p) {
        if (ox0 + p >= a.Wo) break;
        v4i out;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const unsigned o0 = co[p * STRIDE][d], o1 = co[p * STRIDE + 1][d], o2 = co[p * STRIDE + 2][d];
            const unsigned e0 = ce[p * STRIDE][d], e1 = ce[p * STRIDE + 1][d], e2 = ce[p * STRIDE + 2][d];
            if constexpr (AVG) {
                const unsigned so = pk_add_i16(pk_add_i16(o0, o1), pk_add_i16(o2, 0x04800480u));
                const unsigned se = pk_add_i16(pk_add_i16(e0, e1), pk_add_i16(e2, 0x04800480u));
                const unsigned t0 = (se & 0xFFFFu) * 7282u + 32769u, t2 = (se >> 16) * 7282u + 32769u;
                const unsigned t1 = (so & 0xFFFFu) * 7282u + 32769u, t3 = (so >> 16) * 7282u + 32769u;
                const unsigned lo = __builtin_amdgcn_perm(t1, t0, 0x0c0c0602u), hi = __builtin_amdgcn_perm(t3, t2, 0x06020c0cu);
                out[d] = (int)((lo | hi) ^ 0x80808080u);
            } else {
                const unsigned mo = pk_max_i16(pk_max_i16(o0, o1), o2), me = pk_max_i16(pk_max_i16(e0, e1), e2);
                out[d] = (int)__builtin_amdgcn_perm(mo, me, 0x07030501u);
            }
        }
        *(v4i*)((unsigned char*)a.y + ((((long long)n * a.Ho + oy) * a.Wo + ox0 + p) * a.ldc + a.c_off) + q * 16) = out;
    }
}

template <bool AVG>
static hipError_t launch_pool3x3_i8(const PoolArgs& a, hipStream_t s)
{
    const int groups_x = (a.Wo + 3) / 4;
    const long long total = (long long)a.B * a.Ho * groups_x * (a.C / 16);
    if (total <= 0) return hipSuccess;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (a.stride == 1) EE_LAUNCH((pool3x3_i8_kernel<1, AVG>), grid, dim3(256), 0, s, a, groups_x);
    else EE_LAUNCH((pool3x3_i8_kernel<2, AVG>), grid, dim3(256), 0, s, a, groups_x);
    return hipGetLastError();
}

hipError_t launch_maxpool(const PoolArgs& a, int dtype, hipStream_t s)
{
    if (dtype == EE_I8 && a.k == 3 && (a.stride == 1 || a.stride == 2) && a.C % 16 == 0) return launch_pool3x3_i8<false>(a, s);
    const int es = dtype == EE_I8 ? 1 : 2;
    const long long total = (long long)a.B * a.Ho * a.Wo * (a.C * es / 16);
    if (total <= 0) return hipSuccess;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    if (dtype == EE_I8) EE_LAUNCH(maxpool_kernel<1>, dim3(blocks), dim3(256), 0, s, a);
    else EE_LAUNCH(maxpool_kernel<2>, dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_avgpool(const PoolArgs& a, int dtype, hipStream_t s)
{
    if (dtype == EE_I8 && a.k == 3 && (a.stride == 1 || a.stride == 2) && a.C % 16 == 0) return launch_pool3x3_i8<true>(a, s);
    const int es = dtype == EE_I8 ? 1 : 2;
    const long long total = (long long)a.B * a.Ho * a.Wo * (a.C * es / 16);
    if (total <= 0) return hipSuccess;
    if (a.k < 1 || a.k > 15) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    const unsigned magic = (unsigned)(0x100000000ull / (unsigned)(2 * a.k * a.k));
    if (dtype == EE_I8) EE_LAUNCH(avgpool_kernel<1>, dim3(blocks), dim3(256), 0, s, a, magic);
    else EE_LAUNCH(avgpool_kernel<2>, dim3(blocks), dim3(256), 0, s, a, magic);
    return hipGetLastError();
}

// ---- exit head, step 1: global average pool ----------------------------------------------------------
// grid (S pixel splits, B).  Lane = (pixel lane pl, 16-byte channel chunk q); the pixel lanes are reduced
// through LDS into one partial row per workgroup.  int8: the row is added into sums[B][C] with one
// atomic per channel (int32 addition is exact in any order; the buffer is zero on entry, the softmax
// kernel of every head clears what it used).  bf16: the S partial rows of a sample are stored and a
// second small kernel adds them in split order, so the float means never depend on the order in which
// workgroups ran.  (A last-arriving-workgroup reduction inside one kernel would need a device-scope
// release per workgroup, which on this chip writes back the whole L2 of its XCD.)
// Needs C * ES / 16 <= 256.
template <int ES>
__global__ __launch_bounds__(256) void gap_kernel(HeadArgs a, int pix_per_block)
{
    constexpr int NE = 16 / ES;
    __shared__ int red[256 * NE];
    const int cchunks = a.C * ES / 16;
    const int npl = 256 / cchunks;
    const int b = blockIdx.y, S = gridDim.x;
    const int q = (int)threadIdx.x % cchunks, pl = (int)threadIdx.x / cchunks;
    const bool active = pl < npl;
    const int p0 = blockIdx.x * pix_per_block, p1 = min(a.HW, p0 + pix_per_block);
    const long long bs = a.slots ? (long long)a.slots[b] : (long long)b;      // zero-copy compaction: sample b of the batch is slot slots[b] of act
    const unsigned char* x = (const unsigned char*)a.act + bs * a.HW * a.C * ES;
    int acci[NE];
    float accf[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) { acci[e] = 0; accf[e] = 0.f; }
    if (active) {
        int p = p0 + pl;
        for (; p + 3 * npl < p1; p += 4 * npl) {           // four rows in flight per lane
            v4i xv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) xv[u] = *(const v4i*)(x + ((long long)(p + u * npl) * a.C) * ES + q * 16);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if constexpr (ES == 1) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) acci[e] += __builtin_amdgcn_sbfe(xv[u][e >> 2], 8 * (e & 3), 8);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) accf[e] += bf16_to_f32_m((uint16_t)((unsigned)xv[u][e >> 1] >> (16 * (e & 1))));
                }
            }
        }
        for (; p < p1; p += npl) {
            const v4i xv = *(const v4i*)(x + ((long long)p * a.C) * ES + q * 16);
            if constexpr (ES == 1) {
#pragma unroll
                for (int e = 0; e < 16; ++e) acci[e] += __builtin_amdgcn_sbfe(xv[e >> 2], 8 * (e & 3), 8);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) accf[e] += bf16_to_f32_m((uint16_t)((unsigned)xv[e >> 1] >> (16 * (e & 1))));
            }
        }
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            if constexpr (ES == 1) red[pl * a.C + q * NE + e] = acci[e];
            else red[pl * a.C + q * NE + e] = __float_as_int(accf[e]);
        }
    }
    __syncthreads();
    for (int c = threadIdx.x; c < a.C; c += 256) {
        if constexpr (ES == 1) {
            int s = 0;
            for (int l = 0; l < npl; ++l) s += red[l * a.C + c];
            atomicAdd(&a.sums[(long long)b * a.C + c], s);
        } else {
            float s = 0.f;
            for (int l = 0; l < npl; ++l) s += __int_as_float(red[l * a.C + c]);
            if (S == 1) a.sums[(long long)b * a.C + c] = __float_as_int(s / (float)a.HW);
            else a.gap_partial[((long long)b * S + blockIdx.x) * a.C + c] = __float_as_int(s);
        }
    }
}

// bf16: sums[b][c] = (partial[b][0][c] + ... + partial[b][S-1][c]) / HW, 4 channels per lane
__global__ __launch_bounds__(256) void gap_reduce_kernel(HeadArgs a, int S)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;       // (b, c / 4)
    const int c4 = a.C / 4;
    if (idx >= (long long)a.B * c4) return;
    const long long b = idx / c4;
    const int c = (int)(idx - b * c4) * 4;
    const int* rows = a.gap_partial + b * S * a.C + c;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    for (int k = 0; k < S; ++k) {
        const v4i v = *(const v4i*)(rows + (long long)k * a.C);
        s0 += __int_as_float(v[0]); s1 += __int_as_float(v[1]); s2 += __int_as_float(v[2]); s3 += __int_as_float(v[3]);
    }
    // the same rounding as the single-split path: one division per channel
    v4i out = {__float_as_int(s0 / (float)a.HW), __float_as_int(s1 / (float)a.HW), __float_as_int(s2 / (float)a.HW), __float_as_int(s3 / (float)a.HW)};
    *(v4i*)(a.sums + b * a.C + c) = out;
}

static int gap_pixels_per_block(int B, int HW)
{
    const int splits = (512 + B - 1) / B;                    // aim at >= 512 workgroups (256-512 measured equal; 1024 and more are slower:
                                                             // every workgroup ends with one atomic per channel); B * splits <= B + 1024
    int ppb = (HW + splits - 1) / splits;
    if (ppb < 16) ppb = HW < 16 ? HW : 16;
    return ppb;
}

int head_gap_splits(int B, int HW)
{
    if (B <= 0 || HW <= 0) return 0;
    const int ppb = gap_pixels_per_block(B, HW);
    return (HW + ppb - 1) / ppb;
}

hipError_t launch_head_gap(const HeadArgs& a, int dtype, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    const int ppb = gap_pixels_per_block(a.B, a.HW);
    const int splits = (a.HW + ppb - 1) / ppb;
    if (dtype == EE_I8) {
        EE_LAUNCH(gap_kernel<1>, dim3(splits, a.B), dim3(256), 0, s, a, ppb);
    } else {
        // two kernels when the pooling is split: a timed launch takes the first one's begin and the second one's end
        const hipEvent_t t0 = g_launch_start, t1 = g_launch_stop;
        if (splits > 1) g_launch_stop = nullptr;
        EE_LAUNCH(gap_kernel<2>, dim3(splits, a.B), dim3(256), 0, s, a, ppb);
        if (splits > 1) {
            const long long total = (long long)a.B * (a.C / 4);
            g_launch_start = nullptr;
            g_launch_stop = t1;
            EE_LAUNCH(gap_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a, splits);
            g_launch_start = t0;
        }
    }
    return hipGetLastError();
}

// ---- exit head, step 2: FC ------------------------------------------------------------------------------
// logits[b][j] = b_j + sum_c g[b][c] * W[j][c] as a 16 x 16 matrix-core tile per workgroup: rows = 16
// classes (A operand, weight rows read straight from global memory, 16 bytes per lane), columns = 16
// samples (B operand, the pooled features: requantised on the fly for int8; split into a bf16 head and
// a bf16 remainder for bf16 so that the float mean loses nothing that matters).  The 4 wavefronts take
// every 4th 64-byte step of the reduction and add their partial tiles through LDS.
//   v_mfma_i32_16x16x64_i8 / v_mfma_f32_16x16x32_bf16, lane l: row l%16, k-bytes [16*(l/16), +16);
//   D: column l%16, rows 4*(l/16) + v for accumulator register v = 0..3.
typedef float v4f_m __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf_m __attribute__((ext_vector_type(8)));

template <int ES>
__global__ __launch_bounds__(256) void fc_kernel(HeadArgs a)
{
    __shared__ int part[4][256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j0 = blockIdx.x * 16, b0 = blockIdx.y * 16;
    const int r = lane & 15, kq = lane >> 4;
    const int j = j0 + r, b = b0 + r;
    const int CB = a.C * ES;                                   // bytes per weight row (a multiple of 16)
    const int nsteps = (CB + 63) / 64;
    const unsigned char* wrow = (const unsigned char*)a.wfc + (long long)min(j, a.n_cls - 1) * CB;
    const bool jin = j < a.n_cls, bin = b < a.B;
    const v4i zero4 = {0, 0, 0, 0};
    v4i acci = zero4;
    v4f_m accf = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = wave; s0 < nsteps; s0 += 16) {
        v4i wv[4], gv[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {                           // all loads of 4 steps first
            const int kb = (s0 + 4 * u) * 64 + kq * 16;
            const bool kin = kb < CB;
            wv[u] = kin && jin ? *(const v4i*)(wrow + kb) : zero4;
            const int* sp = a.sums + (long long)min(b, a.B - 1) * a.C + kb / ES;
#pragma unroll
            for (int q = 0; q < (ES == 1 ? 4 : 2); ++q) gv[u][q] = kin && bin ? *(const v4i*)(sp + 4 * q) : zero4;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if constexpr (ES == 1) {
                v4i g8 = zero4;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int sum = gv[u][e >> 2][e & 3];
                    int g = a.gap_shift > 0 ? (sum + (1 << (a.gap_shift - 1))) >> a.gap_shift : sum;
                    g = min(max(g, -128), 127);
                    g8[e >> 2] |= (g & 0xFF) << (8 * (e & 3));
                }
                acci = __builtin_amdgcn_mfma_i32_16x16x64_i8(wv[u], g8, acci, 0, 0, 0);
            } else {
                v4i hi = zero4, lo = zero4;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float g = __int_as_float(gv[u][e >> 2][e & 3]);
                    const uint16_t h = f32_to_bf16_rne_m(g);
                    const uint16_t l = f32_to_bf16_rne_m(g - bf16_to_f32_m(h));
                    hi[e >> 1] |= (int)((unsigned)h << (16 * (e & 1)));
                    lo[e >> 1] |= (int)((unsigned)l << (16 * (e & 1)));
                }
                accf = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf_m, wv[u]), __builtin_bit_cast(v8bf_m, hi), accf, 0, 0, 0);
                accf = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf_m, wv[u]), __builtin_bit_cast(v8bf_m, lo), accf, 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) part[wave][v * 64 + lane] = ES == 1 ? acci[v] : __float_as_int(accf[v]);
    __syncthreads();
    const int v = threadIdx.x >> 6;                             // this thread finishes element (class 4*kq + v, sample r)
    const int jj = j0 + 4 * kq + v;
    if (jj >= a.n_cls || !bin) return;
    if constexpr (ES == 1) {
        const int t = part[0][threadIdx.x] + part[1][threadIdx.x] + part[2][threadIdx.x] + part[3][threadIdx.x];
        ((int*)a.logits)[(long long)b * a.n_cls + jj] = t + ((const int*)a.bfc)[jj];
    } else {
        const float t = (__int_as_float(part[0][threadIdx.x]) + __int_as_float(part[1][threadIdx.x])) +
                        (__int_as_float(part[2][threadIdx.x]) + __int_as_float(part[3][threadIdx.x]));
        ((float*)a.logits)[(long long)b * a.n_cls + jj] = a.logit_scale * (t + ((const float*)a.bfc)[jj]);
    }
}

hipError_t launch_head_fc(const HeadArgs& a, int dtype, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    dim3 grid((a.n_cls + 15) / 16, (a.B + 15) / 16);
    if (dtype == EE_I8) EE_LAUNCH(fc_kernel<1>, grid, dim3(256), 0, s, a);
    else EE_LAUNCH(fc_kernel<2>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

// ---- exit head, step 3: softmax top-1 and the exit decision --------------------------------------------------
// 2^30 * 2^(-i/256), i = 0..255, rounded to nearest.
__constant__ uint32_t kExp2[256] = {
#include "exp2_table.inc"
};
static const uint32_t kExp2Host[256] = {
#include "exp2_table.inc"
};
const uint32_t* exp2_table_host() { return kExp2Host; }

template <typename T>
__device__ __forceinline__ T block_reduce(T v, T* scratch, bool is_max)
{
    for (int o = 32; o > 0; o >>= 1) {
        T other = __shfl_xor(v, o, 64);
        v = is_max ? (other > v ? other : v) : v + other;
    }
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[wave] = v;
    __syncthreads();
    T r = scratch[0];
    for (int w = 1; w < 4; ++w) r = is_max ? (scratch[w] > r ? scratch[w] : r) : r + scratch[w];
    return r;
}

// A sample's record for the host: one 16-byte store into pinned host memory.  Both 64-bit words carry the launch's tag, so
// the host sees by itself when a record is complete (an aligned 64-bit word arrives whole): no fence, no counter of
// workgroups and no word behind them on the device side, and the host reads a record as soon as it lands.
__device__ __forceinline__ void host_record(HostOutcome* dst, uint64_t payload, int label, unsigned flag, unsigned tag)
{
    const uint64_t w0 = payload | (uint64_t)tag << EE_OUTCOME_TAG_SHIFT;
    const uint64_t w1 = (uint64_t)(unsigned)label | (uint64_t)(flag & 1u) << 32 | (uint64_t)tag << EE_OUTCOME_TAG_SHIFT;
    const v4i rec = {(int)(unsigned)w0, (int)(unsigned)(w0 >> 32), (int)(unsigned)w1, (int)(unsigned)(w1 >> 32)};
    *(v4i*)dst = rec;
}

// one workgroup per sample.  int8: m = max logit, label = lowest arg-max, S = sum_j T[frac(d_j)] >> (d_j >> f)
// with d_j = m - a_j (a base-2 softmax denominator in Q30); exits iff S <= s_thr.  bf16: float softmax.
// The sample's logits are read once into registers (up to 8 per lane: n_cls <= 2048); the arg-max and the
// denominator travel through one combined reduction.
template <int ES>
__global__ __launch_bounds__(256) void softmax_kernel(HeadArgs a)
{
    __shared__ long long scratch[8];
    __shared__ int scratch_arg[4];
    const int b = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr int PER = 8;
    int vi[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int j = threadIdx.x + 256 * i;
        vi[i] = j < a.n_cls ? ((const int*)a.logits)[(long long)b * a.n_cls + j] : (ES == 1 ? INT32_MIN : __float_as_int(-INFINITY));
    }
    if constexpr (ES == 1) {
        int m = INT32_MIN;
#pragma unroll
        for (int i = 0; i < PER; ++i) m = max(m, vi[i]);
        m = block_reduce<int>(m, (int*)scratch, true);
        int arg = INT32_MAX;
        long long S = 0;
        const int f = a.frac_bits;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int j = threadIdx.x + 256 * i;
            if (j >= a.n_cls) continue;
            const int v = vi[i];
            if (v == m) arg = min(arg, j);
            const long long d = (long long)m - v;
            const long long q = d >> f;
            const long long frac = d & ((1ll << f) - 1);
            const int r = (int)(f >= 8 ? frac >> (f - 8) : frac << (8 - f));
            S += q >= 31 ? 0 : (long long)(kExp2[r] >> q);
        }
        for (int o = 32; o > 0; o >>= 1) {                  // integer sums and minima: exact in any order
            S += __shfl_xor(S, o, 64);
            arg = min(arg, __shfl_xor(arg, o, 64));
        }
        __syncthreads();
        if (lane == 0) { scratch[wave] = S; scratch_arg[wave] = arg; }
        __syncthreads();
        S = scratch[0] + scratch[1] + scratch[2] + scratch[3];
        arg = min(min(scratch_arg[0], scratch_arg[1]), min(scratch_arg[2], scratch_arg[3]));
        // the pooled sums of this sample have been consumed by the FC: leave them zero for the next head
        for (int c = threadIdx.x; c < a.C; c += 256) a.sums[(long long)b * a.C + c] = 0;
        if (threadIdx.x == 0) {
            const float conf = (float)(1073741824.0 / (double)S);
            const uint8_t flag = (uint8_t)(a.last || S <= a.s_thr);
            a.label[b] = arg;
            a.score[b] = S;
            a.conf[b] = conf;
            a.flag[b] = flag;
            if (a.host_out) host_record(a.host_out + b, (uint64_t)S, arg, flag, a.tag);
        }
    } else {
        float m = -INFINITY;
#pragma unroll
        for (int i = 0; i < PER; ++i) m = fmaxf(m, __int_as_float(vi[i]));
        m = block_reduce<float>(m, (float*)scratch, true);
        int arg = INT32_MAX;
        float den = 0.f;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int j = threadIdx.x + 256 * i;
            if (j >= a.n_cls) continue;
            const float z = __int_as_float(vi[i]);
            if (z == m) arg = min(arg, j);
            den += expf(z - m);
        }
        for (int o = 32; o > 0; o >>= 1) {                  // fixed shuffle tree: the float sum is reproducible
            den += __shfl_xor(den, o, 64);
            arg = min(arg, __shfl_xor(arg, o, 64));
        }
        __syncthreads();
        if (lane == 0) { ((float*)scratch)[wave] = den; scratch_arg[wave] = arg; }
        __syncthreads();
        den = ((((float*)scratch)[0] + ((float*)scratch)[1]) + ((float*)scratch)[2]) + ((float*)scratch)[3];
        arg = min(min(scratch_arg[0], scratch_arg[1]), min(scratch_arg[2], scratch_arg[3]));
        if (threadIdx.x == 0) {
            const float conf = 1.0f / den;
            const uint8_t flag = (uint8_t)(a.last || conf >= a.thr);
            a.label[b] = arg;
            a.score[b] = 0;
            a.conf[b] = conf;
            a.flag[b] = flag;
            if (a.host_out) host_record(a.host_out + b, (uint64_t)__float_as_uint(conf), arg, flag, a.tag);
        }
    }
}

hipError_t launch_head_softmax(const HeadArgs& a, int dtype, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    if (dtype == EE_I8) EE_LAUNCH(softmax_kernel<1>, dim3(a.B), dim3(256), 0, s, a);
    else EE_LAUNCH(softmax_kernel<2>, dim3(a.B), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ---- scratch memory that is part of the library image --------------------------------------------------------
// The exit head needs device memory beyond its inputs and outputs: the pooled sums, the partial rows of the
// float pooling and the logits.  ee_exit_head takes them from the context's workspace; ee_exit_head_static
// takes them from this array, so that the call allocates nothing.  Every GPU holds its own copy of the array
// at its own address: the address is looked up once per device, with that device current, and host code only
// ever uses the looked-up pointer (the array's name is not a device address on the host side).
static __device__ __align__(256) unsigned char scratch[EE_STATIC_SCRATCH_BYTES];

hipError_t static_scratch(void** out)
{
    static void* ptr_of_device[64] = {};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    void* p = __atomic_load_n(&ptr_of_device[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        __atomic_store_n(&ptr_of_device[dev], p, __ATOMIC_RELEASE);      // the same value from every thread that races here
    }
    *out = p;
    return hipSuccess;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(v4i* p, long long n16)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const v4i z = {0, 0, 0, 0};
    if (i < n16) p[i] = z;
}

// bytes [0, round-up-to-16(bytes)) of p become zero; a kernel, not a memset node, so that it may be captured
// ---- slot tables of a step: kernel arguments -> device memory ---------------------------------------------
__global__ __launch_bounds__(256) void upload_slots_kernel(SlotTab in, SlotTab out, uint16_t* dst)
{
    dst[threadIdx.x] = in.s[threadIdx.x];
    dst[EE_ZC_MAX_B + threadIdx.x] = out.s[threadIdx.x];
}

hipError_t launch_upload_slots(const SlotTab& in, const SlotTab& out, uint16_t* dst, hipStream_t s)
{
    EE_LAUNCH(upload_slots_kernel, dim3(1), dim3(EE_ZC_MAX_B), 0, s, in, out, dst);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s)
{
    const long long n16 = (long long)((bytes + 15) / 16);
    if (n16 == 0) return hipSuccess;
    EE_LAUNCH(fill_zero_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s, (v4i*)p, n16);
    return hipGetLastError();
}

// ---- compaction: survivors keep their order ---------------------------------------------------------------
// grid (chunks of 16 KiB, b_act).  Every workgroup recomputes its slot's destination = number of
// survivors in front of it with a ballot-style block count over the (<= 1024) flags, then copies its
// chunk with 16-byte accesses.  ring_rows > 0: dst is a ring of that many sample rows and the
// destination row wraps around its end.
__global__ __launch_bounds__(256) void compact_kernel(const uint8_t* flag, const unsigned char* src, unsigned char* dst,
                                                      const int32_t* ids_src, int32_t* ids_dst, int b_act,
                                                      long long sample_bytes, int dst_off, int ring_rows, int* b_rem_out, int* b_rem_out2)
{
    const int b = blockIdx.y;
    int before = 0, total = 0;
    for (int t0 = 0; t0 < b_act; t0 += 256) {
        const int t = t0 + threadIdx.x;
        const int alive = t < b_act && flag[t] == 0;
        before += __syncthreads_count(alive && t < b);
        total += __syncthreads_count(alive);
    }
    if (blockIdx.x == 0 && b == 0 && threadIdx.x == 0) {
        if (b_rem_out) *b_rem_out = total;
        if (b_rem_out2) *b_rem_out2 = total;
    }
    if (flag[b]) return;
    int d = dst_off + before;
    if (ring_rows > 0 && d >= ring_rows) d -= ring_rows;
    if (blockIdx.x == 0 && threadIdx.x == 0 && ids_dst && ids_src) ids_dst[d] = ids_src[b];
    const long long c0 = (long long)blockIdx.x * 16384;
    const v4i* s4 = (const v4i*)(src + (long long)b * sample_bytes + c0);
    v4i* d4 = (v4i*)(dst + (long long)d * sample_bytes + c0);
    const long long n16 = min((long long)1024, (sample_bytes - c0) / 16);
    for (long long i = threadIdx.x; i < n16; i += 256) d4[i] = s4[i];
}

hipError_t launch_compact(const uint8_t* flag, const void* src, void* dst, const int32_t* ids_src, int32_t* ids_dst,
                          int b_act, int64_t sample_bytes, int dst_off, int ring_rows, int* b_rem_out, int* b_rem_out2, hipStream_t s)
{
    if (b_act <= 0) return hipSuccess;
    dim3 grid((unsigned)((sample_bytes + 16383) / 16384), b_act);
    EE_LAUNCH(compact_kernel, grid, dim3(256), 0, s, flag, (const unsigned char*)src, (unsigned char*)dst,
                       ids_src, ids_dst, b_act, (long long)sample_bytes, dst_off, ring_rows, b_rem_out, b_rem_out2);
    return hipGetLastError();
}

// ---- append / admission: whole samples copied to given slots ---------------------------------------------------
// src row = ids ? ids[k] : k  (admission gathers pool rows by request id; refill copies rows in order);
// destination slot = first + k with first = *first_dev when given.
__global__ __launch_bounds__(256) void copy_rows_kernel(const unsigned char* src, unsigned char* dst, const int32_t* gather_ids,
                                                        const int32_t* ids_in, int32_t* ids_out, const int* first_dev, int first,
                                                        int count, long long sample_bytes, int* total_out)
{
    const int k = blockIdx.y;
    const int base = first_dev ? *first_dev : first;
    if (blockIdx.x == 0 && k == 0 && threadIdx.x == 0 && total_out) *total_out = base + count;
    if (blockIdx.x == 0 && threadIdx.x == 0 && ids_out && ids_in) ids_out[base + k] = ids_in[k];
    const long long row = gather_ids ? gather_ids[k] : k;
    const long long c0 = (long long)blockIdx.x * 16384;
    const v4i* s4 = (const v4i*)(src + row * sample_bytes + c0);
    v4i* d4 = (v4i*)(dst + (long long)(base + k) * sample_bytes + c0);
    const long long n16 = min((long long)1024, (sample_bytes - c0) / 16);
    for (long long i = threadIdx.x; i < n16; i += 256) d4[i] = s4[i];
}

hipError_t launch_append(const void* refill, void* dst, const int32_t* refill_ids, int32_t* ids_dst, const int* b_rem_dev,
                         int b_rem_host, int b_incr, int64_t sample_bytes, int* b_merged_out, hipStream_t s)
{
    if (b_incr <= 0) return hipSuccess;
    dim3 grid((unsigned)((sample_bytes + 16383) / 16384), b_incr);
    EE_LAUNCH(copy_rows_kernel, grid, dim3(256), 0, s, (const unsigned char*)refill, (unsigned char*)dst,
                       (const int32_t*)nullptr, refill_ids, ids_dst, b_rem_dev, b_rem_host, b_incr, (long long)sample_bytes, b_merged_out);
    return hipGetLastError();
}

hipError_t launch_admit(const void* pool, void* dst, const int32_t* ids, int b, int64_t sample_bytes, hipStream_t s)
{
    if (b <= 0) return hipSuccess;
    dim3 grid((unsigned)((sample_bytes + 16383) / 16384), b);
    EE_LAUNCH(copy_rows_kernel, grid, dim3(256), 0, s, (const unsigned char*)pool, (unsigned char*)dst, ids,
                       (const int32_t*)nullptr, (int32_t*)nullptr, (const int*)nullptr, 0, b, (long long)sample_bytes, (int*)nullptr);
    return hipGetLastError();
}

}  // namespace ee
