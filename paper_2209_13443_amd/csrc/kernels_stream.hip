// Streaming implicit GEMM (int8) for layers with many pixels, few channels and a short reduction: the folded
// stride-2 first layer (2 x 2 or 4 x 4 taps over 16-channel super-pixels), 3 x 3 / 1 x 3 / 3 x 1 layers over 32
// channels; at most 64 output channels, no residual.  Such layers read and write every pixel once and compute
// little: in the asynchronous-copy kernel a workgroup's set-up and epilogue outweigh its one or two reduction steps.
// Here nothing is staged and the work is a loop:
//   * a wavefront keeps the layer's weights (one v_mfma_i32_32x32x32_i8 A operand per 32 channels and 32-byte block
//     of the reduction, at most 18 of them) and its bias in registers and walks over strips of 32 pixels;
//   * per strip the B operands come straight from global memory: a 32-byte block of the reduction lies inside one
//     kernel row, lane l reads the 16 bytes [16 (l / 32), +16) of it for pixel l % 32 -- one pixel (16 channels) or
//     half a pixel (32 channels); coordinates are clamped so that every load is in range, a tap outside the image
//     becomes zero;
//   * requantisation in the accumulator layout (lane: pixel l % 32, channels 32 j + 8 g + 4 (l / 32) + e for
//     register 4 g + e), the strip's 32 x Co bytes go through the wavefront's own LDS tile into 16-byte stores.
// Wavefronts never wait for one another (no workgroup barrier inside the loop); every wavefront leaves the loop when
// its strips are used up.
#include "ee_internal.hpp"

namespace ee {

typedef int v4i_s __attribute__((ext_vector_type(4)));
typedef int v16i_s __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int stream_med3(int v, int lo, int hi)       // lo <= hi: v clamped to [lo, hi]
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}
__device__ __forceinline__ unsigned stream_div(unsigned n, unsigned d, unsigned magic)   // n / d, magic = floor(2^32 / d) (- 1 for d == 1)
{
    unsigned q = __umulhi(n, magic);
    if (n - q * d >= d) ++q;
    return q;
}

// KH kernel rows of BPR 32-byte blocks each; NT tiles of 32 output channels
template <int KH, int BPR, int NT>
__global__ __launch_bounds__(256) void conv_stream_i8_kernel(ConvArgs a, long long nstrips)
{
    constexpr int NKB = KH * BPR, ROW_PITCH = NT * 32 + 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char stream_lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 31, hi = lane >> 5;
    unsigned char* tile = stream_lds + wave * 32 * ROW_PITCH;
    const unsigned char* wb = (const unsigned char*)a.w;
    v4i_s wreg[NT][NKB], breg[NT][4];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) wreg[j][kb] = *(const v4i_s*)(wb + (size_t)(32 * j + p) * a.Kp + kb * 32 + 16 * hi);
#pragma unroll
        for (int g = 0; g < 4; ++g) breg[j][g] = *(const v4i_s*)((const int*)a.bias + 32 * j + 8 * g + 4 * hi);   // rounding constant included
    }
    const int cr = a.Co >> 4;                                         // 16-byte chunks per output pixel
    const unsigned char* xb0 = (const unsigned char*)a.x;
    const int px_per_block = 32 / a.Ci;                               // 2 (16 channels) or 1 (32 channels)
    // the B operands of one strip: issued one strip ahead, so that their latency hides behind the previous strip's work
    auto load_strip = [&](long long strip, v4i_s* xr, unsigned& okmask) {
        const unsigned m = (unsigned)(strip * 32 + p < a.M ? strip * 32 + p : a.M - 1);    // rows past the end redo the last pixel and are not stored
        const unsigned n = stream_div(m, (unsigned)(a.Ho * a.Wo), a.magic_howo);
        const unsigned rem = m - n * (unsigned)(a.Ho * a.Wo);
        const unsigned oy = stream_div(rem, (unsigned)a.Wo, a.magic_wo), ox = rem - oy * (unsigned)a.Wo;
        const int iy0 = (int)oy * a.stride - a.pad, ix0 = (int)ox * a.stride - a.pad_w;
        okmask = 0;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            const int r = kb / BPR, cb = (kb % BPR) * 32 + 16 * hi;   // kernel row, byte inside the kernel row
            const int s = px_per_block == 2 ? cb >> 4 : cb >> 5, bo = px_per_block == 2 ? 0 : cb & 16;
            const int iy = iy0 + r, ix = ix0 + s;
            if ((unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W) okmask |= 1u << kb;
            // byte offsets inside the batch tensor fit 32 bits (checked when the context is created)
            const unsigned off = (unsigned)(((int)n * a.H + min(max(iy, 0), a.H - 1)) * a.W + min(max(ix, 0), a.W - 1)) * (unsigned)a.Ci + (unsigned)bo;
            xr[kb] = *(const v4i_s*)(xb0 + off);
        }
    };
    // one strip out of operands that are already on their way: matrix instructions, requantisation, stores
    auto compute_strip = [&](long long strip, const v4i_s* xs, unsigned okmask) {
        const long long m0 = strip * 32;
        const v4i_s zero4 = {0, 0, 0, 0};
        v4i_s xm[NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) xm[kb] = (okmask >> kb) & 1u ? xs[kb] : zero4;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            v16i_s acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[j][kb], xm[kb], acc, 0, 0, 0);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                int q[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) q[e] = stream_med3((acc[4 * g + e] + breg[j][g][e]) >> a.shift, a.lo, a.hi);
                const unsigned lo2 = __builtin_amdgcn_perm((unsigned)q[1], (unsigned)q[0], 0x0c0c0400u), hi2 = __builtin_amdgcn_perm((unsigned)q[3], (unsigned)q[2], 0x0c0c0400u);
                *(unsigned*)(tile + p * ROW_PITCH + 32 * j + 8 * g + 4 * hi) = __builtin_amdgcn_perm(hi2, lo2, 0x05040100u);
            }
        }
        // the wavefront's own tile: its LDS accesses execute in program order, only the compiler must keep that order
        __builtin_amdgcn_wave_barrier();
        // 32 * cr <= 64 * NT chunks: exactly NT stores per lane and strip, none of them conditional, so that the wait
        // for the next strip's operands can leave these stores in flight instead of draining the memory queue.  A lane
        // whose chunk or row does not exist stores the strip's last existing chunk or row once more (same bytes).
        const int last_row = (int)(a.M - 1 - m0 < 31 ? a.M - 1 - m0 : 31);
#pragma unroll
        for (int it = 0; it < NT; ++it) {
            const int q = min(lane + 64 * it, 32 * cr - 1);
            const int row = min(q / cr, last_row), ch = (q % cr) * 16;
            *(v4i_s*)((unsigned char*)a.y + (m0 + row) * a.ldc + a.c_off + ch) = *(const v4i_s*)(tile + row * ROW_PITCH + ch);
        }
        __builtin_amdgcn_wave_barrier();
    };
    // Two operand buffers used in turn: while strip i is computed out of one, the loads of strip i + 1 fill the other.
    // The fences keep the compiler from moving the loads behind the work they are meant to overlap.
    const long long step = (long long)gridDim.x * 4;
    long long strip = (long long)blockIdx.x * 4 + wave;
    if (strip >= nstrips) return;
    v4i_s xa[NKB], xb[NKB];
    unsigned oka = 0, okb = 0;
    load_strip(strip, xa, oka);
    for (;;) {
        // always issued (past the end: the last strip once more), so that the number of loads in flight is fixed
        load_strip(strip + step < nstrips ? strip + step : nstrips - 1, xb, okb);
        __builtin_amdgcn_sched_barrier(0);
        compute_strip(strip, xa, oka);
        __builtin_amdgcn_sched_barrier(0);
        strip += step;
        if (strip >= nstrips) break;
        load_strip(strip + step < nstrips ? strip + step : nstrips - 1, xa, oka);
        __builtin_amdgcn_sched_barrier(0);
        compute_strip(strip, xb, okb);
        __builtin_amdgcn_sched_barrier(0);
        strip += step;
        if (strip >= nstrips) break;
    }
}

bool conv_stream_supported(const ConvArgs& a, int es)
{
    if (es != 1 || a.mode != 0 || a.res != nullptr || a.M <= 0) return false;
    if ((a.Ci != 16 && a.Ci != 32) || (a.kw * a.Ci) % 32 != 0) return false;
    if (a.Co > 64 || a.Co % 16 != 0 || a.ldc % 16 != 0 || a.c_off % 16 != 0) return false;
    const int bpr = a.kw * a.Ci / 32;
    return (a.kh == 2 && bpr == 1) || (a.kh == 4 && bpr == 2) || (a.kh == 3 && bpr == 3) || (a.kh == 1 && bpr == 3) || (a.kh == 3 && bpr == 1);
}

template <int KH, int BPR, int NT>
static hipError_t launch_stream_inst(const ConvArgs& a, hipStream_t s)
{
    const long long nstrips = ((long long)a.M + 31) / 32;
    const long long want = (nstrips + 3) / 4;
    const long long cap = KH * BPR * NT <= 6 ? 1024 : 512;            // workgroups per CU the registers allow (4 or 2) x 256 CUs; the loop takes the rest
    const unsigned blocks = (unsigned)(want < cap ? want : cap);
    const size_t lds_bytes = (size_t)4 * 32 * (NT * 32 + 16);
    EE_LAUNCH((conv_stream_i8_kernel<KH, BPR, NT>), dim3(blocks), dim3(256), lds_bytes, s, a, nstrips);
    return hipGetLastError();
}

hipError_t launch_conv_stream(const ConvArgs& a, hipStream_t s)
{
    if (!conv_stream_supported(a, 1)) return hipErrorInvalidValue;
    const int bpr = a.kw * a.Ci / 32;
    const bool two = a.Co > 32;
    if (a.kh == 2 && bpr == 1) return two ? launch_stream_inst<2, 1, 2>(a, s) : launch_stream_inst<2, 1, 1>(a, s);
    if (a.kh == 4 && bpr == 2) return two ? launch_stream_inst<4, 2, 2>(a, s) : launch_stream_inst<4, 2, 1>(a, s);
    if (a.kh == 3 && bpr == 3) return two ? launch_stream_inst<3, 3, 2>(a, s) : launch_stream_inst<3, 3, 1>(a, s);
    if (a.kh == 1 && bpr == 3) return two ? launch_stream_inst<1, 3, 2>(a, s) : launch_stream_inst<1, 3, 1>(a, s);
    return two ? launch_stream_inst<3, 1, 2>(a, s) : launch_stream_inst<3, 1, 1>(a, s);
}

}  // namespace ee
