// 1x1 convolutions (int8) over at most 32 input channels: the expansion layers of inverted-residual blocks, also
// those whose pixels are not 16-byte multiples (12, 20, 24, 28 channels), for which the asynchronous-copy kernel
// needs a zero-padded copy of the whole input.  The reduction is one matrix instruction deep, so there is nothing to
// pipeline and nothing is staged: the layer is a stream of pixels read once and written Co / Ci times wider.
// One wavefront = a strip of 32 pixels:
//   * the strip's activations are the B operand of v_mfma_i32_32x32x32_i8 straight from global memory (lane l:
//     pixel l % 32, reduction bytes [16 (l / 32), +16); bytes past Ci are zero), 32 x Ci contiguous bytes;
//   * per tile of 32 output channels one A operand from the packed weights (rows of 32 bytes, zero padded: 1 KB
//     in one piece per wavefront), one matrix instruction, and the requantisation in the accumulator layout
//     (lane: pixel l % 32, channels 32 j + 8 g + 4 (l / 32) + e for register 4 g + e); the bias sits in LDS,
//     because every lane needs 16 values per tile that are the same for all pixels: read from global memory
//     they cost four times the traffic of the output through the vector memory path;
//   * the strip's 32 x Co output bytes go through LDS so that global stores are 16 bytes per lane along the
//     channels (a whole strip is contiguous when the layer owns the whole pixel).
#include "ee_internal.hpp"

namespace ee {

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int thin_med3(int v, int lo, int hi)       // lo <= hi: v clamped to [lo, hi]
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
    return r;
}

__global__ __launch_bounds__(256) void conv_thin_i8_kernel(ThinConvArgs a, int nt, int row_pitch)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char thin_lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 31, hi = lane >> 5;
    // the bias of all channels once per workgroup: every lane needs 16 of them per tile, the same for all pixels
    int* lbias = (int*)(thin_lds + 4 * 32 * row_pitch);
    for (int i = threadIdx.x; i < nt * 32; i += 256) lbias[i] = ((const int*)a.bias)[i];
    const long long m0 = ((long long)blockIdx.x * 4 + wave) * 32;
    const long long m = m0 + p < a.M ? m0 + p : a.M - 1;           // rows past the end read the last pixel and are not stored
    const unsigned char* xr = (const unsigned char*)a.x + m * a.Ci + 16 * hi;
    v4i_t xb = {0, 0, 0, 0};
#pragma unroll
    for (int d = 0; d < 4; ++d)
        if (16 * hi + 4 * d < a.Ci) xb[d] = *(const int*)(xr + 4 * d);
    unsigned char* tile = thin_lds + wave * 32 * row_pitch;
    __syncthreads();
    for (int j = 0; j < nt; ++j) {
        // weight rows are 32 bytes, zero padded: the wavefront reads 1 KB in one piece
        const v4i_t wa = *(const v4i_t*)((const unsigned char*)a.w + (size_t)(32 * j + p) * 32 + 16 * hi);
        v16i_t acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0;
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wa, xb, acc, 0, 0, 0);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int cl = 32 * j + 8 * g + 4 * hi;
            const v4i_t b4 = *(const v4i_t*)(lbias + cl);                       // the rounding constant is part of the bias
            int q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) q[e] = thin_med3((acc[4 * g + e] + b4[e]) >> a.shift, a.lo, a.hi);
            const unsigned lo2 = __builtin_amdgcn_perm((unsigned)q[1], (unsigned)q[0], 0x0c0c0400u), hi2 = __builtin_amdgcn_perm((unsigned)q[3], (unsigned)q[2], 0x0c0c0400u);
            *(unsigned*)(tile + p * row_pitch + cl) = __builtin_amdgcn_perm(hi2, lo2, 0x05040100u);
        }
    }
    __syncthreads();
    const int cr = a.Co >> 4;                                         // 16-byte chunks per output pixel
    for (int q = lane; q < 32 * cr; q += 64) {
        const int row = q / cr, ch = (q - row * cr) * 16;
        if (m0 + row < a.M) *(v4i_t*)((unsigned char*)a.y + (m0 + row) * a.ldc + a.c_off + ch) = *(const v4i_t*)(tile + row * row_pitch + ch);
    }
}

bool conv_thin_supported(int es, int kh, int kw, int stride, int pad, int pad_w, int ci, int co, int c_tot, int c_off, bool has_res)
{
    return es == 1 && kh == 1 && kw == 1 && stride == 1 && pad == 0 && pad_w == 0 && ci >= 4 && ci <= 32 && ci % 4 == 0 &&
           co % 16 == 0 && co <= 1024 && c_tot % 16 == 0 && c_off % 16 == 0 && !has_res;
}

hipError_t launch_conv_thin(const ThinConvArgs& a, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    const int nt = (a.Co + 31) / 32, row_pitch = nt * 32 + 16;        // + 16: rows 7 dwords apart modulo 8 banks apart
    const size_t lds_bytes = (size_t)4 * 32 * row_pitch + (size_t)nt * 32 * 4;
    if (lds_bytes > 160 * 1024) return hipErrorInvalidValue;
    static const hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void*>(&conv_thin_i8_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (granted != hipSuccess) return granted;
    const long long strips = (a.M + 31) / 32;
    EE_LAUNCH(conv_thin_i8_kernel, dim3((unsigned)((strips + 3) / 4)), dim3(256), lds_bytes, s, a, nt, row_pitch);
    return hipGetLastError();
}

}  // namespace ee
