// First convolution and max-pool of a ResNet-style network (int8) in one launch, for gfx950: the folded stride-2 first layer
// (4 x 4 taps over 16-channel super-pixels, 64 output channels; what conv_stream_i8_kernel runs alone) and the 3 x 3 / 2 max-pool
// with padding 1 behind it.  Layer by layer the convolution's output, the largest tensor of the network, is written once and read
// once for a quarter of its size to come out of the pool; here it only exists in LDS, a tile at a time.
//
// A workgroup (4 wavefronts) walks over tiles of 14 x 8 pooled pixels of one image.  The 29 x 17 convolution outputs under a tile's
// windows are computed in 16 strips of 32, four per wavefront, as in the streaming kernel: weights in registers for good, the activation
// operands straight from global memory, requested two strips ahead through four sets of registers (also across the pooling and into the
// next tile: a strip's operands come out of L2 in about the time two strips take), 16 matrix instructions per strip, requantisation, and the strip's pixels
// go to the tile's LDS image -- the smallest int8 value where the convolution has no output (the pool's padding: every window
// has at least one pixel that exists).  After a barrier the lanes take (pooled pixel, 16 channels) items, 448 per tile: nine 16-byte
// LDS reads, byte-wise maximum on 16-bit halves, one 16-byte store.  A seventh of the convolution is computed twice (the windows'
// overlap between tiles and the last strip's padding); results are those of the two layers bit for bit.
#include "ee_internal.hpp"
#include "ir_device.hpp"

namespace ee {

typedef short v2s_r __attribute__((ext_vector_type(2)));

struct StemTile {
    int Hq, Wq;                // pooled image
    int tiles_x, tiles_y;      // tiles of 14 x 8 pooled pixels per image
    int total;                 // tiles in all
};

constexpr int ST_TW = 14, ST_TH = 8;                       // pooled pixels per tile
constexpr int ST_RW = 2 * ST_TW + 1, ST_RH = 2 * ST_TH + 1;   // convolution outputs under them
constexpr int ST_RPIX = ST_RW * ST_RH;                     // 493
constexpr int ST_STRIPS = (ST_RPIX + 31) / 32;             // 16: four per wavefront
constexpr int ST_ITEMS = 4 * ST_TW * ST_TH;                // (pooled pixel, 16 channels) per tile
static_assert(ST_STRIPS == 16, "four strips per wavefront");
constexpr int ST_PITCH = 64 + 16;                          // bytes per convolution output in LDS

// byte-wise signed maximum of two packed dwords kept as (even bytes << 8, odd bytes in place) 16-bit halves
struct StemMax { v2s_r even, odd; };
__device__ __forceinline__ StemMax stem_split(unsigned d)
{
    const unsigned e = (d << 8) & 0xff00ff00u, o = d & 0xff00ff00u;
    StemMax r;
    __builtin_memcpy(&r.even, &e, 4);
    __builtin_memcpy(&r.odd, &o, 4);
    return r;
}
__device__ __forceinline__ StemMax stem_max(const StemMax& a, unsigned d)
{
    const StemMax b = stem_split(d);
    return StemMax{__builtin_elementwise_max(a.even, b.even), __builtin_elementwise_max(a.odd, b.odd)};
}
__device__ __forceinline__ unsigned stem_join(const StemMax& a)
{
    unsigned e, o;
    __builtin_memcpy(&e, &a.even, 4);
    __builtin_memcpy(&o, &a.odd, 4);
    return ((e >> 8) & 0x00ff00ffu) | o;
}

__global__ __launch_bounds__(256, 2) void stem_pool_i8_kernel(ConvArgs a, void* yq, StemTile t)
{
    constexpr int NKB = 8, NT = 2;                                      // 32-byte blocks of the reduction (4 rows x 2), blocks of 32 output channels
    extern __shared__ __attribute__((aligned(16))) unsigned char stem_lds[];
    const int tid = threadIdx.x, lane = tid & 63, p = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned char* wb = (const unsigned char*)a.w;
    v4i_r wreg[NT][NKB];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) wreg[j][kb] = *(const v4i_r*)(wb + (size_t)(32 * j + p) * a.Kp + kb * 32 + 16 * hi);
    int* const l_bias = (int*)(stem_lds + ST_RPIX * ST_PITCH);         // 64 biases behind the tile's image (rounding constant included)
    if (tid < 64) l_bias[tid] = ((const int*)a.bias)[tid];
    // every weight has arrived before the loop, so that nothing inside it waits for a weight by count
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) asm volatile("" : "+v"(wreg[j][kb]));
    __syncthreads();
    const IrClamp cl = ir_clamp(a.shift, a.lo, a.hi);
    const int tpi = t.tiles_x * t.tiles_y;
    // pooling: this lane's items (pooled pixel, channels): tid and tid + 256
    const int pch = tid & 3;
    int pty[2], ptx[2], poff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int pp = min(tid + 256 * i, ST_ITEMS - 1) >> 2;
        pty[i] = pp / ST_TW; ptx[i] = pp - pty[i] * ST_TW;
        poff[i] = ((2 * pty[i]) * ST_RW + 2 * ptx[i]) * ST_PITCH + 16 * pch;
    }

    struct Tile { int n, py0, px0; };
    auto tile_at = [&](int u) {
        const int n = u / tpi, r0 = u - n * tpi, tyi = r0 / t.tiles_x;
        return Tile{n, ST_TH * tyi, ST_TW * (r0 - tyi * t.tiles_x)};
    };
    auto load_strip = [&](const Tile& tl, int s, v4i_r* xr) {           // unconditional and in range; the folded input carries its own padding
        const unsigned char* xn = (const unsigned char*)a.x + (size_t)tl.n * a.H * a.W * 16;
        const int r = min(32 * s + p, ST_RPIX - 1), ry = r / ST_RW, rx = r - ry * ST_RW;
        const int cy = min(max(2 * tl.py0 - 1 + ry, 0), a.Ho - 1), cx = min(max(2 * tl.px0 - 1 + rx, 0), a.Wo - 1);
        // the four rows and four columns under the clamped output are inside the folded image (it has three rows and columns more than
        // the convolution's output: checked by the launcher), so the eight operands lie at fixed offsets from the first
        const unsigned char* first = xn + (unsigned)((cy * a.W + cx + hi) * 16);
        const unsigned row = (unsigned)a.W * 16;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) xr[kb] = *(const v4i_r*)(first + (kb >> 1) * row + (kb & 1) * 32);
    };
    auto compute_strip = [&](const Tile& tl, int s, const v4i_r* xr) {
        const int r = 32 * s + p, rc = min(r, ST_RPIX - 1), ry = rc / ST_RW, rx = rc - ry * ST_RW;
        const bool exists = (unsigned)(2 * tl.py0 - 1 + ry) < (unsigned)a.Ho && (unsigned)(2 * tl.px0 - 1 + rx) < (unsigned)a.Wo;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            v16i_r acc;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const v4i_r b4 = *(const v4i_r*)(l_bias + 32 * j + 8 * g + 4 * hi);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[4 * g + e] = b4[e];
            }
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(wreg[j][kb], xr[kb], acc, 0, 0, 0);
            v4i_r o = ir_requant_pack(acc, cl);
            if (!exists) o = v4i_r{(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
            if (r < ST_RPIX) *(v4i_r*)(stem_lds + r * ST_PITCH + 32 * j + 16 * hi) = o;
        }
    };
    // strips wave, wave + 4, wave + 8, wave + 12 of a tile through four operand sets; a strip's operands are requested two strips
    // before it is computed, the first two of the next tile behind this tile's last two
    v4i_r xs[4][NKB];
    int u = (int)blockIdx.x;                                            // the same trip count for the whole workgroup
    if (u < t.total) {
        const Tile t0 = tile_at(u);
        load_strip(t0, wave, xs[0]);
        load_strip(t0, wave + 4, xs[1]);
    }
    for (; u < t.total; u += (int)gridDim.x) {
        const Tile tl = tile_at(u);
        const bool more = u + (int)gridDim.x < t.total;
        const Tile tn = tile_at(more ? u + (int)gridDim.x : u);
        const int n = tl.n, py0 = tl.py0, px0 = tl.px0;
        __builtin_amdgcn_sched_barrier(0);
        load_strip(tl, wave + 8, xs[2]);
        __builtin_amdgcn_sched_barrier(0);
        compute_strip(tl, wave, xs[0]);
        __builtin_amdgcn_sched_barrier(0);
        load_strip(tl, wave + 12, xs[3]);
        __builtin_amdgcn_sched_barrier(0);
        compute_strip(tl, wave + 4, xs[1]);
        __builtin_amdgcn_sched_barrier(0);
        load_strip(tn, wave, xs[0]);                                    // past the last tile: this tile's once more (a fixed number of loads)
        __builtin_amdgcn_sched_barrier(0);
        compute_strip(tl, wave + 8, xs[2]);
        __builtin_amdgcn_sched_barrier(0);
        load_strip(tn, wave + 4, xs[1]);
        __builtin_amdgcn_sched_barrier(0);
        compute_strip(tl, wave + 12, xs[3]);
        __syncthreads();                                                // the tile's convolution outputs are in LDS
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (tid + 256 * i >= ST_ITEMS) continue;
            const unsigned char* win = stem_lds + poff[i];
            const v4i_r first = *(const v4i_r*)win;
            StemMax mx[4];
#pragma unroll
            for (int d = 0; d < 4; ++d) mx[d] = stem_split((unsigned)first[d]);
#pragma unroll
            for (int k = 1; k < 9; ++k) {
                const v4i_r v = *(const v4i_r*)(win + ((k / 3) * ST_RW + (k % 3)) * ST_PITCH);
#pragma unroll
                for (int d = 0; d < 4; ++d) mx[d] = stem_max(mx[d], (unsigned)v[d]);
            }
            const int py = py0 + pty[i], px = px0 + ptx[i];
            if (py < t.Hq && px < t.Wq)
                *(v4i_r*)((unsigned char*)yq + ((size_t)(n * t.Hq + py) * t.Wq + px) * 64 + 16 * pch) =
                    v4i_r{(int)stem_join(mx[0]), (int)stem_join(mx[1]), (int)stem_join(mx[2]), (int)stem_join(mx[3])};
        }
        __syncthreads();                                                // the LDS image is free for the next tile
    }
}

// the convolution as the launcher of the streaming kernel sees it (folded input), the pool behind it by its output size
bool stem_pool_supported(const ConvArgs& a, int Hq, int Wq)
{
    if (a.mode != 0 || a.res != nullptr || a.M <= 0 || a.Ci != 16 || a.kh != 4 || a.kw != 4 || a.stride != 1 || a.pad != 0 || a.pad_w != 0) return false;
    if (a.Co != 64 || a.ldc != 64 || a.c_off != 0 || a.Kp < 256 || a.H < a.Ho + 3 || a.W < a.Wo + 3) return false;
    if (Hq != (a.Ho + 2 - 3) / 2 + 1 || Wq != (a.Wo + 2 - 3) / 2 + 1 || Hq < 1 || Wq < 1) return false;
    return (double)(a.M / (a.Ho * a.Wo)) * a.H * a.W * 16 < 2147483648.0;
}

hipError_t launch_stem_pool(const ConvArgs& a, void* yq, int Hq, int Wq, hipStream_t s)
{
    if (!stem_pool_supported(a, Hq, Wq)) return hipErrorInvalidValue;
    StemTile t;
    t.Hq = Hq; t.Wq = Wq;
    t.tiles_x = (Wq + ST_TW - 1) / ST_TW;
    t.tiles_y = (Hq + ST_TH - 1) / ST_TH;
    const long long total = (long long)(a.M / (a.Ho * a.Wo)) * t.tiles_x * t.tiles_y;
    if (total > 0x3fffffff) return hipErrorInvalidValue;
    t.total = (int)total;
    const unsigned blocks = (unsigned)(total < 512 ? total : 512);      // two workgroups on every CU (what matters is the CU's share, not the workgroup's); the loop takes the rest
    EE_LAUNCH(stem_pool_i8_kernel, dim3(blocks), dim3(256), (size_t)ST_RPIX * ST_PITCH + 256, s, a, yq, t);
    return hipGetLastError();
}

}  // namespace ee
