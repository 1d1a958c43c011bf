// global -> LDS (global_load_lds_dwordx4) against global -> registers (global_load_dwordx4): bytes per clock and CU
// when every CU streams tiles of rows out of a buffer that fits L2 / the last-level cache.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef int v4i __attribute__((ext_vector_type(4)));
__device__ __forceinline__ unsigned lds_addr(const void* p) { return (unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)p; }
__device__ __forceinline__ void dma16(unsigned lds_base, const void* base, unsigned voff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(base) : "memory");
}
// MODE 0: LDS DMA, MODE 1: register loads (summed)
// each wave-instruction reads 8 rows x 128 bytes (row pitch `pitch`), like a 128-byte reduction step of the conv kernel
template <int MODE>
__global__ __launch_bounds__(256) void stream(const unsigned char* buf, unsigned region_bytes, unsigned pitch, int iters, int* out)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = lds_addr(lds) + wave * 8192;
    // this workgroup's tile: 256 rows starting at a block-dependent row
    const unsigned rows_total = region_bytes / pitch;
    unsigned row0 = (blockIdx.x * 97u * 64u) % (rows_total - 512);
    const unsigned lrow = wave * 64 + (lane >> 3), chunk = lane & 7;
    unsigned voff = (row0 + lrow) * pitch + chunk * 16;
    v4i acc = {0, 0, 0, 0};
    const unsigned kmax = pitch / 128;
    unsigned k = 0;
    for (int it = 0; it < iters; ++it) {
        // 8 instructions = 64 rows x 128 bytes per wave = 8 KB; 32 KB per workgroup and iteration
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (MODE == 0) dma16(lds0 + j * 1024, buf, voff + j * 8 * pitch);
            else { v4i v; asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(v) : "v"(voff + j * 8 * pitch), "s"(buf) : "memory"); acc += v; }
        }
        if (MODE == 0) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");       // one iteration stays in flight
        voff += 128;
        if (++k == kmax) { k = 0; voff -= pitch; }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (MODE == 1 && acc[0] + acc[1] + acc[2] + acc[3] == 0x12345678) out[0] = 1;
    if (MODE == 0 && lds[threadIdx.x] == 0x7f && lds[threadIdx.x + 999] == 0x11) out[1] = 1;
}
template <int MODE>
void run(const unsigned char* buf, unsigned region, unsigned pitch, int wgs_per_cu, int lds_bytes, int* d)
{
    const int iters = 400, grid = 256 * wgs_per_cu;
    hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
    stream<MODE><<<grid, 256, lds_bytes>>>(buf, region, pitch, 10, d);
    (void)hipEventRecord(e0);
    stream<MODE><<<grid, 256, lds_bytes>>>(buf, region, pitch, iters, d);
    (void)hipEventRecord(e1); (void)hipEventSynchronize(e1);
    float ms; (void)hipEventElapsedTime(&ms, e0, e1);
    const double bytes = (double)grid * iters * 32768;
    printf("%s region %6.1f MB pitch %5u wgs/cu %d: %7.1f us  %6.2f TB/s  %5.1f GB/s per CU = %4.1f B/clk at 2.4 GHz\n", MODE ? "regs" : "lds ", region / 1e6, pitch, wgs_per_cu,
           ms * 1e3, bytes / (ms * 1e-3) / 1e12, bytes / 256 / (ms * 1e-3) / 1e9, bytes / 256 / (ms * 1e-3) / 2.4e9);
}
int main()
{
    unsigned char* buf; (void)hipMalloc(&buf, 512u << 20); (void)hipMemset(buf, 1, 512u << 20);
    int* d; (void)hipMalloc(&d, 8);
    for (unsigned region : {2u << 20, 16u << 20, 128u << 20})
        for (unsigned pitch : {256u, 2304u})
            for (int w : {1, 2, 4}) {
                run<0>(buf, region, pitch, w, 32768, d);
                run<1>(buf, region, pitch, w, 32768, d);
            }
    printf("%s\n", hipGetErrorString(hipDeviceSynchronize()));
    return 0;
}
