// Microbenchmark: LDS read bandwidth per CU with ds_read_b128 (conflict-free pattern), by wavefronts per CU.
// What it decides: whether 64 x 64 outputs per wavefront (1 KB of fragments per matrix instruction) can be fed from LDS.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
typedef int v4i __attribute__((ext_vector_type(4)));
template <int WAVES>
__global__ __launch_bounds__(WAVES * 64) void rd(int iters, int* out)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 16384; i += blockDim.x) ((int*)lds)[i] = i;
    __syncthreads();
    const unsigned char* p = lds + lane * 16 + (wave & 3) * 8192;
    v4i a0 = {0,0,0,0}, a1 = a0, a2 = a0, a3 = a0, a4 = a0, a5 = a0, a6 = a0, a7 = a0;
    const unsigned addr = (unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)p;
    for (int it = 0; it < iters; ++it) {
        v4i b0, b1, b2, b3, b4, b5, b6, b7;
        asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:1024\n\tds_read_b128 %2, %8 offset:2048\n\tds_read_b128 %3, %8 offset:3072\n\t"
                     "ds_read_b128 %4, %8 offset:4096\n\tds_read_b128 %5, %8 offset:5120\n\tds_read_b128 %6, %8 offset:6144\n\tds_read_b128 %7, %8 offset:7168\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(b0), "=&v"(b1), "=&v"(b2), "=&v"(b3), "=&v"(b4), "=&v"(b5), "=&v"(b6), "=&v"(b7) : "v"(addr));
        a0 += b0; a1 += b1; a2 += b2; a3 += b3; a4 += b4; a5 += b5; a6 += b6; a7 += b7;
    }
    v4i s = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;
    if (s[0] + s[1] + s[2] + s[3] == 0x12345678) out[0] = 1;
}
template <int WAVES>
void run(int* d, int wgs_per_cu)
{
    const int iters = 2000, grid = 256 * wgs_per_cu;
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    rd<WAVES><<<grid, WAVES * 64, 65536>>>(10, d);
    hipEventRecord(e0);
    rd<WAVES><<<grid, WAVES * 64, 65536>>>(iters, d);
    hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms, e0, e1);
    const double bytes = (double)grid * WAVES * iters * 8 * 1024;
    printf("waves/wg %d, wgs/cu %d: %.1f us, %.1f GB/s per CU = %.1f B/clk at 2.4 GHz\n", WAVES, wgs_per_cu, ms * 1e3, bytes / 256 / (ms * 1e-3) / 1e9, bytes / 256 / (ms * 1e-3) / 2.4e9);
}
int main()
{
    int* d; hipMalloc(&d, 4);
    run<4>(d, 1); run<4>(d, 2); run<8>(d, 1); run<8>(d, 2); run<16>(d, 1);
    printf("%s\n", hipGetErrorString(hipDeviceSynchronize()));
    return 0;
}
