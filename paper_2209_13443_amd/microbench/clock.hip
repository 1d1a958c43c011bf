// Microbenchmark: the shader clock the chip actually runs at in short and long kernels (s_memtime against the 100 MHz s_memrealtime).
#include <hip/hip_runtime.h>
#include <cstdio>
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256) void spin(int iters, int mfma, unsigned long long* out)
{
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    v16i acc = {0};
    v4i a = {(int)threadIdx.x, 1, 2, 3}, b = {3, 2, 1, (int)blockIdx.x};
    int x = threadIdx.x;
    for (int i = 0; i < iters; ++i) {
        if (mfma) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc, 0, 0, 0);
        else { x = x * 1664525 + 1013904223; x ^= x >> 7; }
    }
    const unsigned long long c1 = clock64(), w1 = wall_clock64();
    if (threadIdx.x == 0) { out[blockIdx.x * 2] = c1 - c0; out[blockIdx.x * 2 + 1] = w1 - w0; }
    if (acc[0] + x == 0x12345) out[0] = 0;
}
int main()
{
    unsigned long long* d; hipMalloc(&d, 16 * 4096);
    unsigned long long h[8192];
    for (int mfma = 0; mfma < 2; ++mfma)
        for (int iters : {200, 2000, 20000, 200000}) {
            for (int rep = 0; rep < 3; ++rep) spin<<<1024, 256>>>(iters, mfma, d);
            hipMemcpy(h, d, 16 * 1024, hipMemcpyDeviceToHost);
            double c = 0, w = 0; for (int i = 0; i < 1024; ++i) { c += h[2 * i]; w += h[2 * i + 1]; }
            printf("%s iters %6d: %.1f core cycles, %.2f us -> %.3f GHz\n", mfma ? "mfma" : "valu", iters, c / 1024, w / 1024 / 100.0, c / w * 0.1);
        }
    return 0;
}
