// Microbenchmark: issue interval of the matrix instructions the convolution kernels use, one and two wavefronts per SIMD,
// independent and dependent accumulators.  (Cycles are the shader clock, s_memtime.)
#include <hip/hip_runtime.h>
#include <cstdio>
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v4acc __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
// MODE 0: 4 independent i8 32x32x32 accumulators; 1: one dependent chain; 2: 4 independent 16x16x64 i8; 3: bf16 32x32x16 x4
template <int MODE>
__global__ __launch_bounds__(256) void k(int iters, unsigned long long* out)
{
    v4i a = {(int)threadIdx.x, 1, 2, 3}, b = {3, 2, 1, (int)blockIdx.x};
    v16i c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    v4acc d0 = {0}, d1 = {0}, d2 = {0}, d3 = {0};
    v16f f0 = {0}, f1 = {0}, f2 = {0}, f3 = {0};
    const unsigned long long t0 = clock64();
    for (int i = 0; i < iters; ++i) {
        if (MODE == 0) {
            c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0); c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0); c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
        } else if (MODE == 1) {
            c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0); c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
            c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0); c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
        } else if (MODE == 2) {
            d0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, d0, 0, 0, 0); d1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, d1, 0, 0, 0);
            d2 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, d2, 0, 0, 0); d3 = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, d3, 0, 0, 0);
        } else {
            v8bf x = __builtin_bit_cast(v8bf, a), y = __builtin_bit_cast(v8bf, b);
            f0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, f0, 0, 0, 0); f1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, f1, 0, 0, 0);
            f2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, f2, 0, 0, 0); f3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, f3, 0, 0, 0);
        }
    }
    const unsigned long long t1 = clock64();
    if (threadIdx.x % 64 == 0) out[blockIdx.x * 4 + threadIdx.x / 64] = t1 - t0;
    int s = c0[0] + c1[1] + c2[2] + c3[3] + d0[0] + d1[1] + d2[2] + d3[3] + (int)(f0[0] + f1[1] + f2[2] + f3[3]);
    if (s == 0x1234567) out[0] = 0;
}
template <int MODE>
void run(unsigned long long* d, int wgs, const char* name)
{
    const int iters = 2000;
    unsigned long long h[4096];
    k<MODE><<<wgs, 256>>>(iters, d); k<MODE><<<wgs, 256>>>(iters, d);
    hipMemcpy(h, d, 8 * 4 * wgs, hipMemcpyDeviceToHost);
    double c = 0; for (int i = 0; i < 4 * wgs; ++i) c += h[i];
    printf("%-28s wgs %4d: %.1f cycles per MFMA per wave\n", name, wgs, c / (4 * wgs) / (4.0 * iters));
}
int main()
{
    unsigned long long* d; hipMalloc(&d, 8 * 4096);
    run<0>(d, 256, "i8 32x32x32, 4 independent"); run<0>(d, 512, "i8 32x32x32, 4 independent");
    run<1>(d, 256, "i8 32x32x32, dependent");
    run<2>(d, 256, "i8 16x16x64, 4 independent"); run<2>(d, 512, "i8 16x16x64, 4 independent");
    run<3>(d, 256, "bf16 32x32x16, 4 independent"); run<3>(d, 512, "bf16 32x32x16, 4 independent");
    return 0;
}
