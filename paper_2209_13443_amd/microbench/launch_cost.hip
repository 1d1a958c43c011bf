// Microbenchmark: host time per kernel launch for small and 1 KB argument blocks (why the slot tables of zero-copy
// compaction are not passed to every convolution launch by value).
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <chrono>
#include <cstdio>
struct Big { unsigned short s[512]; };
__global__ void k_small(int* p) { if (p && threadIdx.x == 9999) *p = 1; }
__global__ void k_big(Big b, int* p) { if (p && threadIdx.x == 9999) *p = b.s[3]; }
int main()
{
    hipStream_t s; hipStreamCreate(&s);
    Big b{};
    const int N = 20000;
    auto t = [&](const char* name, auto f) {
        for (int i = 0; i < 1000; ++i) f();
        hipStreamSynchronize(s);
        auto t0 = std::chrono::steady_clock::now();
        for (int i = 0; i < N; ++i) f();
        auto t1 = std::chrono::steady_clock::now();
        hipStreamSynchronize(s);
        auto t2 = std::chrono::steady_clock::now();
        printf("%-40s host %.2f us per launch, end to end %.2f us per launch\n", name, std::chrono::duration<double, std::micro>(t1 - t0).count() / N,
               std::chrono::duration<double, std::micro>(t2 - t0).count() / N);
    };
    t("hipLaunchKernelGGL small args", [&] { hipLaunchKernelGGL(k_small, dim3(256), dim3(256), 0, s, (int*)nullptr); });
    t("hipExtLaunchKernelGGL small args", [&] { hipExtLaunchKernelGGL(k_small, dim3(256), dim3(256), 0, s, nullptr, nullptr, 0, (int*)nullptr); });
    t("hipLaunchKernelGGL 1 KB args", [&] { hipLaunchKernelGGL(k_big, dim3(256), dim3(256), 0, s, b, (int*)nullptr); });
    t("hipExtLaunchKernelGGL 1 KB args", [&] { hipExtLaunchKernelGGL(k_big, dim3(256), dim3(256), 0, s, nullptr, nullptr, 0, b, (int*)nullptr); });
    return 0;
}
