// Microbenchmark: the time between a dispatch's begin and end time stamps (what a kernel trace reports as a kernel's
// duration) for kernels that do next to nothing: an empty one, one workgroup per sample reading 4 KB and writing a word,
// and the same with a record written to pinned host memory behind a system-scope fence.  The floor under the exit head's
// FC and softmax launches.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <cstdio>
__global__ void k_empty() {}
__global__ void k_read(const int* x, int* y)
{
    int v = 0;
    for (int i = threadIdx.x; i < 1024; i += 256) v += x[blockIdx.x * 1024 + i];
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    if ((threadIdx.x & 63) == 0) atomicAdd(y + blockIdx.x, v);
}
__global__ void k_read_host(const int* x, int* y, int* host, unsigned* counter, unsigned* seq)
{
    int v = 0;
    for (int i = threadIdx.x; i < 1024; i += 256) v += x[blockIdx.x * 1024 + i];
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    if ((threadIdx.x & 63) == 0) atomicAdd(y + blockIdx.x, v);
    __syncthreads();
    if (threadIdx.x == 0) {
        host[blockIdx.x] = y[blockIdx.x];
        __threadfence_system();
        if (atomicAdd(counter, 1u) == gridDim.x - 1u) {     // the last workgroup tells the host
            *counter = 0u;
            __threadfence_system();
            __hip_atomic_store(seq, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}
int main()
{
    hipStream_t s; hipStreamCreate(&s);
    hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
    int *x, *y, *host; unsigned *counter, *seq;
    hipMalloc(&x, 64 * 4096); hipMalloc(&y, 64 * 4); hipMalloc(&counter, 4);
    hipMemset(x, 1, 64 * 4096); hipMemset(y, 0, 64 * 4); hipMemset(counter, 0, 4);
    hipHostMalloc(&host, 64 * 4); hipHostMalloc(&seq, 4);
    auto t = [&](const char* name, auto launch) {
        float sum = 0;
        const int reps = 50;
        for (int i = 0; i < reps + 5; ++i) {
            launch();
            hipStreamSynchronize(s);
            float ms = 0; hipEventElapsedTime(&ms, e0, e1);
            if (i >= 5) sum += ms;
        }
        printf("%-64s %.2f us\n", name, sum / reps * 1000.f);
    };
    t("empty kernel, 1 workgroup", [&] { hipExtLaunchKernelGGL(k_empty, dim3(1), dim3(64), 0, s, e0, e1, 0); });
    t("empty kernel, 256 workgroups of 256", [&] { hipExtLaunchKernelGGL(k_empty, dim3(256), dim3(256), 0, s, e0, e1, 0); });
    t("64 workgroups: 4 KB read, one atomic each", [&] { hipExtLaunchKernelGGL(k_read, dim3(64), dim3(256), 0, s, e0, e1, 0, (const int*)x, y); });
    t("the same + a word to pinned host memory, fence, sequence word", [&] { hipExtLaunchKernelGGL(k_read_host, dim3(64), dim3(256), 0, s, e0, e1, 0, (const int*)x, y, host, counter, seq); });
    return 0;
}
