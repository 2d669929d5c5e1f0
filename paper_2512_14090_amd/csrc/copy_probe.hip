// Plain copy kernel of known size: the calibration run for the HBM traffic counters
// (FETCH_SIZE / WRITE_SIZE per dispatch are scaled by what they read for this copy).
// Built as a stand-alone program by build.build_copy_probe() (python -m paper_2512_14090_amd.build --copy-probe);
// not part of libaiq.so and not built by build().
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef float floatx4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void copy_probe_kernel(const floatx4 *__restrict__ src, floatx4 *__restrict__ dst,
                                                         size_t n4)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

int main(int argc, char **argv)
{
    const size_t mib = argc > 1 ? strtoull(argv[1], nullptr, 10) : 1024;
    const int reps = argc > 2 ? atoi(argv[2]) : 5;
    const size_t bytes = mib << 20, n4 = bytes / 16;
    floatx4 *src = nullptr, *dst = nullptr;
    if (hipMalloc(&src, bytes) != hipSuccess || hipMalloc(&dst, bytes) != hipSuccess) return 1;
    hipMemset(src, 1, bytes);
    hipMemset(dst, 0, bytes);
    hipEvent_t e0, e1;
    hipEventCreate(&e0);
    hipEventCreate(&e1);
    float best = 1e30f;
    for (int r = 0; r < reps; ++r) {
        hipEventRecord(e0, 0);
        hipLaunchKernelGGL(copy_probe_kernel, dim3(256 * 32), dim3(256), 0, 0, src, dst, n4);
        hipEventRecord(e1, 0);
        hipEventSynchronize(e1);
        float ms = 0;
        hipEventElapsedTime(&ms, e0, e1);
        if (ms < best) best = ms;
    }
    if (hipDeviceSynchronize() != hipSuccess) return 2;
    printf("copy_probe: %zu MiB read + %zu MiB written per launch, best %.3f ms, %.1f GB/s (read+write)\n", mib, mib,
           best, 2.0 * bytes / best / 1e6);
    return 0;
}
