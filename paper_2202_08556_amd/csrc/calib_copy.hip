// Calibration tool for HBM traffic counters: copies a buffer of known size with a plain kernel so
// that FETCH_SIZE / WRITE_SIZE read under `rocprofv3 --pmc` can be scaled to bytes.
//   usage: calib_copy [MiB]   (default 1024)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

__global__ __launch_bounds__(256) void calib_copy_kernel(const float4* __restrict__ src,
                                                         float4* __restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

int main(int argc, char** argv)
{
    const size_t mib = argc > 1 ? (size_t)std::atol(argv[1]) : 1024;
    const size_t bytes = mib << 20;
    float4 *a = nullptr, *b = nullptr;
    if (hipMalloc(&a, bytes) != hipSuccess || hipMalloc(&b, bytes) != hipSuccess) {
        std::printf("allocation failed\n");
        return 1;
    }
    (void)hipMemset(a, 1, bytes);
    (void)hipMemset(b, 0, bytes);
    hipEvent_t e0, e1;
    (void)hipEventCreate(&e0);
    (void)hipEventCreate(&e1);
    for (int rep = 0; rep < 5; ++rep) {
        (void)hipEventRecord(e0);
        hipLaunchKernelGGL(calib_copy_kernel, dim3(8192), dim3(256), 0, 0, a, b, bytes / 16);
        (void)hipEventRecord(e1);
        (void)hipEventSynchronize(e1);
        float ms = 0;
        (void)hipEventElapsedTime(&ms, e0, e1);
        std::printf("copy %zu MiB read + %zu MiB written: %.1f us, %.2f TB/s\n", mib, mib, ms * 1e3,
                    2.0 * bytes / ms / 1e9);
    }
    return hipDeviceSynchronize() == hipSuccess ? 0 : 1;
}
