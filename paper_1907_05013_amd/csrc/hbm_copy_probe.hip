// Calibration aid for hardware-counter readings: a plain copy kernel of known size.
// Run under `rocprofv3 --pmc FETCH_SIZE` (then `--pmc WRITE_SIZE`): the counter value per
// dispatch of copy_probe_kernel, divided by the bytes it is known to read (write), gives the
// factor by which the same counter's readings for other kernels are scaled.
//   usage: hbm_copy_probe [MiB per buffer, default 1024] [launches, default 5]
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

__global__ __launch_bounds__(256) void copy_probe_kernel(const float4 *__restrict__ src, float4 *__restrict__ dst, size_t n4)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) dst[i] = src[i];
}

int main(int argc, char **argv)
{
    const size_t mib = argc > 1 ? (size_t)atol(argv[1]) : 1024;
    const int launches = argc > 2 ? atoi(argv[2]) : 5;
    const size_t bytes = mib << 20, n4 = bytes / 16;
    float4 *src = nullptr, *dst = nullptr;
    if (hipMalloc(&src, bytes) != hipSuccess || hipMalloc(&dst, bytes) != hipSuccess) {
        fprintf(stderr, "hipMalloc failed\n");
        return 1;
    }
    hipMemset(src, 1, bytes);
    hipMemset(dst, 0, bytes);
    hipEvent_t e0, e1;
    hipEventCreate(&e0);
    hipEventCreate(&e1);
    copy_probe_kernel<<<4096, 256>>>(src, dst, n4);
    hipDeviceSynchronize();
    hipEventRecord(e0);
    for (int i = 0; i < launches; ++i) copy_probe_kernel<<<4096, 256>>>(src, dst, n4);
    hipEventRecord(e1);
    hipEventSynchronize(e1);
    float ms = 0.f;
    hipEventElapsedTime(&ms, e0, e1);
    printf("copy_probe_kernel: %zu bytes read + %zu bytes written per launch, %d launches, %.3f ms each, %.1f GB/s\n", bytes, bytes,
           launches, ms / launches, 2.0 * bytes * launches / (ms * 1e-3) / 1e9);
    hipFree(src);
    hipFree(dst);
    return 0;
}
