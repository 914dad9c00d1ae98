// Calibration aid for hardware-counter readings: a plain copy kernel of known size.
// Run under `rocprofv3 --pmc FETCH_SIZE` (then `--pmc WRITE_SIZE`): the counter value per
// dispatch of copy_probe_kernel, divided by the bytes it is known to read (write), gives the
// factor by which the same counter's readings for other kernels are scaled.
// Unprofiled, its rate is the practical HBM ceiling of a streaming kernel on this chip: the
// kernel has the shape the element-wise layers use (one 16-byte item per thread, short-lived
// blocks, non-temporal accesses).
//   usage: hbm_copy_probe [MiB per buffer, default 1024] [launches, default 5]
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef float f32x4 __attribute__((ext_vector_type(4)));

#define CK(call)                                                                        \
    do {                                                                                \
        const hipError_t e_ = (call);                                                   \
        if (e_ != hipSuccess) {                                                         \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));           \
            return 1;                                                                   \
        }                                                                               \
    } while (0)

__global__ __launch_bounds__(256) void copy_probe_kernel(const f32x4 *__restrict__ src, f32x4 *__restrict__ dst, size_t n4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

int main(int argc, char **argv)
{
    const size_t mib = argc > 1 ? (size_t)atol(argv[1]) : 1024;
    const int launches = argc > 2 ? atoi(argv[2]) : 5;
    if (mib < 1 || mib > 65536 || launches < 1) {
        fprintf(stderr, "usage: hbm_copy_probe [MiB per buffer 1..65536] [launches >= 1]\n");
        return 1;
    }
    const size_t bytes = mib << 20, n4 = bytes / 16;
    const unsigned blocks = (unsigned)((n4 + 255) / 256);
    f32x4 *src = nullptr, *dst = nullptr;
    CK(hipMalloc(&src, bytes));
    CK(hipMalloc(&dst, bytes));
    CK(hipMemset(src, 1, bytes));
    CK(hipMemset(dst, 0, bytes));
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    copy_probe_kernel<<<blocks, 256>>>(src, dst, n4);
    CK(hipGetLastError());
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int i = 0; i < launches; ++i) copy_probe_kernel<<<blocks, 256>>>(src, dst, n4);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    printf("copy_probe_kernel: %zu bytes read + %zu bytes written per launch, %d launches, %.3f ms each, %.1f GB/s\n", bytes, bytes,
           launches, ms / launches, 2.0 * bytes * launches / (ms * 1e-3) / 1e9);
    CK(hipFree(src));
    CK(hipFree(dst));
    return 0;
}
