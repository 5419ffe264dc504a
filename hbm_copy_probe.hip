// Plain copy kernel of known size: the yardstick for the HBM counters and for what this chip's
// memory system sustains on a pure stream.  Usage: hbm_copy_probe [MiB per buffer] [repeats]
// Prints the bytes one launch reads and writes and the bandwidth from HIP events.
// Not part of the library; build it by hand when profiling:
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops -o hbm_copy_probe hbm_copy_probe.hip
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e_ = (x);                                                              \
        if (e_ != hipSuccess) { std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } \
    } while (0)

__global__ void __launch_bounds__(256) k_plain_copy(float4 *__restrict__ dst, const float4 *__restrict__ src, size_t n4)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) dst[i] = src[i];
}

int main(int argc, char **argv)
{
    const size_t mib = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 2048;
    const int repeats = argc > 2 ? std::atoi(argv[2]) : 20;
    const size_t bytes = mib << 20, n4 = bytes / sizeof(float4);
    float4 *src = nullptr, *dst = nullptr;
    CHECK(hipMalloc(&src, bytes));
    CHECK(hipMalloc(&dst, bytes));
    CHECK(hipMemset(src, 1, bytes));
    CHECK(hipMemset(dst, 0, bytes));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int grid = 256 * 8;
    k_plain_copy<<<grid, 256>>>(dst, src, n4);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    for (int r = 0; r < repeats; ++r) k_plain_copy<<<grid, 256>>>(dst, src, n4);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double per_launch_s = ms / 1e3 / repeats;
    std::printf("plain copy: %zu bytes read + %zu bytes written per launch, %d launches, %.3f ms each, %.1f GB/s (read+write)\n",
                bytes, bytes, repeats + 1, per_launch_s * 1e3, 2.0 * bytes / per_launch_s / 1e9);
    CHECK(hipFree(src));
    CHECK(hipFree(dst));
    return 0;
}
