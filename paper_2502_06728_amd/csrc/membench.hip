// Plain streaming kernels of known size: the achievable HBM ceiling on this GPU and the
// calibration point for rocprofv3's FETCH_SIZE / WRITE_SIZE counters.
//   membench [MiB per buffer = 1024] [iterations = 20]
// copy: reads B bytes and writes B bytes; read: reads B; fill: writes B.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                  \
    do {                                                                          \
        hipError_t e = (x);                                                       \
        if (e != hipSuccess) {                                                    \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e));                \
            return 1;                                                             \
        }                                                                         \
    } while (0)

__global__ __launch_bounds__(256) void copy_kernel(const float4* __restrict__ in,
                                                   float4* __restrict__ out, size_t n16) {
    size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (; i < n16; i += stride) out[i] = in[i];
}

__global__ __launch_bounds__(256) void read_kernel(const float4* __restrict__ in,
                                                   float* __restrict__ sink, size_t n16) {
    size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    float acc = 0.f;
    for (; i < n16; i += stride) {
        const float4 v = in[i];
        acc += v.x + v.y + v.z + v.w;
    }
    if (acc == 123.456f) *sink = acc;
}

__global__ __launch_bounds__(256) void fill_kernel(float4* __restrict__ out, size_t n16) {
    size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    for (; i < n16; i += stride) out[i] = make_float4(1.f, 2.f, 3.f, 4.f);
}

int main(int argc, char** argv) {
    const size_t mib = argc > 1 ? strtoull(argv[1], nullptr, 10) : 1024;
    const int iters = argc > 2 ? atoi(argv[2]) : 20;
    const size_t bytes = mib << 20, n16 = bytes / 16;
    float4 *a, *b;
    float* sink;
    CHECK(hipMalloc(&a, bytes));
    CHECK(hipMalloc(&b, bytes));
    CHECK(hipMalloc(&sink, 4));
    CHECK(hipMemset(a, 1, bytes));
    CHECK(hipMemset(b, 2, bytes));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int grids[] = {256 * 8, 256 * 32, 256 * 128, 0};
    for (int gi = 0; gi < 4; ++gi) {
        const unsigned grid = grids[gi] ? grids[gi] : static_cast<unsigned>((n16 + 255) / 256);
        for (int mode = 0; mode < 3; ++mode) {
            for (int w = 0; w < 2; ++w) {
                if (mode == 0) copy_kernel<<<grid, 256>>>(a, b, n16);
                if (mode == 1) read_kernel<<<grid, 256>>>(a, sink, n16);
                if (mode == 2) fill_kernel<<<grid, 256>>>(b, n16);
            }
            CHECK(hipEventRecord(e0));
            for (int it = 0; it < iters; ++it) {
                if (mode == 0) copy_kernel<<<grid, 256>>>(a, b, n16);
                if (mode == 1) read_kernel<<<grid, 256>>>(a, sink, n16);
                if (mode == 2) fill_kernel<<<grid, 256>>>(b, n16);
            }
            CHECK(hipEventRecord(e1));
            CHECK(hipEventSynchronize(e1));
            float ms;
            CHECK(hipEventElapsedTime(&ms, e0, e1));
            const double moved = (mode == 0 ? 2.0 : 1.0) * bytes * iters;
            printf("%s grid=%u buffer=%zu MiB: %.1f GB/s (%.3f ms per launch)\n",
                   mode == 0 ? "copy" : (mode == 1 ? "read" : "fill"), grid, mib,
                   moved / (ms * 1e-3) / 1e9, ms / iters);
        }
    }
    CHECK(hipGetLastError());
    return 0;
}
