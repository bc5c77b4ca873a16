// Streaming kernels of known size and no arithmetic: the achievable HBM ceilings on this GPU
// and the calibration point for rocprofv3's FETCH_SIZE / WRITE_SIZE counters.
//   membench [MiB per buffer = 1024] [iterations = 20]
// copy: reads B bytes and writes B bytes; read: reads B; fill: writes B.
// Then the two traffic shapes of the optimizer step at chunk 64, k 32, R 4, bf16 gradients and
// parameters, with the launch shape of the library's kernels (one 64-lane workgroup per tile of
// 64 chunks, 16-byte lane accesses) and nothing but loads, a few adds and stores:
//   decompress shape: per tile 8 read streams of 8 KiB (4 replicas x indices, values) plus one
//                     8 KiB stream that is read and rewritten (the parameters);
//   compress shape:   per tile 16 KiB + 8 KiB read (momentum, gradient), 16 KiB + 8 KiB + 8 KiB
//                     written (momentum in place, values, indices).
// Each with plain and with non-temporal accesses.  These are the ceilings the library's kernels
// are measured against: what the memory system gives this access pattern when compute is free.
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

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ f32x4 ld16(const f32x4* p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT>
__device__ __forceinline__ void st16(f32x4* p, f32x4 v) {
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// decompress shape: NS read-only streams + one read-modify-write stream; a workgroup (one
// wavefront) takes PIECE KiB of every stream (PIECE lane accesses of 16 bytes per stream; the
// library's kernels: 8, a tile of 64 chunks); everything is requested before anything is used
template <int NS, int PIECE, bool NTL, bool NTS>
__global__ __launch_bounds__(64) void decompress_shape(const f32x4* __restrict__ payload,
                                                       size_t stream_stride16,
                                                       f32x4* __restrict__ params) {
    const size_t base = static_cast<size_t>(blockIdx.x) * (64 * PIECE) + threadIdx.x;
    f32x4 v[NS][PIECE], th[PIECE];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int i = 0; i < PIECE; ++i)
            v[s][i] = ld16<NTL>(payload + s * stream_stride16 + base + 64 * i);
#pragma unroll
    for (int i = 0; i < PIECE; ++i) th[i] = ld16<NTL>(params + base + 64 * i);
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
        for (int i = 0; i < PIECE; ++i) th[i] += v[s][i];
#pragma unroll
    for (int i = 0; i < PIECE; ++i) st16<NTS>(params + base + 64 * i, th[i]);
}

// compress shape: momentum 16 KiB read and rewritten, gradient 8 KiB read, 8 KiB + 8 KiB written
template <bool NTL, bool NTS>
__global__ __launch_bounds__(64) void compress_shape(const f32x4* __restrict__ grad,
                                                     f32x4* __restrict__ mom,
                                                     f32x4* __restrict__ val,
                                                     f32x4* __restrict__ idx) {
    const size_t t = blockIdx.x;
    const int lane = threadIdx.x;
    f32x4 m[16], g[8];
#pragma unroll
    for (int i = 0; i < 16; ++i) m[i] = ld16<NTL>(mom + t * 1024 + 64 * i + lane);
#pragma unroll
    for (int i = 0; i < 8; ++i) g[i] = ld16<NTL>(grad + t * 512 + 64 * i + lane);
#pragma unroll
    for (int i = 0; i < 16; ++i) m[i] = m[i] * 0.999f + g[i % 8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        st16<NTS>(val + t * 512 + 64 * i + lane, m[i]);
        st16<NTS>(idx + t * 512 + 64 * i + lane, g[i]);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) st16<NTS>(mom + t * 1024 + 64 * i + lane, m[i]);
}

template <typename Launch>
static int time_shape(const char* name, double bytes_per_launch, int iters, Launch launch) {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int w = 0; w < 2; ++w) launch();
    CHECK(hipEventRecord(e0));
    for (int it = 0; it < iters; ++it) launch();
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    printf("%s: %.1f GB/s (%.3f ms per launch, %.1f MB)\n", name,
           bytes_per_launch * iters / (ms * 1e-3) / 1e9, ms / iters, bytes_per_launch / 1e6);
    CHECK(hipGetLastError());
    return 0;
}

// the optimizer step's traffic shapes on `tiles` tiles (35,912 = the OLMo-1B-shaped 1/8 shard)
static int traffic_shapes(int iters) {
    const size_t tiles = 35912;
    const size_t stream16 = tiles * 512;          // 16-byte items of one 8 KiB-per-tile stream
    f32x4 *payload, *params, *mom;
    CHECK(hipMalloc(&payload, stream16 * 16 * 8));
    CHECK(hipMalloc(&params, stream16 * 16));
    CHECK(hipMalloc(&mom, stream16 * 16 * 2));
    CHECK(hipMemset(payload, 0, stream16 * 16 * 8));
    CHECK(hipMemset(params, 0, stream16 * 16));
    CHECK(hipMemset(mom, 0, stream16 * 16 * 2));
    const unsigned grid = static_cast<unsigned>(tiles);
    const double dbytes = static_cast<double>(tiles) * 8192.0 * 10.0;   // 8 + 1 read, 1 written
    const double cbytes = static_cast<double>(tiles) * 1024.0 * (24.0 + 32.0);
    int rc = 0;
    rc |= time_shape("decompress shape (8 read streams + 1 read-write), plain", dbytes, iters, [&] {
        decompress_shape<8, 8, false, false><<<grid, 64>>>(payload, stream16, params); });
    rc |= time_shape("decompress shape, non-temporal loads", dbytes, iters, [&] {
        decompress_shape<8, 8, true, false><<<grid, 64>>>(payload, stream16, params); });
    rc |= time_shape("decompress shape, non-temporal loads and stores", dbytes, iters, [&] {
        decompress_shape<8, 8, true, true><<<grid, 64>>>(payload, stream16, params); });
    // the same traffic in smaller pieces per wavefront (more, lighter wavefronts per SIMD: 72
    // registers of data in flight at 2 KiB, 36 at 1 KiB, against 288 for a whole tile)
    rc |= time_shape("decompress shape, non-temporal loads, 4 KiB of each stream per wavefront",
                     dbytes, iters, [&] {
        decompress_shape<8, 4, true, false><<<2 * grid, 64>>>(payload, stream16, params); });
    rc |= time_shape("decompress shape, non-temporal loads, 2 KiB of each stream per wavefront",
                     dbytes, iters, [&] {
        decompress_shape<8, 2, true, false><<<4 * grid, 64>>>(payload, stream16, params); });
    rc |= time_shape("decompress shape, non-temporal loads, 1 KiB of each stream per wavefront",
                     dbytes, iters, [&] {
        decompress_shape<8, 1, true, false><<<8 * grid, 64>>>(payload, stream16, params); });
    // compress: gradient = payload stream 0, values / indices = payload streams 1 and 2
    rc |= time_shape("compress shape (24 KiB in, 32 KiB out per tile), plain", cbytes, iters, [&] {
        compress_shape<false, false><<<grid, 64>>>(payload, mom, payload + stream16,
                                                   payload + 2 * stream16); });
    rc |= time_shape("compress shape, non-temporal loads", cbytes, iters, [&] {
        compress_shape<true, false><<<grid, 64>>>(payload, mom, payload + stream16,
                                                  payload + 2 * stream16); });
    rc |= time_shape("compress shape, non-temporal loads and stores", cbytes, iters, [&] {
        compress_shape<true, true><<<grid, 64>>>(payload, mom, payload + stream16,
                                                 payload + 2 * stream16); });
    CHECK(hipFree(payload));
    CHECK(hipFree(params));
    CHECK(hipFree(mom));
    return rc;
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
    CHECK(hipFree(a));
    CHECK(hipFree(b));
    return traffic_shapes(iters);
}
