// What this GPU sustains on the resources that bound the redistribution kernels, measured with loops that do
// nothing else: HBM streaming (read only, and read + write), the fp32 matrix instruction and the bf16 matrix
// instruction (register operands only, independent accumulators, once with constant and once with varied data,
// because the chip lowers its clock with the switching activity of the operands), and gathers of whole 128-byte
// lines at random out of a table that each XCD keeps in its own L2 (what the sparse product does with the
// position-minor drafter table), and gathers out of LDS (what a formulation with the drafter values on chip could do).
// A stand-alone program:
//   paper_2506_03206_amd/ceilings
// The published peaks (8 TB/s, 157.3 TFLOP/s fp32, 2.5 PFLOP/s bf16) stay the denominators of every reported
// fraction; these figures only say how much of the gap a kernel could close at all.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CHECK(call)                                                                                      \
    do {                                                                                                 \
        hipError_t e_ = (call);                                                                          \
        if (e_ != hipSuccess) {                                                                          \
            std::fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_));              \
            std::exit(1);                                                                                \
        }                                                                                                \
    } while (0)

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kCus = 256;

// ---- HBM ----------------------------------------------------------------------------------------------------------
// grid-stride float4 stream; each lane keeps a sum so the loads cannot be dropped
__global__ __launch_bounds__(256) void read_stream(const f32x4 *__restrict__ src, size_t n4, float *__restrict__ sink)
{
    float s = 0.f;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n4; i += (size_t)gridDim.x * blockDim.x) {
        const f32x4 v = __builtin_nontemporal_load(src + i);
        s += v.x + v.y + v.z + v.w;
    }
    if (s == 12345.678f) sink[0] = s;   // never true for the data used; keeps the loop alive
}

__global__ __launch_bounds__(256) void copy_stream(const f32x4 *__restrict__ src, f32x4 *__restrict__ dst, size_t n4)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n4; i += (size_t)gridDim.x * blockDim.x)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// varied bit patterns, so that the figures do not flatter the memory with constant data
__global__ __launch_bounds__(256) void fill_stream(f32x4 *__restrict__ dst, size_t n4)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n4; i += (size_t)gridDim.x * blockDim.x) {
        const uint32_t h = (uint32_t)i * 2654435761u;
        f32x4 v;
        v.x = (float)(h & 0xffffu) * 1e-4f;
        v.y = (float)(h >> 16) * 1e-4f;
        v.z = (float)((h * 40503u) >> 12) * 1e-6f;
        v.w = (float)((h ^ (h >> 7)) & 0xfffffu) * 1e-5f;
        dst[i] = v;
    }
}

// ---- matrix instructions ------------------------------------------------------------------------------------------
// NACC independent 32x32 accumulators per wave; operands come from a small table read once
template <int NACC>
__global__ __launch_bounds__(256) void mfma_f32_loop(float *out, const float *in, int iters)
{
    f32x16 acc[NACC];
    for (int i = 0; i < NACC; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const int lane = threadIdx.x % 64;
    float a[4], b[4];
    for (int t = 0; t < 4; ++t) {
        a[t] = in[lane + 64 * t];
        b[t] = in[lane + 64 * (4 + t)];
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < NACC; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[(t + i) % 4], b[t], acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < NACC; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int NACC>
__global__ __launch_bounds__(256) void mfma_bf16_loop(float *out, const float *in, int iters)
{
    f32x16 acc[NACC];
    for (int i = 0; i < NACC; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const int lane = threadIdx.x % 64;
    bf16x8 a[4], b[4];
    for (int t = 0; t < 4; ++t)
        for (int e = 0; e < 8; ++e) {
            a[t][e] = (__bf16)in[lane + 64 * (t * 8 + e)];
            b[t][e] = (__bf16)in[lane + 64 * (32 + t * 8 + e)];
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < NACC; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(t + i) % 4], b[t], acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < NACC; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Mean kernel time over `reps` launches after one untimed launch, in milliseconds, from the dispatches' own begin and
// end timestamps (no launch gaps).  The mean, not the best: under matrix load the clock settles over the first
// launches, and the settled rate is the one a long kernel sees.  launch(r, start, stop) enqueues launch number r.
// ---- line gathers -------------------------------------------------------------------------------------------------
// Eight lanes share one random 128-byte line (16 bytes each), so a wavefront instruction asks for eight lines: the
// access pattern of the sparse product.  Sixteen such loads are in flight per wavefront before the first is used.
// Every XCD (consecutive workgroup ids go to consecutive XCDs) gathers from its own slab of `lines` lines.
__global__ __launch_bounds__(512) void line_gather(const f32x4 *__restrict__ table, uint32_t lines, int iters,
                                                   float *__restrict__ sink)
{
    const uint32_t lane = threadIdx.x & 63, part = lane & 7;
    const f32x4 *slab = table + (size_t)(blockIdx.x % 8) * lines * 8;
    uint32_t state = (blockIdx.x * 512u + threadIdx.x) / 8u * 2654435761u + 12345u;   // the same in the 8 lanes of a line
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        f32x4 g[16];
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            state = state * 1664525u + 1013904223u;
            const uint32_t line = (state >> 8) % lines;
            g[t] = slab[(size_t)line * 8 + part];
        }
#pragma unroll
        for (int t = 0; t < 16; ++t) acc += g[t].x + g[t].y + g[t].z + g[t].w;
    }
    if (acc == 12345.678f) sink[0] = acc;
}

// ---- gathers out of LDS ----------------------------------------------------------------------------------------------
// What a formulation of the sparse product with the drafter values of one position in LDS (128 KB: every kept slot of a
// llama3-sized drafter row) could gather per clock.  WORDS = 1: every lane reads a random 4-byte word (one neighbour of
// one id).  WORDS = 32: the 32 lanes of a half wavefront read the 32 consecutive words of a random 128-byte row (the
// conflict-free pattern of a table bucketed by slot range).  Sixteen reads are in flight per lane before the first is used.
template <int WORDS>
__global__ __launch_bounds__(1024) void lds_gather(int iters, float *__restrict__ sink)
{
    extern __shared__ float slab[];
    constexpr uint32_t kWords = 32768;                 // 128 KB
    for (uint32_t i = threadIdx.x; i < kWords; i += 1024) slab[i] = (float)(i & 255u);
    __syncthreads();
    const uint32_t group = WORDS == 1 ? blockIdx.x * 1024u + threadIdx.x : (blockIdx.x * 1024u + threadIdx.x) / 32u;
    uint32_t state = group * 2654435761u + 12345u;     // the same in the lanes that share a row
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        float g[16];
#pragma unroll
        for (int t = 0; t < 16; t += 2) {              // two addresses per step of the generator: little besides the reads
            state = state * 1664525u + 1013904223u;
            const uint32_t a0 = state >> 17, a1 = (state >> 2) & 32767u;
            g[t] = slab[WORDS == 1 ? a0 : (a0 & ~31u) + (threadIdx.x & 31u)];
            g[t + 1] = slab[WORDS == 1 ? a1 : (a1 & ~31u) + (threadIdx.x & 31u)];
        }
#pragma unroll
        for (int t = 0; t < 16; ++t) acc += g[t];
    }
    if (acc == 12345.678f) sink[0] = acc;
}

template <class F>
static double mean_ms(F launch, int reps = 10)
{
    hipEvent_t t0, t1;
    CHECK(hipEventCreate(&t0));
    CHECK(hipEventCreate(&t1));
    launch(0, t0, t1);
    CHECK(hipDeviceSynchronize());
    double sum = 0.0;
    for (int r = 0; r < reps; ++r) {
        launch(r + 1, t0, t1);
        CHECK(hipEventSynchronize(t1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, t0, t1));
        sum += ms;
    }
    CHECK(hipGetLastError());
    CHECK(hipEventDestroy(t0));
    CHECK(hipEventDestroy(t1));
    return sum / reps;
}

int main()
{
    // HBM: a 1 GiB source, far beyond the 256 MiB last-level cache.  Whole-buffer launches give the long-kernel
    // rate; launches over a 160 MiB window that moves through the buffer (so no launch finds its window cached)
    // give the rate of a kernel as short as the streaming kernels of the library (about 30 us).
    const size_t bytes = size_t(1) << 30, n4 = bytes / sizeof(f32x4);
    const size_t window = size_t(160) << 20, w4 = window / sizeof(f32x4), n_windows = bytes / window;
    f32x4 *src, *dst;
    float *sink;
    CHECK(hipMalloc(&src, bytes));
    CHECK(hipMalloc(&dst, bytes));
    CHECK(hipMalloc(&sink, 4096 * 256 * sizeof(float)));
    hipLaunchKernelGGL(fill_stream, dim3(kCus * 8), dim3(256), 0, 0, src, n4);
    CHECK(hipDeviceSynchronize());
    for (int per_cu : {4, 8, 16}) {
        const dim3 grid(kCus * per_cu), block(256);
        double ms = mean_ms([&](int, hipEvent_t a, hipEvent_t b) {
            hipExtLaunchKernelGGL(read_stream, grid, block, 0, 0, a, b, 0, src, n4, sink);
        });
        std::printf("hbm read         1 GiB, %2d workgroups/CU: %7.3f ms  %6.2f TB/s\n", per_cu, ms, bytes / ms / 1e9);
        ms = mean_ms([&](int r, hipEvent_t a, hipEvent_t b) {
            hipExtLaunchKernelGGL(read_stream, grid, block, 0, 0, a, b, 0, src + (r % n_windows) * w4, w4, sink);
        });
        std::printf("hbm read       160 MiB, %2d workgroups/CU: %7.3f ms  %6.2f TB/s\n", per_cu, ms, window / ms / 1e9);
        ms = mean_ms([&](int, hipEvent_t a, hipEvent_t b) {
            hipExtLaunchKernelGGL(read_stream, grid, block, 0, 0, a, b, 0, src, w4, sink);
        });
        std::printf("read 160 MiB again, %2d workgroups/CU: %7.3f ms  %6.2f TB/s  (same window every launch: fits the "
                    "last-level cache)\n", per_cu, ms, window / ms / 1e9);
        ms = mean_ms([&](int, hipEvent_t a, hipEvent_t b) {
            hipExtLaunchKernelGGL(copy_stream, grid, block, 0, 0, a, b, 0, src, dst, n4);
        });
        std::printf("hbm read+write 2x1 GiB, %2d workgroups/CU: %7.3f ms  %6.2f TB/s\n", per_cu, ms, 2.0 * bytes / ms / 1e9);
        ms = mean_ms([&](int r, hipEvent_t a, hipEvent_t b) {
            hipExtLaunchKernelGGL(copy_stream, grid, block, 0, 0, a, b, 0, src + (r % n_windows) * w4,
                                  dst + (r % n_windows) * w4, w4);
        });
        std::printf("hbm read+write 2x160 MiB, %2d workgroups/CU: %7.3f ms  %6.2f TB/s\n", per_cu, ms, 2.0 * window / ms / 1e9);
    }

    // matrix instructions: a 64 x 64 table of operand values, constant or varied
    float *in;
    CHECK(hipMalloc(&in, 64 * 64 * sizeof(float)));
    std::vector<float> h(64 * 64);
    for (int varied = 0; varied < 2; ++varied) {
        for (int i = 0; i < 64 * 64; ++i)
            h[i] = varied ? (float)((i * 2654435761u) % 1000u) * 1e-3f - 0.5f : 1.0f;
        CHECK(hipMemcpy(in, h.data(), h.size() * sizeof(float), hipMemcpyHostToDevice));
        const char *what = varied ? "varied  " : "constant";
        for (int per_cu : {1, 2}) {   // workgroups of 4 waves per CU: one or two waves per SIMD
            const int grid = kCus * per_cu, iters32 = 1000, iters16 = 2000;
            double ms = mean_ms([&](int, hipEvent_t a, hipEvent_t b) {
                hipExtLaunchKernelGGL(mfma_f32_loop<8>, dim3(grid), dim3(256), 0, 0, a, b, 0, sink, in, iters32);
            });
            std::printf("mfma 32x32x2 f32,   %s data, %d waves/SIMD: %7.3f ms  %7.1f TFLOP/s\n", what, per_cu, ms,
                        (double)grid * 4 * iters32 * 4 * 8 * 4096.0 / ms / 1e9);
            ms = mean_ms([&](int, hipEvent_t a, hipEvent_t b) {
                hipExtLaunchKernelGGL(mfma_bf16_loop<8>, dim3(grid), dim3(256), 0, 0, a, b, 0, sink, in, iters16);
            });
            std::printf("mfma 32x32x16 bf16, %s data, %d waves/SIMD: %7.3f ms  %7.1f TFLOP/s\n", what, per_cu, ms,
                        (double)grid * 4 * iters16 * 4 * 8 * 32768.0 / ms / 1e9);
        }
    }
    // line gathers: per-XCD slabs of 1, 2, 4 (the size of the sparse product's slab at n = 32064) and 8 MiB inside src
    for (int mib : {1, 2, 4, 8}) {
        const uint32_t lines = (uint32_t)((size_t(mib) << 20) / 128);
        for (int per_cu : {2, 4}) {   // workgroups of 8 wavefronts per CU
            const int grid = kCus * per_cu, iters = 64;
            const double ms = mean_ms([&](int, hipEvent_t a, hipEvent_t b) {
                hipExtLaunchKernelGGL(line_gather, dim3(grid), dim3(512), 0, 0, a, b, 0, src, lines, iters, sink);
            });
            const double n_lines = (double)grid * 8 * iters * 16 * 8;   // wavefronts x loads x lines per load
            std::printf("128-byte line gathers, %d MiB slab per XCD, %d workgroups/CU: %7.3f ms  %6.1f G lines/s  %5.1f B/clk/CU  "
                        "%4.2f clk per line and CU (at 2.4 GHz)\n", mib, per_cu, ms, n_lines / ms / 1e6,
                        n_lines * 128 / kCus / (ms * 1e-3 * 2.4e9), ms * 1e-3 * 2.4e9 / (n_lines / kCus));
        }
    }
    // gathers out of a 128 KB LDS array, one workgroup of 16 wavefronts per CU
    CHECK(hipFuncSetAttribute((const void *)lds_gather<1>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    CHECK(hipFuncSetAttribute((const void *)lds_gather<32>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072));
    for (int words : {1, 32}) {
        const int iters = 256;
        const double ms = mean_ms([&](int, hipEvent_t a, hipEvent_t b) {
            if (words == 1)
                hipExtLaunchKernelGGL(lds_gather<1>, dim3(kCus), dim3(1024), 131072, 0, a, b, 0, iters, sink);
            else
                hipExtLaunchKernelGGL(lds_gather<32>, dim3(kCus), dim3(1024), 131072, 0, a, b, 0, iters, sink);
        });
        const double reads = (double)kCus * 1024 * iters * 16;   // 4-byte reads
        std::printf("LDS gathers of %s out of 128 KB, 16 wavefronts/CU: %7.3f ms  %5.1f words per clock and CU (at 2.4 GHz), "
                    "incl. filling the array\n", words == 1 ? "random 4-byte words " : "random 128-byte rows", ms,
                    reads / kCus / (ms * 1e-3 * 2.4e9));
    }
    CHECK(hipFree(src));
    CHECK(hipFree(dst));
    CHECK(hipFree(sink));
    CHECK(hipFree(in));
    return 0;
}
