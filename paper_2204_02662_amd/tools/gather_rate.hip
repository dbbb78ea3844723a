// Random-row gather rate of the memory hierarchy (stand-alone measurement tool).
//
// Gathers random `row_bytes`-byte rows from a table of `table_mb` megabytes, 8 rows in
// flight per lane group, and prints the achieved rows/s and bytes/s.  Sweeping the table
// size shows the L2 (4 MB per XCD), memory-side cache (256 MB) and HBM plateaus that bound
// the aggregation kernel.  Build: hipcc --offload-arch=gfx950 -O3 gather_rate.hip -o gather_rate
// Usage: gather_rate [row_bytes=512] [gathers_per_lane_group=4096] [nt=0] [wavefronts_per_cu=32] [max_table_mb=4096]
//                    [skew=0]
// skew k > 0 (integer) draws the popularity rank as n_rows * u_0 * u_1 * ... * u_k (u_i uniform in
// [0,1), integer arithmetic only) instead of uniformly: a heavy-headed popularity like the source rows
// of a scale-free graph (k = 2: the most popular 0.02 % of the rows receive about 9 % of the gathers, as
// in the R-MAT benchmark graph), with the popular rows scattered over the table.

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

typedef float float4v __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                  \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));               \
            return 1;                                                             \
        }                                                                         \
    } while (0)

__device__ __forceinline__ uint32_t next(uint32_t& s) {  // xorshift32
    s ^= s << 13;
    s ^= s >> 17;
    s ^= s << 5;
    return s;
}

// T lanes of 16 bytes read one row; every lane group walks its own random sequence.
template <bool NT>
__global__ __launch_bounds__(256) void k_gather(const float4v* __restrict__ table, uint32_t n_rows, int lanes_per_row,
                                                int iters, int skew, float* __restrict__ sink) {
    const int tid = blockIdx.x * 256 + threadIdx.x;
    const int group = tid / lanes_per_row, t = tid % lanes_per_row;
    uint32_t s = 0x9E3779B9u * (uint32_t)(group + 1) + 12345u;
    float4v acc = {0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < iters; i += 8) {
        float4v x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            uint32_t r = (uint32_t)(((uint64_t)next(s) * n_rows) >> 32);
            if (skew > 0) {  // popularity rank -> scattered row (odd multiplier: a bijection mod 2^32)
                uint32_t f = 0xFFFFFFFFu;
                for (int j = 0; j < skew; ++j) f = __umulhi(f, next(s));
                const uint32_t rank = __umulhi(f, r);
                r = (uint32_t)(((uint64_t)(rank * 2654435761u) * n_rows) >> 32);
            }
            const float4v* p = table + (size_t)r * lanes_per_row + t;
            x[u] = NT ? __builtin_nontemporal_load(p) : *p;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += x[u];
    }
    if (acc[0] + acc[1] + acc[2] + acc[3] == 123.456f) sink[0] = acc[0];  // keep the loads alive
}

int main(int argc, char** argv) {
    const int row_bytes = argc > 1 ? atoi(argv[1]) : 512;
    const int iters = argc > 2 ? atoi(argv[2]) : 4096;
    const int nt = argc > 3 ? atoi(argv[3]) : 0;
    const int waves_per_cu = argc > 4 ? atoi(argv[4]) : 32;
    const size_t max_mb = argc > 5 ? (size_t)atoll(argv[5]) : 4096;
    const int skew = argc > 6 ? atoi(argv[6]) : 0;
    const int lanes_per_row = row_bytes / 16;
    if (lanes_per_row < 1 || lanes_per_row > 64 || 64 % lanes_per_row) { fprintf(stderr, "bad row size\n"); return 1; }
    const size_t max_bytes = 4ull << 30;
    float4v* table = nullptr;
    float* sink = nullptr;
    CHECK(hipMalloc(&table, max_bytes));
    CHECK(hipMalloc(&sink, 4));
    CHECK(hipMemset(table, 0, max_bytes));
    if (waves_per_cu < 4 || waves_per_cu > 32 || waves_per_cu % 4) { fprintf(stderr, "wavefronts per CU: 4..32, multiple of 4\n"); return 1; }
    const int groups = 256 * waves_per_cu * (64 / lanes_per_row);
    const int blocks = groups * lanes_per_row / 256;
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a));
    CHECK(hipEventCreate(&b));
    printf("row_bytes=%d lane groups=%d gathers each=%d nt=%d wavefronts per CU=%d skew=%d\n", row_bytes, groups, iters, nt,
           waves_per_cu, skew);
    for (size_t mb : {1, 2, 4, 8, 16, 32, 64, 96, 128, 192, 256, 384, 512, 1024, 2048, 4096}) {
        if (mb > max_mb) break;
        const uint32_t n_rows = (uint32_t)((mb << 20) / row_bytes);
        for (int rep = 0; rep < 3; ++rep) {
            CHECK(hipEventRecord(a));
            if (nt) hipLaunchKernelGGL(k_gather<true>, dim3(blocks), dim3(256), 0, 0, table, n_rows, lanes_per_row, iters, skew, sink);
            else hipLaunchKernelGGL(k_gather<false>, dim3(blocks), dim3(256), 0, 0, table, n_rows, lanes_per_row, iters, skew, sink);
            CHECK(hipEventRecord(b));
            CHECK(hipEventSynchronize(b));
            float ms = 0;
            CHECK(hipEventElapsedTime(&ms, a, b));
            if (rep == 2) {
                const double g = (double)groups * iters;
                printf("table %5zu MB: %8.3f ms  %7.2f G rows/s  %7.2f TB/s  %7.2f G lines(128B)/s\n", mb, ms,
                       g / ms / 1e6, g * row_bytes / ms / 1e9, g * ((row_bytes + 127) / 128) / ms / 1e6);
            }
        }
    }
    CHECK(hipFree(table));
    CHECK(hipFree(sink));
    return 0;
}
