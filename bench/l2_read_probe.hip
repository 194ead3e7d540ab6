// l2_read_probe: stand-alone measurement aid, not part of the library.
// How fast do the compute units read data that is already in their XCD's L2, and how much does the
// answer depend on which bytes the lanes of one load instruction ask for?  Every workgroup re-reads
// one small buffer (a copy of which ends up in each XCD's L2) with 128-bit loads, 8 in flight per lane:
//   rows        a quarter wave (16 lanes) reads 256 contiguous bytes: 2 cache lines per quarter wave,
//               8 per instruction -- the pattern of coalesced K/V row loads;
//   half-lines  lane (r = lane / 16, c = lane % 16) reads 16 bytes of row c at byte 16 r + 64 t: a
//               quarter wave touches 16 different lines, 64 line lookups per instruction -- the pattern
//               of loading an MFMA A operand straight from row-major memory (16 rows x 64 bytes).
// usage: l2_read_probe [KiB=2048] [passes over the buffer per workgroup=8]
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef int v4i __attribute__((ext_vector_type(4)));
#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "%s:%d %s\n", __FILE__, __LINE__, hipGetErrorString(e_)); return 1; } } while (0)

constexpr size_t kTrip = 8 * 256;   // vectors one workgroup reads per trip (32 KiB)

__global__ void __launch_bounds__(256) read_rows(const v4i *__restrict__ src, size_t n_vec, int reps, int *sink) {
    v4i acc = {0, 0, 0, 0};
    const size_t trips = n_vec / kTrip;
    const size_t start = ((size_t)blockIdx.x * 37) % trips;   // workgroups do not walk in lockstep
    for (int r = 0; r < reps; ++r)
        for (size_t t = 0; t < trips; ++t) {
            const size_t base = ((start + t) % trips) * kTrip + threadIdx.x;
            v4i x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = src[base + e * 256];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc ^= x[e];
        }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x5eed1234) *sink = 1;   // keeps the loads alive
}

__global__ void __launch_bounds__(256) read_half_lines(const v4i *__restrict__ src, size_t n_vec, int reps, int *sink) {
    v4i acc = {0, 0, 0, 0};
    const size_t trips = n_vec / kTrip;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r = lane >> 4, c = lane & 15;
    const size_t start = ((size_t)blockIdx.x * 37) % trips;
    for (int rp = 0; rp < reps; ++rp)
        for (size_t t = 0; t < trips; ++t) {
            // a wave's share of a trip: 2 groups of 16 rows of 256 bytes (16 vectors per row)
            const size_t base = ((start + t) % trips) * kTrip + (size_t)w * 512 + c * 16 + r;
            v4i x[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = src[base + (e >> 2) * 256 + (e & 3) * 4];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc ^= x[e];
        }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x5eed1234) *sink = 1;
}

int main(int argc, char **argv) {
    const size_t kib = argc > 1 ? strtoull(argv[1], nullptr, 10) : 2048;
    const int reps = argc > 2 ? atoi(argv[2]) : 8;
    const size_t bytes = kib << 10, n_vec = bytes / 16;
    if (kib == 0 || n_vec % kTrip != 0 || reps < 1) { fprintf(stderr, "size must be a positive multiple of 32 KiB\n"); return 1; }
    v4i *src;
    int *sink;
    CHECK(hipMalloc(&src, bytes));
    CHECK(hipMalloc(&sink, 4));
    CHECK(hipMemset(src, 1, bytes));
    CHECK(hipMemset(sink, 0, 4));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    printf("buffer %zu KiB, every workgroup reads it %d times\n", kib, reps);
    for (int g : {256, 512, 1024}) {
        for (int k = 0; k < 2; ++k) {
            float ms = 0.f;
            for (int pass = 0; pass < 2; ++pass) {   // the first pass warms the caches and the clocks
                CHECK(hipEventRecord(e0));
                for (int i = 0; i < 5; ++i) {
                    if (k == 0) read_rows<<<g, 256>>>(src, n_vec, reps, sink);
                    else read_half_lines<<<g, 256>>>(src, n_vec, reps, sink);
                }
                CHECK(hipGetLastError());
                CHECK(hipEventRecord(e1));
                CHECK(hipEventSynchronize(e1));
                CHECK(hipEventElapsedTime(&ms, e0, e1));
            }
            printf("%-10s grid %4d: %8.1f us per launch, %6.2f TB/s into the CUs\n", k ? "half-lines" : "rows", g,
                   ms * 1e3 / 5, (double)g * reps * bytes / (ms * 1e-3 / 5) / 1e12);
        }
    }
    CHECK(hipDeviceSynchronize());
    return 0;
}
