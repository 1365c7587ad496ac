// Streaming-rate reference for MI355X HBM: what trivial-arithmetic kernels with the access
// patterns of the two optimizer kernels sustain, so that their rates can be read against the
// memory system's own limits rather than against the 8 TB/s pin rate alone.
//
//   hbm_stream_bench [elements-per-buffer, default 1557611200 (GPT-2 XL)]
//
// Every lane moves one 16-byte vector per stream with non-temporal accesses.  Two launch
// shapes: one four-wave workgroup per 256-vector tile with no limit on resident waves, and
// one-wave workgroups with an unused LDS reservation that caps the waves resident per
// compute unit (the shape the library launches with).  Buffers are carved from one
// allocation at the stated spacing.  Prints GB/s (read + written bytes over kernel time).
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

typedef float vfloat4 __attribute__((ext_vector_type(4)));
#define GLOBAL __attribute__((address_space(1)))
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); exit(1); } } while (0)

struct Streams { float* r[10]; float* w[10]; };

template <int NR, int NW, int WG>
__global__ __launch_bounds__(WG) void stream_kernel(Streams S, long n4, float c)
{
    const long i = static_cast<long>(blockIdx.x) * WG + threadIdx.x;
    if (i >= n4) return;
    vfloat4 acc = {c, c, c, c};
#pragma unroll
    for (int r = 0; r < NR; ++r) acc += __builtin_nontemporal_load((const GLOBAL vfloat4*)S.r[r] + i);
#pragma unroll
    for (int w = 0; w < NW; ++w)
        __builtin_nontemporal_store(acc * static_cast<float>(w + 1), (GLOBAL vfloat4*)S.w[w] + i);
    if (NW == 0 && acc.x == 12345.678f) S.r[0][0] = acc.y;   // keeps the loads of a read-only pass alive
}

// waves_per_cu = 0: four-wave workgroups, no cap; otherwise one-wave workgroups, each
// reserving floor(160 KiB / waves_per_cu) of LDS (rounded down to 1 KiB) it never touches.
template <int NR, int NW, int WG>
static float time_kernel(const Streams& S, long n4, unsigned lds)
{
    const int grid = static_cast<int>((n4 + WG - 1) / WG);
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    hipLaunchKernelGGL((stream_kernel<NR, NW, WG>), dim3(grid), dim3(WG), lds, 0, S, n4, 1.0f);
    CK(hipGetLastError());
    CK(hipEventRecord(e0, 0));
    const int iters = 5;
    for (int k = 0; k < iters; ++k) hipLaunchKernelGGL((stream_kernel<NR, NW, WG>), dim3(grid), dim3(WG), lds, 0, S, n4, 1.0f);
    CK(hipEventRecord(e1, 0));
    CK(hipEventSynchronize(e1));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return ms / iters;
}

template <int NR, int NW>
static void run(const char* what, const Streams& S, long n, int waves_per_cu = 0)
{
    const long n4 = n / 4;
    char label[128];
    float ms;
    if (waves_per_cu > 0) {
        const unsigned lds = (160u * 1024u / static_cast<unsigned>(waves_per_cu)) & ~1023u;
        ms = time_kernel<NR, NW, 64>(S, n4, lds);
        snprintf(label, sizeof label, "%s [1-wave WGs, %d per CU]", what, waves_per_cu);
    } else {
        ms = time_kernel<NR, NW, 256>(S, n4, 0);
        snprintf(label, sizeof label, "%s", what);
    }
    printf("%-84s %8.3f ms %6.0f GB/s\n", label, ms, static_cast<double>(NR + NW) * n * 4 / ms / 1e6);
    fflush(stdout);
}

int main(int argc, char** argv)
{
    const long n = argc > 1 ? atol(argv[1]) : 1557611200L;
    const size_t GiB = 1ull << 30;
    const double buf_gib = static_cast<double>(n) * 4 / GiB;
    size_t free_b = 0, total_b = 0;
    CK(hipMemGetInfo(&free_b, &total_b));
    const size_t arena_bytes = (free_b - 8 * GiB) / GiB * GiB;
    char* arena = nullptr;
    CK(hipMalloc(reinterpret_cast<void**>(&arena), arena_bytes));
    CK(hipMemset(arena, 0, arena_bytes));
    CK(hipDeviceSynchronize());
    const double arena_gib = static_cast<double>(arena_bytes) / GiB;
    printf("buffers of %.2f GiB in one %.0f GiB allocation\n", buf_gib, arena_gib);
    auto at = [&](double gib) { return reinterpret_cast<float*>(arena + static_cast<size_t>(gib * 512) * (2u << 20)); };
    auto fits = [&](double last_gib) { return last_gib + buf_gib <= arena_gib; };
    const double near = buf_gib <= 6 ? 6 : buf_gib + 0.25;    // adjacent buffers

    Streams S;
    for (int i = 0; i < 10; ++i) { S.r[i] = at(i * near); S.w[i] = at((10 + i) * near); }
    if (fits(19 * near)) {
        run<1, 0>("read 1 stream", S, n);
        run<4, 0>("read 4 streams", S, n);
        run<0, 1>("write 1 stream", S, n);
        run<0, 3>("write 3 streams", S, n);
        run<1, 1>("copy (1 read, 1 write, different buffers)", S, n);
        run<4, 3>("4 reads, 3 writes to other buffers (out of place)", S, n);
    }
    for (double d : {near, 12.0, 24.0, 36.0, 48.0, 60.0}) {
        if (d < near || !fits(3 * d)) continue;
        for (int i = 0; i < 4; ++i) { S.r[i] = at(i * d); S.w[i] = S.r[i]; }
        char what[96];
        snprintf(what, sizeof what, "AdamW pattern: 4 reads, 3 written back in place, %.0f GiB apart", d);
        run<4, 3>(what, S, n);
        run<4, 3>(what, S, n, 12);
        run<4, 3>(what, S, n, 8);
    }
    for (double d : {near, 8.0, 12.0, 16.0, 24.0}) {
        if (d < near || !fits(9 * d)) continue;
        for (int i = 0; i < 10; ++i) { S.r[i] = at(i * d); S.w[i] = S.r[i]; }
        char what[96];
        snprintf(what, sizeof what, "outer pattern (G=8): 10 streams in place, %.0f GiB apart", d);
        run<10, 10>(what, S, n);
        run<10, 10>(what, S, n, 8);
        run<10, 10>(what, S, n, 4);
        snprintf(what, sizeof what, "lazy-start pattern: 10 reads, 2 written in place, %.0f GiB apart", d);
        run<10, 2>(what, S, n);
        run<10, 2>(what, S, n, 8);
        run<10, 2>(what, S, n, 6);
    }
    CK(hipFree(arena));
    return 0;
}
