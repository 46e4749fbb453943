// Stand-alone microbenchmark: fp32 atomic-add throughput with the access pattern that a one-kernel attention
// backward would have.  There the workgroups that own the key tiles of one (sample, head) walk the sample's dQ
// rows in 64 x 64 fp32 tiles and add their partial dQ into them (a "region" below is one such dQ, "ntile" its
// number of tiles).  Plain streaming stores over the same addresses are timed beside the atomics.
// Every index stays inside the one buffer allocated in main(); nothing is read back by the kernels.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("hip error %s line %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)

// region: 64*ntile rows of 64 floats; group = wgs sharing a region
__global__ __launch_bounds__(256) void add_tiles(float* dq, int ntile, int wgs_per_region, int iters, int stagger) {
    const int region = blockIdx.x / wgs_per_region, member = blockIdx.x % wgs_per_region;
    float* base = dq + (size_t)region * ntile * 4096;
    int t = stagger ? (member * ntile / wgs_per_region) % ntile : 0;
    for (int i = 0; i < iters; ++i) {
        float* p = base + (size_t)t * 4096;
#pragma unroll
        for (int r = 0; r < 16; ++r) unsafeAtomicAdd(p + r * 256 + threadIdx.x, 1.0f);
        t = t + 1 == ntile ? 0 : t + 1;
    }
}
__global__ __launch_bounds__(256) void store_tiles(float* dq, int ntile, int wgs_per_region, int iters, int stagger) {
    const int region = blockIdx.x / wgs_per_region, member = blockIdx.x % wgs_per_region;
    float* base = dq + (size_t)region * ntile * 4096;
    int t = stagger ? (member * ntile / wgs_per_region) % ntile : 0;
    for (int i = 0; i < iters; ++i) {
        float* p = base + (size_t)t * 4096;
#pragma unroll
        for (int r = 0; r < 16; ++r) __builtin_nontemporal_store(1.0f, p + r * 256 + threadIdx.x);
        t = t + 1 == ntile ? 0 : t + 1;
    }
}

int main() {
    const int wgs = 512;
    float* dq; size_t bytes = (size_t)wgs * 64 * 4096 * 4;  // enough for every case below
    CK(hipMalloc(&dq, bytes)); CK(hipMemset(dq, 0, bytes));
    hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
    struct Case { int ntile, per_region, stagger; } cases[] = {
        {64, 32, 1}, {64, 32, 0}, {64, 8, 1}, {64, 1, 1}, {16, 8, 1}, {144, 64, 1}};
    for (auto c : cases) for (int kind = 0; kind < 2; ++kind) {
        const int iters = 256;
        auto run = [&]() {
            if (kind == 0) add_tiles<<<wgs, 256>>>(dq, c.ntile, c.per_region, iters, c.stagger);
            else store_tiles<<<wgs, 256>>>(dq, c.ntile, c.per_region, iters, c.stagger);
        };
        run(); CK(hipDeviceSynchronize());
        CK(hipEventRecord(a)); for (int i = 0; i < 5; ++i) run(); CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
        float ms; CK(hipEventElapsedTime(&ms, a, b)); ms /= 5;
        double gb = (double)wgs * iters * 16384 / 1e9;
        printf("%s ntile=%d wgs/region=%d stagger=%d: %.3f ms, %.1f GB/s\n", kind ? "store " : "atomic", c.ntile, c.per_region, c.stagger, ms, gb / ms * 1e3);
        fflush(stdout);
    }
    // sanity: the first region of the last atomic case holds whole numbers
    float h[4]; CK(hipMemcpy(h, dq, 16, hipMemcpyDeviceToHost)); printf("sample values %g %g\n", h[0], h[1]);
    return 0;
}
