// Stand-alone microbenchmark (not part of libvarlen_attn.so): how well does one gfx950 SIMD overlap
// matrix (MFMA) and vector (VALU) work of the kind the attention kernels issue?  No memory traffic,
// no LDS, no barriers: only v_mfma_f32_32x32x16_bf16 and chains of {v_fma, v_exp, v_mul} on 16
// independent values, i.e. the softmax arithmetic.  One workgroup per CU, 1 to 3 waves per SIMD.
// Prints a markdown table of cycles per "unit of work" per SIMD; the kernels' own cycles per tile
// can be held against it (they carry LDS reads, scalar bookkeeping and waits on top).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define CK(x)                                                                  \
    do {                                                                       \
        hipError_t e_ = (x);                                                   \
        if (e_ != hipSuccess) {                                                \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 1;                                                          \
        }                                                                      \
    } while (0)

constexpr int ITERS = 2000;
enum { BURSTS = 0, INTERLEAVED = 1, VALU_ONLY = 2, MFMA_ONLY = 3 };

// One unit of work = NM MFMAs (two accumulation chains) + NG x 16 x {fma, exp2, mul}.
// BURSTS: all MFMAs, then all vector work.  INTERLEAVED: VPER vector instructions after each MFMA.
template <int NM, int NG, int MODE, int VPER>
__global__ void unit_kernel(float* out, long long* stamps, float seed) {
    bf16x8 a, b;
    for (int e = 0; e < 8; e++) { a[e] = (__bf16)(0.01f * threadIdx.x); b[e] = (__bf16)0.5f; }
    f32x16 c0, c1;
    for (int r = 0; r < 16; r++) { c0[r] = 0.f; c1[r] = 0.f; }
    float x[16];
    for (int i = 0; i < 16; i++) x[i] = -(threadIdx.x * 0.001f + i * 0.1f) * seed;
    const long long t0 = clock64();
    for (int it = 0; it < ITERS; it++) {
        if (MODE != VALU_ONLY) {
#pragma unroll
            for (int m = 0; m < NM; m += 2) {
                c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
                c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
            }
        }
        if (MODE == BURSTS) __builtin_amdgcn_sched_barrier(0);
        if (MODE != MFMA_ONLY) {
#pragma unroll
            for (int g = 0; g < NG; g++)
#pragma unroll
                for (int i = 0; i < 16; i++)
                    x[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[i], 0.999f, -0.001f)) * -1.5f;
        }
        if (MODE == INTERLEAVED) {
#pragma unroll
            for (int m = 0; m < NM; m++) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, VPER, 0);  // VPER vector instructions
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    const long long t1 = clock64();
    float r = c0[0] + c1[1];
    for (int i = 0; i < 16; i++) r += x[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
    if (blockIdx.x == 0 && (threadIdx.x & 63) == 0) {
        stamps[2 * (threadIdx.x >> 6)] = t0;
        stamps[2 * (threadIdx.x >> 6) + 1] = t1;
    }
}

// Waves 0..3 (one per SIMD) only issue MFMAs, waves 4..7 only independent vector instructions.
template <int EXP>
__global__ void __launch_bounds__(512) split_kernel(float* out, long long* stamps, int mfma_on, int valu_on, float seed) {
    const int w = threadIdx.x >> 6;
    float r = 0;
    const long long t0 = clock64();
    long long t1 = t0;
    if (w < 4) {
        if (mfma_on) {
            bf16x8 a, b;
            for (int e = 0; e < 8; e++) { a[e] = (__bf16)(0.01f * threadIdx.x); b[e] = (__bf16)0.5f; }
            f32x16 c[4];
            for (int i = 0; i < 4; i++)
                for (int q = 0; q < 16; q++) c[i][q] = 0.f;
            for (int it = 0; it < 2 * ITERS; it++) {
#pragma unroll
                for (int m = 0; m < 16; m++) c[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c[m & 3], 0, 0, 0);
            }
            t1 = clock64();
            for (int i = 0; i < 4; i++) r += c[i][i];
        }
    } else if (valu_on) {
        float x[32];
        for (int i = 0; i < 32; i++) x[i] = -(threadIdx.x * 0.001f + i * 0.1f) * seed;
        for (int it = 0; it < 2 * ITERS; it++) {
#pragma unroll
            for (int rep = 0; rep < 2; rep++)
#pragma unroll
                for (int i = 0; i < 32; i++) x[i] = EXP ? __builtin_amdgcn_exp2f(x[i]) : __builtin_fmaf(x[i], 0.999f, -0.001f);
        }
        t1 = clock64();
        for (int i = 0; i < 32; i++) r += x[i];
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
    if (blockIdx.x == 0 && (threadIdx.x & 63) == 0) {
        stamps[2 * w] = t0;
        stamps[2 * w + 1] = t1;
    }
}

// Pure MFMA loop on operands read from memory, long enough for the clocks to settle: what the
// matrix pipe sustains on zero / constant / random bf16 data, and the shader clock it runs at
// (cycle counter over the 100 MHz real-time counter).  The chip lowers its clock under load.
__global__ void __launch_bounds__(512)
sustained_kernel(const bf16x8* __restrict__ in, float* out, unsigned long long* stamps, int iters) {
    bf16x8 a[4], b[4];
    for (int i = 0; i < 4; i++) {
        a[i] = in[(threadIdx.x * 8 + i) % 4096];
        b[i] = in[(threadIdx.x * 8 + 4 + i) % 4096];
    }
    f32x16 c[4];
    for (int i = 0; i < 4; i++)
        for (int r = 0; r < 16; r++) c[i][r] = 0.f;
    const unsigned long long r0 = __builtin_amdgcn_s_memrealtime(), c0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int m = 0; m < 16; m++)
            c[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m & 3], b[(m >> 2) & 3], c[m & 3], 0, 0, 0);
    }
    const unsigned long long r1 = __builtin_amdgcn_s_memrealtime(), c1 = __builtin_readcyclecounter();
    float r = 0;
    for (int i = 0; i < 4; i++) r += c[i][i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
    if (threadIdx.x == 0) {
        stamps[2 * blockIdx.x] = r1 - r0;
        stamps[2 * blockIdx.x + 1] = c1 - c0;
    }
}

// Two waves per SIMD taking turns: while waves 0..3 (one per SIMD) run their MFMAs, waves 4..7 run their
// vector work, then a workgroup barrier and the roles swap ("ping-pong").  PINGPONG = 0 runs the same
// work without barriers, each wave interleaving VPER vector instructions after every MFMA.  Operands
// come from memory (random data), the run is long enough for the clock to settle, and both the cycle
// counter and the 100 MHz real-time counter are read, so that time per unit includes what the power
// limit does to the clock.
template <int NM, int NG, int PINGPONG, int VPER>
__global__ void __launch_bounds__(512)
turns_kernel(const bf16x8* __restrict__ in, float* out, unsigned long long* stamps, int iters) {
    const int w = threadIdx.x >> 6;
    bf16x8 a[2], b[2];
    for (int i = 0; i < 2; i++) {
        a[i] = in[(threadIdx.x * 4 + i) % 4096];
        b[i] = in[(threadIdx.x * 4 + 2 + i) % 4096];
    }
    f32x16 c0, c1;
    for (int r = 0; r < 16; r++) { c0[r] = 0.f; c1[r] = 0.f; }
    float x[16];
    for (int i = 0; i < 16; i++) x[i] = -(threadIdx.x * 0.001f + i * 0.1f) * (float)a[0][0];
    auto mfmas = [&]() {
#pragma unroll
        for (int m = 0; m < NM; m += 2) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0], b[(m >> 1) & 1], c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1], b[(m >> 1) & 1], c1, 0, 0, 0);
        }
    };
    auto vector_work = [&]() {
#pragma unroll
        for (int g = 0; g < NG; g++)
#pragma unroll
            for (int i = 0; i < 16; i++) x[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[i], 0.999f, -0.001f)) * -1.5f;
    };
    const unsigned long long r0 = __builtin_amdgcn_s_memrealtime(), cy0 = __builtin_readcyclecounter();
    if (PINGPONG) {
        const bool first = w < 4;  // wave-uniform
        for (int it = 0; it < iters; it++) {
            if (first) mfmas(); else vector_work();
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            if (first) vector_work(); else mfmas();
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
        }
    } else {
        for (int it = 0; it < iters; it++) {
            mfmas();
            vector_work();
#pragma unroll
            for (int m = 0; m < NM; m++) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, VPER, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    const unsigned long long r1 = __builtin_amdgcn_s_memrealtime(), cy1 = __builtin_readcyclecounter();
    float r = c0[0] + c1[1];
    for (int i = 0; i < 16; i++) r += x[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = r;
    if ((threadIdx.x & 63) == 0) {  // every wave: without barriers the two waves of a SIMD need not finish together
        unsigned long long* st = stamps + 4 * (blockIdx.x * 8 + w);
        st[0] = r0; st[1] = r1; st[2] = cy0; st[3] = cy1;
    }
}

static int taking_turns(float* out) {
    bf16x8* in;
    unsigned long long* stamps;
    CK(hipMalloc(&in, 4096 * 16));
    CK(hipMalloc(&stamps, 256 * 8 * 32));
    unsigned short* h = (unsigned short*)malloc(4096 * 16);
    unsigned long long* hs = (unsigned long long*)malloc(256 * 8 * 32);
    srand(1);
    for (int i = 0; i < 4096 * 8; i++) {
        const float v = (rand() / (float)RAND_MAX) * 4.f - 2.f;
        unsigned int u;
        memcpy(&u, &v, 4);
        h[i] = (unsigned short)(u >> 16);
    }
    CK(hipMemcpy(in, h, 4096 * 16, hipMemcpyHostToDevice));
    printf("\n| MFMAs per unit | vector work per unit | two waves per SIMD | cycles per unit per SIMD | shader clock GHz | ns per unit per SIMD |\n|---|---|---|---|---|---|\n");
#define RUN3(NM, NG, PP, VPER, LABEL)                                                                         \
    {                                                                                                         \
        const int iters = 60000;                                                                              \
        turns_kernel<NM, NG, PP, VPER><<<256, 512>>>(in, out, stamps, 2000);                                   \
        CK(hipDeviceSynchronize());                                                                           \
        turns_kernel<NM, NG, PP, VPER><<<256, 512>>>(in, out, stamps, iters);                                  \
        CK(hipDeviceSynchronize());                                                                           \
        CK(hipMemcpy(hs, stamps, 256 * 8 * 32, hipMemcpyDeviceToHost));                                       \
        double rt = 0, cy = 0;                                                                                \
        for (int i = 0; i < 256; i++) { /* per workgroup: first start to last end over its waves */           \
            unsigned long long r0 = ~0ull, r1 = 0, c0 = ~0ull, c1 = 0;                                        \
            for (int w = 0; w < 8; w++) {                                                                     \
                const unsigned long long* st = hs + 4 * (i * 8 + w);                                          \
                r0 = st[0] < r0 ? st[0] : r0; r1 = st[1] > r1 ? st[1] : r1;                                   \
                c0 = st[2] < c0 ? st[2] : c0; c1 = st[3] > c1 ? st[3] : c1;                                   \
            }                                                                                                 \
            rt += (double)(r1 - r0); cy += (double)(c1 - c0);                                                 \
        }                                                                                                     \
        printf("| %d | %d x {fma, exp2, mul} | %s | %.0f | %.2f | %.0f |\n", NM, 16 * NG, LABEL,              \
               cy / 256 / iters / 2, cy / rt / 10.0, rt * 10.0 / 256 / iters / 2);                            \
    }
    RUN3(32, 3, 0, 5, "each interleaving its own")
    RUN3(32, 3, 1, 0, "taking turns, barrier between")
    RUN3(24, 2, 0, 4, "each interleaving its own")
    RUN3(24, 2, 1, 0, "taking turns, barrier between")
    RUN3(16, 3, 0, 9, "each interleaving its own")
    RUN3(16, 3, 1, 0, "taking turns, barrier between")
    return 0;
}

static int sustained_mfma(float* out) {
    bf16x8* in;
    unsigned long long* stamps;
    CK(hipMalloc(&in, 4096 * 16));
    CK(hipMalloc(&stamps, 256 * 16));
    unsigned short* h = (unsigned short*)malloc(4096 * 16);
    unsigned long long hs[512];
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    printf("\n| bf16 operands | waves per SIMD | TFLOP/s (256 CUs) | shader clock GHz |\n|---|---|---|---|\n");
    for (int mode = 0; mode < 3; mode++) {
        srand(1);
        for (int i = 0; i < 4096 * 8; i++) {
            const float v = mode == 0 ? 0.0f : mode == 1 ? 0.5f : ((rand() / (float)RAND_MAX) * 4.f - 2.f);
            unsigned int u;
            memcpy(&u, &v, 4);
            h[i] = (unsigned short)(u >> 16);
        }
        CK(hipMemcpy(in, h, 4096 * 16, hipMemcpyHostToDevice));
        for (int threads = 256; threads <= 512; threads += 256) {
            const int iters = 200000 / (threads / 256);
            sustained_kernel<<<256, threads>>>(in, out, stamps, 1000);
            CK(hipDeviceSynchronize());
            CK(hipEventRecord(e0));
            sustained_kernel<<<256, threads>>>(in, out, stamps, iters);
            CK(hipEventRecord(e1));
            CK(hipDeviceSynchronize());
            float ms;
            CK(hipEventElapsedTime(&ms, e0, e1));
            CK(hipMemcpy(hs, stamps, 256 * 16, hipMemcpyDeviceToHost));
            double rt = 0, cy = 0;
            for (int i = 0; i < 256; i++) { rt += (double)hs[2 * i]; cy += (double)hs[2 * i + 1]; }
            const double flops = 256.0 * (threads / 64) * (double)iters * 16 * 32768.0;
            printf("| %s | %d | %.0f | %.2f |\n", mode == 0 ? "all zero" : mode == 1 ? "all 0.5" : "uniform random in [-2, 2)",
                   threads / 256, flops / ms / 1e9, cy / rt / 10.0);
        }
    }
    return 0;
}

int main() {
    float* out;
    long long* stamps;
    CK(hipMalloc(&out, 1 << 22));
    CK(hipMalloc(&stamps, 512));
    long long h[32];
    printf("| MFMAs per unit | vector work per unit | schedule | waves per SIMD | cycles per unit per SIMD | MFMA pipe busy |\n");
    printf("|---|---|---|---|---|---|\n");
#define RUN(NM, NG, MODE, VPER, THREADS, LABEL)                                                              \
    {                                                                                                        \
        unit_kernel<NM, NG, MODE, VPER><<<256, THREADS>>>(out, stamps, 1.0f);                                 \
        CK(hipDeviceSynchronize());                                                                          \
        CK(hipMemcpy(h, stamps, 256, hipMemcpyDeviceToHost));                                                \
        long long lo = h[0], hi = h[1];                                                                      \
        for (int i = 0; i < THREADS / 64; i++) {                                                             \
            lo = h[2 * i] < lo ? h[2 * i] : lo;                                                              \
            hi = h[2 * i + 1] > hi ? h[2 * i + 1] : hi;                                                      \
        }                                                                                                    \
        const double per = (double)(hi - lo) / ITERS / (THREADS / 256);                                      \
        printf("| %d | %d x {fma, exp2, mul} | %s | %d | %.0f | %.0f %% |\n", MODE == VALU_ONLY ? 0 : NM,    \
               MODE == MFMA_ONLY ? 0 : 16 * NG, LABEL, THREADS / 256, per,                                   \
               MODE == VALU_ONLY ? 0.0 : 100.0 * 32 * NM / per);                                             \
    }
    RUN(16, 2, MFMA_ONLY, 0, 256, "MFMA only")
    RUN(16, 2, VALU_ONLY, 0, 256, "vector only")
    RUN(16, 2, VALU_ONLY, 0, 512, "vector only")
    RUN(16, 2, VALU_ONLY, 0, 768, "vector only")
    RUN(16, 2, BURSTS, 0, 256, "bursts")
    RUN(16, 2, BURSTS, 0, 512, "bursts")
    RUN(16, 2, BURSTS, 0, 768, "bursts")
    RUN(16, 2, INTERLEAVED, 6, 256, "interleaved 1:6")
    RUN(16, 2, INTERLEAVED, 6, 512, "interleaved 1:6")
    RUN(16, 2, INTERLEAVED, 6, 768, "interleaved 1:6")
    RUN(24, 2, BURSTS, 0, 512, "bursts")
    RUN(24, 2, BURSTS, 0, 768, "bursts")
    RUN(24, 2, INTERLEAVED, 4, 512, "interleaved 1:4")
    RUN(24, 2, INTERLEAVED, 4, 768, "interleaved 1:4")
    RUN(32, 2, BURSTS, 0, 512, "bursts")
    RUN(32, 2, INTERLEAVED, 3, 512, "interleaved 1:3")
    RUN(32, 3, BURSTS, 0, 512, "bursts")
    RUN(32, 3, INTERLEAVED, 5, 512, "interleaved 1:5")
    printf("\n| waves 0-3 of the CU | waves 4-7 | cycles per MFMA | cycles per vector instruction |\n|---|---|---|---|\n");
#define RUN2(EXP, M, V)                                                                                       \
    {                                                                                                         \
        split_kernel<EXP><<<256, 512>>>(out, stamps, M, V, 1.0f);                                             \
        CK(hipDeviceSynchronize());                                                                           \
        CK(hipMemcpy(h, stamps, 128, hipMemcpyDeviceToHost));                                                 \
        printf("| %s | %s | %.1f | %.2f |\n", M ? "MFMA back to back" : "idle",                               \
               V ? (EXP ? "independent v_exp_f32" : "independent v_fma_f32") : "idle",                        \
               M ? (double)(h[1] - h[0]) / (2 * ITERS) / 16 : 0.0, V ? (double)(h[9] - h[8]) / (2 * ITERS) / 64 : 0.0); \
    }
    RUN2(0, 1, 0) RUN2(0, 0, 1) RUN2(0, 1, 1) RUN2(1, 0, 1) RUN2(1, 1, 1)
    if (sustained_mfma(out)) return 1;
    return taking_turns(out);
}
