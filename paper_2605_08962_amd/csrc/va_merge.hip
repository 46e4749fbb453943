// Merge of partial attention results over disjoint key/value shards (HBM-bound, elementwise):
//     LSE = ln sum_p exp(LSE_p),   O = sum_p exp(LSE_p - LSE) O_p,
// the combination that context parallelism over key shards needs (Section 4.1.2 selects it for
// overlong contexts, Section 5.2 shards long samples for it) and that the forward uses itself when it
// splits the keys of a small launch over several workgroups.  A part with LSE_p = -inf is empty and
// its O_p is never multiplied (it may hold anything).
#include "va_device.h"
#include "va_internal.h"

namespace va {

// One thread per (token, head, 8 consecutive channels).  Parts: PartT [P, T, H, D], lse [P, H, T].
// NP > 0: the number of parts is known at compile time, so that all loads of a thread are in flight
// together (the kernel is bound by HBM latency x bytes in flight otherwise); NP = 0: any P.
template <typename PartT, int NP>
__global__ void __launch_bounds__(256)
merge_kernel(const PartT* __restrict__ o_parts, const float* __restrict__ lse_parts, int P_rt, int T, int H, int D,
             __bf16* __restrict__ o, float* __restrict__ lse) {
    const int P = NP > 0 ? NP : P_rt;
    const int cpr = D / 8;  // chunks per (token, head) row
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)T * H * cpr) return;
    const int c = (int)(idx % cpr);
    const int64_t row = idx / cpr;  // token * H + head
    const int h = (int)(row % H);
    const int64_t t = row / H;
    const size_t lse_stride = (size_t)H * T, o_stride = (size_t)T * H * D;
    const float* lp = lse_parts + (size_t)h * T + t;

    float mx = -INFINITY;
#pragma unroll
    for (int p = 0; p < P; ++p) mx = fmaxf(mx, lp[p * lse_stride]);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float total = -INFINITY;
    if (mx != -INFINITY) {
        float den = 0.f;
#pragma unroll
        for (int p = 0; p < P; ++p) den += __expf(lp[p * lse_stride] - mx);
        total = mx + __logf(den);
        const float inv = 1.f / den;
        const PartT* op = o_parts + (size_t)row * D + 8 * c;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const float x = lp[p * lse_stride];
            if (x == -INFINITY) continue;  // empty part: its O is not read
            const float wgt = __expf(x - mx) * inv;
            if constexpr (sizeof(PartT) == 2) {
                const bf16x8 v = *(const bf16x8*)(op + p * o_stride);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += wgt * (float)v[e];
            } else {
                const float4 v0 = *(const float4*)(op + p * o_stride), v1 = *(const float4*)(op + p * o_stride + 4);
                acc[0] += wgt * v0.x; acc[1] += wgt * v0.y; acc[2] += wgt * v0.z; acc[3] += wgt * v0.w;
                acc[4] += wgt * v1.x; acc[5] += wgt * v1.y; acc[6] += wgt * v1.z; acc[7] += wgt * v1.w;
            }
        }
    }
    bf16x8 out;
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = (__bf16)acc[e];
    *(bf16x8*)(o + (size_t)row * D + 8 * c) = out;
    if (c == 0) lse[(size_t)h * T + t] = total;
}

hipError_t launch_merge(const void* o_parts, bool parts_fp32, const float* lse_parts, int P, int T, int H, int D,
                        void* o, float* lse, hipStream_t stream) {
    const int64_t n = (int64_t)T * H * (D / 8);
    if (n == 0) return hipSuccess;
    dim3 grid((unsigned)((n + 255) / 256)), block(256);
#define VA_MERGE_LAUNCH(PT, NP)                                                                              \
    hipLaunchKernelGGL((merge_kernel<PT, NP>), grid, block, 0, stream, (const PT*)o_parts, lse_parts, P, T, H, D, \
                       (__bf16*)o, lse)
#define VA_MERGE_DISPATCH(PT)                                                \
    switch (P) {                                                             \
        case 1: VA_MERGE_LAUNCH(PT, 1); break;                               \
        case 2: VA_MERGE_LAUNCH(PT, 2); break;                               \
        case 3: VA_MERGE_LAUNCH(PT, 3); break;                               \
        case 4: VA_MERGE_LAUNCH(PT, 4); break;                               \
        case 5: VA_MERGE_LAUNCH(PT, 5); break;                               \
        case 6: VA_MERGE_LAUNCH(PT, 6); break;                               \
        case 7: VA_MERGE_LAUNCH(PT, 7); break;                               \
        case 8: VA_MERGE_LAUNCH(PT, 8); break;                               \
        default: VA_MERGE_LAUNCH(PT, 0); break;                              \
    }
    if (parts_fp32) { VA_MERGE_DISPATCH(float) } else { VA_MERGE_DISPATCH(__bf16) }
#undef VA_MERGE_DISPATCH
#undef VA_MERGE_LAUNCH
    return hipGetLastError();
}

}  // namespace va
