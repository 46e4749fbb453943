// Backward kernels.  P is recomputed from Q, K and the saved LSE (the paper recomputes core
// attention in the backward pass, Section 5 "Selective Activation Offloading").
//
//   delta  : Delta[h,i] = sum_d dO[i,h,d] * O[i,h,d]                       (HBM-bound sweep)
//   dkdv   : one workgroup per (128-row key tile, kv head); loops over the query heads of the
//            group and over 64-row query steps; S = Q K^T is kept with one KEY per lane, so
//            that P and dS are directly the B operands of dV^T += dO^T P and dK^T += Q^T dS
//            (contraction over query rows).
//   dq     : one workgroup per (128-row query tile, query head); loops over 64-row key steps;
//            S^T = K Q^T is kept with one QUERY per lane (as in the forward), so that dS^T is the
//            B operand of dQ^T += K^T dS^T (contraction over key rows).
// Splitting the backward this way needs no atomics and no fp32 dQ buffer, and the result does not
// depend on scheduling order; it recomputes S and dP once more than a fused kernel would.
#include "va_device.h"
#include "va_internal.h"

namespace va {

// ------------------------------------------------------------------------------------------------
// Delta
// ------------------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256)
delta_kernel(const __bf16* __restrict__ dO, const __bf16* __restrict__ O, float* __restrict__ delta,
             int T, int Hq) {
    // 16 lanes per (token, head) row, one 16-byte chunk each
    const int64_t row = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int c = threadIdx.x & 15;
    const int64_t rows = (int64_t)T * Hq;
    float acc = 0.f;
    if (row < rows && c < D / 8) {
        bf16x8 a = *(const bf16x8*)(dO + row * D + c * 8);
        bf16x8 b = *(const bf16x8*)(O + row * D + c * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)b[e];
    }
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 16);
    if (row < rows && c == 0) {
        const int64_t i = row / Hq, h = row % Hq;
        delta[h * T + i] = acc;
    }
}

hipError_t launch_bwd_delta(const BwdArgs& a, hipStream_t stream) {
    const int64_t rows = (int64_t)a.total_tokens * a.num_q_heads;
    dim3 grid((unsigned)((rows + 15) / 16)), block(256);
    auto dO = (const __bf16*)a.dout; auto O = (const __bf16*)a.o;
    switch (a.head_dim) {
        case 64: hipLaunchKernelGGL(delta_kernel<64>, grid, block, 0, stream, dO, O, a.delta, a.total_tokens, a.num_q_heads); break;
        case 80: hipLaunchKernelGGL(delta_kernel<80>, grid, block, 0, stream, dO, O, a.delta, a.total_tokens, a.num_q_heads); break;
        case 96: hipLaunchKernelGGL(delta_kernel<96>, grid, block, 0, stream, dO, O, a.delta, a.total_tokens, a.num_q_heads); break;
        case 128: hipLaunchKernelGGL(delta_kernel<128>, grid, block, 0, stream, dO, O, a.delta, a.total_tokens, a.num_q_heads); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Shared staging of a 64-row [rows, D] tile of a [T, H, D] tensor through registers into LDS.
// ------------------------------------------------------------------------------------------------
template <int D>
struct Stage64 {
    static constexpr int CPR = D / 8;             // 16-byte chunks per row
    static constexpr int CHUNKS = 64 * CPR;
    static constexpr int LOADS = (CHUNKS + 255) / 256;
    u32x4 reg[LOADS];
    // rows [r0, r0+64) of the sample, rows >= L read as zero; base points at (sample row 0, head)
    __device__ __forceinline__ void load(const __bf16* base, size_t row_elems, int r0, int L, int tid) {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            int c = tid + 256 * i;
            int r = c / CPR, cc = c % CPR;
            u32x4 z = {0, 0, 0, 0};
            reg[i] = z;
            if (c < CHUNKS && r0 + r < L) reg[i] = *(const u32x4*)(base + (size_t)(r0 + r) * row_elems + cc * 8);
        }
    }
    __device__ __forceinline__ void store(unsigned char* lds, int stride, int tid) const {
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            int c = tid + 256 * i;
            int r = c / CPR, cc = c % CPR;
            if (c < CHUNKS) *(u32x4*)(lds + r * stride + cc * 16) = reg[i];
        }
    }
};

template <int D>
struct BwdCfg {
    static constexpr int KS = D / 16;
    static constexpr int DB = (D + 31) / 32;
    // LDS bytes per row for tiles read both along rows (16-byte reads) and down columns
    // (transposing reads); DB * 64 bytes are addressable by the transposing reads.
    static constexpr int STR = DB * 64 + 16;
    static constexpr int TILE_BYTES = 64 * STR;
};

__device__ __forceinline__ bf16x8 pack_regs(const f32x16& x, int st) {
    return pack8(x[8 * st + 0], x[8 * st + 1], x[8 * st + 2], x[8 * st + 3], x[8 * st + 4], x[8 * st + 5],
                 x[8 * st + 6], x[8 * st + 7]);
}
__device__ __forceinline__ bf16x8 pack_regs_lo(const f32x16& x, int st, bf16x8 hi) {
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (__bf16)(x[8 * st + e] - (float)hi[e]);
    return r;
}

// ------------------------------------------------------------------------------------------------
// dK, dV
// ------------------------------------------------------------------------------------------------
// One 64-query step for one wave (32 keys).  MASKED steps apply the causal / sample-end mask and
// carry P and dS as bf16 hi + lo (see the forward kernel for why).
template <int D, bool CAUSAL, bool MASKED>
__device__ __forceinline__ void dkdv_step(const unsigned char* qb_, const unsigned char* dob_,
                                          const float* lse2_, const float* delta_, int a_lane, int tr_lane,
                                          const bf16x8 (&kf)[BwdCfg<D>::KS], const bf16x8 (&vf)[BwdCfg<D>::KS],
                                          f32x16 (&dkacc)[BwdCfg<D>::DB], f32x16 (&dvacc)[BwdCfg<D>::DB],
                                          float c2, int q0, int kv, int L, int hh) {
    using C = BwdCfg<D>;
    f32x16 s[2], dp[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[qb][r] = 0.f; dp[qb][r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 aq = *(const bf16x8*)(qb_ + a_lane + qb * 32 * C::STR + ks * 32);
            s[qb] = mfma32(aq, kf[ks], s[qb]);
            bf16x8 ad = *(const bf16x8*)(dob_ + a_lane + qb * 32 * C::STR + ks * 32);
            dp[qb] = mfma32(ad, vf[ks], dp[qb]);
        }
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int qoff = 32 * qb + 8 * r4 + 4 * hh;
            const float4 l4 = *(const float4*)(lse2_ + qoff);
            const float4 d4 = *(const float4*)(delta_ + qoff);
            const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
            const float dv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int r = 4 * r4 + e;
                float p = fast_exp2(__builtin_fmaf(s[qb][r], c2, -lv[e]));
                if (MASKED) {
                    const int q = q0 + qoff + e;
                    const bool ok = q < L && kv < L && (!CAUSAL || kv <= q);
                    p = ok ? p : 0.f;
                }
                s[qb][r] = p;
                dp[qb][r] = p * (dp[qb][r] - dv[e]);
            }
        }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const bf16x8 pb = pack_regs(s[qb], st);
            const bf16x8 dsb = pack_regs(dp[qb], st);
            bf16x8 pl, dsl;
            if (MASKED) { pl = pack_regs_lo(s[qb], st, pb); dsl = pack_regs_lo(dp[qb], st, dsb); }
#pragma unroll
            for (int db = 0; db < C::DB; ++db) {
                const int off = tr_lane + (32 * qb + 16 * st) * C::STR + db * 64;
                bf16x8 ado = cat4(lds_read_tr(dob_ + off), lds_read_tr(dob_ + off + 8 * C::STR));
                dvacc[db] = mfma32(ado, pb, dvacc[db]);
                if (MASKED) dvacc[db] = mfma32(ado, pl, dvacc[db]);
                bf16x8 aq = cat4(lds_read_tr(qb_ + off), lds_read_tr(qb_ + off + 8 * C::STR));
                dkacc[db] = mfma32(aq, dsb, dkacc[db]);
                if (MASKED) dkacc[db] = mfma32(aq, dsl, dkacc[db]);
            }
        }
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, (D <= 64 ? 2 : 1))
dkdv_kernel(const __bf16* __restrict__ Q, const __bf16* __restrict__ K, const __bf16* __restrict__ V,
            const __bf16* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ Delta,
            __bf16* __restrict__ dK, __bf16* __restrict__ dV, const int32_t* __restrict__ hdr,
            const WorkItem* __restrict__ items, int T, int Hq, int Hkv, float scale) {
    using C = BwdCfg<D>;
    constexpr int BUF = 2 * C::TILE_BYTES + 2 * 64 * 4;  // Q tile, dO tile, lse2[64], delta[64]
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF];

    const int item = blockIdx.x / Hkv;
    if (item >= hdr[0]) return;
    const int c = blockIdx.x % Hkv;
    const int g = Hq / Hkv;
    const WorkItem it = items[item];
    const int sb = it.y, L = it.z - it.y, kv0 = it.x - it.y;

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, ln = l & 31, hh = l >> 5;
    const int kv = kv0 + 32 * w + ln;  // this lane's key row inside the sample
    const bool kvalid = kv < L;

    bf16x8 kf[C::KS], vf[C::KS];
    {
        const size_t off = ((size_t)(sb + (kvalid ? kv : 0)) * Hkv + c) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 z = {};
            kf[ks] = kvalid ? *(const bf16x8*)(K + off + 16 * ks) : z;
            vf[ks] = kvalid ? *(const bf16x8*)(V + off + 16 * ks) : z;
        }
    }
    f32x16 dkacc[C::DB], dvacc[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dkacc[db][r] = 0.f; dvacc[db][r] = 0.f; }

    const int first = CAUSAL ? kv0 / BWD_STEP_Q : 0;          // first query step that can see this tile
    const int nsteps = (L + BWD_STEP_Q - 1) / BWD_STEP_Q - first;  // >= 1 because kv0 < L
    const int total = nsteps * g;
    const size_t q_row_elems = (size_t)Hq * D;
    const float c2 = scale * kLog2e;
    const int a_lane = ln * C::STR + hh * 16;
    const int tr_lane = tr_lane_offset(l, C::STR);
    const int wk_lo = kv0 + 32 * w, wk_hi = wk_lo + 31;

    Stage64<D> sq, sdo;
    float lse_reg = 0.f, delta_reg = 0.f;  // threads 0..63 stage lse2 / delta of one query row each
    auto load_step = [&](int idx) {
        const int h = c * g + idx / nsteps;
        const int q0 = (first + idx % nsteps) * BWD_STEP_Q;
        sq.load(Q + ((size_t)sb * Hq + h) * D, q_row_elems, q0, L, tid);
        sdo.load(dO + ((size_t)sb * Hq + h) * D, q_row_elems, q0, L, tid);
        if (tid < 64) {
            const bool ok = q0 + tid < L;
            lse_reg = ok ? LSE[(size_t)h * T + sb + q0 + tid] * kLog2e : 0.f;
            delta_reg = ok ? Delta[(size_t)h * T + sb + q0 + tid] : 0.f;
        }
    };
    auto store_step = [&](int buf) {
        unsigned char* b = lds + buf * BUF;
        sq.store(b, C::STR, tid);
        sdo.store(b + C::TILE_BYTES, C::STR, tid);
        if (tid < 64) {
            ((float*)(b + 2 * C::TILE_BYTES))[tid] = lse_reg;
            ((float*)(b + 2 * C::TILE_BYTES))[64 + tid] = delta_reg;
        }
    };

    load_step(0);
    store_step(0);
    __syncthreads();
    for (int idx = 0; idx < total; ++idx) {
        const bool more = idx + 1 < total;
        if (more) load_step(idx + 1);
        const unsigned char* b = lds + (idx & 1) * BUF;
        const float* lse2_ = (const float*)(b + 2 * C::TILE_BYTES);
        const int q0 = (first + idx % nsteps) * BWD_STEP_Q;
        // causal: a query step entirely above this wave's keys sees none of them
        const bool active = !CAUSAL || q0 + BWD_STEP_Q - 1 >= wk_lo;
        if (active) {
            // Rows past the sample end are staged as zeros and end up only in outputs that are
            // never stored, so the mask is needed under the causal diagonal only; samples shorter
            // than one step take the careful path too (few keys per row, O(1) gradients).
            const bool masked = (CAUSAL && q0 < wk_hi) || (L < BWD_STEP_Q);
            if (masked)
                dkdv_step<D, CAUSAL, true>(b, b + C::TILE_BYTES, lse2_, lse2_ + 64, a_lane, tr_lane, kf, vf,
                                           dkacc, dvacc, c2, q0, kv, L, hh);
            else
                dkdv_step<D, CAUSAL, false>(b, b + C::TILE_BYTES, lse2_, lse2_ + 64, a_lane, tr_lane, kf, vf,
                                            dkacc, dvacc, c2, q0, kv, L, hh);
        }
        if (more) store_step((idx + 1) & 1);
        __syncthreads();
    }

    if (kvalid) {
        __bf16* dkp = dK + ((size_t)(sb + kv) * Hkv + c) * D;
        __bf16* dvp = dV + ((size_t)(sb + kv) * Hkv + c) * D;
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d0 = 32 * db + 8 * r4 + 4 * hh;
                if (d0 < D) {
                    bf16x4 a, b;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        a[e] = (__bf16)(dkacc[db][4 * r4 + e] * scale);
                        b[e] = (__bf16)(dvacc[db][4 * r4 + e]);
                    }
                    *(bf16x4*)(dkp + d0) = a;
                    *(bf16x4*)(dvp + d0) = b;
                }
            }
    }
}

template <int D>
static hipError_t launch_dkdv_d(const BwdArgs& a, hipStream_t stream) {
    dim3 grid((unsigned)(a.max_items_kv * a.num_kv_heads)), block(256);
    auto q = (const __bf16*)a.q; auto k = (const __bf16*)a.k; auto v = (const __bf16*)a.v;
    auto dO = (const __bf16*)a.dout;
    if (a.causal)
        hipLaunchKernelGGL((dkdv_kernel<D, true>), grid, block, 0, stream, q, k, v, dO, a.lse, a.delta,
                           (__bf16*)a.dk, (__bf16*)a.dv, a.sched_hdr_kv, a.items_kv, a.total_tokens,
                           a.num_q_heads, a.num_kv_heads, a.scale);
    else
        hipLaunchKernelGGL((dkdv_kernel<D, false>), grid, block, 0, stream, q, k, v, dO, a.lse, a.delta,
                           (__bf16*)a.dk, (__bf16*)a.dv, a.sched_hdr_kv, a.items_kv, a.total_tokens,
                           a.num_q_heads, a.num_kv_heads, a.scale);
    return hipGetLastError();
}

hipError_t launch_bwd_dkdv(const BwdArgs& a, hipStream_t stream) {
    switch (a.head_dim) {
        case 64: return launch_dkdv_d<64>(a, stream);
        case 80: return launch_dkdv_d<80>(a, stream);
        case 96: return launch_dkdv_d<96>(a, stream);
        case 128: return launch_dkdv_d<128>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

// ------------------------------------------------------------------------------------------------
// dQ
// ------------------------------------------------------------------------------------------------
template <int D, bool CAUSAL, bool MASKED>
__device__ __forceinline__ void dq_step(const unsigned char* kb_, const unsigned char* vb_, int a_lane,
                                        int tr_lane, const bf16x8 (&qf)[BwdCfg<D>::KS],
                                        const bf16x8 (&dof)[BwdCfg<D>::KS], f32x16 (&dqacc)[BwdCfg<D>::DB],
                                        float c2, float lse2, float delta, int kv0, int qrow, int L, int hh) {
    using C = BwdCfg<D>;
    f32x16 s[2], dp[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[b][r] = 0.f; dp[b][r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 ak = *(const bf16x8*)(kb_ + a_lane + b * 32 * C::STR + ks * 32);
            s[b] = mfma32(ak, qf[ks], s[b]);
            bf16x8 av = *(const bf16x8*)(vb_ + a_lane + b * 32 * C::STR + ks * 32);
            dp[b] = mfma32(av, dof[ks], dp[b]);
        }
    }
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p = fast_exp2(__builtin_fmaf(s[b][r], c2, -lse2));
            if (MASKED) {
                const int kv = kv0 + 32 * b + 8 * (r / 4) + 4 * hh + (r % 4);
                const bool ok = kv < L && qrow < L && (!CAUSAL || kv <= qrow);
                p = ok ? p : 0.f;
            }
            dp[b][r] = p * (dp[b][r] - delta);
        }
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const bf16x8 dsb = pack_regs(dp[b], st);
            bf16x8 dsl;
            if (MASKED) dsl = pack_regs_lo(dp[b], st, dsb);
#pragma unroll
            for (int db = 0; db < C::DB; ++db) {
                const int off = tr_lane + (32 * b + 16 * st) * C::STR + db * 64;
                bf16x8 ak = cat4(lds_read_tr(kb_ + off), lds_read_tr(kb_ + off + 8 * C::STR));
                dqacc[db] = mfma32(ak, dsb, dqacc[db]);
                if (MASKED) dqacc[db] = mfma32(ak, dsl, dqacc[db]);
            }
        }
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, (D <= 80 ? 2 : 1))
dq_kernel(const __bf16* __restrict__ Q, const __bf16* __restrict__ K, const __bf16* __restrict__ V,
          const __bf16* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ Delta,
          __bf16* __restrict__ dQ, const int32_t* __restrict__ hdr, const WorkItem* __restrict__ items,
          int T, int Hq, int Hkv, float scale) {
    using C = BwdCfg<D>;
    constexpr int BUF = 2 * C::TILE_BYTES;  // K tile, V tile
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF];

    const int item = blockIdx.x / Hq;
    if (item >= hdr[0]) return;
    const int hp = blockIdx.x % Hq;
    const int kvh = hp % Hkv;
    const int h = kvh * (Hq / Hkv) + hp / Hkv;
    const WorkItem it = items[item];
    const int sb = it.y, L = it.z - it.y, q0 = it.x - it.y;

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, ln = l & 31, hh = l >> 5;
    const int qrow = q0 + 32 * w + ln;
    const bool qvalid = qrow < L;

    bf16x8 qf[C::KS], dof[C::KS];
    float lse2 = 0.f, delta = 0.f;
    {
        const size_t off = ((size_t)(sb + (qvalid ? qrow : 0)) * Hq + h) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 z = {};
            qf[ks] = qvalid ? *(const bf16x8*)(Q + off + 16 * ks) : z;
            dof[ks] = qvalid ? *(const bf16x8*)(dO + off + 16 * ks) : z;
        }
        if (qvalid) {
            lse2 = LSE[(size_t)h * T + sb + qrow] * kLog2e;
            delta = Delta[(size_t)h * T + sb + qrow];
        }
    }
    f32x16 dqacc[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dqacc[db][r] = 0.f;

    const int kv_end = CAUSAL ? min(L, q0 + BWD_TILE_Q) : L;
    const int nsteps = (kv_end + BWD_STEP_KV - 1) / BWD_STEP_KV;
    const size_t kv_row_elems = (size_t)Hkv * D;
    const __bf16* kbase = K + ((size_t)sb * Hkv + kvh) * D;
    const __bf16* vbase = V + ((size_t)sb * Hkv + kvh) * D;
    const float c2 = scale * kLog2e;
    const int a_lane = ln * C::STR + hh * 16;
    const int tr_lane = tr_lane_offset(l, C::STR);
    const int wq_lo = q0 + 32 * w, wq_hi = wq_lo + 31;

    Stage64<D> sk, sv;
    sk.load(kbase, kv_row_elems, 0, L, tid);
    sv.load(vbase, kv_row_elems, 0, L, tid);
    sk.store(lds, C::STR, tid);
    sv.store(lds + C::TILE_BYTES, C::STR, tid);
    __syncthreads();
    for (int j = 0; j < nsteps; ++j) {
        const int kv0 = j * BWD_STEP_KV;
        const bool more = j + 1 < nsteps;
        if (more) {
            sk.load(kbase, kv_row_elems, kv0 + BWD_STEP_KV, L, tid);
            sv.load(vbase, kv_row_elems, kv0 + BWD_STEP_KV, L, tid);
        }
        const unsigned char* b = lds + (j & 1) * BUF;
        const bool active = !CAUSAL || kv0 <= wq_hi;
        if (active) {
            const bool masked = (kv0 + BWD_STEP_KV > L) || (CAUSAL && kv0 + BWD_STEP_KV - 1 > wq_lo);
            if (masked)
                dq_step<D, CAUSAL, true>(b, b + C::TILE_BYTES, a_lane, tr_lane, qf, dof, dqacc, c2, lse2, delta,
                                         kv0, qrow, L, hh);
            else
                dq_step<D, CAUSAL, false>(b, b + C::TILE_BYTES, a_lane, tr_lane, qf, dof, dqacc, c2, lse2, delta,
                                          kv0, qrow, L, hh);
        }
        if (more) {
            unsigned char* nb = lds + ((j + 1) & 1) * BUF;
            sk.store(nb, C::STR, tid);
            sv.store(nb + C::TILE_BYTES, C::STR, tid);
        }
        __syncthreads();
    }

    if (qvalid) {
        __bf16* dqp = dQ + ((size_t)(sb + qrow) * Hq + h) * D;
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                const int d0 = 32 * db + 8 * r4 + 4 * hh;
                if (d0 < D) {
                    bf16x4 a;
#pragma unroll
                    for (int e = 0; e < 4; ++e) a[e] = (__bf16)(dqacc[db][4 * r4 + e] * scale);
                    *(bf16x4*)(dqp + d0) = a;
                }
            }
    }
}

template <int D>
static hipError_t launch_dq_d(const BwdArgs& a, hipStream_t stream) {
    dim3 grid((unsigned)(a.max_items_q * a.num_q_heads)), block(256);
    auto q = (const __bf16*)a.q; auto k = (const __bf16*)a.k; auto v = (const __bf16*)a.v;
    auto dO = (const __bf16*)a.dout;
    if (a.causal)
        hipLaunchKernelGGL((dq_kernel<D, true>), grid, block, 0, stream, q, k, v, dO, a.lse, a.delta,
                           (__bf16*)a.dq, a.sched_hdr_q, a.items_q, a.total_tokens, a.num_q_heads,
                           a.num_kv_heads, a.scale);
    else
        hipLaunchKernelGGL((dq_kernel<D, false>), grid, block, 0, stream, q, k, v, dO, a.lse, a.delta,
                           (__bf16*)a.dq, a.sched_hdr_q, a.items_q, a.total_tokens, a.num_q_heads,
                           a.num_kv_heads, a.scale);
    return hipGetLastError();
}

hipError_t launch_bwd_dq(const BwdArgs& a, hipStream_t stream) {
    switch (a.head_dim) {
        case 64: return launch_dq_d<64>(a, stream);
        case 80: return launch_dq_d<80>(a, stream);
        case 96: return launch_dq_d<96>(a, stream);
        case 128: return launch_dq_d<128>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace va
