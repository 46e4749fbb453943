// Backward kernels.  P is recomputed from Q, K and the saved LSE (the paper recomputes core
// attention in the backward pass, Section 6 "Selective Activation Offloading").
//
//   (row statistics: per (head, row) LSE * log2(e) and -Delta = -sum_d dO * O; every dQ workgroup
//    computes them for its own 128 rows while it loads its fragments and writes them to the workspace,
//    where the dK/dV kernel, launched after it, finds them.  Delta is stored negated so that the dK/dV
//    kernel can load it straight into the accumulator of dP = dO V^T and get dP - Delta for free.)
//   dkdv   : one workgroup per (128-row key tile, kv head); loops over the query heads of the
//            group and over 64-row query steps; S = Q K^T is kept with one KEY per lane, so
//            that P and dS are directly the B operands of dV^T += dO^T P and dK^T += Q^T dS
//            (contraction over query rows).
//   dq     : one workgroup per (128-row query tile, query head); loops over 64-row key steps;
//            S^T = K Q^T is kept with one QUERY per lane (as in the forward), so that dS^T is the
//            B operand of dQ^T += K^T dS^T (contraction over key rows).  Two forms: dq_kernel (head_dim 80:
//            phases, four LDS stages) and dq_kernel_direct (64, 96 and 128: operands read at use, two
//            stages, more workgroups per CU).
// Splitting the backward this way needs no atomics and no fp32 dQ buffer, and the result does not
// depend on scheduling order; it recomputes S and dP once more than a fused kernel would.
//
// Staging is the forward's: 64-row tiles go straight from HBM/L2 into XOR-swizzled LDS tiles with
// direct-to-LDS loads, three stages deep, one barrier per step, completion tracked with vmcnt.
//
// The file is compiled three times (VA_BWD_PART): part 0 holds everything but the head_dim 128 dK/dV
// and dQ kernels, which parts 1 and 2 build under a different instruction-scheduling strategy of the
// compiler (measured 7 % and up to 7 % faster there, slower for the other head sizes; part 1 also with
// MFMA results in ordinary vector registers, see build.py).
#include "va_device.h"
#include "va_internal.h"

#ifndef VA_BWD_PART
#define VA_BWD_PART 0
#endif

namespace va {
hipError_t launch_dkdv_128(const BwdArgs& a, hipStream_t stream);  // part 1
hipError_t launch_dq_128(const BwdArgs& a, hipStream_t stream);    // part 2

template <int D>
struct BwdCfg {
    using T = LdsTile<D>;
    static constexpr int KS = D / 16;
    static constexpr int DB = (D + 31) / 32;
    static constexpr int TILE = 64 * T::ROWB;        // one 64-row tile in LDS
    static constexpr int NI = TileDma<D, 64>::NI;    // load instructions per wave per tile
    static constexpr int STAT_BYTES = 4 * 128;       // per wave: 16 x lse2, 16 x delta
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
// One 64-query step for one wave (32 keys).  MASKED steps apply the causal / sample-end mask and, where
// `lo` is set (wave-uniform), carry P and dS as bf16 hi + lo (see the forward kernel for why).
//   qt, dot : LDS tiles of Q and dO (64 rows);  stat: per 16 rows {16 x lse2, 16 x delta}
//   aaddr   : per-lane offsets of the row-wise 16-byte reads, taddr: of the transposing reads
template <int D, bool CAUSAL, bool MASKED>
__device__ __forceinline__ void dkdv_step(const unsigned char* qt, const unsigned char* dot,
                                          const unsigned char* stat, const int (&aaddr)[BwdCfg<D>::KS],
                                          const int (&taddr)[BwdCfg<D>::DB][2],
                                          const bf16x8 (&kf)[BwdCfg<D>::KS], const bf16x8 (&vf)[BwdCfg<D>::KS],
                                          f32x16 (&dkacc)[BwdCfg<D>::DB], f32x16 (&dvacc)[BwdCfg<D>::DB],
                                          float c2, int q0, int kv, int L, int hh, bool lo = MASKED) {
    using C = BwdCfg<D>;
    constexpr int ROWB = C::T::ROWB;
    // without the causal mask every masked step carries lo parts, next to the hi parts' MFMAs; under it few
    // steps do (`lo`), in a pass of their own behind one wave-uniform branch
    constexpr bool LO_INLINE = MASKED && !CAUSAL;
    // The two 32-query halves of the step are handled one after the other, so that only one half's
    // scores and dP (2 x 16 registers) are live at a time.
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        // keep the instruction scheduler from hoisting the second half's LDS reads over the first
        // half: it would hold both halves' operands in registers and spill
        if (qb) __builtin_amdgcn_sched_barrier(0);
        f32x16 s, dp;
        float lv[16];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            const int qoff = 32 * qb + 8 * r4 + 4 * hh;  // 4 consecutive query rows, inside one 16-row block
            const unsigned char* sp = stat + (qoff >> 4) * 128 + (qoff & 15) * 4;
            const float4 l4 = *(const float4*)(sp);
            const float4 d4 = *(const float4*)(sp + 64);
            lv[4 * r4 + 0] = l4.x; lv[4 * r4 + 1] = l4.y; lv[4 * r4 + 2] = l4.z; lv[4 * r4 + 3] = l4.w;
            // dP accumulates on top of -Delta
            dp[4 * r4 + 0] = d4.x; dp[4 * r4 + 1] = d4.y; dp[4 * r4 + 2] = d4.z; dp[4 * r4 + 3] = d4.w;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 aq = *(const bf16x8*)(qt + aaddr[ks] + qb * 32 * ROWB);
            s = mfma32(aq, kf[ks], s);
            bf16x8 ad = *(const bf16x8*)(dot + aaddr[ks] + qb * 32 * ROWB);
            dp = mfma32(ad, vf[ks], dp);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p = fast_exp2(__builtin_fmaf(s[r], c2, -lv[r]));
            if (MASKED) {
                const int q = q0 + 32 * qb + 8 * (r / 4) + 4 * hh + (r % 4);
                const bool ok = q < L && kv < L && (!CAUSAL || kv <= q);
                p = ok ? p : 0.f;
            }
            s[r] = p;
            dp[r] = p * dp[r];
        }
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const bf16x8 pb = pack_regs(s, st);
            const bf16x8 dsb = pack_regs(dp, st);
            bf16x8 pl, dsl;
            if (LO_INLINE) { pl = pack_regs_lo(s, st, pb); dsl = pack_regs_lo(dp, st, dsb); }
            const int rowoff = (32 * qb + 16 * st) * ROWB;
#pragma unroll
            for (int db = 0; db < C::DB; ++db) {
                bf16x8 ado = cat4(lds_read_tr(dot + rowoff + taddr[db][0]), lds_read_tr(dot + rowoff + taddr[db][1]));
                dvacc[db] = mfma32(ado, pb, dvacc[db]);
                if (LO_INLINE) dvacc[db] = mfma32(ado, pl, dvacc[db]);
                bf16x8 aq = cat4(lds_read_tr(qt + rowoff + taddr[db][0]), lds_read_tr(qt + rowoff + taddr[db][1]));
                dkacc[db] = mfma32(aq, dsb, dkacc[db]);
                if (LO_INLINE) dkacc[db] = mfma32(aq, dsl, dkacc[db]);
            }
        }
        if (MASKED && CAUSAL && lo) {
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const bf16x8 pl = pack_regs_lo(s, st, pack_regs(s, st));
                const bf16x8 dsl = pack_regs_lo(dp, st, pack_regs(dp, st));
                const int rowoff = (32 * qb + 16 * st) * ROWB;
#pragma unroll
                for (int db = 0; db < C::DB; ++db) {
                    bf16x8 ado = cat4(lds_read_tr(dot + rowoff + taddr[db][0]), lds_read_tr(dot + rowoff + taddr[db][1]));
                    dvacc[db] = mfma32(ado, pl, dvacc[db]);
                    bf16x8 aq = cat4(lds_read_tr(qt + rowoff + taddr[db][0]), lds_read_tr(qt + rowoff + taddr[db][1]));
                    dkacc[db] = mfma32(aq, dsl, dkacc[db]);
                }
            }
        }
    }
}

// ---- the mask-free step, cut into phases whose LDS operands are fetched one phase ahead ----
// An LDS read takes a few hundred cycles to return while an MFMA issues every 32; left to itself
// the compiler puts each read right in front of the MFMA that consumes it and the matrix pipe
// waits most of the time.  Here every phase first ISSUES the reads of the next phase into a second
// set of registers and then runs its own MFMAs / vector work on operands that arrived long ago;
// sched_barriers keep the phases apart.
template <int D>
struct DkdvOpsA {  // operands of S = Q K^T and dP = dO V^T for one 32-query half
    bf16x8 q[BwdCfg<D>::KS], d[BwdCfg<D>::KS];
};
template <int D>
struct DkdvOpsC {  // operands of dV^T += dO^T P and dK^T += Q^T dS for one half
    bf16x8 o[2][BwdCfg<D>::DB], q[2][BwdCfg<D>::DB];
};
template <int D, int HALF>
__device__ __forceinline__ void dkdv_load_A(const unsigned char* stage, const int (&aaddr)[BwdCfg<D>::KS],
                                            DkdvOpsA<D>& f, f32x16& dp, int hh) {
    using C = BwdCfg<D>;
    constexpr int ROWB = C::T::ROWB;
    const unsigned char* stat = stage + 2 * C::TILE;
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) {
        f.q[ks] = *(const bf16x8*)(stage + aaddr[ks] + HALF * 32 * ROWB);
        f.d[ks] = *(const bf16x8*)(stage + C::TILE + aaddr[ks] + HALF * 32 * ROWB);
    }
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {  // dP accumulates on top of -Delta
        const int qoff = 32 * HALF + 8 * r4 + 4 * hh;
        const float4 d4 = *(const float4*)(stat + (qoff >> 4) * 128 + (qoff & 15) * 4 + 64);
        dp[4 * r4 + 0] = d4.x; dp[4 * r4 + 1] = d4.y; dp[4 * r4 + 2] = d4.z; dp[4 * r4 + 3] = d4.w;
    }
}
template <int D, int HALF>
__device__ __forceinline__ void dkdv_load_lse(const unsigned char* stage, float (&lv)[16], int hh) {
    const unsigned char* stat = stage + 2 * BwdCfg<D>::TILE;
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
        const int qoff = 32 * HALF + 8 * r4 + 4 * hh;
        const float4 l4 = *(const float4*)(stat + (qoff >> 4) * 128 + (qoff & 15) * 4);
        lv[4 * r4 + 0] = l4.x; lv[4 * r4 + 1] = l4.y; lv[4 * r4 + 2] = l4.z; lv[4 * r4 + 3] = l4.w;
    }
}
template <int D, int HALF>
__device__ __forceinline__ void dkdv_load_C(const unsigned char* stage, const int (&taddr)[BwdCfg<D>::DB][2],
                                            DkdvOpsC<D>& f) {
    using C = BwdCfg<D>;
    constexpr int ROWB = C::T::ROWB;
#pragma unroll
    for (int st = 0; st < 2; ++st) {
        const unsigned char* qt = stage + (32 * HALF + 16 * st) * ROWB;
        const unsigned char* dot = qt + C::TILE;
#pragma unroll
        for (int db = 0; db < C::DB; ++db) {
            f.o[st][db] = cat4(lds_read_tr(dot + taddr[db][0]), lds_read_tr(dot + taddr[db][1]));
            f.q[st][db] = cat4(lds_read_tr(qt + taddr[db][0]), lds_read_tr(qt + taddr[db][1]));
        }
    }
}
template <int D>
__device__ __forceinline__ void dkdv_run_A(const DkdvOpsA<D>& f, const bf16x8 (&kf)[BwdCfg<D>::KS],
                                           const bf16x8 (&vf)[BwdCfg<D>::KS], f32x16& s, f32x16& dp) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < BwdCfg<D>::KS; ++ks) {
        s = mfma32(f.q[ks], kf[ks], s);
        dp = mfma32(f.d[ks], vf[ks], dp);
    }
}
// P = exp2(S c2 - lse2) and dS = P (dP - Delta), rounded to bf16 (vector ALU only)
__device__ __forceinline__ void dkdv_run_B(const f32x16& s, const f32x16& dp, const float (&lv)[16], float c2,
                                           bf16x8 (&pb)[2], bf16x8 (&dsb)[2]) {
    f32x16 p, ds;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        p[r] = fast_exp2(__builtin_fmaf(s[r], c2, -lv[r]));
        ds[r] = p[r] * dp[r];
    }
#pragma unroll
    for (int st = 0; st < 2; ++st) {
        pb[st] = pack_regs(p, st);
        dsb[st] = pack_regs(ds, st);
    }
}
template <int D>
__device__ __forceinline__ void dkdv_run_C(const DkdvOpsC<D>& f, const bf16x8 (&pb)[2], const bf16x8 (&dsb)[2],
                                           f32x16 (&dkacc)[BwdCfg<D>::DB], f32x16 (&dvacc)[BwdCfg<D>::DB]) {
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int db = 0; db < BwdCfg<D>::DB; ++db) {
            dvacc[db] = mfma32(f.o[st][db], pb[st], dvacc[db]);
            dkacc[db] = mfma32(f.q[st][db], dsb[st], dkacc[db]);
        }
}

// The same work cut differently: S alone, then dP, dV and dK with the vector work in their shadow.
// A wave that has just issued an MFMA cannot issue anything for about 16 cycles and is then free for
// about 16 more before the matrix pipe takes the next one (measured: up to 3 vector instructions per
// MFMA cost nothing, further ones about 4.5 cycles each).  Vector work that does not depend on the
// MFMAs around it is therefore cheapest when spread between them.
template <int D>
__device__ __forceinline__ void dkdv_run_S(const DkdvOpsA<D>& f, const bf16x8 (&kf)[BwdCfg<D>::KS], f32x16& s) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < BwdCfg<D>::KS; ++ks) s = mfma32(f.q[ks], kf[ks], s);
}
template <int D>
__device__ __forceinline__ void dkdv_run_dP(const DkdvOpsA<D>& f, const bf16x8 (&vf)[BwdCfg<D>::KS], f32x16& dp) {
#pragma unroll
    for (int ks = 0; ks < BwdCfg<D>::KS; ++ks) dp = mfma32(f.d[ks], vf[ks], dp);
}
// rounds of {1 MFMA, DS_PER LDS reads, VALU_PER vector instructions} for the region that ends here
template <int N_MFMA, int DS_PER, int VALU_PER>
__device__ __forceinline__ void dkdv_interleave() {
#pragma unroll
    for (int i = 0; i < N_MFMA; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (DS_PER) __builtin_amdgcn_sched_group_barrier(0x100, DS_PER, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);
    }
}

// Load K of the 2*NI + 1 direct-to-LDS loads of one dK/dV step: K = 0 the stats, then NI loads of the Q
// tile, then NI of the dO tile.  K beyond that is a no-op, so callers can name slots freely.
template <int D, int K>
__device__ __forceinline__ void dkdv_issue_part(bool ragged, const TileDma<D, 64>& dma, const unsigned char* q,
                                                const unsigned char* dO, const unsigned char* st,
                                                uint32_t stat_off, uint32_t lds, int wave) {
    constexpr int NI = BwdCfg<D>::NI;
    if constexpr (K == 0) {
        dma4(st, stat_off, lds + 2 * BwdCfg<D>::TILE + (wave & 1) * 256);
    } else if constexpr (K <= NI) {
        dma.template issue_one<K - 1>(q, ragged, lds, wave);
    } else if constexpr (K <= 2 * NI) {
        dma.template issue_one<K - 1 - NI>(dO, ragged, lds + BwdCfg<D>::TILE, wave);
    }
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, (D <= 80 ? 2 : 1))
dkdv_kernel(const __bf16* __restrict__ Q, const __bf16* __restrict__ K, const __bf16* __restrict__ V,
            const __bf16* __restrict__ dO, const float2* __restrict__ stats,
            __bf16* __restrict__ dK, __bf16* __restrict__ dV, const int32_t* __restrict__ hdr,
            const WorkItem* __restrict__ items, int max_items, int T, int Hq, int Hkv, float scale,
            unsigned long long* __restrict__ clock_probe) {
    using C = BwdCfg<D>;
    using LT = LdsTile<D>;
    constexpr int STAGE = 2 * C::TILE + C::STAT_BYTES;  // Q tile, dO tile, stats
    constexpr int PER = 2 * C::NI + 1;                  // loads per wave per step
    // LDS stages: four where two workgroups per CU are out of reach anyway or still fit (head_dim 64),
    // three at head_dim 80, where the fourth would cost the second workgroup
    constexpr int NST = D == 80 ? 3 : 4;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE];

    int item, c;  // work item and kv head (see xcd_item_head)
    xcd_item_head(blockIdx.x, max_items, Hkv, Hkv, hdr[1], item, c);
    // (integer division runs on the vector ALU: without this, everything derived from the two, the
    // staging pointers included, would be kept in vector registers and advanced there)
    item = __builtin_amdgcn_readfirstlane(item); c = __builtin_amdgcn_readfirstlane(c);
    if (item >= hdr[0]) return;
    ClockProbe wg_clock;
    wg_clock.begin(clock_probe);
    stagger_wave_priority();
    const int g = Hq / Hkv;
    const WorkItem it = items[item];
    // same for the whole workgroup: tell the compiler, so that everything derived stays in SGPRs
    const int sb = __builtin_amdgcn_readfirstlane(it.y), L = __builtin_amdgcn_readfirstlane(it.z - it.y),
              kv0 = __builtin_amdgcn_readfirstlane(it.x - it.y);

    const int tid = threadIdx.x, w = uniform_wave_id(), l = tid & 63, ln = l & 31, hh = l >> 5;
    const int kv = kv0 + 32 * w + ln;  // this lane's key row inside the sample
    const bool kvalid = kv < L;

    const int first = CAUSAL ? kv0 / BWD_STEP_Q : 0;               // first query step that can see this tile
    const int nsteps = (L + BWD_STEP_Q - 1) / BWD_STEP_Q - first;  // >= 1 because kv0 < L
    // Steps [0, n_head) sit on the causal diagonal, steps [n_tail, nsteps) hold the sample's ragged
    // end (its out-of-range rows are staged as copies of the last row and must be masked); samples
    // shorter than one step are all "careful".  Steps in between need no mask in any wave.
    const int n_head = (L < BWD_STEP_Q) ? nsteps : (CAUSAL ? min(2, nsteps) : 0);
    const int n_tail = max(n_head, nsteps - ((L % BWD_STEP_Q) ? 1 : 0));

    // Staging state: pointers to the next (head, step) to issue, advanced by additions only.  Every
    // quantity here is wave-uniform (scalar registers).  Loads are issued unconditionally: once the
    // last step has been issued the state stops advancing and later calls fetch that step again into
    // a stage nobody will read, so that the loop needs no branches around its loads and the count of
    // outstanding loads per step is the same everywhere.
    const uint32_t q_row_bytes = (uint32_t)Hq * D * 2;
    TileDma<D, 64> dma;  // Q and dO share the offsets
    dma.init(q_row_bytes, L, w, l);
    // stats: a wave fetches {lse2, -Delta} of 32 rows (waves w and w + 2 fetch the same ones): lanes
    // [0,16) lse2 and [16,32) -Delta of the first 16 rows, lanes [32,64) the same of the next 16
    const int srow = 32 * (w & 1) + 16 * (l >> 5) + (l & 15);
    const int last_q0 = (L - 1) / BWD_STEP_Q * BWD_STEP_Q;
    const uint32_t stat_full = (uint32_t)srow * 8 + ((l >> 4) & 1) * 4;
    const uint32_t stat_last = (uint32_t)min(srow, L - 1 - last_q0) * 8 + ((l >> 4) & 1) * 4;
    const uint32_t lds0 = lds_address(lds);
    const int total = g * nsteps;
    const bool ragged_sample = (L % BWD_STEP_Q) != 0;
    const int64_t step_q = (int64_t)BWD_STEP_Q * q_row_bytes, step_st = (int64_t)BWD_STEP_Q * 8;
    const int64_t wrap_q = (int64_t)D * 2 - (int64_t)(nsteps - 1) * step_q;       // last step of a head -> first of the next
    const int64_t wrap_st = (int64_t)T * 8 - (int64_t)(nsteps - 1) * step_st;
    const size_t qoff0 = ((size_t)(sb + first * BWD_STEP_Q) * Hq + (size_t)c * g) * D * 2;
    const unsigned char* nxt_q = (const unsigned char*)Q + qoff0;
    const unsigned char* nxt_do = (const unsigned char*)dO + qoff0;
    const unsigned char* nxt_st = (const unsigned char*)(stats + (size_t)c * g * T + sb + first * BWD_STEP_Q);
    int nxt_s = 0, nxt_n = 0, iss_stage = 0;
    // the step the current round of loads belongs to (set by begin_issue)
    bool iss_ragged = false;
    const unsigned char *iss_q = nullptr, *iss_do = nullptr, *iss_st = nullptr;
    uint32_t iss_lds = 0;
    auto begin_issue = [&]() {
        iss_q = nxt_q; iss_do = nxt_do; iss_st = nxt_st;
        iss_ragged = ragged_sample && nxt_s == nsteps - 1;
        iss_lds = lds0 + iss_stage * STAGE;
        iss_stage = iss_stage == NST - 1 ? 0 : iss_stage + 1;
        const bool more = nxt_n + 1 < total;
        const bool wrap = nxt_s == nsteps - 1;
        const int64_t aq = more ? (wrap ? wrap_q : step_q) : 0, as = more ? (wrap ? wrap_st : step_st) : 0;
        nxt_q += aq; nxt_do += aq; nxt_st += as;
        nxt_s = more ? (wrap ? 0 : nxt_s + 1) : nxt_s;
        nxt_n += more ? 1 : 0;
    };
    auto issue_stat = [&]() {
        dma4(iss_st, iss_ragged ? stat_last : stat_full, iss_lds + 2 * C::TILE + (w & 1) * 256);
    };
    // slot S of 6 per step carries loads S and S + 6
#define VA_DKDV_ISSUE_SLOT(S)                                                                             \
    dkdv_issue_part<D, (S)>(iss_ragged, dma, iss_q, iss_do, iss_st, iss_ragged ? stat_last : stat_full,   \
                            iss_lds, w);                                                                  \
    dkdv_issue_part<D, (S) + 6>(iss_ragged, dma, iss_q, iss_do, iss_st, 0, iss_lds, w);
    auto issue_all = [&]() {
        begin_issue();
        issue_stat();
        dma.issue_tile(iss_q, iss_ragged, iss_lds, w);
        dma.issue_tile(iss_do, iss_ragged, iss_lds + C::TILE, w);
    };

    int aaddr[C::KS], taddr[C::DB][2];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) aaddr[ks] = LT::off(ln, 2 * ks + hh);
#pragma unroll
    for (int db = 0; db < C::DB; ++db) {
        taddr[db][0] = LT::tr_off(l, 0, db);
        taddr[db][1] = LT::tr_off(l, 8, db);
    }

    // prologue: NST - 1 steps in flight plus this lane's K and V fragments; all waited for once (see the
    // forward kernel for why the register loads must not be left pending at loop entry)
#pragma unroll
    for (int i = 0; i < NST - 1; ++i) issue_all();
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
    wait_vmcnt<0>();
    wg_barrier();
    if constexpr (D > 80) {  // one wave per SIMD: see park_in_acc_registers
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) { park_in_acc_registers(kf[ks]); park_in_acc_registers(vf[ks]); }
    }

    f32x16 dkacc[C::DB], dvacc[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) { dkacc[db][r] = 0.f; dvacc[db][r] = 0.f; }
    const float c2 = scale * kLog2e;
    const int wk_lo = kv0 + 32 * w;
    // causal: only rows near a sample's start hold few terms, and those meet key tile 0 only
    const bool lo_steps = !CAUSAL || kv0 == 0;

    // Stage protocol.  Step i lives in stage i % NST.  VA_DKDV_SYNC() ends the part of step idx that
    // reads stage idx - 1: it waits until step idx + 1 has landed (with four stages step idx + 2,
    // issued one sync earlier, may stay in flight), passes the barrier, after which every wave is done
    // with stage idx - 1, and refills that stage with step idx + NST - 1.
    int stage_i = 0;  // stage of the current step ("idx" in the comment above)
#define VA_DKDV_SYNC()                                                               \
        wait_vmcnt<(NST - 3) * PER>();                                                   \
        wg_barrier();
#define VA_DKDV_ADVANCE()                                                            \
        stage_i = stage_i == NST - 1 ? 0 : stage_i + 1;
#define VA_DKDV_CAREFUL(st)                                                          \
    {                                                                                    \
        const unsigned char* b = lds + stage_i * STAGE;                                  \
        const int q0 = (first + (st)) * BWD_STEP_Q;                                      \
        /* causal: a query step entirely above this wave's keys sees none of them; every other  \
           step here takes the masked variant (a superset of the plain one) to keep code small */ \
        if (!CAUSAL || q0 + BWD_STEP_Q - 1 >= wk_lo)                                     \
            dkdv_step<D, CAUSAL, true>(b, b + C::TILE, b + 2 * C::TILE, aaddr, taddr, kf, vf, dkacc, dvacc, \
                                       c2, q0, kv, L, hh, lo_steps);                     \
        VA_DKDV_SYNC()                                                                   \
        issue_all();                                                                     \
        VA_DKDV_ADVANCE()                                                                \
    }

    // The mask-free step in phases.  Per half: phase A (S, dP MFMAs), phase B (vector ALU), phase C (dV, dK
    // MFMAs); each phase also issues the LDS reads of the phase after it.  The step's sync
    // sits at its start: it only has to retire stage idx - 1, and having stage idx + 1
    // published early lets the last phase fetch the next step's first operands.
    DkdvOpsA<D> fa;
    DkdvOpsC<D> fc;
    f32x16 s, dpa, dpb;  // dP accumulators of the even / odd half, preloaded with -Delta
    float lv[16];
    bf16x8 pb[2], dsb[2];
    // STAGE_TAG: the step's stage where the caller knows it (-1 otherwise); with it the LDS addresses of the
    // operand reads are per-lane offsets plus immediates instead of vector additions per step
    auto phased = [&](auto stage_tag) {
        constexpr int KNOWN = decltype(stage_tag)::value;
        VA_DKDV_SYNC()
        const int si = KNOWN >= 0 ? KNOWN : stage_i;
        const unsigned char* cur = lds + si * STAGE;
        const unsigned char* nxt = lds + (si == NST - 1 ? 0 : si + 1) * STAGE;
        // half 0 (the scalar bookkeeping of this step's loads runs behind its MFMAs)
        dkdv_load_lse<D, 0>(cur, lv, hh);
        dkdv_run_S<D>(fa, kf, s);
        begin_issue();
        __builtin_amdgcn_sched_barrier(0);
        VA_DKDV_ISSUE_SLOT(0)
        VA_DKDV_ISSUE_SLOT(1)
        dkdv_load_C<D, 0>(cur, taddr, fc);
        dkdv_run_dP<D>(fa, vf, dpa);
        dkdv_run_B(s, dpa, lv, c2, pb, dsb);
        dkdv_run_C<D>(fc, pb, dsb, dkacc, dvacc);
        dkdv_load_A<D, 1>(cur, aaddr, fa, dpb, hh);
        dkdv_interleave<C::KS, 8 * C::DB / C::KS, 14>();   // dP; dV/dK operand reads; P
        dkdv_interleave<4 * C::DB, 2, 2>();                // dV, dK; next half's S/dP operand reads; dS
        __builtin_amdgcn_sched_barrier(0);
        VA_DKDV_ISSUE_SLOT(2)
        // half 1
        dkdv_load_lse<D, 1>(cur, lv, hh);
        dkdv_run_S<D>(fa, kf, s);
        __builtin_amdgcn_sched_barrier(0);
        VA_DKDV_ISSUE_SLOT(3)
        VA_DKDV_ISSUE_SLOT(4)
        dkdv_load_C<D, 1>(cur, taddr, fc);
        dkdv_run_dP<D>(fa, vf, dpb);
        dkdv_run_B(s, dpb, lv, c2, pb, dsb);
        dkdv_run_C<D>(fc, pb, dsb, dkacc, dvacc);
        dkdv_load_A<D, 0>(nxt, aaddr, fa, dpa, hh);  // next step (dropped after the last one)
        dkdv_interleave<C::KS, 8 * C::DB / C::KS, 14>();   // dP; dV/dK operand reads; P
        dkdv_interleave<4 * C::DB, 2, 2>();                // dV, dK; next half's S/dP operand reads; dS
        __builtin_amdgcn_sched_barrier(0);
        VA_DKDV_ISSUE_SLOT(5)
        VA_DKDV_ADVANCE()
    };

    // Masked steps (the causal diagonal, the one that holds the sample's end) take the simple form: in
    // phases, with the mask and the lo parts on top, they were measured no faster even at one wave per SIMD.
    for (int hg = 0; hg < g; ++hg) {
        int st = 0;
        for (; st < n_head; ++st) VA_DKDV_CAREFUL(st)
        if (st < n_tail) {
            dkdv_load_A<D, 0>(lds + stage_i * STAGE, aaddr, fa, dpa, hh);
            using Unknown = std::integral_constant<int, -1>;
            if constexpr (D == 64) {  // (elsewhere the four copies of the step cost registers the kernel does not have)
                for (; st < n_tail && stage_i != 0; ++st) phased(Unknown{});
                for (; st + NST <= n_tail; st += NST) {  // whole rounds of the stages, each stage a constant
                    phased(std::integral_constant<int, 0>{});
                    phased(std::integral_constant<int, 1>{});
                    phased(std::integral_constant<int, 2>{});
                    phased(std::integral_constant<int, 3>{});
                }
            }
            for (; st < n_tail; ++st) phased(Unknown{});
        }
        for (; st < nsteps; ++st) VA_DKDV_CAREFUL(st)
    }
    wait_vmcnt<0>();  // the surplus loads issued near the end must land before this LDS is given away
#undef VA_DKDV_SYNC
#undef VA_DKDV_ISSUE_SLOT
#undef VA_DKDV_ADVANCE
#undef VA_DKDV_CAREFUL

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
    wg_clock.end(clock_probe);
}

template <int D>
static hipError_t launch_dkdv_d(const BwdArgs& a, hipStream_t stream) {
    dim3 grid((unsigned)(a.max_items_kv * a.num_kv_heads)), block(256);
    auto q = (const __bf16*)a.q; auto k = (const __bf16*)a.k; auto v = (const __bf16*)a.v;
    auto dO = (const __bf16*)a.dout;
    auto st = (const float2*)a.stats;
    if (a.causal)
        hipLaunchKernelGGL((dkdv_kernel<D, true>), grid, block, 0, stream, q, k, v, dO, st,
                           (__bf16*)a.dk, (__bf16*)a.dv, a.sched_hdr_kv, a.items_kv, (int)a.max_items_kv, a.total_tokens,
                           a.num_q_heads, a.num_kv_heads, a.scale, a.clock_probe_dkdv);
    else
        hipLaunchKernelGGL((dkdv_kernel<D, false>), grid, block, 0, stream, q, k, v, dO, st,
                           (__bf16*)a.dk, (__bf16*)a.dv, a.sched_hdr_kv, a.items_kv, (int)a.max_items_kv, a.total_tokens,
                           a.num_q_heads, a.num_kv_heads, a.scale, a.clock_probe_dkdv);
    return hipGetLastError();
}

#if VA_BWD_PART == 0
hipError_t launch_bwd_dkdv(const BwdArgs& a, hipStream_t stream) {
    switch (a.head_dim) {
        case 64: return launch_dkdv_d<64>(a, stream);
        case 80: return launch_dkdv_d<80>(a, stream);
        case 96: return launch_dkdv_d<96>(a, stream);
        case 128: return launch_dkdv_128(a, stream);
        default: return hipErrorInvalidValue;
    }
}
#elif VA_BWD_PART == 1
hipError_t launch_dkdv_128(const BwdArgs& a, hipStream_t stream) { return launch_dkdv_d<128>(a, stream); }
#endif

// ------------------------------------------------------------------------------------------------
// dQ
// ------------------------------------------------------------------------------------------------
// The step that holds the sample's end, for the kernel without the causal mask (under it the masked steps
// run in phases, see dq_kernel): keys and rows beyond the sample are masked, dS goes through its MFMAs as
// bf16 hi + lo.  Operands are read right before use.
template <int D>
__device__ __forceinline__ void dq_end_step(const unsigned char* kt, const unsigned char* vt,
                                            const int (&aaddr)[BwdCfg<D>::KS], const int (&taddr)[BwdCfg<D>::DB][2],
                                            const bf16x8 (&qf)[BwdCfg<D>::KS], const bf16x8 (&dof)[BwdCfg<D>::KS],
                                            f32x16 (&dqacc)[BwdCfg<D>::DB], float c2, float lse2, float ndelta,
                                            int kv0, int qrow, int L, int hh) {
    using C = BwdCfg<D>;
    constexpr int ROWB = C::T::ROWB;
    f32x16 s[2], dp[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[b][r] = 0.f; dp[b][r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 ak = *(const bf16x8*)(kt + aaddr[ks] + b * 32 * ROWB);
            s[b] = mfma32(ak, qf[ks], s[b]);
            bf16x8 av = *(const bf16x8*)(vt + aaddr[ks] + b * 32 * ROWB);
            dp[b] = mfma32(av, dof[ks], dp[b]);
        }
    }
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p = fast_exp2(__builtin_fmaf(s[b][r], c2, -lse2));
            const int kv = kv0 + 32 * b + 8 * (r / 4) + 4 * hh + (r % 4);
            p = (kv < L && qrow < L) ? p : 0.f;
            dp[b][r] = p * (dp[b][r] + ndelta);
        }
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const bf16x8 dsb = pack_regs(dp[b], st);
            const bf16x8 dsl = pack_regs_lo(dp[b], st, dsb);
            const int rowoff = (32 * b + 16 * st) * ROWB;
#pragma unroll
            for (int db = 0; db < C::DB; ++db) {
                bf16x8 ak = cat4(lds_read_tr(kt + rowoff + taddr[db][0]), lds_read_tr(kt + rowoff + taddr[db][1]));
                dqacc[db] = mfma32(ak, dsb, dqacc[db]);
                dqacc[db] = mfma32(ak, dsl, dqacc[db]);
            }
        }
}

// ---- the mask-free dQ step in phases (see the dK/dV kernel): S | dP with exp in its shadow | dQ
// with dS in its shadow; the LDS operands of a phase are read one phase ahead ----
template <int D>
struct DqOpsA {  // operands of S^T = K Q^T or dP^T = V dO^T for the step's two 32-key blocks
    bf16x8 a[2][BwdCfg<D>::KS];
};
template <int D>
struct DqOpsT {  // K^T operands of dQ^T += K^T dS^T: key block b, 16-key step st, 32-channel block db
    bf16x8 a[2][2][BwdCfg<D>::DB];
};
template <int D>
__device__ __forceinline__ void dq_load_A(const unsigned char* tile, const int (&aaddr)[BwdCfg<D>::KS], DqOpsA<D>& f) {
    constexpr int ROWB = BwdCfg<D>::T::ROWB;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int ks = 0; ks < BwdCfg<D>::KS; ++ks) f.a[b][ks] = *(const bf16x8*)(tile + aaddr[ks] + b * 32 * ROWB);
}
template <int D>
__device__ __forceinline__ void dq_load_T(const unsigned char* kt, const int (&taddr)[BwdCfg<D>::DB][2], DqOpsT<D>& f) {
    constexpr int ROWB = BwdCfg<D>::T::ROWB;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int db = 0; db < BwdCfg<D>::DB; ++db) {
                const unsigned char* p0 = kt + (32 * b + 16 * st) * ROWB;
                f.a[b][st][db] = cat4(lds_read_tr(p0 + taddr[db][0]), lds_read_tr(p0 + taddr[db][1]));
            }
}
// acc[b] = init + sum_ks ops[b][ks] x frag[ks]
template <int D>
__device__ __forceinline__ void dq_run_A(const DqOpsA<D>& f, const bf16x8 (&frag)[BwdCfg<D>::KS], const f32x16& init,
                                         f32x16 (&acc)[2]) {
#pragma unroll
    for (int ks = 0; ks < BwdCfg<D>::KS; ++ks)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[b] = mfma32(f.a[b][ks], frag[ks], ks == 0 ? init : acc[b]);
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, (D <= 80 ? 2 : 1))
dq_kernel(const __bf16* __restrict__ Q, const __bf16* __restrict__ K, const __bf16* __restrict__ V,
          const __bf16* __restrict__ dO, const __bf16* __restrict__ O, const float* __restrict__ LSE,
          float2* __restrict__ stats, __bf16* __restrict__ dQ, const int32_t* __restrict__ hdr, const WorkItem* __restrict__ items,
          int max_items, int T, int Hq, int Hkv, float scale, unsigned long long* __restrict__ clock_probe) {
    using C = BwdCfg<D>;
    using LT = LdsTile<D>;
    constexpr int STAGE = 2 * C::TILE;  // K tile, V tile
    constexpr int NST = 4;              // LDS stages
    constexpr int PER = 2 * C::NI;      // loads per wave per step
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * STAGE];

    int item, hp;
    xcd_item_head(blockIdx.x, max_items, Hq, Hkv, hdr[1], item, hp);
    item = __builtin_amdgcn_readfirstlane(item); hp = __builtin_amdgcn_readfirstlane(hp);  // see dkdv_kernel
    if (item >= hdr[0]) return;
    ClockProbe wg_clock;
    wg_clock.begin(clock_probe);
    const int kvh = hp % Hkv;
    const int h = kvh * (Hq / Hkv) + hp / Hkv;
    const WorkItem it = items[item];
    // same for the whole workgroup: tell the compiler, so that everything derived stays in SGPRs
    const int sb = __builtin_amdgcn_readfirstlane(it.y), L = __builtin_amdgcn_readfirstlane(it.z - it.y),
              q0 = __builtin_amdgcn_readfirstlane(it.x - it.y);

    const int tid = threadIdx.x, w = uniform_wave_id(), l = tid & 63, ln = l & 31, hh = l >> 5;
    const int qrow = q0 + 32 * w + ln;
    const bool qvalid = qrow < L;

    const int kv_end = CAUSAL ? min(L, q0 + BWD_TILE_Q) : L;
    const int nsteps = (kv_end + BWD_STEP_KV - 1) / BWD_STEP_KV;
    const int n_plain = CAUSAL ? min(L, q0 + 1) / BWD_STEP_KV : L / BWD_STEP_KV;
    const unsigned char* kbase = (const unsigned char*)(K + ((size_t)sb * Hkv + kvh) * D);
    const unsigned char* vbase = (const unsigned char*)(V + ((size_t)sb * Hkv + kvh) * D);
    const uint32_t row_bytes = (uint32_t)Hkv * D * 2;
    TileDma<D, 64, D == 80> dma;
    dma.init(row_bytes, L, w, l);
    const uint32_t lds0 = lds_address(lds);
    // Staging, as in the dK/dV kernel: pointers advanced by additions, loads issued unconditionally
    // (after the last step the same step is fetched again into a stage nobody reads), so that every
    // step has the same number of loads in flight and the loop needs no branches around them.
    const int64_t step_bytes = (int64_t)BWD_STEP_KV * row_bytes;
    const bool ragged_sample = (L % BWD_STEP_KV) != 0;
    const int last_step = (L + BWD_STEP_KV - 1) / BWD_STEP_KV - 1;  // the one holding the sample's end
    const unsigned char *nxt_k = kbase, *nxt_v = vbase;
    int nxt_j = 0, iss_stage = 0;
    bool iss_ragged = false;
    const unsigned char *iss_k = nullptr, *iss_v = nullptr;
    uint32_t iss_lds = 0;
    auto begin_issue = [&]() {
        iss_k = nxt_k; iss_v = nxt_v;
        iss_ragged = ragged_sample && nxt_j == last_step;
        iss_lds = lds0 + iss_stage * STAGE;
        iss_stage = iss_stage == NST - 1 ? 0 : iss_stage + 1;
        const bool more = nxt_j + 1 < nsteps;
        const int64_t adv = more ? step_bytes : 0;
        nxt_k += adv; nxt_v += adv;
        nxt_j += more ? 1 : 0;
    };
    auto issue_all = [&]() {
        begin_issue();
        dma.issue_tile(iss_k, iss_ragged, iss_lds, w);
        dma.issue_tile(iss_v, iss_ragged, iss_lds + C::TILE, w);
    };

    int aaddr[C::KS], taddr[C::DB][2];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) aaddr[ks] = LT::off(ln, 2 * ks + hh);
#pragma unroll
    for (int db = 0; db < C::DB; ++db) {
        taddr[db][0] = LT::tr_off(l, 0, db);
        taddr[db][1] = LT::tr_off(l, 8, db);
    }

    issue_all();
    issue_all();
    issue_all();
    bf16x8 qf[C::KS], dof[C::KS];
    float lse2 = 0.f, ndelta = 0.f;  // ndelta = -Delta
    {
        const size_t off = ((size_t)(sb + (qvalid ? qrow : 0)) * Hq + h) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 z = {};
            qf[ks] = qvalid ? *(const bf16x8*)(Q + off + 16 * ks) : z;
            dof[ks] = qvalid ? *(const bf16x8*)(dO + off + 16 * ks) : z;
        }
        // Row statistics of this lane's row: Delta = sum_d dO * O (each half of the wave sums its 8 of
        // every 16 columns), and the saved LSE in base 2.  Written out for the dK/dV kernel.
        float part = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 z = {};
            const bf16x8 of = qvalid ? *(const bf16x8*)(O + off + 16 * ks) : z;
#pragma unroll
            for (int e = 0; e < 8; ++e) part = __builtin_fmaf((float)dof[ks][e], (float)of[e], part);
        }
        ndelta = -xhalf_sum(part);
        if (qvalid) {
            lse2 = LSE[(size_t)h * T + sb + qrow] * kLog2e;
            if (hh == 0) stats[(size_t)h * T + sb + qrow] = make_float2(lse2, ndelta);
        }
    }
    wait_vmcnt<0>();
    wg_barrier();
    if constexpr (D > 80) {  // one wave per SIMD: see park_in_acc_registers
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) { park_in_acc_registers(qf[ks]); park_in_acc_registers(dof[ks]); }
    }

    f32x16 dqacc[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dqacc[db][r] = 0.f;
    const float c2 = scale * kLog2e;
    // causal: only a sample's first rows hold few terms, and only those need dS as bf16 hi + lo
    const bool lo_steps = !CAUSAL || q0 == 0;

    // Stage protocol as in the dK/dV kernel: step i lives in stage i % 4; the sync at the start of a step
    // waits until step i + 1 has landed (step i + 2 may stay in flight) and passes the barrier, after
    // which every wave is done with step i - 1, whose stage this step's loads refill.
    int stage_i = 0;
    int j = 0;
    f32x16 nd16, zero16;  // -Delta of this lane's row as the starting value of dP; 0 for S
#pragma unroll
    for (int r = 0; r < 16; ++r) { nd16[r] = ndelta; zero16[r] = 0.f; }
    DqOpsA<D> fa;  // K rows for S, then V rows for dP
    DqOpsA<D> fv;
    DqOpsT<D> ft;
    f32x16 s[2], dp[2];
    dq_load_A<D>(lds + stage_i * STAGE, aaddr, fa);
    // One key step in phases.  Masked steps (the causal diagonal, the sample's end) zero P outside the
    // mask; fully masked waves run them all the same, they would only wait at the next barrier.
    auto step = [&](auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        wait_vmcnt<PER>();
        wg_barrier();
        const unsigned char* cur = lds + stage_i * STAGE;
        const unsigned char* nxt = lds + (stage_i == NST - 1 ? 0 : stage_i + 1) * STAGE;
        // S^T = K Q^T; meanwhile fetch the V rows and do the scalar bookkeeping of this step's loads
        dq_load_A<D>(cur + C::TILE, aaddr, fv);
        dq_run_A<D>(fa, qf, zero16, s);
        begin_issue();
        __builtin_amdgcn_sched_barrier(0);
        dma.issue_tile(iss_k, iss_ragged, iss_lds, w);
        // dP^T = V dO^T - Delta with P = exp2(c2 S - lse2) in its shadow; meanwhile fetch K^T
        dq_load_T<D>(cur, taddr, ft);
        dq_run_A<D>(fv, dof, nd16, dp);
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float p = fast_exp2(__builtin_fmaf(s[b][r], c2, -lse2));
                if (MASKED) {
                    const int kv = j * BWD_STEP_KV + 32 * b + 8 * (r / 4) + 4 * hh + (r % 4);
                    const bool ok = kv < L && qrow < L && (!CAUSAL || kv <= qrow);
                    p = ok ? p : 0.f;
                }
                s[b][r] = p;
            }
        dkdv_interleave<2 * C::KS, 4 * C::DB / C::KS, 8>();
        __builtin_amdgcn_sched_barrier(0);
        dma.issue_tile(iss_v, iss_ragged, iss_lds + C::TILE, w);
        // dQ^T += K^T dS^T with dS = P (dP - Delta) in its shadow; meanwhile fetch the next step's K rows
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
#pragma unroll
                for (int e = 0; e < 8; ++e) dp[b][8 * st + e] *= s[b][8 * st + e];
                const bf16x8 dsb = pack_regs(dp[b], st);
#pragma unroll
                for (int db = 0; db < C::DB; ++db) dqacc[db] = mfma32(ft.a[b][st][db], dsb, dqacc[db]);
            }
        dq_load_A<D>(nxt, aaddr, fa);
        dkdv_interleave<4 * C::DB, 2 * C::KS / (4 * C::DB) + 1, 6>();
        __builtin_amdgcn_sched_barrier(0);
        if (MASKED && lo_steps) {  // the lo parts of dS, on the K^T operands still in registers
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    const bf16x8 dsl = pack_regs_lo(dp[b], st, pack_regs(dp[b], st));
#pragma unroll
                    for (int db = 0; db < C::DB; ++db) dqacc[db] = mfma32(ft.a[b][st][db], dsl, dqacc[db]);
                }
        }
        stage_i = stage_i == NST - 1 ? 0 : stage_i + 1;
    };
    for (; j < n_plain; ++j) step(std::false_type{});
    if constexpr (CAUSAL) {
        for (; j < nsteps; ++j) step(std::true_type{});
    } else {
        // Without the causal mask the only masked step is the one holding the sample's end: it takes the
        // simple form (the phased one with hi + lo in every such step needs more registers than there are).
        // Its sync sits at its end: the step's own stage was published by the sync before.
        for (; j < nsteps; ++j) {
            dq_end_step<D>(lds + stage_i * STAGE, lds + stage_i * STAGE + C::TILE, aaddr, taddr, qf, dof,
                           dqacc, c2, lse2, ndelta, j * BWD_STEP_KV, qrow, L, hh);
            wait_vmcnt<PER>();
            wg_barrier();
            issue_all();
            stage_i = stage_i == NST - 1 ? 0 : stage_i + 1;
        }
    }
    wait_vmcnt<0>();  // the surplus loads issued near the end must land before this LDS is given away

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
    wg_clock.end(clock_probe);
}

// ------------------------------------------------------------------------------------------------
// dQ with the operands read right before their MFMAs: the dQ kernel of head_dim 64, 96 and 128.
//
// dq_kernel above keeps three sets of operands in flight (its phases) and four LDS stages.  At head_dim 96 and
// 128 that takes 400 registers and 128 KB: one workgroup per CU, whose start (Q, dO, O, LSE, three stages of
// K/V, all waited for) and end (stores) then run with nothing beside them; a query tile under the causal mask
// has only (q0 + 128) / 64 key steps to spread that over: measured, the fixed cost of an item was about 8 of
// its steps, and the matrix pipes were 41 % busy on the LLM batch against 60 % elsewhere.
// This form keeps 32 keys of S and dP live at a time, double-buffers K/V in two LDS stages and fits 256
// registers at head_dim 128 (150 at 64), so two (three at 64) workgroups share a CU and one's start and end
// hide behind the others' steps.  Same arithmetic per element as dq_kernel (P, dP - Delta, dS rounded to
// bf16, hi + lo where rows can have few keys).  Measured against dq_kernel:
//   head_dim 128: the LLM batch's dQ 2.23 -> 1.79 ms, 16384-token causal samples 6.33 -> 5.33 ms, the same
//     without the mask 5.73 -> 5.24 ms, 512-token causal samples 0.63 -> 0.44 ms; head_dim 96: 20-26 % faster;
//   head_dim 64: the ViT batch's dQ 3.89 -> 3.81 ms, batches of 64..1024-token samples 9-15 % faster;
//   head_dim 80: slower (32.6 against 30.6 ms on the long/short mix; its 20 KB tiles and three partly masked
//     loads per tile leave it short of registers at three workgroups per CU), so head_dim 80 keeps dq_kernel.
// (The operands that only the matrix cores touch are left to the compiler here: parked in the accumulation
// half they pin 128 of the 256 registers there and the vector half spills.)
// ------------------------------------------------------------------------------------------------
template <int D, bool CAUSAL, bool MASKED>
__device__ __forceinline__ void dq_plain_step(const unsigned char* kt, const unsigned char* vt,
                                              const int (&aaddr)[BwdCfg<D>::KS], const int (&taddr)[BwdCfg<D>::DB][2],
                                              const bf16x8 (&qf)[BwdCfg<D>::KS], const bf16x8 (&dof)[BwdCfg<D>::KS],
                                              f32x16 (&dqacc)[BwdCfg<D>::DB], float c2, float lse2,
                                              const f32x16& ndelta16, int kv0, int qrow, int L, int hh, bool lo) {
    using C = BwdCfg<D>;
    constexpr int ROWB = C::T::ROWB;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        if (b) __builtin_amdgcn_sched_barrier(0);  // keep the second block's operand reads behind the first block
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 ak = *(const bf16x8*)(kt + aaddr[ks] + b * 32 * ROWB);
            s = mfma32(ak, qf[ks], s);
            bf16x8 av = *(const bf16x8*)(vt + aaddr[ks] + b * 32 * ROWB);
            // -Delta is where the dP accumulation starts: a 16-register constant read as the first MFMA's addend
            dp = mfma32(av, dof[ks], ks == 0 ? ndelta16 : dp);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p = fast_exp2(__builtin_fmaf(s[r], c2, -lse2));
            if (MASKED) {
                const int kv = kv0 + 32 * b + 8 * (r / 4) + 4 * hh + (r % 4);
                const bool ok = kv < L && qrow < L && (!CAUSAL || kv <= qrow);
                p = ok ? p : 0.f;
            }
            dp[r] *= p;
        }
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const bf16x8 dsb = pack_regs(dp, st);
            const int rowoff = (32 * b + 16 * st) * ROWB;
#pragma unroll
            for (int db = 0; db < C::DB; ++db) {
                bf16x8 ak = cat4(lds_read_tr(kt + rowoff + taddr[db][0]), lds_read_tr(kt + rowoff + taddr[db][1]));
                dqacc[db] = mfma32(ak, dsb, dqacc[db]);
            }
        }
        if (MASKED && lo) {  // wave-uniform: the lo parts of dS, in a pass of their own (as in dq_kernel)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const bf16x8 dsl = pack_regs_lo(dp, st, pack_regs(dp, st));
                const int rowoff = (32 * b + 16 * st) * ROWB;
#pragma unroll
                for (int db = 0; db < C::DB; ++db) {
                    bf16x8 ak = cat4(lds_read_tr(kt + rowoff + taddr[db][0]), lds_read_tr(kt + rowoff + taddr[db][1]));
                    dqacc[db] = mfma32(ak, dsl, dqacc[db]);
                }
            }
        }
    }
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, (D <= 80 ? 3 : 2))
dq_kernel_direct(const __bf16* __restrict__ Q, const __bf16* __restrict__ K, const __bf16* __restrict__ V,
              const __bf16* __restrict__ dO, const __bf16* __restrict__ O, const float* __restrict__ LSE,
              float2* __restrict__ stats, __bf16* __restrict__ dQ, const int32_t* __restrict__ hdr,
              const WorkItem* __restrict__ items, int max_items, int T, int Hq, int Hkv, float scale,
              unsigned long long* __restrict__ clock_probe) {
    using C = BwdCfg<D>;
    using LT = LdsTile<D>;
    constexpr int STAGE = 2 * C::TILE;  // K tile, V tile
    // two LDS stages: step j + 1 loads while step j computes (a third stage, tried at head_dim 64, was slower:
    // 16 more registers for nothing that the other workgroups on the CU do not already cover)
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * STAGE];

    int item, hp;
    xcd_item_head(blockIdx.x, max_items, Hq, Hkv, hdr[1], item, hp);
    item = __builtin_amdgcn_readfirstlane(item); hp = __builtin_amdgcn_readfirstlane(hp);
    if (item >= hdr[0]) return;
    ClockProbe wg_clock;
    wg_clock.begin(clock_probe);
    const int kvh = hp % Hkv;
    const int h = kvh * (Hq / Hkv) + hp / Hkv;
    const WorkItem it = items[item];
    const int sb = __builtin_amdgcn_readfirstlane(it.y), L = __builtin_amdgcn_readfirstlane(it.z - it.y),
              q0 = __builtin_amdgcn_readfirstlane(it.x - it.y);
    const int tid = threadIdx.x, w = uniform_wave_id(), l = tid & 63, ln = l & 31, hh = l >> 5;
    const int qrow = q0 + 32 * w + ln;
    const bool qvalid = qrow < L;

    const int kv_end = CAUSAL ? min(L, q0 + BWD_TILE_Q) : L;
    const int nsteps = (kv_end + BWD_STEP_KV - 1) / BWD_STEP_KV;
    const int n_plain = CAUSAL ? min(L, q0 + 1) / BWD_STEP_KV : L / BWD_STEP_KV;
    const unsigned char* kbase = (const unsigned char*)(K + ((size_t)sb * Hkv + kvh) * D);
    const unsigned char* vbase = (const unsigned char*)(V + ((size_t)sb * Hkv + kvh) * D);
    const uint32_t row_bytes = (uint32_t)Hkv * D * 2;
    TileDma<D, 64> dma;
    dma.init(row_bytes, L, w, l);
    const uint32_t lds0 = lds_address(lds);
    const int64_t step_bytes = (int64_t)BWD_STEP_KV * row_bytes;
    const bool ragged_sample = (L % BWD_STEP_KV) != 0;
    const int last_step = (L + BWD_STEP_KV - 1) / BWD_STEP_KV - 1;  // the one holding the sample's end
    // loads of step j into stage j % 2; a step past the item's last one is not loaded
    // (the ragged step in a branch of its own, with the flag a constant on either side: a select between the two
    // offset tables on a run-time flag makes the compiler index them through memory, and it then moves them into
    // LDS, at 32 bytes per lane: bank conflicts in every load that reads them)
    auto issue_step = [&](int j) {
        if (j < nsteps) {
            const uint32_t st = lds0 + (j & 1) * STAGE;
            if (ragged_sample && j == last_step) {
                dma.issue_tile(kbase + (size_t)j * step_bytes, true, st, w);
                dma.issue_tile(vbase + (size_t)j * step_bytes, true, st + C::TILE, w);
            } else {
                dma.issue_tile(kbase + (size_t)j * step_bytes, false, st, w);
                dma.issue_tile(vbase + (size_t)j * step_bytes, false, st + C::TILE, w);
            }
        }
    };
    int aaddr[C::KS], taddr[C::DB][2];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) aaddr[ks] = LT::off(ln, 2 * ks + hh);
#pragma unroll
    for (int db = 0; db < C::DB; ++db) {
        taddr[db][0] = LT::tr_off(l, 0, db);
        taddr[db][1] = LT::tr_off(l, 8, db);
    }

    issue_step(0);
    bf16x8 qf[C::KS], dof[C::KS];
    float lse2 = 0.f, ndelta = 0.f;  // ndelta = -Delta
    {
        const size_t off = ((size_t)(sb + (qvalid ? qrow : 0)) * Hq + h) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 z = {};
            qf[ks] = qvalid ? *(const bf16x8*)(Q + off + 16 * ks) : z;
            dof[ks] = qvalid ? *(const bf16x8*)(dO + off + 16 * ks) : z;
        }
        // row statistics of this lane's row, as in dq_kernel (same order of operations)
        float part = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 z = {};
            const bf16x8 of = qvalid ? *(const bf16x8*)(O + off + 16 * ks) : z;
#pragma unroll
            for (int e = 0; e < 8; ++e) part = __builtin_fmaf((float)dof[ks][e], (float)of[e], part);
        }
        ndelta = -xhalf_sum(part);
        if (qvalid) {
            lse2 = LSE[(size_t)h * T + sb + qrow] * kLog2e;
            if (hh == 0) stats[(size_t)h * T + sb + qrow] = make_float2(lse2, ndelta);
        }
    }
    // (everything waited for here, once: see the forward kernel for why the register loads must not be left
    // pending at loop entry)
    wait_vmcnt<0>();

    f32x16 dqacc[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) dqacc[db][r] = 0.f;
    const float c2 = scale * kLog2e;
    // causal: only a sample's first rows hold few terms.  Without the mask every masked step (the one holding the
    // sample's end) carries lo parts; the flag is hidden from the compiler all the same, so that the lo pass stays
    // behind a branch of its own: folded into the step it costs the kernel 10 registers it does not have.
    f32x16 ndelta16;
#pragma unroll
    for (int r = 0; r < 16; ++r) ndelta16[r] = ndelta;
    asm volatile("" : "+v"(ndelta16));  // one set of registers for the whole kernel, not a refill per block
    int always = 1;
    asm volatile("" : "+s"(always));
    const bool lo_steps = CAUSAL ? q0 == 0 : always != 0;

    // Step j: its loads (issued during step j - 1) have landed; the barrier publishes them and tells that every
    // wave is done with step j - 1, whose stage the loads of step j + 1 may now overwrite.
    // PARITY: j % 2 where the caller knows it (-1 otherwise).  The mask-free loop runs two steps per iteration with
    // the stage a constant in each, so that the LDS addresses of the operand reads are the per-lane offsets plus an
    // immediate instead of one vector addition per address and step.
    auto step = [&](int j, auto masked_tag, auto parity_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        constexpr int PARITY = decltype(parity_tag)::value;
        wait_vmcnt<0>();
        wg_barrier();
        issue_step(j + 1);
        const unsigned char* st = lds + (PARITY >= 0 ? PARITY : (j & 1)) * STAGE;
        dq_plain_step<D, CAUSAL, MASKED>(st, st + C::TILE, aaddr, taddr, qf, dof, dqacc, c2, lse2, ndelta16,
                                         j * BWD_STEP_KV, qrow, L, hh, lo_steps);
    };
    using Unknown = std::integral_constant<int, -1>;
    int j = 0;
    for (; j + 1 < n_plain; j += 2) {
        step(j, std::false_type{}, std::integral_constant<int, 0>{});
        step(j + 1, std::false_type{}, std::integral_constant<int, 1>{});
    }
    for (; j < n_plain; ++j) step(j, std::false_type{}, Unknown{});
    for (; j < nsteps; ++j) step(j, std::true_type{}, Unknown{});
    wait_vmcnt<0>();

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
    wg_clock.end(clock_probe);
}

template <int D>
static hipError_t launch_dq_d(const BwdArgs& a, hipStream_t stream) {
    dim3 grid((unsigned)(a.max_items_q * a.num_q_heads)), block(256);
    auto q = (const __bf16*)a.q; auto k = (const __bf16*)a.k; auto v = (const __bf16*)a.v;
    auto dO = (const __bf16*)a.dout;
    auto o = (const __bf16*)a.o;
    auto st = (float2*)a.stats;
    if constexpr (D != 80) {  // (head_dim 80 keeps the phased dq_kernel: see dq_kernel_direct)
        if (a.causal)
            hipLaunchKernelGGL((dq_kernel_direct<D, true>), grid, block, 0, stream, q, k, v, dO, o, a.lse, st,
                               (__bf16*)a.dq, a.sched_hdr_q, a.items_q, (int)a.max_items_q, a.total_tokens,
                               a.num_q_heads, a.num_kv_heads, a.scale, a.clock_probe_dq);
        else
            hipLaunchKernelGGL((dq_kernel_direct<D, false>), grid, block, 0, stream, q, k, v, dO, o, a.lse, st,
                               (__bf16*)a.dq, a.sched_hdr_q, a.items_q, (int)a.max_items_q, a.total_tokens,
                               a.num_q_heads, a.num_kv_heads, a.scale, a.clock_probe_dq);
    } else {
        if (a.causal)
            hipLaunchKernelGGL((dq_kernel<D, true>), grid, block, 0, stream, q, k, v, dO, o, a.lse, st,
                               (__bf16*)a.dq, a.sched_hdr_q, a.items_q, (int)a.max_items_q, a.total_tokens,
                               a.num_q_heads, a.num_kv_heads, a.scale, a.clock_probe_dq);
        else
            hipLaunchKernelGGL((dq_kernel<D, false>), grid, block, 0, stream, q, k, v, dO, o, a.lse, st,
                               (__bf16*)a.dq, a.sched_hdr_q, a.items_q, (int)a.max_items_q, a.total_tokens,
                               a.num_q_heads, a.num_kv_heads, a.scale, a.clock_probe_dq);
    }
    return hipGetLastError();
}

#if VA_BWD_PART == 2
hipError_t launch_dq_128(const BwdArgs& a, hipStream_t stream) { return launch_dq_d<128>(a, stream); }
#elif VA_BWD_PART == 0
hipError_t launch_bwd_dq(const BwdArgs& a, hipStream_t stream) {
    switch (a.head_dim) {
        case 64: return launch_dq_d<64>(a, stream);
        case 80: return launch_dq_d<80>(a, stream);
        case 96: return launch_dq_d<96>(a, stream);
        case 128: return launch_dq_128(a, stream);
        default: return hipErrorInvalidValue;
    }
}
#endif

}  // namespace va
