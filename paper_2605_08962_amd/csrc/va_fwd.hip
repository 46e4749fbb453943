// Forward kernel: one workgroup (4 waves) per (128-row query tile, query head).
//
// Orientation.  Each wave owns 32 query rows and computes the TRANSPOSED score tile
// S^T[kv][q] = K Q^T, so that in the MFMA result layout one lane holds one query column and 16
// key rows per 32-key block.  Row max and row sum of the softmax are then lane-local loops
// plus one exchange between the two wave halves, the running max and the rescale factor are
// per-lane scalars, and P^T (cast to bf16) already is the B operand of O^T = V^T P^T.  V^T is
// read from a row-major LDS tile with the transposing LDS read.  K/V tiles of 64 rows are
// double-buffered in LDS; the next tile's global loads are in flight during the MFMAs.
#include "va_device.h"
#include "va_internal.h"

namespace va {

template <int D>
struct FwdCfg {
    static constexpr int BQ = FWD_TILE_Q, BKV = FWD_TILE_KV;
    static constexpr int KS = D / 16;                  // 16-deep steps of QK^T
    static constexpr int DB = (D + 31) / 32;           // 32-wide blocks of O^T rows
    static constexpr int KSTR = D * 2 + 16;            // LDS bytes per K row (odd multiple of 16)
    // LDS bytes per V row: smallest size >= DB*64 that is 32 mod 128, which measured fastest for
    // the transposing reads (rows 4 apart then start 32 banks apart)
    static constexpr int VSTR = (DB * 64 - 32 + 127) / 128 * 128 + 32;
    static constexpr int K_BYTES = BKV * KSTR, V_BYTES = BKV * VSTR;
    static constexpr int CHUNKS_PER_ROW = D / 8;       // 16-byte chunks
    static constexpr int CHUNKS = BKV * CHUNKS_PER_ROW;
    static constexpr int LOADS = (CHUNKS + 255) / 256;
};

// The running maximum m is only a reference point for the exponentials; it is moved (and O, l
// rescaled) only when some row of the wave would otherwise produce P above 2^kRescaleLog2.  After
// the first tiles of a sample that almost never happens, which saves the rescale multiplies.
constexpr float kRescaleLog2 = 8.0f;

// One 64-key tile for one wave: S^T = K Q^T, online softmax, O^T += V^T P^T.
// BOUNDARY tiles apply the sample-end / causal mask and carry P as bf16 hi + lo: they are where
// rows with only a handful of keys live (short samples, the first rows under the causal mask),
// whose outputs are O(1), so a single bf16 rounding of P would eat most of the 1e-2 tolerance.
template <int D, bool CAUSAL, bool BOUNDARY>
__device__ __forceinline__ void tile_step(const unsigned char* kb, const unsigned char* vb, int k_lane,
                                          int v_lane, const bf16x8 (&qf)[FwdCfg<D>::KS],
                                          f32x16 (&oacc)[FwdCfg<D>::DB], float& m, float& lsum,
                                          float c2, int kv0, int L, int qrow, int hh) {
    using C = FwdCfg<D>;
    f32x16 s[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 a = *(const bf16x8*)(kb + k_lane + b * 32 * C::KSTR + ks * 32);
            s[b] = mfma32(a, qf[ks], s[b]);
        }
    }
    bool ok[2][16];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int kv = kv0 + 32 * b + 8 * (r / 4) + 4 * hh + (r % 4);
            ok[b][r] = !BOUNDARY || (kv < L && (!CAUSAL || kv <= qrow));
            if (!ok[b][r]) s[b][r] = kMaskedScore;
        }
    float mx = s[0][0];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[b][r]);
    mx = xhalf_max(mx);
    if (__builtin_amdgcn_ballot_w64((mx - m) * c2 > kRescaleLog2) != 0) {  // wave-uniform
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2((m - m_new) * c2);
        m = m_new;
        lsum *= alpha;
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    const float mc = m * c2;
    float rs = 0.f;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p = fast_exp2(__builtin_fmaf(s[b][r], c2, -mc));
            p = ok[b][r] ? p : 0.f;
            rs += p;
            s[b][r] = p;
        }
    lsum += rs;

    bf16x8 pb[2][2], plo[2][2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            pb[b][st] = pack8(s[b][8 * st + 0], s[b][8 * st + 1], s[b][8 * st + 2], s[b][8 * st + 3],
                              s[b][8 * st + 4], s[b][8 * st + 5], s[b][8 * st + 6], s[b][8 * st + 7]);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                plo[b][st][e] = BOUNDARY ? (__bf16)(s[b][8 * st + e] - (float)pb[b][st][e]) : (__bf16)0.f;
        }
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const unsigned char* p0 = vb + v_lane + (32 * b + 16 * st) * C::VSTR + db * 64;
                bf16x8 a = cat4(lds_read_tr(p0), lds_read_tr(p0 + 8 * C::VSTR));
                oacc[db] = mfma32(a, pb[b][st], oacc[db]);
                if (BOUNDARY) oacc[db] = mfma32(a, plo[b][st], oacc[db]);
            }
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, 2)
fwd_kernel(const __bf16* __restrict__ Q, const __bf16* __restrict__ K, const __bf16* __restrict__ V,
           __bf16* __restrict__ O, float* __restrict__ LSE, const int32_t* __restrict__ hdr,
           const WorkItem* __restrict__ items, int T, int Hq, int Hkv, float scale) {
    using C = FwdCfg<D>;
    constexpr int BUF = C::K_BYTES + C::V_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF];

    const int item = blockIdx.x / Hq;
    if (item >= hdr[0]) return;
    // Heads: consecutive workgroups walk the kv heads first, so that (with Hkv a multiple of the
    // 8 XCDs) every XCD's L2 only ever sees its own kv heads.
    const int hp = blockIdx.x % Hq;
    const int kvh = hp % Hkv;
    const int h = kvh * (Hq / Hkv) + hp / Hkv;
    const WorkItem it = items[item];
    const int sb = it.y, L = it.z - it.y, q0 = it.x - it.y;  // q0: tile start inside the sample

    const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, ln = l & 31, hh = l >> 5;
    const int qrow = q0 + 32 * w + ln;  // this lane's query row inside the sample
    const bool qvalid = qrow < L;

    bf16x8 qf[C::KS];
    {
        const __bf16* qp = Q + ((size_t)(sb + (qvalid ? qrow : 0)) * Hq + h) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 z = {};
            qf[ks] = qvalid ? *(const bf16x8*)(qp + 16 * ks) : z;
        }
    }

    const int kv_end = CAUSAL ? min(L, q0 + C::BQ) : L;
    const int ntiles = (kv_end + C::BKV - 1) / C::BKV;
    // tiles [0, n_plain) need no mask in any wave: whole tiles below the sample end and, under the
    // causal mask, entirely at or below the tile's first query row
    const int n_plain = CAUSAL ? min(L, q0 + 1) / C::BKV : L / C::BKV;
    const int wq_lo = q0 + 32 * w, wq_hi = wq_lo + 31;  // this wave's query rows

    // staging: thread -> (row, 16-byte chunk) of the 64-row K and V tiles
    const __bf16* kbase = K + ((size_t)sb * Hkv + kvh) * D;
    const __bf16* vbase = V + ((size_t)sb * Hkv + kvh) * D;
    const size_t row_elems = (size_t)Hkv * D;
    u32x4 kreg[C::LOADS], vreg[C::LOADS];
    auto load_tile = [&](int kv0) {
#pragma unroll
        for (int i = 0; i < C::LOADS; ++i) {
            int c = tid + 256 * i;
            int r = c / C::CHUNKS_PER_ROW, cc = c % C::CHUNKS_PER_ROW;
            u32x4 z = {0, 0, 0, 0};
            kreg[i] = z;
            vreg[i] = z;
            if (c < C::CHUNKS && kv0 + r < L) {
                size_t off = (size_t)(kv0 + r) * row_elems + cc * 8;
                kreg[i] = *(const u32x4*)(kbase + off);
                vreg[i] = *(const u32x4*)(vbase + off);
            }
        }
    };
    auto store_tile = [&](int buf) {
        unsigned char* kb = lds + buf * BUF;
        unsigned char* vb = kb + C::K_BYTES;
#pragma unroll
        for (int i = 0; i < C::LOADS; ++i) {
            int c = tid + 256 * i;
            int r = c / C::CHUNKS_PER_ROW, cc = c % C::CHUNKS_PER_ROW;
            if (c < C::CHUNKS) {
                *(u32x4*)(kb + r * C::KSTR + cc * 16) = kreg[i];
                *(u32x4*)(vb + r * C::VSTR + cc * 16) = vreg[i];
            }
        }
    };
    f32x16 oacc[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m = kMaskedScore, lsum = 0.f;
    const float c2 = scale * kLog2e;

    const int k_lane = ln * C::KSTR + hh * 16;
    const int v_lane = tr_lane_offset(l, C::VSTR);

    load_tile(0);
    store_tile(0);
    __syncthreads();

    int j = 0;
    for (; j < n_plain; ++j) {  // no masks, every wave active: no branches around the tile step
        const bool more = j + 1 < ntiles;
        if (more) load_tile((j + 1) * C::BKV);
        const unsigned char* kb = lds + (j & 1) * BUF;
        tile_step<D, CAUSAL, false>(kb, kb + C::K_BYTES, k_lane, v_lane, qf, oacc, m, lsum, c2,
                                    j * C::BKV, L, qrow, hh);
        if (more) store_tile((j + 1) & 1);
        __syncthreads();
    }
    for (; j < ntiles; ++j) {  // the sample's ragged last tile and the causal diagonal
        const int kv0 = j * C::BKV;
        const bool more = j + 1 < ntiles;
        if (more) load_tile(kv0 + C::BKV);
        const unsigned char* kb = lds + (j & 1) * BUF;
        // causal: a wave whose rows all lie above this key tile has nothing to add
        if (!CAUSAL || kv0 <= wq_hi) {
            const bool boundary = (kv0 + C::BKV > L) || (CAUSAL && kv0 + C::BKV - 1 > wq_lo);
            if (boundary)
                tile_step<D, CAUSAL, true>(kb, kb + C::K_BYTES, k_lane, v_lane, qf, oacc, m, lsum, c2,
                                           kv0, L, qrow, hh);
            else
                tile_step<D, CAUSAL, false>(kb, kb + C::K_BYTES, k_lane, v_lane, qf, oacc, m, lsum, c2,
                                            kv0, L, qrow, hh);
        }
        if (more) store_tile((j + 1) & 1);
        __syncthreads();
    }

    // The row sum stays in fp32 on the vector ALU: summing the bf16-rounded P on the matrix cores
    // instead was measured to cost up to 1e-3 in LSE, the whole tolerance.
    const float ltot = xhalf_sum(lsum);
    const float inv = 1.f / ltot;
    if (qvalid) {
        __bf16* op = O + ((size_t)(sb + qrow) * Hq + h) * D;
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                int d0 = 32 * db + 8 * r4 + 4 * hh;
                if (d0 < D) {
                    bf16x4 o4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[db][4 * r4 + e] * inv);
                    *(bf16x4*)(op + d0) = o4;
                }
            }
        if (hh == 0) LSE[(size_t)h * T + sb + qrow] = m * scale + __logf(ltot);
    }
}

template <int D>
static hipError_t launch_d(const FwdArgs& a, hipStream_t stream) {
    dim3 grid((unsigned)(a.max_items * a.num_q_heads)), block(256);
    auto q = (const __bf16*)a.q; auto k = (const __bf16*)a.k; auto v = (const __bf16*)a.v;
    if (a.causal)
        hipLaunchKernelGGL((fwd_kernel<D, true>), grid, block, 0, stream, q, k, v, (__bf16*)a.o, a.lse,
                           a.sched_hdr, a.items, a.total_tokens, a.num_q_heads, a.num_kv_heads, a.scale);
    else
        hipLaunchKernelGGL((fwd_kernel<D, false>), grid, block, 0, stream, q, k, v, (__bf16*)a.o, a.lse,
                           a.sched_hdr, a.items, a.total_tokens, a.num_q_heads, a.num_kv_heads, a.scale);
    return hipGetLastError();
}

hipError_t launch_fwd(const FwdArgs& a, hipStream_t stream) {
    switch (a.head_dim) {
        case 64: return launch_d<64>(a, stream);
        case 80: return launch_d<80>(a, stream);
        case 96: return launch_d<96>(a, stream);
        case 128: return launch_d<128>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace va
