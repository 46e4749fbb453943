// Forward kernel: one workgroup (4 waves) per (128-row query tile, query head).
//
// Orientation.  Each wave owns 32 query rows and computes the TRANSPOSED score tile
// S^T[kv][q] = K Q^T, so that in the MFMA result layout one lane holds one query column and 16
// key rows per 32-key block.  Row max and row sum of the softmax are then lane-local loops
// plus one exchange between the two wave halves, the running max and the rescale factor are
// per-lane scalars, and P^T (cast to bf16) already is the B operand of O^T = V^T P^T.  V^T is
// read from a row-major LDS tile with the transposing LDS read.
//
// Staging.  K and V tiles of 64 rows (32 at head_dim 128) go from HBM/L2 straight into LDS (direct-to-LDS loads, no
// registers in between).  K is triple-buffered and V double-buffered: while tile j is computed,
// V(j+1) and K(j+2) are in flight, which covers the L2/HBM latency that a one-tile-ahead register
// prefetch was measured to expose (about a third of the kernel time).
#include "va_device.h"
#include "va_internal.h"

namespace va {

template <int D>
struct FwdCfg {
    using T = LdsTile<D>;
    // Key tiles of 64 rows; 32 at head_dim 128, where the smaller tiles (and the 16 score registers they save)
    // are what lets three workgroups share a CU instead of two.
    static constexpr int BQ = FWD_TILE_Q, BKV = D == 128 ? 32 : FWD_TILE_KV;
    static constexpr int NB = BKV / 32;                // 32-key blocks of S^T per tile
    static constexpr int KS = D / 16;                  // 16-deep steps of QK^T
    static constexpr int DB = (D + 31) / 32;           // 32-wide blocks of O^T rows
    static constexpr int TILE = BKV * T::ROWB;         // bytes of one K or V tile in LDS
    static constexpr int NI = TileDma<D, BKV>::NI;     // load instructions per wave per tile
};

// The running maximum m is only a reference point for the exponentials; it is moved (and O, l
// rescaled) only when some row of the wave would otherwise produce P above 2^kRescaleLog2.  After
// the first tiles of a sample that almost never happens, which saves the rescale multiplies.
constexpr float kRescaleLog2 = 8.0f;

// One key tile (FwdCfg<D>::BKV rows) for one wave: S^T = K Q^T, online softmax, O^T += V^T P^T.
// BOUNDARY tiles apply the sample-end / causal mask.  LO tiles also carry P as bf16 hi + lo: a
// sample's first 64 keys, when a mask falls into them, are where rows with only a handful of keys live
// (samples shorter than a tile, the first rows under the causal mask); their outputs are O(1), so a
// single bf16 rounding of P would eat most of the 1e-2 tolerance.  A row that reaches any other
// boundary tile sees at least 64 keys, and the rounding errors of its P average out.
// `issue` is called with slot numbers 0..3 spread over the step (FIRST_SLOT..3 only, for a caller that
// has already run the earlier ones): the caller hangs the tile loads of the iterations ahead on
// them, so that they trickle into the memory pipeline between the MFMAs instead of queueing up
// behind every other wave's right after the barrier.
template <int D, bool CAUSAL, bool BOUNDARY, int FIRST_SLOT = 0, bool LO = false, typename Issue>
__device__ __forceinline__ void tile_step(const unsigned char* kb, const unsigned char* vb,
                                          const int (&kaddr)[FwdCfg<D>::KS],
                                          const int (&vaddr)[FwdCfg<D>::DB][2],
                                          const bf16x8 (&qf)[FwdCfg<D>::KS],
                                          f32x16 (&oacc)[FwdCfg<D>::DB], float& m, float& lsum,
                                          float c2, int kv0, int L, int qrow, int hh, Issue& issue) {
    using C = FwdCfg<D>;
    constexpr int ROWB = C::T::ROWB;
    constexpr int NB = C::NB;
    f32x16 s[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 a = *(const bf16x8*)(kb + kaddr[ks] + b * 32 * ROWB);
            s[b] = mfma32(a, qf[ks], s[b]);
        }
        if (FIRST_SLOT <= b) issue(b);
    }
    if (NB == 1 && FIRST_SLOT <= 1) issue(1);
    bool ok[NB][16];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int kv = kv0 + 32 * b + 8 * (r / 4) + 4 * hh + (r % 4);
            ok[b][r] = !BOUNDARY || (kv < L && (!CAUSAL || kv <= qrow));
            if (!ok[b][r]) s[b][r] = kMaskedScore;
        }
    float mx = s[0][0];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[b][r]);
    mx = xhalf_max(mx);
    if (__builtin_amdgcn_ballot_w64((mx - m) * c2 > kRescaleLog2) != 0) {  // wave-uniform
        const float m_new = fmaxf(m, mx);
        const float alpha = fast_exp2((m - m_new) * c2);
        m = m_new;
        lsum *= alpha;
        // In-place multiplies (tied operands): written as plain C++ the compiler builds the scaled
        // accumulators in fresh registers and pays 2 x 16 x DB register copies in EVERY iteration to
        // merge the two paths, as much as rescaling unconditionally would cost.
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
            // (s_nop first: alpha comes straight out of v_exp_f32, and the hardware needs one idle
            // issue slot between a transcendental op and a consumer the compiler cannot see)
            asm volatile(
                "s_nop 1\n\t"
                "v_mul_f32 %0, %16, %0\n\tv_mul_f32 %1, %16, %1\n\tv_mul_f32 %2, %16, %2\n\tv_mul_f32 %3, %16, %3\n\t"
                "v_mul_f32 %4, %16, %4\n\tv_mul_f32 %5, %16, %5\n\tv_mul_f32 %6, %16, %6\n\tv_mul_f32 %7, %16, %7\n\t"
                "v_mul_f32 %8, %16, %8\n\tv_mul_f32 %9, %16, %9\n\tv_mul_f32 %10, %16, %10\n\tv_mul_f32 %11, %16, %11\n\t"
                "v_mul_f32 %12, %16, %12\n\tv_mul_f32 %13, %16, %13\n\tv_mul_f32 %14, %16, %14\n\tv_mul_f32 %15, %16, %15"
                : "+v"(oacc[db][0]), "+v"(oacc[db][1]), "+v"(oacc[db][2]), "+v"(oacc[db][3]), "+v"(oacc[db][4]),
                  "+v"(oacc[db][5]), "+v"(oacc[db][6]), "+v"(oacc[db][7]), "+v"(oacc[db][8]), "+v"(oacc[db][9]),
                  "+v"(oacc[db][10]), "+v"(oacc[db][11]), "+v"(oacc[db][12]), "+v"(oacc[db][13]),
                  "+v"(oacc[db][14]), "+v"(oacc[db][15])
                : "v"(alpha));
    }
    const float mc = m * c2;
    float rs = 0.f;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float p = fast_exp2(__builtin_fmaf(s[b][r], c2, -mc));
            p = ok[b][r] ? p : 0.f;
            rs += p;
            s[b][r] = p;
        }
    lsum += rs;

    bf16x8 pb[NB][2], plo[NB][2];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            pb[b][st] = pack8(s[b][8 * st + 0], s[b][8 * st + 1], s[b][8 * st + 2], s[b][8 * st + 3],
                              s[b][8 * st + 4], s[b][8 * st + 5], s[b][8 * st + 6], s[b][8 * st + 7]);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                plo[b][st][e] = LO ? (__bf16)(s[b][8 * st + e] - (float)pb[b][st][e]) : (__bf16)0.f;
        }
    issue(2);
#pragma unroll
    for (int db = 0; db < C::DB; ++db) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const unsigned char* p0 = vb + (32 * b + 16 * st) * ROWB;
                bf16x8 a = cat4(lds_read_tr(p0 + vaddr[db][0]), lds_read_tr(p0 + vaddr[db][1]));
                oacc[db] = mfma32(a, pb[b][st], oacc[db]);
                if (LO) oacc[db] = mfma32(a, plo[b][st], oacc[db]);
            }
        if (db == 0) issue(3);
    }
}

// A mask-free tile taken on trust: the reference maximum m is NOT looked at, P = exp2(c2 (S - m)) is
// formed directly and only the row sums are checked afterwards.  m is merely a reference point, so
// any P below kTrustLimit is as good as one below 1 (fp32 and bf16 share their exponent range); once
// the first tile of a sample has set m, later tiles essentially never exceed it by 2^30.  If some
// row of the wave does (or overflows to infinity), nothing has been accumulated yet: the function
// returns false and the caller repeats the tile with tile_step, which moves m.  This removes the
// maximum search (one instruction per two scores) from the common path.
constexpr float kTrustLimit = 1073741824.0f;  // 2^30
// (slots 0 and 1 of `issue` have run when it returns false, all four when it returns true)
template <int D, typename Issue>
__device__ __forceinline__ bool tile_step_trusting(const unsigned char* kb, const unsigned char* vb,
                                                   const int (&kaddr)[FwdCfg<D>::KS],
                                                   const int (&vaddr)[FwdCfg<D>::DB][2],
                                                   const bf16x8 (&qf)[FwdCfg<D>::KS],
                                                   f32x16 (&oacc)[FwdCfg<D>::DB], float m, float& lsum, float c2,
                                                   Issue& issue) {
    using C = FwdCfg<D>;
    constexpr int ROWB = C::T::ROWB;
    constexpr int NB = C::NB;
    f32x16 s[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 a = *(const bf16x8*)(kb + kaddr[ks] + b * 32 * ROWB);
            s[b] = mfma32(a, qf[ks], s[b]);
        }
        issue(b);
    }
    if (NB == 1) issue(1);
    const float mc = m * c2;
    float rs = 0.f;
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            s[b][r] = fast_exp2(__builtin_fmaf(s[b][r], c2, -mc));
            rs += s[b][r];
        }
    if (__builtin_amdgcn_ballot_w64(!(rs <= kTrustLimit)) != 0) return false;  // wave-uniform, rare
    lsum += rs;
    issue(2);
#pragma unroll
    for (int db = 0; db < C::DB; ++db) {
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const bf16x8 pb = pack8(s[b][8 * st + 0], s[b][8 * st + 1], s[b][8 * st + 2], s[b][8 * st + 3],
                                        s[b][8 * st + 4], s[b][8 * st + 5], s[b][8 * st + 6], s[b][8 * st + 7]);
                const unsigned char* p0 = vb + (32 * b + 16 * st) * ROWB;
                bf16x8 a = cat4(lds_read_tr(p0 + vaddr[db][0]), lds_read_tr(p0 + vaddr[db][1]));
                oacc[db] = mfma32(a, pb, oacc[db]);
            }
        if (db == 0) issue(3);
    }
    return true;
}

// Workgroups per CU the kernel is compiled for (registers) and its LDS allows.  At head_dim 64 the general
// form fits four (126 registers, 40 KB) and needs them: held to three by LDS padding it measured 12 % slower on
// 8192-token samples, to two 18 %.  The lean form is compiled for three: under the causal mask it takes 149 registers
// and spills at 128.
template <int D, bool CAUSAL>
constexpr int kFwdWgsPerCu = D == 64 ? 4 : (D <= 80 || D == 128) ? 3 : 2;
template <int D>
constexpr int kFwdLeanWgsPerCu = (D <= 80 || D == 128) ? 3 : 2;

// One work item: the query tile `wid` names (see xcd_item_head), all its key tiles.  `lds` is the workgroup's
// staging memory, 5 tiles (K x3, then V x2).
// LEAN (batches of short samples): loads past the item's last tile are not issued.  The general form
// issues them regardless (they re-fetch the last tile into a free slot), which keeps its loop free of
// branches and its wait counts constant; an item of one or two tiles, though, then waits for two more
// memory round trips than it has use for, and in that regime the round trips are all there is.
template <int D, bool CAUSAL, bool LEAN = false>
__device__ __forceinline__ void fwd_work_item(unsigned wid, unsigned char* lds, const __bf16* __restrict__ Q,
                                              const __bf16* __restrict__ K, const __bf16* __restrict__ V,
                                              __bf16* __restrict__ O, float* __restrict__ LSE,
                                              const int32_t* __restrict__ hdr, const WorkItem* __restrict__ items,
                                              int max_items, int T, int Hq, int Hkv, float scale, int S,
                                              float* __restrict__ part_o, float* __restrict__ part_lse,
                                              unsigned long long* __restrict__ clock_probe) {
    using C = FwdCfg<D>;
    using LT = LdsTile<D>;

    // S > 1: the key tiles of every query tile are split into S consecutive chunks, one workgroup
    // each, which write partial results (fp32 O and LSE per chunk) that a merge kernel combines.  Used
    // for launches too small to fill the chip (few heads, one mid-length sample).
    const int ch = S > 1 ? (int)(wid % S) : 0;
    const unsigned bid = S > 1 ? wid / S : wid;
    int item, hp;
    // (LEAN: always the item-major order, which is what the scheduler picks for short samples anyway; not
    // reading it from the header lets the work item's own load start at once, next to the header's)
    xcd_item_head(bid, max_items, Hq, Hkv, LEAN ? 1 : hdr[1], item, hp);
    // (integer division runs on the vector ALU; make the results scalar again, so that what is derived
    // from them stays in scalar registers)
    item = __builtin_amdgcn_readfirstlane(item); hp = __builtin_amdgcn_readfirstlane(hp);
    if (!LEAN && item >= hdr[0]) return;
    ClockProbe wg_clock;
    wg_clock.begin(clock_probe);
    // Head slots count the kv heads first, so that (with Hkv a multiple of the 8 XCDs) every XCD's L2
    // only ever sees its own kv heads.
    const int kvh = hp % Hkv;
    const int h = kvh * (Hq / Hkv) + hp / Hkv;
    // (LEAN: an entry past the live ones is inside the list's memory, whatever it holds; it is only looked at
    // after the check)
    const WorkItem it = items[item];
    if (LEAN && item >= hdr[0]) return;
    // same for the whole workgroup: tell the compiler, so that everything derived stays in SGPRs
    const int sb = __builtin_amdgcn_readfirstlane(it.y), L = __builtin_amdgcn_readfirstlane(it.z - it.y),
              q0 = __builtin_amdgcn_readfirstlane(it.x - it.y);  // q0: tile start inside the sample

    const int tid = threadIdx.x, w = uniform_wave_id(), l = tid & 63, ln = l & 31, hh = l >> 5;
    const int qrow = q0 + 32 * w + ln;  // this lane's query row inside the sample
    const bool qvalid = qrow < L;

    const int kv_end = CAUSAL ? min(L, q0 + C::BQ) : L;
    const int ntiles = (kv_end + C::BKV - 1) / C::BKV;
    // tiles [0, n_plain) need no mask in any wave: whole tiles below the sample end and, under the
    // causal mask, entirely at or below the tile's first query row
    // (rows that meet fewer than 64 keys before any mask do so in the first 64 / BKV tiles, which then all count
    // as masked tiles and carry P as hi + lo, whatever the tile size)
    const int keys_unmasked = CAUSAL ? min(L, q0 + 1) : L;
    const bool few_keys = keys_unmasked < 64;
    const int n_plain = few_keys ? 0 : keys_unmasked / C::BKV;
    const int n_lo = few_keys ? 64 / C::BKV : 0;
    const int jb = S > 1 ? ntiles * ch / S : 0, je = S > 1 ? ntiles * (ch + 1) / S : ntiles;  // this chunk's tiles
    if (jb >= je) {  // fewer tiles than chunks: an empty part (its O is never read)
        if (qvalid && hh == 0) part_lse[((size_t)ch * Hq + h) * T + sb + qrow] = -INFINITY;
        return;
    }

    const unsigned char* kbase = (const unsigned char*)(K + ((size_t)sb * Hkv + kvh) * D);
    const unsigned char* vbase = (const unsigned char*)(V + ((size_t)sb * Hkv + kvh) * D);
    const uint32_t row_bytes = (uint32_t)Hkv * D * 2;
    unsigned char* const kbuf = lds;
    unsigned char* const vbuf = lds + 3 * C::TILE;
    TileDma<D, C::BKV> dma;  // K and V share the offsets: same shape, same row pitch
    dma.init(row_bytes, L, w, l);
    const uint32_t lds0 = lds_address(lds);
    // Staging: K tiles run two iterations ahead in three LDS slots, V tiles one ahead in two.  The
    // pointers advance by additions; loads are issued unconditionally (past the last tile of this
    // workgroup the last one is fetched again, into a slot nobody reads any more), so that every
    // iteration has the same number of loads in flight and nothing branches around them.
    const int64_t tile_bytes = (int64_t)C::BKV * row_bytes;
    const bool ragged_sample = (L % C::BKV) != 0;
    const int last_tile = (L + C::BKV - 1) / C::BKV - 1;  // the tile holding the sample's end
    auto tile_ptr = [&](const unsigned char* base, int j) { return base + (size_t)min(j, je - 1) * tile_bytes; };
    auto load_tile = [&](const unsigned char* base, int j, uint32_t lds_tile) {
        dma.issue_tile(tile_ptr(base, j), ragged_sample && min(j, je - 1) == last_tile, lds_tile, w);
    };
    // per-lane LDS offsets: K rows read along the row (A operand of S^T), V read down the columns
    int kaddr[C::KS], vaddr[C::DB][2];
#pragma unroll
    for (int ks = 0; ks < C::KS; ++ks) kaddr[ks] = LT::off(ln, 2 * ks + hh);
#pragma unroll
    for (int db = 0; db < C::DB; ++db) {
        vaddr[db][0] = LT::tr_off(l, 0, db);
        vaddr[db][1] = LT::tr_off(l, 8, db);
    }

    f32x16 oacc[C::DB];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m = kMaskedScore, lsum = 0.f;
    const float c2 = scale * kLog2e;

    // prologue: K(0), V(0), K(1) and this lane's Q fragments.  Everything is waited for here, once:
    // the compiler cannot see the direct-to-LDS loads, and if the Q loads were still pending in its
    // bookkeeping at loop entry it would put a wait for ALL outstanding loads into every iteration.
    load_tile(kbase, jb, lds0);
    load_tile(vbase, jb, lds0 + 3 * C::TILE);
    if (!LEAN || jb + 1 < je) load_tile(kbase, jb + 1, lds0 + C::TILE);
    bf16x8 qf[C::KS];
    {
        const __bf16* qp = Q + ((size_t)(sb + (qvalid ? qrow : 0)) * Hq + h) * D + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            bf16x8 z = {};
            qf[ks] = qvalid ? *(const bf16x8*)(qp + 16 * ks) : z;
        }
    }
    wait_vmcnt<0>();
    wg_barrier();

    int kslot = 0;  // (j - jb) % 3
    int vslot = 0;  // (j - jb) % 2
    int j = jb;
    // Iteration j first fixes what it will load (V(j+1) into the other V slot, K(j+2) into the K slot
    // of tile j-1) and then lets the tile step issue those 2 NI loads in four portions, V first.
    const unsigned char *iss_v = nullptr, *iss_k = nullptr;
    uint32_t iss_v_lds = 0, iss_k_lds = 0;
    bool iss_v_ragged = false, iss_k_ragged = false;
    bool do_v = true, do_k = true;  // LEAN: whether tiles j + 1 and j + 2 exist (wave-uniform)
    auto issue = [&](int slot) {  // slot is a compile-time constant after inlining
        constexpr int NI = C::NI, HALF = (NI + 1) / 2;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            if (slot == (i < HALF ? 0 : 1) && (!LEAN || do_v)) dma.issue_one_rt(i, iss_v, iss_v_ragged, iss_v_lds, w);
            if (slot == (i < HALF ? 2 : 3) && (!LEAN || do_k)) dma.issue_one_rt(i, iss_k, iss_k_ragged, iss_k_lds, w);
        }
    };
#define VA_FWD_ITER_BEGIN()                                                                \
        const int kv0 = j * C::BKV;                                                            \
        iss_v = tile_ptr(vbase, j + 1);                                                        \
        iss_k = tile_ptr(kbase, j + 2);                                                        \
        iss_v_ragged = ragged_sample && min(j + 1, je - 1) == last_tile;                       \
        iss_k_ragged = ragged_sample && min(j + 2, je - 1) == last_tile;                       \
        iss_v_lds = lds0 + (3 + (vslot ^ 1)) * C::TILE;                                        \
        iss_k_lds = lds0 + (kslot == 0 ? 2 : kslot - 1) * C::TILE; /* slot (j + 2 - jb) % 3 */ \
        if (LEAN) { do_v = j + 1 < je; do_k = j + 2 < je; }                                    \
        const unsigned char* kb = kbuf + kslot * C::TILE;                                      \
        const unsigned char* vb = vbuf + vslot * C::TILE;
    // K(j+1) and V(j+1) must have landed; K(j+2), issued last, may stay in flight (LEAN: if it was issued).
#define VA_FWD_ITER_END()                                                                  \
        if (!LEAN || do_k) wait_vmcnt<C::NI>(); else wait_vmcnt<0>();                          \
        wg_barrier();                                                                          \
        kslot = kslot == 2 ? 0 : kslot + 1;                                                    \
        vslot ^= 1;

    // a sample's first keys behind a mask: rows with very few keys (hi + lo P)
    if constexpr (C::BKV == 64) {
        if (few_keys && j == 0) {
            VA_FWD_ITER_BEGIN()
            tile_step<D, CAUSAL, true, 0, true>(kb, vb, kaddr, vaddr, qf, oacc, m, lsum, c2, kv0, L, qrow, hh, issue);
            VA_FWD_ITER_END()
            ++j;
        }
    } else {
        for (; j < min(n_lo, je); ++j) {
            VA_FWD_ITER_BEGIN()
            tile_step<D, CAUSAL, true, 0, true>(kb, vb, kaddr, vaddr, qf, oacc, m, lsum, c2, kv0, L, qrow, hh, issue);
            VA_FWD_ITER_END()
        }
    }
    if (j < min(n_plain, je)) {  // the first mask-free tile sets the reference maximum
        VA_FWD_ITER_BEGIN()
        tile_step<D, CAUSAL, false>(kb, vb, kaddr, vaddr, qf, oacc, m, lsum, c2, kv0, L, qrow, hh, issue);
        VA_FWD_ITER_END()
        ++j;
    }
    for (; j < min(n_plain, je); ++j) {  // no masks, every wave active, maximum taken on trust
        VA_FWD_ITER_BEGIN()
        // (measured: worth 2 % at head_dim 64 and 80, where the vector ALU is the busier pipe, 1.5 % at 128)
        if (!tile_step_trusting<D>(kb, vb, kaddr, vaddr, qf, oacc, m, lsum, c2, issue))
            tile_step<D, CAUSAL, false, 2>(kb, vb, kaddr, vaddr, qf, oacc, m, lsum, c2, kv0, L, qrow, hh, issue);
        VA_FWD_ITER_END()
    }
    for (; j < je; ++j) {  // the sample's ragged last tile and the causal diagonal
        VA_FWD_ITER_BEGIN()
        // Every wave takes the masked variant here, also one whose rows see the whole tile or none of it
        // (causal: rows above the key tile; such a wave adds exact zeros).  A second variant in this loop
        // makes the compiler keep two sets of accumulator registers, and letting the idle wave skip the
        // step costs 30 to 60 registers for the branch around it (one workgroup per CU less at head_dim
        // 64): it has to wait at the barrier for the other waves anyway.
        tile_step<D, CAUSAL, true>(kb, vb, kaddr, vaddr, qf, oacc, m, lsum, c2, kv0, L, qrow, hh, issue);
        VA_FWD_ITER_END()
    }
    wait_vmcnt<0>();  // the surplus loads issued near the end must land before this LDS is given away
#undef VA_FWD_ITER_BEGIN
#undef VA_FWD_ITER_END

    // The row sum stays in fp32 on the vector ALU: summing the bf16-rounded P on the matrix cores
    // instead was measured to cost up to 1e-3 in LSE, the whole tolerance.
    const float ltot = xhalf_sum(lsum);
    // (a row can have met no key at all only in a chunk of a split launch: under the causal mask
    // the chunk may lie entirely beyond the row; its part is empty)
    const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
    const float row_lse = ltot > 0.f ? m * scale + __logf(ltot) : -INFINITY;
    if (qvalid) {
        if (S > 1) {
            float* op = part_o + (((size_t)ch * T + sb + qrow) * Hq + h) * D;
#pragma unroll
            for (int db = 0; db < C::DB; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    int d0 = 32 * db + 8 * r4 + 4 * hh;
                    if (d0 < D)
                        *(float4*)(op + d0) = make_float4(oacc[db][4 * r4 + 0] * inv, oacc[db][4 * r4 + 1] * inv,
                                                          oacc[db][4 * r4 + 2] * inv, oacc[db][4 * r4 + 3] * inv);
                }
            if (hh == 0) part_lse[((size_t)ch * Hq + h) * T + sb + qrow] = row_lse;
            wg_clock.end(clock_probe);
            return;
        }
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
        if (hh == 0) LSE[(size_t)h * T + sb + qrow] = row_lse;
    }
    wg_clock.end(clock_probe);
}

template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, (kFwdWgsPerCu<D, CAUSAL>))
fwd_kernel(const __bf16* __restrict__ Q, const __bf16* __restrict__ K, const __bf16* __restrict__ V,
           __bf16* __restrict__ O, float* __restrict__ LSE, const int32_t* __restrict__ hdr,
           const WorkItem* __restrict__ items, int max_items, int T, int Hq, int Hkv, float scale, int S,
           float* __restrict__ part_o, float* __restrict__ part_lse, unsigned long long* __restrict__ clock_probe) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[5 * FwdCfg<D>::TILE];  // K x3, then V x2
    fwd_work_item<D, CAUSAL>(blockIdx.x, lds, Q, K, V, O, LSE, hdr, items, max_items, T, Hq, Hkv, scale, S, part_o,
                             part_lse, clock_probe);
}

// The same for batches of short samples only (the caller's max_seqlen says so): the LEAN form of the work
// item.  There an item is one or two tile steps, a workgroup lives for a few microseconds, nearly all of it
// waiting for memory round trips one after the other (measured at 64-token samples: item record, first
// tiles, and two more for loads past the last tile), and the launch is bound by that chain and by the rate
// at which workgroups start, not by bandwidth or arithmetic.  (A variant that starts only as many workgroups
// as fit on the chip and lets each walk the list was measured slower than this one: the hardware handing the
// next item to whichever CU has room is worth more than the saved workgroup starts.)
template <int D, bool CAUSAL>
__global__ void __launch_bounds__(256, (kFwdLeanWgsPerCu<D>))
fwd_kernel_lean(const __bf16* __restrict__ Q, const __bf16* __restrict__ K, const __bf16* __restrict__ V,
                __bf16* __restrict__ O, float* __restrict__ LSE, const int32_t* __restrict__ hdr,
                const WorkItem* __restrict__ items, int max_items, int T, int Hq, int Hkv, float scale,
                unsigned long long* __restrict__ clock_probe) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[5 * FwdCfg<D>::TILE];
    fwd_work_item<D, CAUSAL, true>(blockIdx.x, lds, Q, K, V, O, LSE, hdr, items, max_items, T, Hq, Hkv, scale, 1,
                                   nullptr, nullptr, clock_probe);
}

template <int D>
static hipError_t launch_d(const FwdArgs& a, hipStream_t stream) {
    dim3 grid((unsigned)(a.max_items * a.num_q_heads * a.kv_splits)), block(256);
    auto q = (const __bf16*)a.q; auto k = (const __bf16*)a.k; auto v = (const __bf16*)a.v;
    if (a.lean) {  // batches of short samples (see fwd_kernel_lean); never with split keys
        if (a.causal)
            hipLaunchKernelGGL((fwd_kernel_lean<D, true>), grid, block, 0, stream, q, k, v, (__bf16*)a.o, a.lse,
                               a.sched_hdr, a.items, (int)a.max_items, a.total_tokens, a.num_q_heads, a.num_kv_heads,
                               a.scale, a.clock_probe);
        else
            hipLaunchKernelGGL((fwd_kernel_lean<D, false>), grid, block, 0, stream, q, k, v, (__bf16*)a.o, a.lse,
                               a.sched_hdr, a.items, (int)a.max_items, a.total_tokens, a.num_q_heads, a.num_kv_heads,
                               a.scale, a.clock_probe);
        return hipGetLastError();
    }
    if (a.causal)
        hipLaunchKernelGGL((fwd_kernel<D, true>), grid, block, 0, stream, q, k, v, (__bf16*)a.o, a.lse,
                           a.sched_hdr, a.items, (int)a.max_items, a.total_tokens, a.num_q_heads, a.num_kv_heads, a.scale,
                           a.kv_splits, a.part_o, a.part_lse, a.clock_probe);
    else
        hipLaunchKernelGGL((fwd_kernel<D, false>), grid, block, 0, stream, q, k, v, (__bf16*)a.o, a.lse,
                           a.sched_hdr, a.items, (int)a.max_items, a.total_tokens, a.num_q_heads, a.num_kv_heads, a.scale,
                           a.kv_splits, a.part_o, a.part_lse, a.clock_probe);
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
