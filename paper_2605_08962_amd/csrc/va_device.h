// Device-side helpers for the gfx950 kernels: vector types, MFMA, LDS transposing reads,
// cross-half exchange.  Lane layouts used throughout (wave64, v_mfma_f32_32x32x16_bf16):
//   A operand: lane l holds A[m = l % 32][k = 8*(l/32) .. 8*(l/32)+7]
//   B operand: lane l holds B[k = 8*(l/32) .. +7][n = l % 32]
//   C/D      : lane l, register r holds C[m = 8*(r/4) + 4*(l/32) + r%4][n = l % 32]
// A C tile X[m][n] therefore already is the B operand of a product that contracts over m,
// provided the A operand enumerates k in the order  k(l/32, e) = 8*(e/4) + 4*(l/32) + e%4
// per 16-wide step (registers 0..7 = step 0, 8..15 = step 1).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace va {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define VA_LDS __attribute__((address_space(3)))

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// max / sum of x between lane l and lane l ^ 32 (v_permlane32_swap exchanges the upper half of
// its first operand with the lower half of its second).
__device__ __forceinline__ float xhalf_max(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// ds_read_b64_tr_b16: inside each group of 16 lanes, lane 4*k + j supplies the LDS address of
// elements [row k][cols 4j .. 4j+3] of a 4 x 16 block of 16-bit values; lane i receives
// [rows 0..3][col i].  Two of them give one 8-deep MFMA A operand of a row-major tile read
// "down the columns".
__device__ __forceinline__ bf16x4 lds_read_tr(const unsigned char* p) {
    s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 VA_LDS*)(p));
    return __builtin_bit_cast(bf16x4, r);
}
__device__ __forceinline__ bf16x8 cat4(bf16x4 a, bf16x4 b) {
    return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}
// Per-lane byte offset, inside a row-major LDS tile with `stride` bytes per row, of the address
// this lane supplies to lds_read_tr for the block whose origin is (row 0, col 0) for lanes 0..15,
// col 16 for lanes 16..31, and 4 rows further down for lanes 32..63.
__device__ __forceinline__ int tr_lane_offset(int lane, int stride) {
    return (4 * (lane >> 5) + ((lane & 15) >> 2)) * stride + (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
}

// ------------------------------------------------------------------------------------------------
// LDS tiles filled by direct-to-LDS loads (global_load_lds_dwordx4).
// (The layout functions are host-callable as well: a CPU test checks their bank properties.)
//
// Such a load writes the 64 lanes' 16-byte chunks to 1024 CONTIGUOUS LDS bytes, so rows cannot be
// padded against bank conflicts.  Instead the 16-byte chunks of a row are permuted: logical chunk c
// of row r lives in slot c ^ swz(r).  swz is chosen so that (a) 16 consecutive rows read at one
// logical chunk (MFMA A operand read along the row) and (b) 4 consecutive rows read over one
// 64-byte span (transposing read down the columns) both cover all 64 banks exactly once.
// Rows are 128 bytes for head_dim 64 and 256 bytes for 96 (4 slots unused) and 128; head_dim 80 has a
// packed layout of its own (LdsTile<80>).
// ------------------------------------------------------------------------------------------------
#define VA_GLOBAL __attribute__((address_space(1)))

template <int D>
struct LdsTile {
    static constexpr int ROWB = D <= 64 ? 128 : 256;  // bytes per row
    static constexpr int SLOTS = ROWB / 16;
    static constexpr int CHUNKS = D / 8;              // slots that hold data
    static constexpr int BLOCK_POS = 16 * SLOTS;      // 16-byte positions in a block of 16 rows
    __host__ __device__ __forceinline__ static constexpr int swz(int r) {
        if (ROWB == 256) return ((r & 3) << 2) | ((r >> 2) & 3);
        const int x = (r >> 1) & 7;
        return ((x & 1) << 2) | (x >> 1);
    }
    __host__ __device__ __forceinline__ static constexpr int off(int r, int c) { return r * ROWB + ((c ^ swz(r)) << 4); }
    // Byte offset this lane passes to lds_read_tr for the 4 x 16 block at rows row0.., columns
    // 32*db + (0 or 16).. of the tile; row0 must be a multiple of 8 (see tr_lane_offset).
    __host__ __device__ __forceinline__ static int tr_off(int lane, int row0, int db) {
        const int r = row0 + 4 * (lane >> 5) + ((lane & 15) >> 2);
        const int c = 4 * db + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
        return off(r, c) + 8 * (lane & 1);
    }
    // Which (row of the block, logical chunk) lives at 16-byte position p of a 16-row block; false
    // for a position that holds no data.  The inverse of off(), used to aim the direct-to-LDS loads.
    __host__ __device__ __forceinline__ static constexpr bool locate(int p, int& r, int& c) {
        r = p / SLOTS;
        c = (p % SLOTS) ^ swz(r);
        return CHUNKS == SLOTS || c < CHUNKS;
    }
};

// head_dim 80: 160-byte rows, stored without padding (a 64-row tile takes 10 KB instead of 16 KB, which
// is what lets three forward and two backward workgroups share a CU).  Ten chunks per row rule out an
// XOR swizzle, so each block of 16 rows (2560 bytes = 10 segments of 256 bytes = 16 positions) is laid
// out by hand.  With a = r / 4 and b = r % 4 inside the block, chunk c of row r sits in
//     segment 2a + c/4  (c < 8)   or   segment c  (c = 8, 9),     position 4b + (c + a) % 4.
// (a) For one c the 16 rows occupy 16 different positions, so a row-wise 16-byte read of 16 rows covers
// all 64 banks once.  (b) For one a (4 rows) and one group of 4 chunks the 16 (row, chunk) pairs do too,
// which is the footprint of half a transposing read.  (c) Chunks 0-3 and 4-7 of a row are adjacent in
// LDS (rotated), so four lanes of a load still fetch 64 contiguous bytes from memory.
template <>
struct LdsTile<80> {
    static constexpr int ROWB = 160;  // nominal: a block of 16 rows is 16 * ROWB bytes
    static constexpr int CHUNKS = 10;
    static constexpr int BLOCK_POS = 160;
    __host__ __device__ __forceinline__ static constexpr int pos(int r, int c) {  // r in [0, 16)
        const int a = r >> 2, b = r & 3;
        const int seg = c < 8 ? 2 * a + (c >> 2) : c;
        return 16 * seg + 4 * b + ((c + a) & 3);
    }
    __host__ __device__ __forceinline__ static constexpr int off(int r, int c) { return (r >> 4) * (16 * ROWB) + 16 * pos(r & 15, c); }
    // Columns 80..95 of the third 32-column block do not exist: the lanes that would address them
    // re-read chunks 8 and 9 (same addresses as their partner lanes; the results are never used).
    __host__ __device__ __forceinline__ static int tr_off(int lane, int row0, int db) {
        const int r = row0 + 4 * (lane >> 5) + ((lane & 15) >> 2);
        int c = 4 * db + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
        if (c >= CHUNKS) c -= 2;
        return off(r, c) + 8 * (lane & 1);
    }
    __host__ __device__ __forceinline__ static constexpr bool locate(int p, int& r, int& c) {
        const int seg = p >> 4, b = (p >> 2) & 3, e = p & 3;
        int a = 0;
        if (seg < 8) { a = seg >> 1; c = 4 * (seg & 1) + ((e - a) & 3); }
        else { c = seg; a = (e - c) & 3; }
        r = 4 * a + b;
        return true;
    }
};

// One direct-to-LDS load: every active lane fetches 16 bytes from base + its own byte offset; lane
// i's data lands at lds_addr + 16 * i (lds_addr is a wave-uniform LDS byte address and goes through
// M0; base is wave-uniform and stays in scalar registers).  Written as inline assembly on purpose: the compiler
// then does not see an LDS write in flight and so does not put a wait for ALL outstanding loads in
// front of every LDS read (which is what it does for the equivalent builtin, and which would
// serialise the prefetch with the compute).  The price is that completion must be waited for by
// hand (wait_vmcnt) before the barrier that publishes the tile.
// (readfirstlane of a value the compiler already knows to be uniform folds away; it is there for the
// cases it cannot prove, because an "s" operand must never be handed a vector register.  The statements
// name M0 as clobbered: they overwrite it, and the compiler may keep a value of its own there.)
__device__ __forceinline__ uint64_t uniform_u64(const void* p) {
    const uint64_t b = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ void dma16(const void* base, uint32_t byte_off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 : : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(byte_off), "s"(uniform_u64(base)) : "memory", "m0");
}
// The same load for the lanes named in `lanes` only (a wave-uniform bit mask).  The execution mask is
// narrowed inside the assembly statement and put back behind the load, so that the compiler sees no
// branch: an `if (lane is active)` around the load costs a saved-exec branch per load and, worse, cuts
// the loop body into basic blocks across which nothing is scheduled.  Must be reached by all 64 lanes.
__device__ __forceinline__ void dma16_lanes(const void* base, uint32_t byte_off, uint32_t lds_addr, uint64_t lanes) {
    uint64_t saved;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, %4\n\ts_mov_b32 m0, %1\n\t"
                 "global_load_lds_dwordx4 %2, %3\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved)
                 : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(byte_off), "s"(uniform_u64(base)),
                   "s"(lanes)
                 : "memory", "m0");
}
// Same with 4 bytes per lane: lane i's dword lands at lds_addr + 4 * i.
__device__ __forceinline__ void dma4(const void* base, uint32_t byte_off, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2"
                 : : "s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(byte_off), "s"(uniform_u64(base)) : "memory", "m0");
}
// LDS byte address (what M0 and ds instructions use) of a pointer into a __shared__ array.
__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(VA_LDS const unsigned char*)p;
}
// Gives the waves that share a SIMD different, fixed issue priorities (by the parity of their
// hardware wave slot).  Workgroups of equal work start together and, with equal priority, stay in
// lock-step: both waves of a SIMD want the matrix pipe at the same time, then the vector ALU at the
// same time, and each pipe idles while the other is fought over (measured: MFMA-busy + VALU-busy
// = 100 %, co-execution < 20 %).  With unequal priorities one wave runs unhindered and the other
// fills the gaps, so its MFMAs run under the first one's vector work and vice versa.
__device__ __forceinline__ void stagger_wave_priority() {
    const unsigned slot = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 4);  // HW_ID[3:0]: wave slot in the SIMD
    if (slot & 1) __builtin_amdgcn_s_setprio(2); else __builtin_amdgcn_s_setprio(0);
}

// Optional clock probe of a compute kernel: when `probe` is not null, every workgroup adds the time
// it was resident in ticks of the 100 MHz real-time counter to probe[0] and in shader cycles to
// probe[1].  Their ratio is the shader clock the kernel actually ran at (the chip lowers it under
// load).  Two scalar clock reads and, for one lane, two atomics per workgroup.
struct ClockProbe {
    unsigned long long rt0 = 0, cc0 = 0;
    __device__ __forceinline__ void begin(const unsigned long long* probe) {
        if (probe) { rt0 = __builtin_amdgcn_s_memrealtime(); cc0 = __builtin_readcyclecounter(); }
    }
    __device__ __forceinline__ void end(unsigned long long* probe) const {
        if (probe && threadIdx.x == 0) {
            atomicAdd(&probe[0], (unsigned long long)(__builtin_amdgcn_s_memrealtime() - rt0));
            atomicAdd(&probe[1], (unsigned long long)(__builtin_readcyclecounter() - cc0));
        }
    }
};

// Workgroup id -> (work item, head slot) for a launch of n_items x heads workgroups; head slot hp stands
// for kv head hp % kv_heads and member hp / kv_heads of its group of query heads.  Workgroup ids are
// dealt round-robin to the 8 XCDs, each with an L2 of its own.  With kv_heads a multiple of 8, XCD x
// gets the kv heads x, x + 8, ... and all their query heads.  It walks the (cost-sorted) work list in
// chunks of `chunk` items and finishes a chunk for one kv head (all query heads of the group side by
// side: they read the same K/V) before it takes the chunk for its next kv head.
//   chunk = kXcdChunk (long samples): the workgroups running together on an XCD stream the K/V (or
//     Q/dO) of ONE kv head where an item-major order interleaves all of the XCD's heads; the same bytes
//     serve more workgroups and stay in L2 for longer (HBM-side traffic of a 65536-token sample halved).
//   chunk = 1 (short samples only; item-major): the workgroups of all heads of an item run together and
//     read whole token rows of Q/K/V at once.  Nothing is re-read in this regime, and visiting every
//     DRAM row once instead of once per head of the XCD is worth 10 % at 128-token samples.  The head
//     slots are rotated by the item index there, so that an XCD reads every head in turn: with a fixed
//     pair of heads per XCD all its requests have the same two byte offsets inside the token rows, and the
//     memory side serves them 5-25 % slower (measured: 64-token samples at head_dim 64, forward 193 -> 155 us,
//     dQ 311 -> 237 us, dK/dV 339 -> 289 us; no difference in the chunked order, where L2 serves the reads).
// The scheduler kernel picks the chunk from the longest sample and leaves it in its header.
constexpr int kXcdChunk = 128;
constexpr int kXcdChunkMinLen = 1024;  // longest sample from which the chunked order is used
__host__ __device__ __forceinline__ void xcd_item_head(unsigned bid, int n_items, int heads, int kv_heads, int chunk,
                                                       int& item, int& hp) {
    if (kv_heads % 8 != 0) {
        item = (int)(bid / (unsigned)heads);
        hp = (int)(bid % (unsigned)heads);
        if (chunk == 1) hp = (int)((unsigned)(hp + item) % (unsigned)heads);  // (see chunk = 1 above)
        return;
    }
    const unsigned C = (unsigned)chunk;
    const unsigned g = (unsigned)(heads / kv_heads), kx = (unsigned)kv_heads / 8;
    const unsigned x = bid % 8, k = bid / 8;        // k-th workgroup of XCD x
    const unsigned full = (unsigned)n_items / C * C;  // items in whole chunks
    const unsigned per_chunk = C * g;                 // workgroups of one (chunk, kv head)
    unsigned kvslot, i, gq;
    if (k < full * g * kx) {
        const unsigned c = k / (per_chunk * kx), rem = k % (per_chunk * kx);
        kvslot = rem / per_chunk;
        i = c * C + (rem % per_chunk) / g;
        gq = rem % g;
    } else {
        const unsigned kk = k - full * g * kx, r = (unsigned)n_items - full;
        kvslot = kk / (r * g);
        i = full + (kk % (r * g)) / g;
        gq = kk % g;
    }
    item = (int)i;
    hp = (int)(x + 8 * kvslot + (unsigned)kv_heads * gq);
    if (C == 1) hp = (int)(((unsigned)hp + i) % (unsigned)heads);
}

// Index of this wave inside its workgroup, as a value the compiler knows to be wave-uniform.
__device__ __forceinline__ int uniform_wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// Per-lane source offsets of the direct-to-LDS loads that fill one LdsTile of ROWS rows of a
// [rows, heads, D] tensor, split over the 4 waves of the workgroup.  The offsets are relative to
// the tile's first row; they are computed once per kernel, so that issuing a tile costs no vector
// ALU work.  `last` holds the offsets for the sample's ragged last tile, where rows past the sample
// end re-read its last row (finite data that the caller masks).
// MASK_BY_BRANCH: partly active loads sit behind an `if (lane active)` instead of narrowing the execution
// mask in assembly.  The branch cuts the caller's loop body into blocks; one kernel (dQ at head_dim 80,
// at its register limit) is faster that way because the compiler then hoists less across the loads.
template <int D, int ROWS, bool MASK_BY_BRANCH = false>
struct TileDma {
    using T = LdsTile<D>;
    // 64-row tiles: one block of 16 rows per wave.  32-row tiles (head_dim 128 forward): 8 rows per wave, for the
    // layouts whose rows hold data in every slot.
    static_assert(ROWS == 64 || (ROWS == 32 && (D == 64 || D == 128)), "tile shape");
    static constexpr int RPW = ROWS / 4;                                            // rows per wave
    static constexpr int WAVE_POS = ROWS == 64 ? T::BLOCK_POS : RPW * (T::ROWB / 16);  // 16-byte positions per wave
    static constexpr int NI = (WAVE_POS + 63) / 64;      // load instructions per wave per tile
    static constexpr int WAVE_BYTES = RPW * T::ROWB;     // LDS bytes of one wave's rows
    uint32_t full[NI], last[NI];
    // lanes of load instruction i that hold data (a compile-time constant of the layout)
    __device__ __forceinline__ static constexpr uint64_t lane_mask(int i) {
        uint64_t m = 0;
        for (int lane = 0; lane < 64; ++lane) {
            const int p = 64 * i + lane;
            int r = 0, c = 0;
            if (ROWS == 32 ? p < WAVE_POS : (p < T::BLOCK_POS && T::locate(p, r, c))) m |= 1ull << lane;
        }
        return m;
    }
    struct LaneMasks { uint64_t m[NI]; };
    __device__ __forceinline__ static constexpr LaneMasks lane_masks() {
        LaneMasks k{};
        for (int i = 0; i < NI; ++i) k.m[i] = lane_mask(i);
        return k;
    }
    // load instruction i (known after unrolling) of a tile
    __device__ __forceinline__ static void load(int i, const unsigned char* src, uint32_t off, uint32_t lds_addr) {
        constexpr LaneMasks k = lane_masks();
        const uint64_t m = k.m[i];
        if (m == ~0ull) dma16(src, off, lds_addr);
        else if (!MASK_BY_BRANCH) dma16_lanes(src, off, lds_addr, m);
        else if ((m >> (threadIdx.x & 63)) & 1) dma16(src, off, lds_addr);
    }
    // row_bytes: bytes between consecutive rows of the tensor; L: rows in the sample
    __device__ __forceinline__ void init(uint32_t row_bytes, int L, int wave, int lane) {
        const int last_r0 = (L - 1) / ROWS * ROWS;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int p = 64 * i + lane;  // position inside this wave's block
            int r = 0, c = 0;
            if constexpr (ROWS == 64) {
                T::locate(p < T::BLOCK_POS ? p : 0, r, c);  // (a lane without data gets some valid offset; it never loads)
            } else {  // 8 rows per wave: the swizzle goes by the row inside the tile
                constexpr int SLOTS = T::ROWB / 16;
                r = (p < WAVE_POS ? p : 0) / SLOTS;
                c = ((p < WAVE_POS ? p : 0) % SLOTS) ^ T::swz(RPW * wave + r);
            }
            const int row = RPW * wave + r;
            full[i] = (uint32_t)row * row_bytes + c * 16;
            last[i] = (uint32_t)min(row, L - 1 - last_r0) * row_bytes + c * 16;
        }
    }
    // LDS byte address of load instruction i of `wave` in the tile at `tile`
    __device__ __forceinline__ static uint32_t dest(uint32_t tile, int wave, int i) {
        return tile + wave * WAVE_BYTES + i * 1024;
    }
    // base: first byte of the sample's row 0 at this head; r0: first row of the tile; tile: LDS byte
    // address of the tile; wave: uniform_wave_id()
    __device__ __forceinline__ void issue(const unsigned char* base, uint32_t row_bytes, int r0, int L,
                                          uint32_t tile, int wave) const {
        const unsigned char* src = base + (size_t)r0 * row_bytes;
        const bool ragged = r0 + ROWS > L;  // wave-uniform
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const uint32_t off = ragged ? last[i] : full[i];
            load(i, src, off, dest(tile, wave, i));
        }
    }
    // All loads of a tile whose first row's bytes at this head start at src.
    __device__ __forceinline__ void issue_tile(const unsigned char* src, bool ragged, uint32_t tile, int wave) const {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const uint32_t off = ragged ? last[i] : full[i];
            load(i, src, off, dest(tile, wave, i));
        }
    }
    // Load instruction i of a tile, i known after unrolling (same as issue_one<i>).
    __device__ __forceinline__ void issue_one_rt(int i, const unsigned char* src, bool ragged, uint32_t tile, int wave) const {
        const uint32_t off = ragged ? last[i] : full[i];
        load(i, src, off, dest(tile, wave, i));
    }
    // One of the NI load instructions of a tile: src = first byte of the tile's first row at this
    // head.  Lets a caller spread a tile's loads over its compute phases: a wave that issues them
    // back to back right after a barrier queues up behind every other wave doing the same and sits
    // in the issue stage for hundreds of cycles.
    template <int I>
    __device__ __forceinline__ void issue_one(const unsigned char* src, bool ragged, uint32_t tile, int wave) const {
        static_assert(I >= 0 && I < NI, "no such load");
        const uint32_t off = ragged ? last[I] : full[I];
        load(I, src, off, dest(tile, wave, I));
    }
};

// Wait until at most N of this wave's vector-memory loads (direct-to-LDS ones included) are still
// outstanding; LDS and scalar counters are left alone.
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// Workgroup barrier without the memory fence of __syncthreads (which would wait for every
// outstanding load, including the prefetches that are meant to stay in flight).
__device__ __forceinline__ void wg_barrier() {
    asm volatile("" ::: "memory");
    // this wave's own LDS reads must have returned before another wave may refill the tile
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0), vmcnt and expcnt untouched
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// Asks the instruction scheduler to lay out the current straight-line region as N_MFMA rounds of
// {2 LDS reads, 1 MFMA, 5 vector-ALU instructions}.  Used where a region holds matrix work and
// vector work that do not depend on each other (software-pipelined loops): left alone the
// scheduler emits them as two blocks and the wave leaves one pipe idle at a time.
template <int N_MFMA, int DS_AHEAD = 10, int DS_PER = 2, int VALU_PER = 5>
__device__ __forceinline__ void interleave_mfma_valu() {
    // LDS reads run DS_AHEAD instructions ahead of the MFMAs that consume them: an LDS read takes a
    // few hundred cycles to return, an MFMA issues every 32
    __builtin_amdgcn_sched_group_barrier(0x100, DS_AHEAD, 0);
#pragma unroll
    for (int i = 0; i < N_MFMA; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);         // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, DS_PER, 0);    // DS read
        __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER, 0);  // VALU
    }
}

// Moves a loop-invariant MFMA operand into the accumulation half of the register file.  A kernel that
// runs one wave per SIMD has 512 registers, but the vector ALU only reaches the 256 "architectural"
// ones; when those run short the compiler parks MFMA RESULTS in the other half and pays one copy
// instruction per register every time the vector ALU needs them (64 per step for S and dP).  The
// matrix instructions read their A/B operands from either half, so operands that only they touch
// are the right thing to keep there.
__device__ __forceinline__ void park_in_acc_registers(bf16x8& x) { asm volatile("" : "+a"(x)); }

// Forces x to be computed by this point of the program: without it the compiler sinks a value's
// whole computation into the later block that first uses it, i.e. out of the pipeline slot that was
// meant to overlap it with matrix work.
__device__ __forceinline__ void pin_here(bf16x8& x) { asm volatile("" : "+v"(x)); }

__device__ __forceinline__ bf16x8 pack8(float a0, float a1, float a2, float a3, float a4, float a5, float a6, float a7) {
    bf16x8 r;
    r[0] = (__bf16)a0; r[1] = (__bf16)a1; r[2] = (__bf16)a2; r[3] = (__bf16)a3;
    r[4] = (__bf16)a4; r[5] = (__bf16)a5; r[6] = (__bf16)a6; r[7] = (__bf16)a7;
    return r;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kMaskedScore = -1.0e30f;  // finite stand-in for -inf: keeps 0 * score finite

}  // namespace va
