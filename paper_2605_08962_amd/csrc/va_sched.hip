// Length-aware tile scheduler.
//
// The paper's motivation is the imbalance that mixed long and short samples cause (Section 2.2,
// Section 4.1.1) and it picks its attention algorithm for its work partitioning on long inputs
// (Section 6, "Efficient Operators").  On one GPU the same problem shows up inside a single
// launch: a 64k-token sample packed with hundreds of short ones.  This kernel turns cu_seqlens
// into a list of row tiles sorted by decreasing cost (the number of partner tiles a tile loops
// over), entirely on the device.  The compute kernels launch one workgroup per (list entry,
// head) in list order, so the hardware dispatcher hands out the heaviest tiles first and the
// light ones fill the tail (longest-processing-time-first list scheduling).
#include <vector>

#include "va_device.h"
#include "va_internal.h"

namespace va {

constexpr int SCHED_THREADS = 1024;

SchedLayout sched_layout(int64_t total_tokens, int64_t num_seqs, int tile_rows) {
    SchedLayout lay;
    lay.max_items = total_tokens / tile_rows + num_seqs;  // >= sum_s ceil(L_s / tile_rows)
    lay.tile_off_ofs = 16 * sizeof(int32_t);
    size_t p = lay.tile_off_ofs + (size_t)(num_seqs + 1) * sizeof(int32_t);
    lay.items_ofs = (p + 15) / 16 * 16;
    p = lay.items_ofs + (size_t)lay.max_items * sizeof(WorkItem);
    lay.end_ofs = (p + 255) / 256 * 256;
    return lay;
}

// Exclusive scan of one value per thread over the block; returns the exclusive prefix and
// writes the block total to *total.  `buf` holds SCHED_THREADS ints (the first 16 are used).
// Inside a wave the scan runs on lane shuffles; the 16 wave totals meet in LDS (two barriers in all, where a
// scan through LDS alone takes twenty: at a few thousand samples the scans were most of this kernel's time).
__device__ int block_exclusive_scan(int v, int* buf, int* total) {
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    int incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (lane == 63) buf[wave] = incl;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < SCHED_THREADS / 64; ++w) {
        const int x = buf[w];
        before += w < wave ? x : 0;
        all += x;
    }
    *total = all;
    __syncthreads();  // buf may be refilled by the next scan
    return before + incl - v;
}

// Samples whose clamped bounds and tile offsets the kernel keeps in LDS (3 x 4 bytes each).  A batch with up to
// three times as many keeps the tile offsets there, which is what the per-tile searches walk, and reads the
// bounds of the sample found from cu_seqlens; beyond that the searches read the workspace (same results, slower).
constexpr int SCHED_CACHE = 8192;
constexpr int SCHED_CACHE_OFFSETS = 3 * SCHED_CACHE;

struct SchedJob {  // one work list
    int R, U, mode, max_items;
    int32_t *hdr, *tile_off;
    WorkItem* items;
};

// One workgroup per work list (the backward builds two at a time).
__global__ void __launch_bounds__(SCHED_THREADS)
sched_kernel(const int32_t* __restrict__ cu, int B, int T, SchedJob job0, SchedJob job1) {
    __shared__ int scan_buf[SCHED_THREADS];
    __shared__ int bins[SCHED_BINS];
    __shared__ int cache_l[3 * SCHED_CACHE + 1];
    __shared__ int longest;
    const SchedJob job = blockIdx.x == 0 ? job0 : job1;
    const int R = job.R, U = job.U, mode = job.mode;
    int32_t* __restrict__ const hdr = job.hdr;
    int32_t* __restrict__ const tile_off = job.tile_off;
    WorkItem* __restrict__ const items = job.items;
    const bool cached = B <= SCHED_CACHE;                              // (uniform) bounds and offsets in LDS
    const bool cached_offsets = !cached && B <= SCHED_CACHE_OFFSETS;   // (uniform) offsets only
    int* const beg_l = cache_l;
    int* const end_l = cache_l + SCHED_CACHE;
    int* const toff_l = cached ? cache_l + 2 * SCHED_CACHE : cache_l;
    const int t = threadIdx.x;
    if (t == 0) longest = 0;
    __syncthreads();

    // 1. tile_off[s] = number of tiles of samples 0..s-1
    int carry = 0;
    for (int base = 0; base < B; base += SCHED_THREADS) {
        int s = base + t;
        int n = 0;
        if (s < B) {
            int begin, end;
            sched_sample_rows(cu[s], cu[s + 1], T, begin, end);
            if (cached) { beg_l[s] = begin; end_l[s] = end; }
            const int len = end - begin;
            n = (len + R - 1) / R;
            if (len >= kXcdChunkMinLen) longest = len;  // (any such length will do: only the threshold matters)
        }
        int total;
        int ex = block_exclusive_scan(n, scan_buf, &total);
        if (s < B) {
            tile_off[s] = carry + ex;
            if (cached || cached_offsets) toff_l[s] = carry + ex;
        }
        carry += total;
    }
    // (a well-formed batch has at most max_items tiles; one that is not loses the surplus instead of
    // writing past the list)
    const int n_items = min(carry, job.max_items);
    if (t == 0) {
        tile_off[B] = n_items;
        hdr[0] = n_items;
        hdr[1] = longest >= kXcdChunkMinLen ? kXcdChunk : 1;  // work order of the compute kernels (xcd_item_head)
    }
    for (int i = t; i < SCHED_BINS; i += SCHED_THREADS) bins[i] = 0;
    __syncthreads();  // also makes tile_off (global, written by this block) visible to the block

    // the sample that holds tile idx of the batch (largest s with tile_off[s] <= idx), its rows and the tile's cost
    auto locate = [&](int idx, int& begin, int& end, int& tile) {
        int lo = 0, hi = B;
        if (cached) {
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (toff_l[mid] <= idx) lo = mid; else hi = mid;
            }
            begin = beg_l[lo]; end = end_l[lo]; tile = idx - toff_l[lo];
        } else if (cached_offsets) {
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (toff_l[mid] <= idx) lo = mid; else hi = mid;
            }
            sched_sample_rows(cu[lo], cu[lo + 1], T, begin, end);
            tile = idx - toff_l[lo];
        } else {
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (tile_off[mid] <= idx) lo = mid; else hi = mid;
            }
            sched_sample_rows(cu[lo], cu[lo + 1], T, begin, end);
            tile = idx - tile_off[lo];
        }
        return sched_tile_cost(end - begin, tile, R, U, mode);
    };

    // 2. histogram of costs
    for (int idx = t; idx < n_items; idx += SCHED_THREADS) {
        int begin, end, tile;
        atomicAdd(&bins[locate(idx, begin, end, tile)], 1);
    }
    __syncthreads();

    // 3. start position of each cost class, heaviest class first
    {
        constexpr int PER = SCHED_BINS / SCHED_THREADS;
        int loc[PER];
        int sum = 0;
        for (int i = 0; i < PER; ++i) {  // thread t owns descending costs
            loc[i] = bins[SCHED_BINS - 1 - (t * PER + i)];
            sum += loc[i];
        }
        int total;
        int ex = block_exclusive_scan(sum, scan_buf, &total);
        for (int i = 0; i < PER; ++i) {
            bins[SCHED_BINS - 1 - (t * PER + i)] = ex;
            ex += loc[i];
        }
    }
    __syncthreads();

    // 4. scatter (the order inside one cost class is arbitrary; results do not depend on it)
    for (int idx = t; idx < n_items; idx += SCHED_THREADS) {
        int begin, end, tile;
        const int pos = atomicAdd(&bins[locate(idx, begin, end, tile)], 1);
        items[pos] = make_int4(begin + tile * R, begin, end, tile);
    }
}

static SchedJob make_job(int tile_rows, int partner_rows, CostMode mode, void* ws, const SchedLayout& lay) {
    char* base = (char*)ws;
    return SchedJob{tile_rows, partner_rows, (int)mode, (int)lay.max_items, (int32_t*)base,
                    (int32_t*)(base + lay.tile_off_ofs), (WorkItem*)(base + lay.items_ofs)};
}

hipError_t launch_scheduler(const int32_t* cu_seqlens, int num_seqs, int total_tokens, int tile_rows,
                            int partner_rows, CostMode mode, void* ws, const SchedLayout& lay, hipStream_t stream) {
    const SchedJob job = make_job(tile_rows, partner_rows, mode, ws, lay);
    hipLaunchKernelGGL(sched_kernel, dim3(1), dim3(SCHED_THREADS), 0, stream, cu_seqlens, num_seqs, total_tokens,
                       job, job);
    return hipGetLastError();
}

hipError_t launch_scheduler_pair(const int32_t* cu_seqlens, int num_seqs, int total_tokens, int tile_rows_a,
                                 int partner_rows_a, CostMode mode_a, void* ws_a, const SchedLayout& lay_a,
                                 int tile_rows_b, int partner_rows_b, CostMode mode_b, void* ws_b,
                                 const SchedLayout& lay_b, hipStream_t stream) {
    hipLaunchKernelGGL(sched_kernel, dim3(2), dim3(SCHED_THREADS), 0, stream, cu_seqlens, num_seqs, total_tokens,
                       make_job(tile_rows_a, partner_rows_a, mode_a, ws_a, lay_a),
                       make_job(tile_rows_b, partner_rows_b, mode_b, ws_b, lay_b));
    return hipGetLastError();
}

int64_t schedule_on_host(const int32_t* cu, int B, int T, int R, int U, CostMode mode, int64_t max_items,
                         WorkItem* items) {
    // counting sort by cost class, heaviest first; inside a class the tiles keep their (sample, tile) order
    std::vector<int64_t> start(SCHED_BINS + 1, 0);
    int64_t n = 0;
    for (int pass = 0; pass < 2; ++pass) {
        int64_t seen = 0;
        for (int s = 0; s < B && seen < max_items; ++s) {
            int begin, end;
            sched_sample_rows(cu[s], cu[s + 1], T, begin, end);
            const int L = end - begin;
            for (int t = 0; t * (int64_t)R < L && seen < max_items; ++t, ++seen) {
                const int c = sched_tile_cost(L, t, R, U, (int)mode);
                if (pass == 0) ++start[SCHED_BINS - 1 - c + 1];
                else items[start[SCHED_BINS - 1 - c]++] = make_int4(begin + t * R, begin, end, t);
            }
        }
        if (pass == 0) {
            n = seen;
            for (int i = 0; i < SCHED_BINS; ++i) start[i + 1] += start[i];
        }
    }
    return n;
}

// One workgroup walks cu_seqlens; every thread notes what it sees wrong, the block ORs the notes.
__global__ void __launch_bounds__(SCHED_THREADS)
check_cu_seqlens_kernel(const int32_t* __restrict__ cu, int B, int T, int32_t* __restrict__ verdict) {
    int bad = 0;
    for (int s = threadIdx.x; s < B; s += SCHED_THREADS) bad |= cu[s] > cu[s + 1];
    if (threadIdx.x == 0) bad |= cu[0] != 0 || cu[B] != T;
    bad = __syncthreads_or(bad);
    if (threadIdx.x == 0) *verdict = bad ? 1 : 0;
}

hipError_t launch_check_cu_seqlens(const int32_t* cu_seqlens, int num_seqs, int total_tokens, int32_t* verdict,
                                   hipStream_t stream) {
    hipLaunchKernelGGL(check_cu_seqlens_kernel, dim3(1), dim3(SCHED_THREADS), 0, stream, cu_seqlens, num_seqs,
                       total_tokens, verdict);
    return hipGetLastError();
}

}  // namespace va
