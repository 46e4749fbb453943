// Internal host-side declarations shared by the translation units of libvarlen_attn.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace va {

// Scheduler work item: one tile of `rows` consecutive rows of one sample.
//   x = first packed row of the tile, y = first packed row of the sample,
//   z = one past the sample's last packed row, w = tile index inside the sample.
typedef int4 WorkItem;

// How the cost of a tile (the number of partner tiles it loops over) is derived.
enum CostMode {
    COST_FULL = 0,          // every tile of a sample meets the whole sample
    COST_CAUSAL_QUERY = 1,  // query tile t meets keys [0, end of tile t]
    COST_CAUSAL_KEY = 2     // key tile t meets queries [start of tile t, L)
};

// Layout of the scheduler's part of a workspace (all int32):
//   [0] n_items   [1..15] reserved   [16 .. 16+B] tile offsets per sample   then the work items.
struct SchedLayout {
    size_t tile_off_ofs;  // bytes
    size_t items_ofs;     // bytes, 16-byte aligned
    size_t end_ofs;       // bytes, 256-byte aligned
    int64_t max_items;
};
SchedLayout sched_layout(int64_t total_tokens, int64_t num_seqs, int tile_rows);

// Rows [begin, end) of a sample, from cu[s] and cu[s+1] as they stand on the device.  For a well-formed
// cu_seqlens this changes nothing; for one that breaks the precondition it keeps every work item inside
// [0, T), so that the attention kernels never address memory outside the tensors.
__host__ __device__ inline void sched_sample_rows(int cu_s, int cu_s1, int T, int& begin, int& end) {
    begin = cu_s < 0 ? 0 : (cu_s > T ? T : cu_s);
    end = cu_s1 < begin ? begin : (cu_s1 > T ? T : cu_s1);
}
constexpr int SCHED_BINS = 4096;  // cost classes of the counting sort; costs above SCHED_BINS-1 share the top one
// Cost of tile t (R rows) of a sample of L rows: the number of partner tiles of U rows it visits.
__host__ __device__ inline int sched_tile_cost(int L, int t, int R, int U, int mode) {
    int span;
    if (mode == COST_FULL) span = L;
    else if (mode == COST_CAUSAL_QUERY) span = L < (t + 1) * R ? L : (t + 1) * R;
    else span = L - t * R;
    const int c = (span + U - 1) / U;
    return c < SCHED_BINS - 1 ? c : SCHED_BINS - 1;
}
// The same work list on the host (cu_seqlens in host memory): every tile once, by decreasing cost, tiles of
// equal cost in (sample, tile) order.  items holds max_items entries; returns the number written.
int64_t schedule_on_host(const int32_t* cu_seqlens, int num_seqs, int total_tokens, int tile_rows, int partner_rows,
                         CostMode mode, int64_t max_items, WorkItem* items);

// Enqueue the scheduler: fills header, tile offsets and the cost-sorted work list at `ws`.
hipError_t launch_scheduler(const int32_t* cu_seqlens, int num_seqs, int total_tokens, int tile_rows,
                            int partner_rows, CostMode mode, void* ws, const SchedLayout& lay, hipStream_t stream);

// Two work lists in one launch (one workgroup each): what the backward needs.
hipError_t launch_scheduler_pair(const int32_t* cu_seqlens, int num_seqs, int total_tokens, int tile_rows_a,
                                 int partner_rows_a, CostMode mode_a, void* ws_a, const SchedLayout& lay_a,
                                 int tile_rows_b, int partner_rows_b, CostMode mode_b, void* ws_b,
                                 const SchedLayout& lay_b, hipStream_t stream);

// Enqueue the check of cu_seqlens' contents: *verdict (device) = 0 if cu[0] = 0, cu never decreases and
// cu[num_seqs] = total_tokens, else 1.
hipError_t launch_check_cu_seqlens(const int32_t* cu_seqlens, int num_seqs, int total_tokens, int32_t* verdict,
                                   hipStream_t stream);

struct FwdArgs {
    const void *q, *k, *v;
    void* o;
    float* lse;
    const int32_t* sched_hdr;
    const WorkItem* items;
    int64_t max_items;
    int total_tokens, num_q_heads, num_kv_heads, head_dim, causal;
    float scale;
    int kv_splits;    // >= 1; > 1: every query tile's keys are split over that many workgroups
    float* part_o;    // kv_splits > 1: fp32 [kv_splits, T, Hq, D] partial outputs
    float* part_lse;  // kv_splits > 1: fp32 [kv_splits, Hq, T]
    unsigned long long* clock_probe;  // null, or 2 counters (see ClockProbe)
    bool lean;  // batches of short samples (the caller's max_seqlen says so), kv_splits == 1: the lean kernel form
};
constexpr int kShortBatchMaxSeqlen = 1024;  // max_seqlen hint up to which a batch counts as "short samples only"
constexpr int FWD_TILE_Q = 128;
constexpr int FWD_TILE_KV = 64;
hipError_t launch_fwd(const FwdArgs& a, hipStream_t stream);

struct BwdArgs {
    const void *dout, *q, *k, *v, *o;
    const float* lse;
    float* stats;  // fp32 [Hq, T, 2] scratch: LSE * log2(e) and Delta per (head, row)
    void *dq, *dk, *dv;
    const int32_t* sched_hdr_kv;
    const WorkItem* items_kv;
    int64_t max_items_kv;
    const int32_t* sched_hdr_q;
    const WorkItem* items_q;
    int64_t max_items_q;
    int total_tokens, num_q_heads, num_kv_heads, head_dim, causal;
    float scale;
    unsigned long long *clock_probe_dkdv, *clock_probe_dq;  // null, or 2 counters each (see ClockProbe)
};
constexpr int BWD_TILE_KV = 128;  // rows of K/V one dK/dV workgroup owns
constexpr int BWD_STEP_Q = 64;    // query rows it stages per step
constexpr int BWD_TILE_Q = 128;   // rows of Q one dQ workgroup owns
constexpr int BWD_STEP_KV = 64;   // key rows it stages per step
// O = sum_p exp(LSE_p - LSE) O_p over parts [P, T, H, D] (bf16 or fp32) with lse [P, H, T].
hipError_t launch_merge(const void* o_parts, bool parts_fp32, const float* lse_parts, int P, int T, int H, int D,
                        void* o, float* lse, hipStream_t stream);

hipError_t launch_bwd_dkdv(const BwdArgs& a, hipStream_t stream);
hipError_t launch_bwd_dq(const BwdArgs& a, hipStream_t stream);

}  // namespace va
