/*
 * varlen_attn.h -- C ABI of the MI355X (gfx950) variable-length packed self-attention library.
 *
 * The operation.  The paper trains multimodal LLMs on packed sequences: samples of different
 * lengths are concatenated into one token stream and must not attend to each other (Section
 * 2.1, hybrid packing, Fig. 3c).  Encoder (ViT) attention is full inside a sample (Section 2.2;
 * Section 4.1.1: the Ulysses state keeps full attention per rank), LLM attention is causal
 * (Section 4.1.1, parallelism selection rationale), and the attention layers use an exact tiled
 * algorithm (Section 6, "Efficient Operators").  The paper prints no formula; the library
 * computes the textbook one.  For sample s with rows [cu[s], cu[s+1]), query head h and kv head
 * c = h / (Hq / Hkv):
 *
 *     S_ij  = softmax_scale * <Q[i,h,:], K[j,c,:]>,   j in the same sample, and j <= i if causal
 *     LSE_i = ln sum_j exp(S_ij)                       (natural log, scale inside)
 *     O[i,h,:] = sum_j exp(S_ij - LSE_i) * V[j,c,:]
 *
 * and the gradients of sum(O * dO) with respect to Q, K and V.  Inputs and O/dQ/dK/dV are bf16,
 * products accumulate in fp32 on the matrix cores, LSE is fp32.
 *
 * Pointers.  Every tensor pointer is a DEVICE pointer owned by the caller and must be 16-byte
 * aligned; `p` is a HOST pointer.  The library never allocates, frees or synchronises: all work
 * is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the default stream), and the
 * buffers must stay alive until the stream has run it.  Outputs are fully overwritten.  The
 * workspace is scratch; its contents mean nothing between calls, and two calls that share one
 * workspace must be ordered on one stream.  The calls may be recorded under HIP stream capture:
 * the work list is rebuilt on the device inside every call, so a recorded graph stays valid when
 * the buffers' contents change, cu_seqlens included, as long as the sizes in `p` stay the same.
 *
 * Layouts (row-major, contiguous):
 *     q, o, dout, dq : bf16 [total_tokens, num_q_heads,  head_dim]
 *     k, v, dk, dv   : bf16 [total_tokens, num_kv_heads, head_dim]
 *     lse            : fp32 [num_q_heads, total_tokens]
 *     cu_seqlens     : int32 [num_seqs + 1], cu[0] = 0, non-decreasing, cu[num_seqs] = total_tokens
 * Empty samples (cu[s] == cu[s+1]) are legal.  The contents of cu_seqlens live on the device and
 * are NOT validated.  The scheduler clamps every sample to rows inside [0, total_tokens) and the
 * work list to the size the workspace holds, so an array that breaks the precondition gives
 * meaningless results but no access outside the tensors; varlen_attn_check_cu_seqlens tells.
 *
 * Errors.  Every argument the host can see is validated before anything is launched; on error
 * nothing has been enqueued.  total_tokens == 0 or num_seqs == 0 returns VA_OK with no launch.
 */
#ifndef VARLEN_ATTN_H
#define VARLEN_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    VA_OK = 0,
    VA_ERR_NULL_PTR = 1,            /* a required pointer is NULL */
    VA_ERR_BAD_SHAPE = 2,           /* negative size or count, heads < 1, Hq % Hkv != 0, causal not 0/1,
                                       max_seqlen < 0, kv_splits or num_parts out of range */
    VA_ERR_UNSUPPORTED = 3,         /* head_dim not in {64, 80, 96, 128}, or device is not gfx950 */
    VA_ERR_WORKSPACE_TOO_SMALL = 4, /* workspace_bytes below the *_workspace_bytes() answer */
    VA_ERR_BAD_SCALE = 5,           /* softmax_scale is NaN, infinite or negative */
    VA_ERR_HIP = 6,                 /* a HIP call failed; see varlen_attn_last_hip_error() */
    VA_ERR_MISALIGNED = 7,          /* a tensor or workspace pointer is not 16-byte aligned */
    VA_ERR_BAD_CU_SEQLENS = 8,      /* varlen_attn_check_cu_seqlens only: the device array breaks the precondition */
    VA_ERR_SCRATCH_LIMIT = 9        /* varlen_attn_fwd_static_scratch only: the call needs more scratch than
                                       VA_STATIC_SCRATCH_BYTES */
};

typedef struct {
    int32_t total_tokens;  /* T   >= 0 */
    int32_t num_seqs;      /* B   >= 0 */
    int32_t num_q_heads;   /* Hq  >= 1 */
    int32_t num_kv_heads;  /* Hkv >= 1, Hq % Hkv == 0; q head h reads kv head h / (Hq/Hkv) */
    int32_t head_dim;      /* D in {64, 80, 96, 128} */
    int32_t causal;        /* 0: full attention inside a sample; 1: j <= i inside a sample */
    float softmax_scale;   /* finite, >= 0 (0 is legal: uniform attention) */
    int32_t max_seqlen;    /* optional hint, 0 = unknown: the caller's promise that no sample is longer than
                              this.  The work list is built on the device from cu_seqlens, so nothing is
                              sized by it and a wrong value never makes a result wrong; the host uses it
                              where it must decide before the device has seen the lengths: the automatic
                              kv_splits choice, and the tile shape for batches of short samples only
                              (see varlen_attn_fwd).  Must be >= 0. */
    int32_t kv_splits;     /* an extension, forward only; a tuning hint that never changes results beyond
                              rounding: 0 = automatic, 1 = never split, 2..VA_MAX_KV_SPLITS = that many
                              workgroups share the keys of each query tile (see varlen_attn_fwd) */
} varlen_attn_params;
enum { VA_MAX_KV_SPLITS = 8, VA_MAX_MERGE_PARTS = 64 };

/* Bytes of device scratch the forward / backward call needs for these sizes (0 on bad params). */
size_t varlen_attn_fwd_workspace_bytes(const varlen_attn_params *p);
size_t varlen_attn_bwd_workspace_bytes(const varlen_attn_params *p);

/*
 * Forward: writes o and lse.  Steps (all on the device): a length-aware scheduler turns
 * cu_seqlens into a list of 128-row query tiles ordered by decreasing cost; one workgroup per
 * (tile, head) streams the sample's K/V through LDS, S = QK^T and PV on bf16 MFMA, online softmax.
 * A launch too small to fill the GPU (few heads, one mid-length sample: what a rank sees in the
 * sequence-parallel state of Section 4.1.1) is split further: kv_splits workgroups share the keys of
 * each query tile, write fp32 partial results into the workspace, and a merge kernel combines them
 * (same formula as varlen_attn_merge).  The workspace size accounts for it.
 * A batch of short samples only (0 < max_seqlen <= 1024, keys not split) takes a leaner form of the same
 * kernel, which issues no load past a tile list's end: there a workgroup lives for one to a few tile steps
 * and its time is a chain of memory round trips, so the two spare ones matter (measured 1.1-1.3x at 64..256
 * tokens per sample).  The results are bit-identical to those without the hint, also when the hint is wrong.
 */
int varlen_attn_fwd(const varlen_attn_params *p,
                    const void *q, const void *k, const void *v,
                    const int32_t *cu_seqlens,
                    void *o, float *lse,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The forward for callers that can neither allocate device memory nor hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and
 * results as varlen_attn_fwd, bit for bit, minus the workspace: the scratch the call needs (the
 * scheduler's work list and, when the keys of a query tile are split, the fp32 partial results) lives in
 * an array of VA_STATIC_SCRATCH_BYTES that is part of the library's device code.  Every GPU the library
 * runs on holds its own copy of it from the first call there until the process ends.  The call allocates
 * nothing and calls no allocating routine; the first call on a device looks the array's address up
 * (hipGetSymbolAddress) and keeps it.
 * Limit: a call whose varlen_attn_fwd_workspace_bytes(p) exceeds VA_STATIC_SCRATCH_BYTES returns
 * VA_ERR_SCRATCH_LIMIT with nothing launched (kv_splits = 1 shrinks the need to the work list: 16 bytes per
 * 128 tokens and 20 per sample).
 * All calls on one GPU share that GPU's array, whatever their stream or thread: calls that overlap in time
 * on one GPU race on it and must be ordered by the caller (one stream, or events).  Nothing in it has to
 * start at zero: every call rewrites what it reads.
 */
enum { VA_STATIC_SCRATCH_BYTES = 32 << 20 };
int varlen_attn_fwd_static_scratch(const varlen_attn_params *p,
                                   const void *q, const void *k, const void *v,
                                   const int32_t *cu_seqlens,
                                   void *o, float *lse, void *hip_stream);

/*
 * Backward: writes dq, dk, dv from dout and the forward's saved o and lse (P is recomputed from
 * q, k and lse, as the paper's recomputation of core attention implies, Section 6 "Selective
 * Activation Offloading").  dk and dv are summed over the query heads that share a kv head.
 * Two kernels, no atomics, results are bit-reproducible: dQ per query tile (it also forms
 * Delta_i = <dout_i, o_i> from `o` as stored, in bf16, and leaves it with lse in the workspace),
 * then dK and dV per key tile.  Rows whose softmax is nearly one-hot feel the rounding of `o`
 * through Delta: dS = P (dP - Delta) is a small difference of large terms there.
 */
int varlen_attn_bwd(const varlen_attn_params *p,
                    const void *dout, const void *q, const void *k, const void *v,
                    const void *o, const float *lse,
                    const int32_t *cu_seqlens,
                    void *dq, void *dk, void *dv,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Merge of partial attention results over disjoint key/value shards: what context parallelism needs
 * after every rank has attended to one shard of the keys (Section 4.1.2 selects context parallelism
 * for overlong contexts; Section 5.2 shards long samples for it).  For every (row, head)
 *     LSE = ln sum_p exp(LSE_p),    O = sum_p exp(LSE_p - LSE) * O_p.
 * A part with LSE_p = -infinity held no key for that row: its weight is 0 and its O_p is not read.
 * If all parts are empty, O = 0 and LSE = -infinity.
 *   p          uses total_tokens, num_q_heads, head_dim (the other fields must still be valid)
 *   o_parts    DEVICE bf16 [num_parts, total_tokens, num_q_heads, head_dim], 16-byte aligned
 *   lse_parts  DEVICE fp32 [num_parts, num_q_heads, total_tokens]
 *   o, lse     DEVICE outputs, bf16 [T, Hq, D] and fp32 [Hq, T]; must not alias the parts
 * 1 <= num_parts <= VA_MAX_MERGE_PARTS.  Asynchronous on hip_stream, no workspace.
 */
int varlen_attn_merge(const varlen_attn_params *p, int32_t num_parts, const void *o_parts,
                      const float *lse_parts, void *o, float *lse, void *hip_stream);

/*
 * Checks the CONTENTS of cu_seqlens, which live on the device and which no other call looks at:
 * cu[0] = 0, cu[s] <= cu[s+1] for every sample, cu[num_seqs] = total_tokens (the precondition on a
 * packed batch: Section 2.1, hybrid packing keeps samples apart inside one stream).  A batch that
 * breaks it makes the attention kernels read outside the tensors.  For callers that cannot vouch
 * for their packing code; varlen_attn_fwd / varlen_attn_bwd never call it.
 *   workspace: at least 16 bytes of device scratch, 16-byte aligned (the verdict is written there).
 * Unlike every other call this one SYNCHRONISES hip_stream: it copies the verdict back (4 bytes)
 * before it returns.  It must not be called while the stream is being captured.
 * Returns VA_OK, VA_ERR_BAD_CU_SEQLENS, or an argument error (nothing launched then).
 * num_seqs == 0 is checked on the host: it is VA_OK exactly if total_tokens == 0.
 */
int varlen_attn_check_cu_seqlens(const varlen_attn_params *p, const int32_t *cu_seqlens, void *workspace,
                                 size_t workspace_bytes, void *hip_stream);

/* Static, NUL-terminated description of a status code. */
const char *varlen_attn_status_string(int status);

/* hipError_t (as int) of the last failed HIP call on this thread, 0 if none. */
int varlen_attn_last_hip_error(void);

/*
 * Number of scheduler work items the forward (which = 0), the backward dK/dV pass (1) or the
 * backward dQ pass (2) launches at most for these sizes: the grid is this times the head count
 * of that pass.  Host arithmetic only; for tests and benchmarks.
 */
int64_t varlen_attn_max_work_items(const varlen_attn_params *p, int which);

/*
 * The scheduler's work list (Section 2.2 and 4.1.1: mixed long and short samples; Section 6, "Efficient
 * Operators": work partitioning) computed on the HOST from a host copy of cu_seqlens, with the arithmetic
 * the device scheduler uses: per sample the rows [begin, end) clamped into [0, total_tokens), tiles of 128
 * rows, a tile's cost = the number of 64-row partner tiles it visits, heaviest first (equal costs in
 * sample-then-tile order here; the device list may order them differently), at most
 * varlen_attn_max_work_items() tiles.  For tests and for callers that want to inspect the balance; the
 * compute calls never use it.
 *   which            0 forward query tiles, 1 backward key tiles (dK/dV), 2 backward query tiles (dQ)
 *   cu_seqlens_host  HOST int32 [num_seqs + 1]; need NOT obey the precondition (that is the point of the clamp)
 *   items            HOST int32 [items_capacity][4] (out): first row, sample begin, sample end, tile index
 * Returns the number of tiles written, or -1 on bad arguments (items_capacity below max_work_items included).
 */
int64_t varlen_attn_schedule_host(const varlen_attn_params *p, int which, const int32_t *cu_seqlens_host,
                                  int32_t *items, int64_t items_capacity);

/*
 * Length-balanced partition of a group's samples into `bins` subsets (one per rank): the step in
 * front of the attention kernels in the paper's pipeline (Section 5.1, decentralized grouped
 * reordering: after the sample sizes of a group of ranks are gathered, the samples are reordered
 * "using the Karp algorithm").  The paper says no more; this is the k-way Karmarkar-Karp largest
 * differencing method, or greedy longest-processing-time-first scheduling for comparison.
 * HOST pointers only, no GPU work, thread-safe.
 *   lengths      int32 [num_seqs], each >= 0
 *   cost of a sample of length L = lin_cost * L + quad_cost * L * L   (both finite, >= 0;
 *                  attention is the quadratic term)
 *   equal_counts 1: bin sizes differ by at most one sample (fixed microbatch size per rank);
 *                  0: any sizes
 *   bin_of       int32 [num_seqs] (out): the bin of every sample; bin 0 is the most expensive
 *                  one for the differencing method
 *   bin_cost     double [bins] (out, may be NULL): summed cost per bin
 * Ties: equal costs go to the lower sample index, equally cheap bins to the lower bin.
 * Errors: VA_ERR_BAD_SHAPE (negative count or length, bins < 1, unknown method),
 * VA_ERR_BAD_SCALE (cost coefficients), VA_ERR_NULL_PTR.  num_seqs == 0 returns VA_OK.
 */
enum { VA_PARTITION_KARMARKAR_KARP = 0, VA_PARTITION_LPT = 1 };
int varlen_attn_balance_partition(const int32_t *lengths, int32_t num_seqs, int32_t bins, int32_t method,
                                  int32_t equal_counts, double lin_cost, double quad_cost,
                                  int32_t *bin_of, double *bin_cost);

/*
 * Per-kernel timing for benchmarks.  While enabled (process-wide), every kernel this library
 * launches is bracketed by two HIP events recorded on the caller's stream; launches are not
 * synchronised and results are unchanged.  Enabling drops earlier samples.  profile_read() waits
 * for the recorded events of one kernel kind and returns their summed duration (milliseconds) and
 * count.  Events are created with hipEventCreate: do not leave this on in a loop that must not
 * allocate, and read or re-enable now and then so the sample list does not grow without bound.
 */
enum {
    VA_KERNEL_SCHED = 0, /* tile scheduler (1 launch per forward, 1 per backward: both of its lists) */
    VA_KERNEL_FWD = 1,   /* forward attention */
    VA_KERNEL_DKDV = 2,  /* backward: dK, dV */
    VA_KERNEL_DQ = 3,    /* backward: dQ (also forms Delta = rowsum(dO * O) and writes the per-row statistics
                            dK/dV reads; launched first) */
    VA_KERNEL_MERGE = 4  /* merge of partial results (varlen_attn_merge, split forward) */
};
int varlen_attn_profile_enable(int on);
int varlen_attn_profile_read(int kernel, double *total_ms, int64_t *launches);

/*
 * Shader-clock probe for benchmarks (the chip lowers its clock under matrix-core load, which moves
 * the attainable fraction of the published peak).  device_counters: DEVICE uint64 [6], 8-byte
 * aligned, owned and zeroed by the caller, alive until the last launch made while it was set has
 * finished; NULL (the default) switches the probe off.  While set (process-wide), every workgroup of
 * the forward, dK/dV and dQ kernels adds its residence time to [0], [2], [4] in ticks of the 100 MHz
 * constant clock and to [1], [3], [5] in shader cycles: [1]/[0] * 0.1 is the forward's average clock
 * in GHz.  Two clock reads and two atomics per workgroup; results are unchanged.
 */
int varlen_attn_profile_clock_probe(unsigned long long *device_counters);

#ifdef __cplusplus
}
#endif
#endif /* VARLEN_ATTN_H */
