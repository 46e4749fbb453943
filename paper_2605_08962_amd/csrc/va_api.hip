// C-ABI entry points of libvarlen_attn.so: argument validation, workspace carving, launches.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/varlen_attn.h"
#include "va_internal.h"

// Scratch of varlen_attn_fwd_static_scratch: device memory that belongs to the library's code object, one
// copy per GPU.  In host code this name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[VA_STATIC_SCRATCH_BYTES];

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return VA_ERR_HIP;
}

// Optional per-kernel timing: while enabled, each kernel launch is bracketed by two events recorded
// on the caller's stream.  Nothing synchronises until varlen_attn_profile_read().
struct ProfSample { int kernel; hipEvent_t a, b; };
std::mutex g_prof_mutex;
bool g_prof_on = false;
std::vector<ProfSample> g_prof_samples;
unsigned long long* g_clock_probe = nullptr;  // device, 6 counters, caller-owned (see the header)

unsigned long long* clock_probe_slot(int pair) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    return g_clock_probe ? g_clock_probe + 2 * pair : nullptr;
}

struct ProfScope {
    bool on = false;
    ProfSample s{};
    hipStream_t stream;
    ProfScope(int kernel, hipStream_t st) : stream(st) {
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        if (!g_prof_on) return;
        if (hipEventCreate(&s.a) != hipSuccess) return;
        if (hipEventCreate(&s.b) != hipSuccess) { (void)hipEventDestroy(s.a); return; }
        s.kernel = kernel;
        on = hipEventRecord(s.a, stream) == hipSuccess;
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(s.b, stream);
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        g_prof_samples.push_back(s);
    }
};

void prof_clear_locked() {
    for (auto& s : g_prof_samples) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
    g_prof_samples.clear();
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

int check_params(const varlen_attn_params* p) {
    if (!p) return VA_ERR_NULL_PTR;
    if (p->total_tokens < 0 || p->num_seqs < 0 || p->num_q_heads < 1 || p->num_kv_heads < 1 ||
        p->num_q_heads % p->num_kv_heads != 0 || (p->causal != 0 && p->causal != 1) || p->max_seqlen < 0 ||
        p->kv_splits < 0 || p->kv_splits > VA_MAX_KV_SPLITS)
        return VA_ERR_BAD_SHAPE;
    if (p->head_dim != 64 && p->head_dim != 80 && p->head_dim != 96 && p->head_dim != 128)
        return VA_ERR_UNSUPPORTED;
    if (!std::isfinite(p->softmax_scale) || p->softmax_scale < 0.f) return VA_ERR_BAD_SCALE;
    // grid sizes and packed offsets are 32-bit in places: keep the launch within them
    int64_t items = (int64_t)p->total_tokens / 64 + p->num_seqs;
    if (items * p->num_q_heads * std::max(p->kv_splits, 1) >= (int64_t)1 << 31) return VA_ERR_BAD_SHAPE;
    return VA_OK;
}

// The current device must be a gfx950; checked once per device.
int check_device() {
    static thread_local int checked_dev = -1;
    static thread_local int checked_rc = VA_OK;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev == checked_dev) return checked_rc;
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return hip_fail(e);
    checked_dev = dev;
    checked_rc = std::strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? VA_OK : VA_ERR_UNSUPPORTED;
    return checked_rc;
}

// How many workgroups share the keys of one query tile in the forward.  Splitting only pays when the
// launch cannot fill the chip: fewer workgroups than the 256 CUs can hold at once (3 per CU at
// head_dim <= 80, else 2), and samples long enough that every chunk still gets two key tiles (judged by
// the caller's max_seqlen if it gave one, else by the average sample).
bool short_batch(const varlen_attn_params* p) { return p->max_seqlen > 0 && p->max_seqlen <= va::kShortBatchMaxSeqlen; }

int fwd_kv_splits(const varlen_attn_params* p) {
    if (p->kv_splits >= 1) return p->kv_splits;
    const int64_t wgs = ((int64_t)p->total_tokens / va::FWD_TILE_Q + p->num_seqs) * p->num_q_heads;
    const int64_t slots = 256 * (p->head_dim <= 80 ? 3 : 2);
    const int64_t sample_len = p->max_seqlen > 0 ? std::min(p->max_seqlen, p->total_tokens) : p->total_tokens / p->num_seqs;
    const int64_t tiles_per_sample = sample_len / va::FWD_TILE_KV;
    int64_t s = std::min<int64_t>(std::min<int64_t>(slots / std::max<int64_t>(wgs, 1), tiles_per_sample / 2), VA_MAX_KV_SPLITS);
    return (int)std::max<int64_t>(s, 1);
}

struct FwdLayout {
    va::SchedLayout sched;
    int splits;
    size_t part_o_ofs, part_lse_ofs, end;
};

FwdLayout fwd_layout(const varlen_attn_params* p) {
    FwdLayout f;
    f.sched = va::sched_layout(p->total_tokens, p->num_seqs, va::FWD_TILE_Q);
    f.splits = fwd_kv_splits(p);
    f.part_o_ofs = f.part_lse_ofs = f.end = f.sched.end_ofs;
    if (f.splits > 1) {
        const size_t rows = (size_t)p->total_tokens * p->num_q_heads;
        f.part_lse_ofs = f.part_o_ofs + (size_t)f.splits * rows * p->head_dim * sizeof(float);
        f.end = (f.part_lse_ofs + (size_t)f.splits * rows * sizeof(float) + 255) / 256 * 256;
    }
    return f;
}

struct BwdLayout {
    va::SchedLayout kv, q;
    size_t kv_ofs, q_ofs, stats_ofs, end;
};

BwdLayout bwd_layout(const varlen_attn_params* p) {
    BwdLayout b;
    b.kv = va::sched_layout(p->total_tokens, p->num_seqs, va::BWD_TILE_KV);
    b.q = va::sched_layout(p->total_tokens, p->num_seqs, va::BWD_TILE_Q);
    b.kv_ofs = 0;
    b.q_ofs = b.kv.end_ofs;
    b.stats_ofs = b.q_ofs + b.q.end_ofs;
    b.end = b.stats_ofs + ((size_t)p->total_tokens * p->num_q_heads * 2 * sizeof(float) + 255) / 256 * 256;
    return b;
}

}  // namespace

extern "C" {

size_t varlen_attn_fwd_workspace_bytes(const varlen_attn_params* p) {
    if (check_params(p) != VA_OK) return 0;
    if (p->total_tokens == 0 || p->num_seqs == 0) return va::sched_layout(0, 0, va::FWD_TILE_Q).end_ofs;
    return fwd_layout(p).end;
}

size_t varlen_attn_bwd_workspace_bytes(const varlen_attn_params* p) {
    if (check_params(p) != VA_OK) return 0;
    return bwd_layout(p).end;
}

int64_t varlen_attn_max_work_items(const varlen_attn_params* p, int which) {
    if (check_params(p) != VA_OK) return 0;
    int rows = which == 0 ? va::FWD_TILE_Q : which == 1 ? va::BWD_TILE_KV : va::BWD_TILE_Q;
    return va::sched_layout(p->total_tokens, p->num_seqs, rows).max_items;
}

int64_t varlen_attn_schedule_host(const varlen_attn_params* p, int which, const int32_t* cu_seqlens_host,
                                  int32_t* items, int64_t items_capacity) {
    if (check_params(p) != VA_OK || which < 0 || which > 2 || !cu_seqlens_host || !items) return -1;
    const int rows = which == 0 ? va::FWD_TILE_Q : which == 1 ? va::BWD_TILE_KV : va::BWD_TILE_Q;
    const int partner = which == 0 ? va::FWD_TILE_KV : which == 1 ? va::BWD_STEP_Q : va::BWD_STEP_KV;
    const va::CostMode mode = !p->causal ? va::COST_FULL : which == 1 ? va::COST_CAUSAL_KEY : va::COST_CAUSAL_QUERY;
    const int64_t max_items = va::sched_layout(p->total_tokens, p->num_seqs, rows).max_items;
    if (items_capacity < max_items) return -1;
    static_assert(sizeof(va::WorkItem) == 4 * sizeof(int32_t), "work items are four int32");
    return va::schedule_on_host(cu_seqlens_host, p->num_seqs, p->total_tokens, rows, partner, mode, max_items,
                                (va::WorkItem*)items);
}

int varlen_attn_fwd(const varlen_attn_params* p, const void* q, const void* k, const void* v,
                    const int32_t* cu_seqlens, void* o, float* lse, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
    int rc = check_params(p);
    if (rc != VA_OK) return rc;
    if (p->total_tokens == 0 || p->num_seqs == 0) return VA_OK;
    if (!q || !k || !v || !cu_seqlens || !o || !lse || !workspace) return VA_ERR_NULL_PTR;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(workspace) ||
        ((uintptr_t)lse & 3u) || ((uintptr_t)cu_seqlens & 3u))
        return VA_ERR_MISALIGNED;
    const FwdLayout fl = fwd_layout(p);
    const va::SchedLayout& lay = fl.sched;
    if (workspace_bytes < fl.end) return VA_ERR_WORKSPACE_TOO_SMALL;
    rc = check_device();
    if (rc != VA_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;

    hipError_t e;
    {
        ProfScope ps(VA_KERNEL_SCHED, stream);
        e = va::launch_scheduler(cu_seqlens, p->num_seqs, p->total_tokens, va::FWD_TILE_Q, va::FWD_TILE_KV,
                                 p->causal ? va::COST_CAUSAL_QUERY : va::COST_FULL, workspace, lay, stream);
    }
    if (e != hipSuccess) return hip_fail(e);
    va::FwdArgs a;
    a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
    a.sched_hdr = (const int32_t*)workspace;
    a.items = (const va::WorkItem*)((const char*)workspace + lay.items_ofs);
    a.max_items = lay.max_items;
    a.total_tokens = p->total_tokens; a.num_q_heads = p->num_q_heads; a.num_kv_heads = p->num_kv_heads;
    a.head_dim = p->head_dim; a.causal = p->causal; a.scale = p->softmax_scale;
    a.kv_splits = fl.splits;
    a.part_o = (float*)((char*)workspace + fl.part_o_ofs);
    a.part_lse = (float*)((char*)workspace + fl.part_lse_ofs);
    a.clock_probe = clock_probe_slot(0);
    a.lean = short_batch(p) && fl.splits == 1;
    {
        ProfScope ps(VA_KERNEL_FWD, stream);
        e = va::launch_fwd(a, stream);
    }
    if (e != hipSuccess) return hip_fail(e);
    if (fl.splits > 1) {
        ProfScope ps(VA_KERNEL_MERGE, stream);
        e = va::launch_merge(a.part_o, true, a.part_lse, fl.splits, p->total_tokens, p->num_q_heads, p->head_dim,
                             o, lse, stream);
        if (e != hipSuccess) return hip_fail(e);
    }
    return VA_OK;
}

namespace {
// Address of `scratch` on the current device, looked up once per device (with that device current).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int static_scratch_ptr(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return VA_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!ptr) return hip_fail(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return VA_OK;
}
}  // namespace

int varlen_attn_fwd_static_scratch(const varlen_attn_params* p, const void* q, const void* k, const void* v,
                                   const int32_t* cu_seqlens, void* o, float* lse, void* hip_stream) {
    int rc = check_params(p);
    if (rc != VA_OK) return rc;
    if (p->total_tokens == 0 || p->num_seqs == 0) return VA_OK;
    if (fwd_layout(p).end > (size_t)VA_STATIC_SCRATCH_BYTES) return VA_ERR_SCRATCH_LIMIT;
    rc = check_device();
    if (rc != VA_OK) return rc;
    void* ptr = nullptr;
    rc = static_scratch_ptr(&ptr);
    if (rc != VA_OK) return rc;
    return varlen_attn_fwd(p, q, k, v, cu_seqlens, o, lse, ptr, (size_t)VA_STATIC_SCRATCH_BYTES, hip_stream);
}

int varlen_attn_merge(const varlen_attn_params* p, int32_t num_parts, const void* o_parts, const float* lse_parts,
                      void* o, float* lse, void* hip_stream) {
    int rc = check_params(p);
    if (rc != VA_OK) return rc;
    if (num_parts < 1 || num_parts > VA_MAX_MERGE_PARTS) return VA_ERR_BAD_SHAPE;
    if (p->total_tokens == 0) return VA_OK;
    if (!o_parts || !lse_parts || !o || !lse) return VA_ERR_NULL_PTR;
    if (!aligned16(o_parts) || !aligned16(o) || ((uintptr_t)lse & 3u) || ((uintptr_t)lse_parts & 3u))
        return VA_ERR_MISALIGNED;
    rc = check_device();
    if (rc != VA_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    ProfScope ps(VA_KERNEL_MERGE, stream);
    hipError_t e = va::launch_merge(o_parts, false, lse_parts, num_parts, p->total_tokens, p->num_q_heads,
                                    p->head_dim, o, lse, stream);
    if (e != hipSuccess) return hip_fail(e);
    return VA_OK;
}

int varlen_attn_check_cu_seqlens(const varlen_attn_params* p, const int32_t* cu_seqlens, void* workspace,
                                 size_t workspace_bytes, void* hip_stream) {
    int rc = check_params(p);
    if (rc != VA_OK) return rc;
    if (p->num_seqs == 0) return p->total_tokens == 0 ? VA_OK : VA_ERR_BAD_CU_SEQLENS;
    if (!cu_seqlens || !workspace) return VA_ERR_NULL_PTR;
    if (((uintptr_t)cu_seqlens & 3u) || !aligned16(workspace)) return VA_ERR_MISALIGNED;
    if (workspace_bytes < 16) return VA_ERR_WORKSPACE_TOO_SMALL;
    rc = check_device();
    if (rc != VA_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    hipError_t e = va::launch_check_cu_seqlens(cu_seqlens, p->num_seqs, p->total_tokens, (int32_t*)workspace, stream);
    if (e != hipSuccess) return hip_fail(e);
    int32_t verdict = 1;
    e = hipMemcpyAsync(&verdict, workspace, sizeof(verdict), hipMemcpyDeviceToHost, stream);
    if (e != hipSuccess) return hip_fail(e);
    e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return hip_fail(e);
    return verdict == 0 ? VA_OK : VA_ERR_BAD_CU_SEQLENS;
}

int varlen_attn_bwd(const varlen_attn_params* p, const void* dout, const void* q, const void* k,
                    const void* v, const void* o, const float* lse, const int32_t* cu_seqlens,
                    void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
    int rc = check_params(p);
    if (rc != VA_OK) return rc;
    if (p->total_tokens == 0 || p->num_seqs == 0) return VA_OK;
    if (!dout || !q || !k || !v || !o || !lse || !cu_seqlens || !dq || !dk || !dv || !workspace)
        return VA_ERR_NULL_PTR;
    if (!aligned16(dout) || !aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) ||
        !aligned16(dq) || !aligned16(dk) || !aligned16(dv) || !aligned16(workspace) ||
        ((uintptr_t)lse & 3u) || ((uintptr_t)cu_seqlens & 3u))
        return VA_ERR_MISALIGNED;
    BwdLayout lay = bwd_layout(p);
    if (workspace_bytes < lay.end) return VA_ERR_WORKSPACE_TOO_SMALL;
    rc = check_device();
    if (rc != VA_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;

    hipError_t e;
    {   // both work lists (key tiles for dK/dV, query tiles for dQ) in one launch, one workgroup each
        ProfScope ps(VA_KERNEL_SCHED, stream);
        e = va::launch_scheduler_pair(cu_seqlens, p->num_seqs, p->total_tokens, va::BWD_TILE_KV, va::BWD_STEP_Q,
                                      p->causal ? va::COST_CAUSAL_KEY : va::COST_FULL, ws + lay.kv_ofs, lay.kv,
                                      va::BWD_TILE_Q, va::BWD_STEP_KV,
                                      p->causal ? va::COST_CAUSAL_QUERY : va::COST_FULL, ws + lay.q_ofs, lay.q, stream);
    }
    if (e != hipSuccess) return hip_fail(e);

    va::BwdArgs a;
    a.dout = dout; a.q = q; a.k = k; a.v = v; a.o = o; a.lse = lse;
    a.stats = (float*)(ws + lay.stats_ofs);
    a.dq = dq; a.dk = dk; a.dv = dv;
    a.sched_hdr_kv = (const int32_t*)(ws + lay.kv_ofs);
    a.items_kv = (const va::WorkItem*)(ws + lay.kv_ofs + lay.kv.items_ofs);
    a.max_items_kv = lay.kv.max_items;
    a.sched_hdr_q = (const int32_t*)(ws + lay.q_ofs);
    a.items_q = (const va::WorkItem*)(ws + lay.q_ofs + lay.q.items_ofs);
    a.max_items_q = lay.q.max_items;
    a.total_tokens = p->total_tokens; a.num_q_heads = p->num_q_heads; a.num_kv_heads = p->num_kv_heads;
    a.head_dim = p->head_dim; a.causal = p->causal; a.scale = p->softmax_scale;
    a.clock_probe_dkdv = clock_probe_slot(1);
    a.clock_probe_dq = clock_probe_slot(2);
    // dQ first: it also writes the row statistics {LSE * log2 e, -Delta} that dK/dV reads
    {
        ProfScope ps(VA_KERNEL_DQ, stream);
        e = va::launch_bwd_dq(a, stream);
    }
    if (e != hipSuccess) return hip_fail(e);
    {
        ProfScope ps(VA_KERNEL_DKDV, stream);
        e = va::launch_bwd_dkdv(a, stream);
    }
    if (e != hipSuccess) return hip_fail(e);
    return VA_OK;
}

const char* varlen_attn_status_string(int status) {
    switch (status) {
        case VA_OK: return "ok";
        case VA_ERR_NULL_PTR: return "a required pointer is NULL";
        case VA_ERR_BAD_SHAPE: return "bad shape: negative size or count, head counts, causal flag, kv_splits, or launch too large";
        case VA_ERR_UNSUPPORTED: return "unsupported: head_dim must be 64, 80, 96 or 128 and the device gfx950";
        case VA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case VA_ERR_BAD_SCALE: return "softmax_scale must be finite and >= 0";
        case VA_ERR_HIP: return "a HIP call failed";
        case VA_ERR_MISALIGNED: return "a tensor or workspace pointer is not 16-byte aligned";
        case VA_ERR_BAD_CU_SEQLENS: return "cu_seqlens must start at 0, never decrease and end at total_tokens";
        case VA_ERR_SCRATCH_LIMIT: return "the call needs more scratch than the library's static array holds (VA_STATIC_SCRATCH_BYTES)";
        default: return "unknown status";
    }
}

int varlen_attn_last_hip_error(void) { return g_last_hip_error; }

int varlen_attn_profile_enable(int on) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (on) prof_clear_locked();
    g_prof_on = on != 0;
    return VA_OK;
}

int varlen_attn_profile_read(int kernel, double* total_ms, int64_t* launches) {
    if (!total_ms || !launches) return VA_ERR_NULL_PTR;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    double sum = 0.0;
    int64_t n = 0;
    for (auto& s : g_prof_samples) {
        if (s.kernel != kernel) continue;
        hipError_t e = hipEventSynchronize(s.b);
        if (e != hipSuccess) return hip_fail(e);
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, s.a, s.b);
        if (e != hipSuccess) return hip_fail(e);
        sum += ms;
        ++n;
    }
    *total_ms = sum;
    *launches = n;
    return VA_OK;
}

int varlen_attn_profile_clock_probe(unsigned long long* device_counters) {
    if (((uintptr_t)device_counters & 7u) != 0) return VA_ERR_MISALIGNED;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    g_clock_probe = device_counters;
    return VA_OK;
}

}  // extern "C"
