// C-ABI of libpard (see include/pard.h): argument checks, plan upload, kernel launches.
#include <cstring>
#include <mutex>
#include <new>

#include "pard_device.hpp"

using namespace pard;

struct pard_plan {
    HostPlan host;
    PlanDev dev;
    void* blob = nullptr;      // one device allocation holding every plan table
    uint32_t* drawn = nullptr; // inside blob: scratch of pard_sub_latency, PARD_MAX_WAIT_SAMPLES * S words
    int device = 0;
    int num_cus = 1;
};

namespace {

constexpr int64_t kHeaderBytes = 256;      // workspace header: word 0 = status bits

int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

// Built-in scratch buffer of pard_estimate_drop_static.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address is looked up once per device and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[PARD_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of the current device's copy of the scratch buffer (nullptr on failure).
void* static_scratch_for_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return nullptr; }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

// Hands the accumulated status bits to the caller and starts the next call from zero.
__global__ void take_status_kernel(uint32_t* __restrict__ src, uint32_t* __restrict__ dst) {
    if (threadIdx.x == 0 && blockIdx.x == 0) { *dst = *src; *src = 0u; }
}

// What the estimate calls themselves use of a workspace: the header alone on the on-chip path, header and
// sort buffers for larger snapshots.
// Layout of a workspace: header | one word per snapshot (marks of the on-chip path) | what the large-snapshot
// path or pard_compact keep there.
int64_t marks_bytes(const pard_plan* p) { return align256((int64_t)p->host.K * 4); }

int64_t estimate_need(const pard_plan* p, int64_t n, int64_t max_snap) {
    if (max_snap <= PARD_FUSED_SNAPSHOT_CAPACITY) return kHeaderBytes + marks_bytes(p);
    return kHeaderBytes + marks_bytes(p) + sort_workspace_bytes(p->host.K, p->host.S, n);
}

// Behind the compaction's own region: what pard_estimate_drop_compact stages for it (survivors of the snapshot
// before each of its queues, one survivor slot per request).
int64_t staging_bytes(const pard_plan* p, int64_t n, int64_t max_snap) {
    if (!compact_per_snapshot(max_snap)) return 0;
    return align256((int64_t)p->host.K * p->host.S * 4) + align256(n * 4);
}

// What pard_workspace_bytes reports: enough for the estimate calls, for pard_compact and for the call that does both.
int64_t workspace_need(const pard_plan* p, int64_t n, int64_t max_snap) {
    int64_t need = compact_workspace_bytes(n, p->host.K) + staging_bytes(p, n, max_snap);
    if (max_snap > PARD_FUSED_SNAPSHOT_CAPACITY) {
        int64_t s = sort_workspace_bytes(p->host.K, p->host.S, n);
        if (s > need) need = s;
    }
    return kHeaderBytes + marks_bytes(p) + need;
}

}  // namespace

extern "C" {

int pard_plan_check(const pard_plan_desc_t* desc, int64_t* total_paths, int32_t* max_path_len) {
    try {
        HostPlan hp;
        int rc = build_host_plan(desc, hp);
        if (rc != PARD_OK) return rc;
        if (total_paths) *total_paths = hp.total_paths;
        if (max_path_len) *max_path_len = hp.max_path_len;
        return PARD_OK;
    } catch (...) {
        return PARD_E_BAD_SHAPE;
    }
}

int pard_plan_create(pard_plan_t** out, const pard_plan_desc_t* desc) {
    if (!out) return PARD_E_NULL;
    *out = nullptr;
    pard_plan* p = nullptr;
    try {
        p = new pard_plan();
        int rc = build_host_plan(desc, p->host);
        if (rc != PARD_OK) { delete p; return rc; }
    } catch (...) {
        delete p;
        return PARD_E_BAD_SHAPE;
    }
    const HostPlan& h = p->host;
    const int64_t b_recs = align256((int64_t)h.recs.size() * (int64_t)sizeof(StageRec));
    const int64_t b_lat = align256((int64_t)h.lat.size() * 4);
    const int64_t b_dep = align256((int64_t)h.dag_entry_ptr.size() * 4);
    const int64_t b_est = align256((int64_t)h.entry_stage.size() * 4 + 4);
    const int64_t b_een = align256((int64_t)h.entry_end.size() * 4 + 4);
    const int64_t b_edg = align256((int64_t)h.entry_dag.size() * 4 + 4);
    const int64_t b_drw = align256((int64_t)PARD_MAX_WAIT_SAMPLES * h.S * 4);
    const int64_t b_spl = align256((int64_t)h.split_in.size() * 8);
    const int64_t total = b_recs + b_lat + b_dep + b_est + b_een + b_edg + 2 * b_spl + b_drw;
    if (hipGetDevice(&p->device) != hipSuccess || hipMalloc(&p->blob, (size_t)total) != hipSuccess) {
        (void)hipGetLastError();
        delete p;
        return PARD_E_HIP;
    }
    char* base = static_cast<char*>(p->blob);
    int64_t off = 0;
    auto put = [&](const void* src, size_t bytes, int64_t span) -> char* {
        char* dst = base + off;
        off += span;
        if (bytes && hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice) != hipSuccess) return nullptr;
        return dst;
    };
    char* d_recs = put(h.recs.data(), h.recs.size() * sizeof(StageRec), b_recs);
    char* d_lat = put(h.lat.data(), h.lat.size() * 4, b_lat);
    char* d_dep = put(h.dag_entry_ptr.data(), h.dag_entry_ptr.size() * 4, b_dep);
    char* d_est = put(h.entry_stage.data(), h.entry_stage.size() * 4, b_est);
    char* d_een = put(h.entry_end.data(), h.entry_end.size() * 4, b_een);
    char* d_edg = put(h.entry_dag.data(), h.entry_dag.size() * 4, b_edg);
    char* d_spi = put(h.split_in.data(), h.split_in.size() * 8, b_spl);
    char* d_spw = put(h.split_whole.data(), h.split_whole.size() * 8, b_spl);
    p->drawn = reinterpret_cast<uint32_t*>(base + off);
    if (!d_recs || !d_lat || !d_dep || !d_est || !d_een || !d_edg || !d_spi || !d_spw) {
        (void)hipGetLastError();
        (void)hipFree(p->blob);
        delete p;
        return PARD_E_HIP;
    }
    {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, p->device) == hipSuccess && prop.multiProcessorCount > 0)
            p->num_cus = prop.multiProcessorCount;
        else
            (void)hipGetLastError();
    }
    PlanDev& d = p->dev;
    d.K = h.K; d.S = h.S; d.shared = h.shared; d.any_fcfs = h.any_fcfs ? 1 : 0;
    d.uniform_mode = h.uniform_mode;
    d.max_entries_per_dag = h.max_entries_per_dag;
    d.presorted_ok = h.short_form_everywhere ? 1 : 0;
    d.recs = reinterpret_cast<const StageRec*>(d_recs);
    d.lat = reinterpret_cast<const int32_t*>(d_lat);
    d.dag_entry_ptr = reinterpret_cast<const int32_t*>(d_dep);
    d.entry_stage = reinterpret_cast<const int32_t*>(d_est);
    d.entry_end = reinterpret_cast<const int32_t*>(d_een);
    d.entry_dag = reinterpret_cast<const int32_t*>(d_edg);
    d.split_in = reinterpret_cast<const int64_t*>(d_spi);
    d.split_whole = reinterpret_cast<const int64_t*>(d_spw);
    d.total_entries = (int64_t)h.entry_stage.size();
    *out = p;
    return PARD_OK;
}

int pard_plan_destroy(pard_plan_t* plan) {
    if (!plan) return PARD_OK;
    int rc = PARD_OK;
    if (plan->blob && hipFree(plan->blob) != hipSuccess) { (void)hipGetLastError(); rc = PARD_E_HIP; }
    delete plan;
    return rc;
}

int pard_plan_info(const pard_plan_t* plan, int64_t* total_paths, int32_t* max_path_len) {
    if (!plan) return PARD_E_NULL;
    if (total_paths) *total_paths = plan->host.total_paths;
    if (max_path_len) *max_path_len = plan->host.max_path_len;
    return PARD_OK;
}

int pard_workspace_bytes(const pard_plan_t* plan, int64_t max_requests, int64_t max_snapshot_requests,
                         int64_t* bytes) {
    if (!plan || !bytes) return PARD_E_NULL;
    if (max_requests < 0 || max_requests >= ((int64_t)1 << 30) || max_snapshot_requests < 0) return PARD_E_BAD_SHAPE;
    if (max_snapshot_requests > PARD_FUSED_SNAPSHOT_CAPACITY &&
        !sort_supported(plan->host.K, plan->host.S, max_requests, max_snapshot_requests)) return PARD_E_UNSUPPORTED;
    *bytes = workspace_need(plan, max_requests, max_snapshot_requests);
    return PARD_OK;
}

static int estimate_drop_impl(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                              const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                              const int32_t* d_snap_ptr, const int32_t* d_now, const int64_t* d_sub, bool consistent,
                              int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                              void* d_workspace, int64_t workspace_bytes, void* stream, bool own_buffer = false,
                              bool stage_survivors = false) {
    if (!plan || !d_snap_ptr || !d_now || !d_seg_ptr) return PARD_E_NULL;
    if (n < 0 || n >= ((int64_t)1 << 30) || max_snapshot_requests < 0) return PARD_E_BAD_SHAPE;
    if (n > 0 && (!d_deadline || !d_stage || !d_est || !d_drop || !d_order)) return PARD_E_NULL;
    if (n > 0 && plan->host.any_fcfs && !d_arrival) return PARD_E_NULL;
    const bool fused = max_snapshot_requests <= PARD_FUSED_SNAPSHOT_CAPACITY;
    if (!fused && !sort_supported(plan->host.K, plan->host.S, n, max_snapshot_requests)) return PARD_E_UNSUPPORTED;
    if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255) != 0 ||
        // a caller's workspace must be the size pard_workspace_bytes reports (it also serves pard_compact); the
        // library's own buffer only has to hold what this call uses
        workspace_bytes < (own_buffer ? estimate_need(plan, n, max_snapshot_requests)
                                      : workspace_need(plan, n, max_snapshot_requests))) return PARD_E_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t* status = static_cast<uint32_t*>(d_workspace);
    hipError_t e;
    if (fused) {
        FusedArgs a{};
        a.plan = plan->dev;
        a.arrival = d_arrival; a.deadline = d_deadline; a.stage = d_stage;
        a.snap_ptr = d_snap_ptr; a.now = d_now;
        a.est = d_est; a.drop = d_drop; a.order = d_order; a.seg_ptr = d_seg_ptr;
        a.sub = d_sub;
        a.status = status;
        a.todo = reinterpret_cast<uint32_t*>(static_cast<char*>(d_workspace) + kHeaderBytes);
        if (stage_survivors) {
            // the compaction's region starts with its per-snapshot counts; the staging arrays follow the region
            char* region = static_cast<char*>(d_workspace) + kHeaderBytes + marks_bytes(plan);
            char* stage = region + compact_workspace_bytes(n, plan->host.K);
            a.kept = reinterpret_cast<uint32_t*>(region);
            a.loc_ptr = reinterpret_cast<int32_t*>(stage);
            a.staged = reinterpret_cast<int32_t*>(stage + align256((int64_t)plan->host.K * plan->host.S * 4));
        }
        a.cap = (int32_t)max_snapshot_requests;
        a.consistent = consistent ? 1 : 0;
        a.n = n;
        e = launch_fused(a, s);
    } else {
        SortArgs a{};
        a.plan = plan->dev;
        a.n = n;
        a.max_snapshot = max_snapshot_requests;
        a.arrival = d_arrival; a.deadline = d_deadline; a.stage = d_stage;
        a.snap_ptr = d_snap_ptr; a.now = d_now;
        a.est = d_est; a.drop = d_drop; a.order = d_order; a.seg_ptr = d_seg_ptr;
        a.sub = d_sub;
        a.consistent = consistent ? 1 : 0;
        a.status = status;
        a.workspace = static_cast<char*>(d_workspace) + kHeaderBytes + marks_bytes(plan);
        a.num_cus = plan->num_cus;
        e = launch_sort_path(a, s);
    }
    return e == hipSuccess ? PARD_OK : PARD_E_HIP;
}

int pard_estimate_drop(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                       const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                       const int32_t* d_snap_ptr, const int32_t* d_now,
                       int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                       void* d_workspace, int64_t workspace_bytes, void* stream) {
    return estimate_drop_impl(plan, n, max_snapshot_requests, d_arrival, d_deadline, d_stage, d_snap_ptr, d_now, nullptr, false,
                              d_est, d_drop, d_order, d_seg_ptr, d_workspace, workspace_bytes, stream);
}

int pard_estimate_drop_static(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                              const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                              const int32_t* d_snap_ptr, const int32_t* d_now,
                              int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                              uint32_t* d_status, void* stream) {
    if (!plan) return PARD_E_NULL;
    if (n < 0 || n >= ((int64_t)1 << 30) || max_snapshot_requests < 0) return PARD_E_BAD_SHAPE;
    // what the call will use of the buffer: the header alone on the on-chip path, header + sort buffers above it
    if (max_snapshot_requests > PARD_FUSED_SNAPSHOT_CAPACITY &&
        !sort_supported(plan->host.K, plan->host.S, n, max_snapshot_requests)) return PARD_E_UNSUPPORTED;
    if (estimate_need(plan, n, max_snapshot_requests) > (int64_t)PARD_STATIC_SCRATCH_BYTES) return PARD_E_SCRATCH;
    void* ptr = static_scratch_for_current_device();
    if (!ptr) return PARD_E_HIP;
    const int rc = estimate_drop_impl(plan, n, max_snapshot_requests, d_arrival, d_deadline, d_stage, d_snap_ptr, d_now, nullptr,
                                      false, d_est, d_drop, d_order, d_seg_ptr, ptr, (int64_t)PARD_STATIC_SCRATCH_BYTES, stream, true);
    if (rc != PARD_OK) return rc;
    if (d_status) {
        take_status_kernel<<<1, 64, 0, static_cast<hipStream_t>(stream)>>>(static_cast<uint32_t*>(ptr), d_status);
        if (hipGetLastError() != hipSuccess) return PARD_E_HIP;
    }
    return PARD_OK;
}

int pard_estimate_drop_compact(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                               const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                               const int32_t* d_snap_ptr, const int32_t* d_now,
                               int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                               int32_t* d_surv_idx, int32_t* d_surv_ptr,
                               void* d_workspace, int64_t workspace_bytes, void* between_event, void* stream) {
    if (!plan || !d_surv_ptr) return PARD_E_NULL;
    if (n > 0 && !d_surv_idx) return PARD_E_NULL;
    const bool prepared = n > 0 && max_snapshot_requests >= 0 && compact_per_snapshot(max_snapshot_requests);
    int rc = estimate_drop_impl(plan, n, max_snapshot_requests, d_arrival, d_deadline, d_stage, d_snap_ptr, d_now, nullptr, false,
                                d_est, d_drop, d_order, d_seg_ptr, d_workspace, workspace_bytes, stream, false, prepared);
    if (rc != PARD_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (between_event && hipEventRecord(static_cast<hipEvent_t>(between_event), s) != hipSuccess) {
        (void)hipGetLastError();
        return PARD_E_HIP;
    }
    if (!prepared)
        return pard_compact(plan, n, max_snapshot_requests, d_order, d_seg_ptr, d_drop, d_surv_idx, d_surv_ptr, d_workspace,
                            workspace_bytes, stream);
    char* region = static_cast<char*>(d_workspace) + kHeaderBytes + marks_bytes(plan);
    char* stage = region + compact_workspace_bytes(n, plan->host.K);
    CompactArgs a{};
    a.num_segments = plan->host.K * plan->host.S;
    a.stages = plan->host.S;
    a.max_snapshot = max_snapshot_requests;
    a.n = n;
    a.order = d_order; a.seg_ptr = d_seg_ptr; a.drop = d_drop;
    a.surv_idx = d_surv_idx; a.surv_ptr = d_surv_ptr;
    a.status = static_cast<uint32_t*>(d_workspace);
    a.workspace = region;
    a.kept = reinterpret_cast<const uint32_t*>(region);
    a.loc_ptr = reinterpret_cast<const int32_t*>(stage);
    a.staged = reinterpret_cast<const int32_t*>(stage + align256((int64_t)plan->host.K * plan->host.S * 4));
    return launch_compact(a, s) == hipSuccess ? PARD_OK : PARD_E_HIP;
}

int pard_estimate_drop_sub(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                           const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                           const int32_t* d_snap_ptr, const int32_t* d_now, const int64_t* d_sub,
                           int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                           void* d_workspace, int64_t workspace_bytes, void* stream) {
    if (!d_sub) return PARD_E_NULL;
    return estimate_drop_impl(plan, n, max_snapshot_requests, d_arrival, d_deadline, d_stage, d_snap_ptr, d_now, d_sub, false,
                              d_est, d_drop, d_order, d_seg_ptr, d_workspace, workspace_bytes, stream);
}

int pard_estimate_drop_consistent(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                                  const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                                  const int32_t* d_snap_ptr, const int32_t* d_now, const int64_t* d_sub,
                                  int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                                  void* d_workspace, int64_t workspace_bytes, void* stream) {
    return estimate_drop_impl(plan, n, max_snapshot_requests, d_arrival, d_deadline, d_stage, d_snap_ptr, d_now, d_sub, true,
                              d_est, d_drop, d_order, d_seg_ptr, d_workspace, workspace_bytes, stream);
}

int pard_estimate_drop_ranked(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                              const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                              const int32_t* d_snap_ptr, const int32_t* d_now,
                              int32_t* d_est, uint8_t* d_drop, int32_t* d_order, int32_t* d_seg_ptr,
                              void* d_workspace, int64_t workspace_bytes, void* stream) {
    const int rc = estimate_drop_impl(plan, n, max_snapshot_requests, d_arrival, d_deadline, d_stage, d_snap_ptr, d_now, nullptr,
                                      false, d_est, d_drop, d_order, d_seg_ptr, d_workspace, workspace_bytes, stream);
    if (rc != PARD_OK) return rc;
    RankedArgs a{};
    a.plan = plan->dev;
    a.n = n;
    a.deadline = d_deadline; a.now = d_now;
    a.order = d_order; a.seg_ptr = d_seg_ptr;
    a.est = d_est; a.drop = d_drop;
    a.max_snapshot = max_snapshot_requests;
    a.num_cus = plan->num_cus;
    return launch_ranked(a, static_cast<hipStream_t>(stream)) == hipSuccess ? PARD_OK : PARD_E_HIP;
}

int pard_queue_lengths(const pard_plan_t* plan, int64_t n, const int32_t* d_stage, const int32_t* d_snap_ptr,
                       int32_t* d_qlen, void* stream) {
    if (!plan || !d_snap_ptr || !d_qlen) return PARD_E_NULL;
    if (n < 0 || n >= ((int64_t)1 << 30)) return PARD_E_BAD_SHAPE;
    if (n > 0 && !d_stage) return PARD_E_NULL;
    hipError_t e = launch_queue_lengths(plan->dev, n, d_stage, d_snap_ptr, d_qlen, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PARD_OK : PARD_E_HIP;
}

static int sub_latency_impl(const pard_plan_t* plan, const int32_t* d_qlen, const int32_t* d_qdelay, int32_t variant,
                            int64_t lambda_num, int64_t lambda_den, int32_t num_samples,
                            const int32_t* d_samples, const uint32_t* d_picks, int64_t* d_sub, void* stream) {
    if (!plan || !d_qlen || !d_sub) return PARD_E_NULL;
    if (variant < PARD_SUB_FULL || variant > PARD_SUB_BACK) return PARD_E_BAD_SHAPE;
    SubArgs a{};
    a.plan = plan->dev;
    a.qlen = d_qlen;
    a.qdelay = d_qdelay;
    a.variant = variant;
    a.sub = reinterpret_cast<unsigned long long*>(d_sub);
    if (variant == PARD_SUB_FULL) {
        if (lambda_den <= 0 || lambda_num < 0 || lambda_num > lambda_den) return PARD_E_BAD_SHAPE;
        if (lambda_num == 0) a.variant = PARD_SUB_LOWER;                 // F^-1(0) = 0
        else if (lambda_num == lambda_den) a.variant = PARD_SUB_UPPER;   // F^-1(1) = sum d_i
        else {
            if (num_samples < 1 || num_samples > PARD_MAX_WAIT_SAMPLES) return PARD_E_BAD_SHAPE;
            if (!d_samples || !d_picks) return PARD_E_NULL;
            if (plan->host.max_lat > PARD_MAX_WAIT_LATENCY) return PARD_E_UNSUPPORTED;
            // ceil(lambda * M), in 1..M
            const unsigned __int128 num = (unsigned __int128)lambda_num * (unsigned)num_samples + (unsigned __int128)(lambda_den - 1);
            a.rank = (int64_t)(num / (unsigned __int128)lambda_den);
            a.num_samples = num_samples;
            a.samples = d_samples;
            a.picks = d_picks;
            a.drawn = plan->drawn;
        }
    }
    hipError_t e = launch_sub_latency(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PARD_OK : PARD_E_HIP;
}

int pard_sub_latency(const pard_plan_t* plan, const int32_t* d_qlen, int32_t variant,
                     int64_t lambda_num, int64_t lambda_den, int32_t num_samples,
                     const int32_t* d_samples, const uint32_t* d_picks, int64_t* d_sub, void* stream) {
    return sub_latency_impl(plan, d_qlen, nullptr, variant, lambda_num, lambda_den, num_samples, d_samples, d_picks, d_sub, stream);
}

int pard_sub_latency_q(const pard_plan_t* plan, const int32_t* d_qlen, const int32_t* d_qdelay, int32_t variant,
                       int64_t lambda_num, int64_t lambda_den, int32_t num_samples,
                       const int32_t* d_samples, const uint32_t* d_picks, int64_t* d_sub, void* stream) {
    if (!d_qdelay) return PARD_E_NULL;
    return sub_latency_impl(plan, d_qlen, d_qdelay, variant, lambda_num, lambda_den, num_samples, d_samples, d_picks, d_sub, stream);
}

int pard_queue_delay(const pard_plan_t* plan, int32_t series_len, int64_t window_us, const int32_t* d_time,
                     const int32_t* d_delay, const int32_t* d_now, int32_t* d_q, void* stream) {
    if (!plan || !d_now || !d_q) return PARD_E_NULL;
    if (series_len < 0 || series_len > PARD_MAX_DELAY_SAMPLES || window_us < 1 || window_us > 0x7fffffff) return PARD_E_BAD_SHAPE;
    if (series_len > 0 && (!d_time || !d_delay)) return PARD_E_NULL;
    hipError_t e = launch_queue_delay(plan->host.K, plan->host.S, series_len, (uint32_t)window_us, d_time, d_delay, d_now, d_q,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PARD_OK : PARD_E_HIP;
}

int pard_priority_modes(const pard_plan_t* plan, int32_t series_len, int32_t window, const int32_t* d_rate,
                        const int32_t* d_prev_mode, int32_t* d_mode, void* stream) {
    if (!plan || !d_rate || !d_mode) return PARD_E_NULL;
    if (series_len < 1 || window < 1) return PARD_E_BAD_SHAPE;
    hipError_t e = launch_priority_modes(plan->dev, series_len, window, d_rate, d_prev_mode, d_mode,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PARD_OK : PARD_E_HIP;
}

int pard_plan_set_modes(pard_plan_t* plan, const int32_t* d_mode, void* stream) {
    if (!plan || !d_mode) return PARD_E_NULL;
    const int64_t count = (int64_t)plan->host.D * plan->host.S;
    hipError_t e = launch_set_modes(const_cast<StageRec*>(plan->dev.recs), d_mode, count, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return PARD_E_HIP;
    plan->host.uniform_mode = -1;          // the stages' modes now live on the device only
    plan->dev.uniform_mode = -1;
    return PARD_OK;
}

int pard_reactive_drop(const pard_plan_t* plan, int32_t policy, int64_t n,
                       const int32_t* d_arrival, const int32_t* d_deadline, const int32_t* d_stage,
                       const int32_t* d_snap_ptr, const int32_t* d_now, const int32_t* d_order, const int32_t* d_seg_ptr,
                       uint8_t* d_drop, int32_t* d_first_kept, void* stream) {
    if (!plan || !d_now) return PARD_E_NULL;
    if (n < 0 || n >= ((int64_t)1 << 30) || (policy != PARD_REACTIVE_WINDOW_SCAN && policy != PARD_REACTIVE_SLO_SPLIT))
        return PARD_E_BAD_SHAPE;
    if (n > 0 && (!d_deadline || !d_drop)) return PARD_E_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (policy == PARD_REACTIVE_WINDOW_SCAN) {
        if (!d_seg_ptr || !d_first_kept || (n > 0 && !d_order)) return PARD_E_NULL;
        e = launch_window_scan(plan->dev, n, d_deadline, d_order, d_seg_ptr, d_now, d_drop, d_first_kept, s);
    } else {
        if (!d_snap_ptr || (n > 0 && (!d_arrival || !d_stage))) return PARD_E_NULL;
        if (!plan->host.split_fits) return PARD_E_UNSUPPORTED;
        e = launch_slo_split(plan->dev, n, d_arrival, d_deadline, d_stage, d_snap_ptr, d_now, d_drop, s);
    }
    return e == hipSuccess ? PARD_OK : PARD_E_HIP;
}

int pard_compact(const pard_plan_t* plan, int64_t n, int64_t max_snapshot_requests,
                 const int32_t* d_order, const int32_t* d_seg_ptr, const uint8_t* d_drop,
                 int32_t* d_surv_idx, int32_t* d_surv_ptr,
                 void* d_workspace, int64_t workspace_bytes, void* stream) {
    if (!plan || !d_seg_ptr || !d_surv_ptr) return PARD_E_NULL;
    if (n < 0 || n >= ((int64_t)1 << 30) || max_snapshot_requests < 0) return PARD_E_BAD_SHAPE;
    if (n > 0 && (!d_order || !d_drop || !d_surv_idx)) return PARD_E_NULL;
    if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) & 255) != 0 ||
        workspace_bytes < kHeaderBytes + marks_bytes(plan) + compact_workspace_bytes(n, plan->host.K)) return PARD_E_WORKSPACE;
    CompactArgs a{};
    a.num_segments = plan->host.K * plan->host.S;
    a.stages = plan->host.S;
    a.max_snapshot = max_snapshot_requests;
    a.n = n;
    a.order = d_order; a.seg_ptr = d_seg_ptr; a.drop = d_drop;
    a.surv_idx = d_surv_idx; a.surv_ptr = d_surv_ptr;
    a.status = static_cast<uint32_t*>(d_workspace);
    a.workspace = static_cast<char*>(d_workspace) + kHeaderBytes + marks_bytes(plan);
    hipError_t e = launch_compact(a, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? PARD_OK : PARD_E_HIP;
}

const char* pard_strerror(int status) {
    switch (status) {
        case PARD_OK: return "ok";
        case PARD_E_NULL: return "a required pointer is NULL";
        case PARD_E_BAD_SHAPE: return "bad shape: snapshots, stages or request count out of range";
        case PARD_E_BAD_BATCH: return "batch size outside 1..64";
        case PARD_E_BAD_WORKERS: return "worker count outside 1..2^20";
        case PARD_E_BAD_LATENCY: return "negative latency";
        case PARD_E_BAD_DAG: return "malformed DAG: bad offsets, edge out of range, self loop or cycle";
        case PARD_E_TOO_MANY_PATHS: return "DAG expands to too many paths";
        case PARD_E_WORKSPACE: return "workspace missing, misaligned or too small";
        case PARD_E_HIP: return "HIP runtime error";
        case PARD_E_BAD_MODE: return "unknown order mode";
        case PARD_E_SCRATCH: return "the call needs more than the library's built-in scratch buffer holds (PARD_STATIC_SCRATCH_BYTES)";
        case PARD_E_UNSUPPORTED: return "not supported: bits of the snapshot bound plus bits of the queue count above 32 on the large-snapshot path, or a latency above 2^25 us for the sampled batch wait";
        default: return "unknown status";
    }
}

}  // extern "C"
