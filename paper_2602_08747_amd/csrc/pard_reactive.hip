// Reactive dropping policies on the same snapshots (paper Section 5.1, "Baselines"): what the proactive
// estimate is compared with.  Both are data-parallel over the queues the estimate call has ordered.
//
// Window scan (the policy the paper describes for Nexus): the queue is scanned in the order given with a
// window of one batch; the scan stops at the first window whose requests can all still finish the current
// module, and everything before it is dropped.  With n requests in the queue and batch size B the window at
// position p holds w = min(B, n - p) requests, runs as a batch of w and ends at now + lat[w]; it fits when no
// deadline in it is earlier.  Three steps:
//   1. every window of full size at once: a request is "late" when its deadline is before now + lat[B]; a
//      wave holds the late bits of 64 consecutive queue slots and of the 64 after them, a window fits when
//      its B bits are clear; the lowest fitting position of a queue is kept with an atomic minimum
//   2. queues without a fitting full window: one wave per queue tries the cut-off windows at the queue's end
//      (fewer than 64 requests, each window size has its own latency)
//   3. drop[request] = its queue position is before the first fitting window.
//
// Per-module SLO split (Clipper++): a request is dropped once the time since it was sent exceeds the budgets
// of the modules up to and including its own, SLO * P_k / T_k, with P_k the summed execution durations along
// the longest way from a source to its module and T_k the longest whole path through it (both tabulated in the
// plan).  now - arrival > SLO P_k / T_k  <=>  (now - arrival) T_k > SLO P_k  in integers: no division.
#include "pard_device.hpp"

namespace pard {

namespace {

constexpr int kRxThreads = 256;
constexpr int kRxChunks = 16;                            // chunks of 64 queue slots a wave walks
constexpr int kRxTile = kRxThreads / kWave * kRxChunks * kWave;   // queue slots per workgroup
constexpr int32_t kNoWindow = 0x7fffffff;

// The queue that holds slot j: the last g in [lo, hi] with seg_ptr[g] <= j (queues may be empty).
__device__ __forceinline__ int queue_of_slot(const int32_t* seg_ptr, int64_t j, int lo, int hi) {
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int64_t)seg_ptr[mid] <= j) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__global__ void window_init_kernel(int32_t* first, int32_t num_queues) {
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g < num_queues) first[g] = kNoWindow;
}

struct WindowArgs {
    PlanDev plan;
    int64_t n;
    const int32_t *deadline, *order, *seg_ptr, *now;
    uint8_t* drop;
    int32_t* first;
};

// Step 1.
__global__ __launch_bounds__(kRxThreads) void window_scan_kernel(WindowArgs A) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int G = A.plan.K * A.plan.S, S = A.plan.S;
    const int64_t t0 = ((int64_t)blockIdx.x * (kRxThreads / kWave) + wave) * (kRxChunks * kWave);
    if (t0 >= A.n) return;
    int64_t t1 = t0 + (kRxChunks + 1) * kWave;            // one chunk of look-ahead
    if (t1 > A.n) t1 = A.n;
    const int g_lo = queue_of_slot(A.seg_ptr, t0, 0, G - 1), g_hi = queue_of_slot(A.seg_ptr, t1 - 1, g_lo, G - 1);

    // state of the previous chunk, whose windows are settled once the late bits of this chunk are known
    unsigned long long late_prev = 0;
    int g_prev = 0;
    int32_t pos_prev = 0, batch_prev = 0;
    bool start_prev = false;                                // the lane's slot starts a window of full size
    for (int c = 0; c <= kRxChunks; ++c) {
        const int64_t j = t0 + (int64_t)c * kWave + lane;
        const bool in = j < A.n;
        int g = g_lo;
        int32_t pos = 0, batch = 1;
        bool late = false, start = false;
        if (in) {
            g = queue_of_slot(A.seg_ptr, j, g_lo, g_hi);
            const int u = g / S;
            const StageRec& r = A.plan.recs[A.plan.shared ? g - u * S : g];
            const int32_t a = A.seg_ptr[g], len = A.seg_ptr[g + 1] - a;
            pos = (int32_t)(j - a);
            batch = r.B;
            const int32_t dl = A.deadline[A.order[j]];
            late = (int64_t)A.now[u] + (int64_t)r.latB > (int64_t)dl;
            start = c < kRxChunks && pos + batch <= len;    // the look-ahead chunk starts no windows of this wave
        }
        const unsigned long long late_now = __ballot(late);
        if (c > 0) {
            // the B slots from the previous chunk's lane on: bits lane.. of late_prev, then the low bits of late_now
            const unsigned long long seen = (late_prev >> lane) | (lane ? late_now << (kWave - lane) : 0ull);
            const unsigned long long mask = batch_prev >= kWave ? ~0ull : (1ull << batch_prev) - 1ull;
            const bool fits = start_prev && (seen & mask) == 0ull;
            // the lowest fitting position of a queue inside this chunk reports it
            const int g_left = __shfl_up(g_prev, 1);
            const bool fits_left = __shfl_up((int)fits, 1) != 0;
            if (fits && (lane == 0 || !fits_left || g_left != g_prev)) {
                if (__hip_atomic_load(A.first + g_prev, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > pos_prev)
                    atomicMin(A.first + g_prev, pos_prev);
            }
        }
        late_prev = late_now;
        g_prev = g; pos_prev = pos; batch_prev = batch; start_prev = start;
    }
}

// Step 2: one wave per queue.
__global__ __launch_bounds__(kWave) void window_tail_kernel(WindowArgs A) {
    const int lane = threadIdx.x;
    const int g = blockIdx.x, S = A.plan.S;
    const int32_t a = A.seg_ptr[g], len = A.seg_ptr[g + 1] - a;
    const int32_t found = A.first[g];
    if (found != kNoWindow) return;
    const int u = g / S;
    const int rec = A.plan.shared ? g - u * S : g;
    const int32_t B = A.plan.recs[rec].B;
    const int32_t* lat = A.plan.lat + (int64_t)rec * PARD_LAT_ENTRIES;
    const int64_t now = A.now[u];
    // the windows that are cut off by the queue's end hold fewer than B <= 64 requests: the last `cnt` slots
    const int32_t cnt = len < kWave - 1 ? len : kWave - 1;
    const int32_t my_pos = len - cnt + lane;
    const bool have = lane < cnt;
    const int64_t dl = have ? (int64_t)A.deadline[A.order[(int64_t)a + my_pos]] : 0;
    const int32_t p0 = len >= B ? len - B + 1 : 0;          // first position whose window is cut off
    int32_t first = len;
    for (int32_t p = p0; p < len; ++p) {
        const int32_t w = len - p;
        const int64_t batch_end = now + (int64_t)lat[w - 1];
        if (__ballot(have && my_pos >= p && batch_end > dl) == 0ull) { first = p; break; }
    }
    if (lane == 0) A.first[g] = first;
}

// Step 3.
__global__ __launch_bounds__(kRxThreads) void window_mask_kernel(WindowArgs A) {
    const int G = A.plan.K * A.plan.S;
    const int64_t t0 = (int64_t)blockIdx.x * kRxTile;
    int64_t t1 = t0 + kRxTile;
    if (t1 > A.n) t1 = A.n;
    if (t0 >= t1) return;
    const int g_lo = queue_of_slot(A.seg_ptr, t0, 0, G - 1), g_hi = queue_of_slot(A.seg_ptr, t1 - 1, g_lo, G - 1);
    for (int64_t j = t0 + threadIdx.x; j < t1; j += kRxThreads) {
        const int g = queue_of_slot(A.seg_ptr, j, g_lo, g_hi);
        A.drop[A.order[j]] = (int32_t)(j - A.seg_ptr[g]) < A.first[g] ? 1 : 0;
    }
}

struct SplitArgs {
    PlanDev plan;
    int64_t n;
    const int32_t *arrival, *deadline, *stage, *snap_ptr, *now;
    uint8_t* drop;
};

// The snapshot that holds request r: the last u in [lo, hi] with snap_ptr[u] <= r.
__device__ __forceinline__ int snapshot_of_request(const int32_t* snap_ptr, int64_t r, int lo, int hi) {
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int64_t)snap_ptr[mid] <= r) lo = mid; else hi = mid - 1;
    }
    return lo;
}

constexpr int kSplitPerThread = 4;
__global__ __launch_bounds__(kRxThreads) void slo_split_kernel(SplitArgs A) {
    const int64_t t0 = (int64_t)blockIdx.x * (kRxThreads * kSplitPerThread);
    int64_t t1 = t0 + kRxThreads * kSplitPerThread;
    if (t1 > A.n) t1 = A.n;
    if (t0 >= t1) return;
    const int K = A.plan.K, S = A.plan.S;
    const int u_lo = snapshot_of_request(A.snap_ptr, t0, 0, K - 1), u_hi = snapshot_of_request(A.snap_ptr, t1 - 1, u_lo, K - 1);
#pragma unroll
    for (int i = 0; i < kSplitPerThread; ++i) {
        const int64_t r = t0 + (int64_t)i * kRxThreads + threadIdx.x;
        if (r >= t1) continue;
        const int u = snapshot_of_request(A.snap_ptr, r, u_lo, u_hi);
        const int k = clamp_stage(A.stage[r], S);
        const int64_t rec = (int64_t)(A.plan.shared ? 0 : u) * S + k;
        const int64_t way_in = A.plan.split_in[rec], whole = A.plan.split_whole[rec];
        const int64_t used = (int64_t)A.now[u] - (int64_t)A.arrival[r];
        const int64_t slo = (int64_t)A.deadline[r] - (int64_t)A.arrival[r];
        // |used|, |slo| < 2^33 and the path sums are below 2^30 (checked when the plan was made): the products fit 64 bits
        A.drop[r] = (whole == 0 ? used > slo : used * whole > slo * way_in) ? 1 : 0;
    }
}

}  // namespace

hipError_t launch_window_scan(const PlanDev& plan, int64_t n, const int32_t* deadline, const int32_t* order, const int32_t* seg_ptr,
                              const int32_t* now, uint8_t* drop, int32_t* first, hipStream_t stream) {
    WindowArgs a{plan, n, deadline, order, seg_ptr, now, drop, first};
    const int G = plan.K * plan.S;
    window_init_kernel<<<(G + 255) / 256, 256, 0, stream>>>(first, G);
    if (n > 0) {
        const int64_t per_block = (int64_t)(kRxThreads / kWave) * kRxChunks * kWave;
        window_scan_kernel<<<(unsigned)((n + per_block - 1) / per_block), kRxThreads, 0, stream>>>(a);
    }
    window_tail_kernel<<<(unsigned)G, kWave, 0, stream>>>(a);
    if (n > 0) window_mask_kernel<<<(unsigned)((n + kRxTile - 1) / kRxTile), kRxThreads, 0, stream>>>(a);
    return hipGetLastError();
}

hipError_t launch_slo_split(const PlanDev& plan, int64_t n, const int32_t* arrival, const int32_t* deadline, const int32_t* stage,
                            const int32_t* snap_ptr, const int32_t* now, uint8_t* drop, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    SplitArgs a{plan, n, arrival, deadline, stage, snap_ptr, now, drop};
    const int64_t per_block = kRxThreads * kSplitPerThread;
    slo_split_kernel<<<(unsigned)((n + per_block - 1) / per_block), kRxThreads, 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace pard
