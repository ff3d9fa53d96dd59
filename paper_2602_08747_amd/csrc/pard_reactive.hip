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
constexpr int32_t kNoWindow = 0x7fffffff;

// The queue that holds slot j: the last g in [lo, hi] with seg_ptr[g] <= j (queues may be empty).  The slot is the
// same in every lane of a wave and all 64 lanes call this: each round the lanes probe 64 evenly spaced queues at
// once, so thousands of queues take three dependent loads instead of fifteen.
__device__ __forceinline__ int queue_of_slot_wave(const int32_t* seg_ptr, int64_t j, int lo, int hi, int lane) {
    while (hi > lo) {
        const int step = (hi - lo + kWave - 1) / kWave;
        const int probe = lo + (lane + 1) * step;
        const bool le = probe <= hi && (int64_t)seg_ptr[probe] <= j;       // offsets never fall: these lanes are a prefix
        const int below = __popcll(__ballot(le));
        lo += below * step;
        hi = lo + step - 1 < hi ? lo + step - 1 : hi;
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
    int32_t mask_cap;                                       // snapshots of at most this many requests get their mask from
                                                            // window_mask_snapshot_kernel (0: none do)
};

// What a lane keeps about the queue its slots are in; reloaded only when the queue changes along the walk.
struct QueueView {
    int g;
    int32_t start, len, batch;
    int64_t batch_end;                                      // now + lat[B]
};

__device__ __forceinline__ void look_at_queue(const WindowArgs& A, int g, QueueView& q) {
    const int S = A.plan.S;
    const int u = g / S;
    const StageRec& r = A.plan.recs[A.plan.shared ? g - u * S : g];
    q.g = g;
    q.start = A.seg_ptr[g];
    q.len = A.seg_ptr[g + 1] - q.start;
    q.batch = r.B;
    q.batch_end = (int64_t)A.now[u] + (int64_t)r.latB;
}

// Step 1.  A wave walks kRxChunks chunks of 64 slots plus one chunk of look-ahead.  All its loads are issued before
// anything is decided: the slots' request ids first, then the deadlines they point at (two round trips to memory
// for the whole walk instead of two per chunk).
__global__ __launch_bounds__(kRxThreads) void window_scan_kernel(WindowArgs A) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int G = A.plan.K * A.plan.S;
    const int64_t t0 = ((int64_t)blockIdx.x * (kRxThreads / kWave) + wave) * (kRxChunks * kWave);
    if (t0 >= A.n) return;
    int64_t t1 = t0 + (kRxChunks + 1) * kWave;            // one chunk of look-ahead
    if (t1 > A.n) t1 = A.n;
    const int g_lo = queue_of_slot_wave(A.seg_ptr, t0, 0, G - 1, lane), g_hi = queue_of_slot_wave(A.seg_ptr, t1 - 1, g_lo, G - 1, lane);
    // A walk that lies inside one queue has nothing to add once a fitting window before its first slot is known
    // (workgroups start roughly in the order of the slots, so the earlier part of a queue has usually reported).
    if (g_lo == g_hi) {
        const int32_t known = __hip_atomic_load(A.first + g_lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((int64_t)known <= t0 - (int64_t)A.seg_ptr[g_lo]) return;
    }
    int32_t req[kRxChunks + 1], dl[kRxChunks + 1];
#pragma unroll
    for (int c = 0; c <= kRxChunks; ++c) {
        const int64_t j = t0 + (int64_t)c * kWave + lane;
        req[c] = j < t1 ? A.order[j] : -1;
    }
#pragma unroll
    for (int c = 0; c <= kRxChunks; ++c) dl[c] = req[c] >= 0 ? A.deadline[req[c]] : 0;

    QueueView q;
    look_at_queue(A, g_lo, q);
    // state of the previous chunk, whose windows are settled once the late bits of this chunk are known
    unsigned long long late_prev = 0;
    int g_prev = 0;
    int32_t pos_prev = 0, batch_prev = 0;
    bool start_prev = false;                                // the lane's slot starts a window of full size
    int reported = -1;                                      // the highest queue this wave has reported a position for
#pragma unroll
    for (int c = 0; c <= kRxChunks; ++c) {
        const int64_t j = t0 + (int64_t)c * kWave + lane;
        const bool in = j < t1;
        int32_t pos = 0;
        bool late = false, start = false;
        if (in) {
            // the slots of a lane rise along the walk, so its queue only moves forward (empty queues are stepped over)
            while (q.g < g_hi && j >= (int64_t)q.start + q.len) look_at_queue(A, q.g + 1, q);
            pos = (int32_t)(j - q.start);
            late = q.batch_end > (int64_t)dl[c];
            start = c < kRxChunks && pos + q.batch <= q.len;   // the look-ahead chunk starts no windows of this wave
        }
        const int g = in ? q.g : g_lo;
        const int32_t batch = in ? q.batch : 1;
        const unsigned long long late_now = __ballot(late);
        if (c > 0) {
            // the B slots from the previous chunk's lane on: bits lane.. of late_prev, then the low bits of late_now
            const unsigned long long seen = (late_prev >> lane) | (lane ? late_now << (kWave - lane) : 0ull);
            const unsigned long long mask = batch_prev >= kWave ? ~0ull : (1ull << batch_prev) - 1ull;
            const bool fits = start_prev && (seen & mask) == 0ull;
            // the lowest fitting position of a queue inside this chunk reports it
            const int g_left = __shfl_up(g_prev, 1);
            const bool fits_left = __shfl_up((int)fits, 1) != 0;
            // ... once per wave: positions rise along the walk, so a queue that has reported has nothing lower to add
            const bool reports = fits && g_prev > reported && (lane == 0 || !fits_left || g_left != g_prev);
            if (reports) {
                if (__hip_atomic_load(A.first + g_prev, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > pos_prev)
                    atomicMin(A.first + g_prev, pos_prev);
            }
            const unsigned long long who = __ballot(reports);
            if (who) reported = __builtin_amdgcn_readlane(g_prev, 63 - __clzll((long long)who));   // queues rise with the lanes
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

// Step 3.  The queue slots of a snapshot hold exactly the snapshot's own requests, which are neighbours in the
// request arrays: a snapshot of at most kMaskCap requests gets one workgroup that collects its decisions in LDS by
// request and writes them out in request order (one byte per request written straight from the queue slots costs a
// write request per cache line touched: 126 us for 33.5 million requests against 38 this way).
constexpr int kMaskCap = 16384;
constexpr int kMaskThreads = 256;
__global__ __launch_bounds__(kMaskThreads) void window_mask_snapshot_kernel(WindowArgs A) {
    __shared__ __align__(16) uint8_t mask[kMaskCap];
    __shared__ int32_t qstart[PARD_MAX_STAGES + 1];
    __shared__ int32_t qfirst[PARD_MAX_STAGES];
    const int S = A.plan.S, u = blockIdx.x, tid = threadIdx.x;
    const int64_t lo = A.seg_ptr[(int64_t)u * S], hi = A.seg_ptr[(int64_t)(u + 1) * S];
    const int64_t m = hi - lo;
    if (lo < 0 || hi > A.n || m <= 0 || m > (int64_t)A.mask_cap) return;          // larger ones: window_mask_kernel
    if (tid <= S) qstart[tid] = A.seg_ptr[(int64_t)u * S + tid];
    if (tid < S) qfirst[tid] = A.first[(int64_t)u * S + tid];
    for (int i = tid * 4; i < (int)m; i += kMaskThreads * 4) *reinterpret_cast<uint32_t*>(&mask[i]) = 0u;
    __syncthreads();
    const bool vec = (reinterpret_cast<uintptr_t>(A.order) & 15) == 0 && (lo & 3) == 0;
    for (int64_t j0 = lo + (int64_t)tid * 4; j0 < hi; j0 += kMaskThreads * 4) {
        int32_t req[4];
        if (vec && j0 + 3 < hi) {
            const int4 v = *reinterpret_cast<const int4*>(A.order + j0);
            req[0] = v.x; req[1] = v.y; req[2] = v.z; req[3] = v.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) req[c] = j0 + c < hi ? A.order[j0 + c] : -1;
        }
        int g = 0, top = S - 1;                              // the queue of slot j0: the last g with qstart[g] <= j0
        while (g < top) {
            const int mid = (g + top + 1) >> 1;
            if ((int64_t)qstart[mid] <= j0) g = mid; else top = mid - 1;
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int64_t j = j0 + c;
            if (j >= hi) break;
            while (g < S - 1 && j >= (int64_t)qstart[g + 1]) ++g;
            const uint8_t d = (int32_t)(j - qstart[g]) < qfirst[g] ? 1 : 0;
            const int64_t at = (int64_t)req[c] - lo;
            if (at >= 0 && at < m) mask[at] = d;
            else if (req[c] >= 0 && (int64_t)req[c] < A.n) A.drop[req[c]] = d;      // not from this snapshot's range
        }
    }
    __syncthreads();
    uint8_t* out = A.drop + lo;
    if ((reinterpret_cast<uintptr_t>(out) & 15) == 0) {
        for (int i = tid * 16; i < (int)m; i += kMaskThreads * 16) {
            if (i + 15 < (int)m) *reinterpret_cast<uint4*>(out + i) = *reinterpret_cast<const uint4*>(&mask[i]);
            else for (int c = i; c < (int)m; ++c) out[c] = mask[c];
        }
    } else {
        for (int i = tid; i < (int)m; i += kMaskThreads) out[i] = mask[i];
    }
}

// Larger snapshots: the same walk as in step 1 (a wave takes kRxChunks chunks of 64 slots, request ids loaded up
// front), one byte per slot written at its request's place.
__global__ __launch_bounds__(kRxThreads) void window_mask_kernel(WindowArgs A) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int G = A.plan.K * A.plan.S, S = A.plan.S;
    const int64_t t0 = ((int64_t)blockIdx.x * (kRxThreads / kWave) + wave) * (kRxChunks * kWave);
    if (t0 >= A.n) return;
    int64_t t1 = t0 + kRxChunks * kWave;
    if (t1 > A.n) t1 = A.n;
    const int g_lo = queue_of_slot_wave(A.seg_ptr, t0, 0, G - 1, lane), g_hi = queue_of_slot_wave(A.seg_ptr, t1 - 1, g_lo, G - 1, lane);
    // snapshots the other kernel takes care of; a walk that only meets such snapshots has nothing to do
    auto taken = [&](int g) {
        const int u = g / S;
        const int64_t size = (int64_t)A.seg_ptr[(int64_t)(u + 1) * S] - (int64_t)A.seg_ptr[(int64_t)u * S];
        return size <= (int64_t)A.mask_cap;
    };
    if (A.mask_cap > 0) {
        bool all_taken = true;
        for (int u = g_lo / S; u <= g_hi / S; ++u) all_taken = all_taken && taken(u * S);
        if (all_taken) return;
    }
    int32_t req[kRxChunks];
#pragma unroll
    for (int c = 0; c < kRxChunks; ++c) {
        const int64_t j = t0 + (int64_t)c * kWave + lane;
        req[c] = j < t1 ? A.order[j] : -1;
    }
    // the slots of a lane rise along the walk, so its queue only moves forward (empty queues are stepped over)
    int g = g_lo;
    int32_t start = A.seg_ptr[g_lo], end = A.seg_ptr[g_lo + 1], first = A.first[g_lo];
    bool skip = A.mask_cap > 0 && taken(g_lo);
#pragma unroll
    for (int c = 0; c < kRxChunks; ++c) {
        const int64_t j = t0 + (int64_t)c * kWave + lane;
        if (j < t1) {
            while (g < g_hi && j >= (int64_t)end) {
                ++g; start = end; end = A.seg_ptr[g + 1]; first = A.first[g];
                if (A.mask_cap > 0 && g % S == 0) skip = taken(g);
            }
            if (!skip) A.drop[req[c]] = (int32_t)(j - start) < first ? 1 : 0;
        }
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

constexpr int kSplitPerThread = 4;                      // consecutive requests of a thread (16-byte loads when the arrays allow it)
__global__ __launch_bounds__(kRxThreads) void slo_split_kernel(SplitArgs A) {
    const int64_t t0 = (int64_t)blockIdx.x * (kRxThreads * kSplitPerThread);
    int64_t t1 = t0 + kRxThreads * kSplitPerThread;
    if (t1 > A.n) t1 = A.n;
    if (t0 >= t1) return;
    const int K = A.plan.K, S = A.plan.S;
    const int u_lo = snapshot_of_request(A.snap_ptr, t0, 0, K - 1), u_hi = snapshot_of_request(A.snap_ptr, t1 - 1, u_lo, K - 1);
    const int64_t r0 = t0 + (int64_t)threadIdx.x * kSplitPerThread;
    if (r0 >= t1) return;
    const bool vec = ((reinterpret_cast<uintptr_t>(A.arrival) | reinterpret_cast<uintptr_t>(A.deadline) |
                       reinterpret_cast<uintptr_t>(A.stage)) & 15) == 0 && r0 + 3 < t1;
    int32_t arr[4], dl[4], st[4];
    if (vec) {
        // one pass over the requests: streaming loads and stores (131 -> 118 us on 33.5 M requests)
        const pard_v4i a4 = __builtin_nontemporal_load(reinterpret_cast<const pard_v4i*>(A.arrival + r0));
        const pard_v4i d4 = __builtin_nontemporal_load(reinterpret_cast<const pard_v4i*>(A.deadline + r0));
        const pard_v4i s4 = __builtin_nontemporal_load(reinterpret_cast<const pard_v4i*>(A.stage + r0));
        arr[0] = a4.x; arr[1] = a4.y; arr[2] = a4.z; arr[3] = a4.w;
        dl[0] = d4.x; dl[1] = d4.y; dl[2] = d4.z; dl[3] = d4.w;
        st[0] = s4.x; st[1] = s4.y; st[2] = s4.z; st[3] = s4.w;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const bool ok = r0 + i < t1;
            arr[i] = ok ? A.arrival[r0 + i] : 0;
            dl[i] = ok ? A.deadline[r0 + i] : 0;
            st[i] = ok ? A.stage[r0 + i] : 0;
        }
    }
    int u = snapshot_of_request(A.snap_ptr, r0, u_lo, u_hi);              // then forward: the four are consecutive
    int64_t now = A.now[u];
    uint32_t bits = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t r = r0 + i;
        if (r >= t1) break;
        while (u < u_hi && r >= (int64_t)A.snap_ptr[u + 1]) { ++u; now = A.now[u]; }
        const int k = clamp_stage(st[i], S);
        const int64_t rec = (int64_t)(A.plan.shared ? 0 : u) * S + k;
        const int64_t way_in = A.plan.split_in[rec], whole = A.plan.split_whole[rec];
        const int64_t used = now - (int64_t)arr[i];
        const int64_t slo = (int64_t)dl[i] - (int64_t)arr[i];
        // |used|, |slo| < 2^33 and the path sums are below 2^30 (checked when the plan was made): the products fit 64 bits
        const bool drop = whole == 0 ? used > slo : used * whole > slo * way_in;
        bits |= (drop ? 1u : 0u) << (8 * i);
    }
    if (r0 + 3 < t1 && (reinterpret_cast<uintptr_t>(A.drop) & 3) == 0) {
        stream_store(reinterpret_cast<uint32_t*>(A.drop + r0), bits);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (r0 + i < t1) A.drop[r0 + i] = (uint8_t)((bits >> (8 * i)) & 1u);
    }
}

}  // namespace

hipError_t launch_window_scan(const PlanDev& plan, int64_t n, const int32_t* deadline, const int32_t* order, const int32_t* seg_ptr,
                              const int32_t* now, uint8_t* drop, int32_t* first, hipStream_t stream) {
    WindowArgs a{plan, n, deadline, order, seg_ptr, now, drop, first, 0};
    const int G = plan.K * plan.S;
    // snapshots of a few thousand requests on average: one workgroup per snapshot writes its mask (smaller ones
    // would leave most of a workgroup idle, and the host cannot see the single sizes)
    if (n / plan.K >= 1024 && n / plan.K <= kMaskCap) a.mask_cap = kMaskCap;
    window_init_kernel<<<(G + 255) / 256, 256, 0, stream>>>(first, G);
    if (n > 0) {
        const int64_t per_block = (int64_t)(kRxThreads / kWave) * kRxChunks * kWave;
        window_scan_kernel<<<(unsigned)((n + per_block - 1) / per_block), kRxThreads, 0, stream>>>(a);
    }
    window_tail_kernel<<<(unsigned)G, kWave, 0, stream>>>(a);
    if (n > 0) {
        const int64_t per_block = (int64_t)(kRxThreads / kWave) * kRxChunks * kWave;
        if (a.mask_cap > 0) window_mask_snapshot_kernel<<<(unsigned)plan.K, kMaskThreads, 0, stream>>>(a);
        window_mask_kernel<<<(unsigned)((n + per_block - 1) / per_block), kRxThreads, 0, stream>>>(a);
    }
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
