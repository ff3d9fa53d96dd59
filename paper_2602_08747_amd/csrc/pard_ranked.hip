// Ranked downstream positions: a variant of the estimate in which a request does not join the
// back of every later queue but takes the place its budget gives it there.
//
// The paper keeps every worker queue in remaining-budget order (Section 3.3), so at a later
// stage i the requests ahead of a newcomer with deadline d are the ones that order serves first:
// those with deadline <= d under low budget first (the ones already there win ties), those with
// deadline >= d under high budget first, the whole queue in arrival order.  The estimate is
//   est = cost_k(pos) + max over the paths through k of sum over later stages i of cost_i(ahead_i(d))
// (Section 3.2 Eq.(4) and the DAG maximum), everything else as in the plain estimate.
//
// It runs after the plain call, on its outputs: the queues are sorted then, so ahead_i(d) is a
// binary search over queue i's slots (deadline looked up through order[]).  One thread per queue
// slot: neighbouring threads hold neighbouring deadlines of one queue, so their searches walk the
// same slots.  The downstream sum depends on the request now, so the path CSR is walked per
// request; the cost of each later stage is computed once per request and kept in LDS.
#include "pard_device.hpp"

namespace pard {

namespace {

constexpr int kRThreads = 64;                          // one wave per workgroup: a thread's LDS row is private
constexpr unsigned long long kUnset = ~0ull;

// the queue g with seg_ptr[g] <= j < seg_ptr[g+1], among queues lo..hi
__device__ __forceinline__ int64_t queue_of(const int32_t* seg_ptr, int64_t lo, int64_t hi, int64_t j) {
    int64_t a = lo, b = hi + 1;                        // answer in [a, b)
    while (b - a > 1) {
        const int64_t mid = (a + b) >> 1;
        if ((int64_t)seg_ptr[mid] <= j) a = mid; else b = mid;
    }
    return a;
}

__global__ __launch_bounds__(kRThreads) void ranked_estimate_kernel(RankedArgs A) {
    extern __shared__ unsigned long long memo[];       // [S][kRThreads]: cost of later stage i for this thread's request
    const PlanDev& P = A.plan;
    const int tid = threadIdx.x;
    const int S = P.S;
    const int64_t segs = (int64_t)P.K * S;
    const int64_t tiles = (A.n + kRThreads - 1) / kRThreads;
    for (int64_t tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const int64_t j0 = tile * kRThreads, j1 = j0 + kRThreads - 1 < A.n - 1 ? j0 + kRThreads - 1 : A.n - 1;
        const int64_t g_first = queue_of(A.seg_ptr, 0, segs - 1, j0), g_last = queue_of(A.seg_ptr, g_first, segs - 1, j1);
        const int64_t j = j0 + tid;
        if (j >= A.n) continue;
        const int64_t g = queue_of(A.seg_ptr, g_first, g_last, j);
        const int32_t u = (int32_t)(g / S), k = (int32_t)(g - (int64_t)u * S);
        const int64_t rec0 = P.shared ? 0 : (int64_t)u * S;
        const int32_t r = A.order[j];
        if ((uint32_t)r >= (uint64_t)A.n) continue;
        const int32_t d = A.deadline[r];
        for (int i = 0; i < S; ++i) memo[i * kRThreads + tid] = kUnset;
        const int32_t dag = P.shared ? 0 : u;
        const int32_t e_lo = P.dag_entry_ptr[dag], e_hi = P.dag_entry_ptr[dag + 1];
        unsigned long long best = 0;
        for (int32_t e = e_lo; e < e_hi; ++e) {
            if (P.entry_stage[e] != k) continue;
            const int32_t end = P.entry_end[e];
            unsigned long long sum = 0;
            for (int32_t t = e + 1; t < end; ++t) {
                const int32_t i = P.entry_stage[t];
                unsigned long long c = memo[i * kRThreads + tid];
                if (c == kUnset) {
                    const StageRec sr = P.recs[rec0 + i];
                    const int64_t start = A.seg_ptr[(int64_t)u * S + i], stop = A.seg_ptr[(int64_t)u * S + i + 1];
                    const int32_t mode = P.uniform_mode >= 0 ? P.uniform_mode : (sr.mode & 0xFF);
                    int64_t lo = start, hi = stop;     // first slot the newcomer does not have to let pass
                    if (mode == PARD_ORDER_FCFS) {
                        lo = stop;
                    } else {
                        while (lo < hi) {
                            const int64_t mid = (lo + hi) >> 1;
                            const int32_t rm = A.order[mid];
                            const int32_t dm = (uint32_t)rm < (uint64_t)A.n ? A.deadline[rm] : 0;
                            const bool passes = mode == PARD_ORDER_HBF ? dm >= d : dm <= d;
                            if (passes) lo = mid + 1; else hi = mid;
                        }
                    }
                    c = stage_cost(sr, (uint32_t)(lo - start), P.lat + (rec0 + i) * PARD_LAT_ENTRIES);
                    memo[i * kRThreads + tid] = c;
                }
                sum += c;
            }
            best = sum > best ? sum : best;
        }
        const StageRec own = P.recs[rec0 + k];
        const uint64_t e64 = stage_cost(own, (uint32_t)(j - (int64_t)A.seg_ptr[g]), P.lat + (rec0 + k) * PARD_LAT_ENTRIES) + best;
        int32_t est;
        uint8_t drp;
        finish_request(e64, A.now[u], d, est, drp);
        A.est[r] = est;
        A.drop[r] = drp;
    }
}

// Snapshots that fit LDS: one workgroup per snapshot first lays the deadlines out by queue slot
// in LDS, so a search step is one LDS read instead of two dependent global loads.
constexpr int kRSnapEntries = 1024;                    // path entries of a DAG kept in LDS (longer lists are read in place)

template <int kRSnapThreads>
__global__ __launch_bounds__(kRSnapThreads) void ranked_snapshot_kernel(RankedArgs A) {
    extern __shared__ unsigned long long lds[];         // memo [S][kRSnapThreads], then the deadlines by slot
    __shared__ StageRec recs[PARD_MAX_STAGES];
    __shared__ int32_t qstart[PARD_MAX_STAGES + 1];     // queue starts inside the snapshot
    __shared__ uint32_t ent[kRSnapEntries];             // stage | (end of the entry's path) << 8
    const PlanDev& P = A.plan;
    const int tid = threadIdx.x;
    const int S = P.S;
    unsigned long long* memo = lds;
    int32_t* dls = reinterpret_cast<int32_t*>(lds + (size_t)S * kRSnapThreads);
    const int32_t u = blockIdx.x;
    const int64_t a0 = A.seg_ptr[(int64_t)u * S], a1 = A.seg_ptr[(int64_t)(u + 1) * S];
    if (a0 < 0 || a1 < a0 || a1 > A.n || a1 - a0 > A.max_snapshot) return;   // larger than promised: reported by the plain call
    const int m = (int)(a1 - a0);
    const int64_t rec0 = P.shared ? 0 : (int64_t)u * S;
    const int32_t dag = P.shared ? 0 : u;
    const int32_t e_lo = P.dag_entry_ptr[dag], n_entries = P.dag_entry_ptr[dag + 1] - e_lo;
    const bool cached = n_entries <= kRSnapEntries;
    for (int j = tid; j < m; j += kRSnapThreads) {
        const int32_t r = A.order[a0 + j];
        dls[j] = (uint32_t)r < (uint64_t)A.n ? A.deadline[r] : 0;
    }
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(P.recs + rec0);
        uint32_t* dst = reinterpret_cast<uint32_t*>(recs);
        for (int i = tid; i < S * (int)(sizeof(StageRec) / 4); i += kRSnapThreads) dst[i] = src[i];
        for (int i = tid; i <= S; i += kRSnapThreads) qstart[i] = (int32_t)((int64_t)A.seg_ptr[(int64_t)u * S + i] - a0);
        if (cached)
            for (int e = tid; e < n_entries; e += kRSnapThreads)
                ent[e] = (uint32_t)P.entry_stage[e_lo + e] | ((uint32_t)(P.entry_end[e_lo + e] - e_lo) << 8);
    }
    __syncthreads();
    auto entry_stage = [&](int e) -> int { return cached ? (int)(ent[e] & 0xFFu) : P.entry_stage[e_lo + e]; };
    auto entry_end = [&](int e) -> int { return cached ? (int)(ent[e] >> 8) : P.entry_end[e_lo + e] - e_lo; };
    const int32_t now = A.now[u];
    for (int j = tid; j < m; j += kRSnapThreads) {
        int k = 0;                                      // the queue of slot j: the last one that starts at or before it
        while (k + 1 < S && qstart[k + 1] <= j) ++k;
        const int32_t d = dls[j];
        for (int i = 0; i < S; ++i) memo[i * kRSnapThreads + tid] = kUnset;
        unsigned long long best = 0;
        for (int e = 0; e < n_entries; ++e) {
            if (entry_stage(e) != k) continue;
            const int end = entry_end(e);
            unsigned long long sum = 0;
            for (int t = e + 1; t < end; ++t) {
                const int i = entry_stage(t);
                unsigned long long c = memo[i * kRSnapThreads + tid];
                if (c == kUnset) {
                    const int start = qstart[i], stop = qstart[i + 1];
                    const int32_t mode = P.uniform_mode >= 0 ? P.uniform_mode : (recs[i].mode & 0xFF);
                    int lo = start, hi = stop;           // first slot the newcomer does not have to let pass
                    if (mode == PARD_ORDER_FCFS) {
                        lo = stop;
                    } else {
                        while (lo < hi) {
                            const int mid = (lo + hi) >> 1;
                            const int32_t dm = dls[mid];
                            const bool passes = mode == PARD_ORDER_HBF ? dm >= d : dm <= d;
                            if (passes) lo = mid + 1; else hi = mid;
                        }
                    }
                    c = stage_cost(recs[i], (uint32_t)(lo - start), P.lat + (rec0 + i) * PARD_LAT_ENTRIES);
                    memo[i * kRSnapThreads + tid] = c;
                }
                sum += c;
            }
            best = sum > best ? sum : best;
        }
        const uint64_t e64 = stage_cost(recs[k], (uint32_t)(j - qstart[k]), P.lat + (rec0 + k) * PARD_LAT_ENTRIES) + best;
        const int32_t r = A.order[a0 + j];
        if ((uint32_t)r >= (uint64_t)A.n) continue;
        int32_t est;
        uint8_t drp;
        finish_request(e64, now, d, est, drp);
        A.est[r] = est;
        A.drop[r] = drp;
    }
}

}  // namespace

hipError_t launch_ranked(const RankedArgs& a, hipStream_t stream) {
    if (a.n <= 0) return hipSuccess;
    // the largest workgroup whose per-thread rows and the snapshot's deadlines fit 64 KB of LDS
    const int64_t cap = a.max_snapshot < 1 ? 1 : a.max_snapshot;
    auto lds_bytes = [&](int threads) { return (size_t)a.plan.S * threads * sizeof(unsigned long long) + (size_t)((cap + 1) & ~(int64_t)1) * 4; };
    if (a.max_snapshot <= PARD_FUSED_SNAPSHOT_CAPACITY) {
        const unsigned K = (unsigned)a.plan.K;
        if (lds_bytes(512) <= 64 * 1024 && cap > 2048) { ranked_snapshot_kernel<512><<<K, 512, lds_bytes(512), stream>>>(a); return hipGetLastError(); }
        if (lds_bytes(256) <= 64 * 1024 && cap > 512) { ranked_snapshot_kernel<256><<<K, 256, lds_bytes(256), stream>>>(a); return hipGetLastError(); }
        if (lds_bytes(128) <= 64 * 1024) { ranked_snapshot_kernel<128><<<K, 128, lds_bytes(128), stream>>>(a); return hipGetLastError(); }
    }                                                   // else: many stages, the general kernel
    int64_t grid = (a.n + kRThreads - 1) / kRThreads;
    if (grid > 64 * (int64_t)a.num_cus) grid = 64 * (int64_t)a.num_cus;
    ranked_estimate_kernel<<<(unsigned)grid, kRThreads, (size_t)a.plan.S * kRThreads * sizeof(unsigned long long), stream>>>(a);
    return hipGetLastError();
}

}  // namespace pard
