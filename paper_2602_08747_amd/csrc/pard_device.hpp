// Device-side view of a plan and the small arithmetic helpers every kernel shares.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "pard_host.hpp"

namespace pard {

constexpr int kWave = 64;
constexpr uint64_t kCostCap = (uint64_t)1 << 40;   // per-term clamp, see stage_cost()
constexpr int32_t kInt32Max = 0x7fffffff;

// Plan tables in device memory (passed to kernels by value).
struct PlanDev {
    int32_t K, S, shared, any_fcfs;
    int32_t uniform_mode;              // >= 0 when all stages share one order mode
    int32_t max_entries_per_dag;
    int32_t presorted_ok;              // every stage admits the 32-bit short-queue form (see HostPlan)
    const StageRec* recs;              // [D*S]
    const int32_t* lat;                // [D*S*64]
    const int32_t* dag_entry_ptr;      // [D+1]
    const int32_t* entry_stage;        // [E]
    const int32_t* entry_end;          // [E]
    const int32_t* entry_dag;          // [E]
    const int64_t* split_in;           // [D*S] per-module SLO split: longest way in (see HostPlan)
    const int64_t* split_whole;        // [D*S] longest whole path through the stage
    int64_t total_entries;             // E
};

// Status bits a kernel may raise in the workspace's status word.
enum : uint32_t {
    kStatusSnapshotTooLarge = 1u       // a snapshot exceeded the promised bound
};

__device__ __forceinline__ uint32_t magic_div_dev(uint32_t n, uint32_t m, uint32_t sh) {
    uint32_t t = __umulhi(m, n);
    return (t + ((n - t) >> (sh & 0xFF))) >> (sh >> 8);
}

// int32 -> uint32 preserving order, then the per-mode queue key: ascending key order
// is the queue order (Section 3.3: LBF = smallest remaining budget first, HBF = largest).
__device__ __forceinline__ uint32_t order_key(int32_t mode, int32_t deadline, int32_t arrival) {
    uint32_t d = (uint32_t)deadline ^ 0x80000000u;
    if (mode == PARD_ORDER_HBF) return ~d;
    if (mode == PARD_ORDER_FCFS) return (uint32_t)arrival ^ 0x80000000u;
    return d;
}

__device__ __forceinline__ int32_t clamp_stage(int32_t s, int32_t S) {
    return s < 0 ? 0 : (s >= S ? S - 1 : s);
}

// 64-bit by 32-bit division, kept out of line: it is long and almost never taken.
static __device__ __noinline__ uint64_t wide_div(uint64_t x, uint32_t d) { return x / d; }

// Eq.(2) in snapshot form with `a` requests ahead (0 <= a < 2^31):
//   floor(ceil(a/B) * lat[B] / W) + lat[min(B, a+1)]
// clamped to 2^40.  With lat[B] = aW * W + bW (bW < W) and q batches ahead, floor(q * lat[B] / W) is
// q * aW + floor(q * bW / W): what is left to divide fits 32 bits unless W is huge, while q * lat[B] itself
// passes 2^32 as soon as a queue is long.  Clamping every term at 2^40 keeps 64-bit sums of up to 65 terms
// exact-or-saturated: any sum that reaches the clamp is far above INT32_MAX even after
// adding the most negative `now`, so the reported estimate and the drop decision are
// the same as with unbounded integers.
__device__ __forceinline__ uint64_t stage_cost(const StageRec& r, uint32_t a, const int32_t* lat_row) {
    uint32_t q = magic_div_dev(a + (uint32_t)r.B - 1u, r.mB, r.shB);
    const uint64_t p = (uint64_t)q * r.bW;
    uint64_t wait = (uint64_t)q * r.aW;
    if ((p >> 32) == 0) wait += magic_div_dev((uint32_t)p, r.mW, r.shW);
    else wait += wide_div(p, (uint32_t)r.W);
    uint32_t ex = (a + 1u >= (uint32_t)r.B) ? (uint32_t)r.latB : (uint32_t)lat_row[a];
    uint64_t c = wait + ex;
    return c < kCostCap ? c : kCostCap;
}

// The same cost for a short queue (a < 2^13), without 32x32 multiplies or integer
// division when the stage allows it (kStageFast):
//   q = ceil(a/B) = trunc((a + B - 1 + 0.5) * (1/B))        exact: the true value sits at
//       least 0.5/B from an integer and the two float roundings move it by < 0.002 * 0.5/B
//   latB = aW*W + bW  =>  floor(q*latB/W) = q*aW + floor(q*bW/W)
//   p = q*bW < 2^21 (bW < W <= 256), floor(p/W) = trunc((p + 0.5) * (1/W))   exact: p + 0.5
//       is a float, the true value sits at least 0.5/W from an integer, error < 0.25/W
//   q*aW < 2^31 (aW < 2^18), so everything fits 32 bits.
__device__ __forceinline__ uint64_t stage_cost_short(const StageRec& r, uint32_t a, const int32_t* lat_row) {
    if (r.mode & kStageFast) {
        const uint32_t q = (uint32_t)(((float)(a + (uint32_t)r.B - 1u) + 0.5f) * r.rcpB);
        const uint32_t p = __umul24(q, r.bW);
        const uint32_t wait = __umul24(q, r.aW) + (uint32_t)(((float)p + 0.5f) * r.rcpW);
        const uint32_t ex = (a + 1u >= (uint32_t)r.B) ? (uint32_t)r.latB : (uint32_t)lat_row[a];
        return (uint64_t)wait + ex;
    }
    return stage_cost(r, a, lat_row);
}

// est (clamped) and the drop decision from the 64-bit estimate:
//   drop = min(now + e64, INT32_MAX) > deadline.
// A deadline of INT32_MAX can never be exceeded by the clamped finish time; for any smaller
// deadline the clamp does not change the comparison.
__device__ __forceinline__ void finish_request(uint64_t e64, int32_t now, int32_t deadline,
                                               int32_t& est, uint8_t& drop) {
    est = e64 > (uint64_t)kInt32Max ? kInt32Max : (int32_t)e64;
    const int64_t fin = (int64_t)now + (int64_t)e64;
    drop = ((deadline != kInt32Max) & (fin > (int64_t)deadline)) ? 1 : 0;
}

__device__ __forceinline__ uint32_t lane_id() {
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Inclusive prefix sum across the 64 lanes of a wave, on the vector ALU's data-parallel
// primitives: four shifts inside each row of 16 lanes, then the last lane of rows 0 and 2 is
// added to rows 1 and 3, and lane 31 to the upper half.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xF, 0xF, false);    // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xF, 0xF, false);    // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);    // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);    // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);    // row_bcast:15 into rows 1, 3
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);    // row_bcast:31 into rows 2, 3
    return v;
}

// Estimates and decisions are written once and not read again by the call that writes them: streaming stores
// (they leave the caches early and do not push out what the next kernel reads).
typedef int pard_v4i __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void stream_store(int4* p, int4 v) {
    pard_v4i x = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(x, reinterpret_cast<pard_v4i*>(p));
}
__device__ __forceinline__ void stream_store(uint32_t* p, uint32_t v) { __builtin_nontemporal_store(v, p); }

// Where a snapshot's staged survivors start inside the snapshot's own stretch of the staging array.  Snapshots
// of equal size start at equal distances; if every one staged its few survivors at its very start, they would
// all fall into the same few memory channels (measured: the kernel that moves them ran at an eighth of the
// bandwidth).  Eight consecutive snapshots therefore start at eight different eighths of the free room.
__host__ __device__ __forceinline__ uint32_t staging_shift(int64_t u, uint32_t requests, uint32_t survivors) {
    return ((uint32_t)(u & 7) * ((requests - survivors) >> 3)) & ~15u;
}

// ---- launchers implemented in the .hip files (host functions) ----------------

struct FusedArgs {
    PlanDev plan;
    const int32_t *arrival, *deadline, *stage, *snap_ptr, *now;
    int32_t *est;
    uint8_t* drop;
    int32_t *order, *seg_ptr;
    const int64_t* sub;                // [K*S] downstream latency per (snapshot, stage), or null: walk the paths
    uint32_t* status;
    uint32_t* todo;                    // [K] scratch, or null: snapshots left to the general kernel by the one for
                                       // snapshots that come in queue order
    // survivor compaction in the same pass (all three null otherwise):
    uint32_t* kept;                    // [K] out: survivors of every snapshot
    int32_t* staged;                   // [n] out: a snapshot's survivors in queue order from its first request's place on
    int32_t* loc_ptr;                  // [K*S] out: survivors of the snapshot before each of its queues
    int32_t cap;                       // promised bound on a snapshot's size
    int32_t consistent;                // positions count only the kept requests ahead
    int64_t n;                         // total requests (bounds every index derived from snap_ptr)
};
hipError_t launch_fused(const FusedArgs& a, hipStream_t stream);
// Snapshots whose requests already come in queue order (launch_fused tries this first when it applies).
constexpr int kPresortedMaxStages = 6;
bool presorted_path_covers(const FusedArgs& a);
hipError_t launch_presorted(const FusedArgs& a, hipStream_t stream);
// Snapshots of at most 128 requests, one wave each (launch_fused hands these over itself).
bool wave_path_covers(const FusedArgs& a);
hipError_t launch_wave(const FusedArgs& a, hipStream_t stream);

struct SortArgs {
    PlanDev plan;
    int64_t n;
    int64_t max_snapshot;              // promised bound on a snapshot's size
    const int32_t *arrival, *deadline, *stage, *snap_ptr, *now;
    int32_t* est;
    uint8_t* drop;
    int32_t *order, *seg_ptr;
    const int64_t* sub;                // as in FusedArgs
    int32_t consistent;                // as in FusedArgs
    uint32_t* status;
    void* workspace;                   // sort_workspace_bytes(K, S, n) bytes, 256-byte aligned
    int32_t num_cus;
};
int64_t sort_workspace_bytes(int32_t K, int32_t S, int64_t n);
bool sort_supported(int32_t K, int32_t S, int64_t n, int64_t max_snapshot);
hipError_t launch_sort_path(const SortArgs& a, hipStream_t stream);

struct RankedArgs {
    PlanDev plan;
    int64_t n;
    const int32_t *deadline, *now;
    const int32_t *order, *seg_ptr;    // the plain call's queues
    int32_t* est;                      // rewritten
    uint8_t* drop;
    int64_t max_snapshot;              // promised bound on a snapshot's size
    int32_t num_cus;
};
hipError_t launch_ranked(const RankedArgs& a, hipStream_t stream);

struct CompactArgs {
    int32_t num_segments;              // K*S
    int32_t stages;                    // S
    int64_t max_snapshot;              // promised bound on a snapshot's size
    int64_t n;
    const int32_t *order, *seg_ptr;
    const uint8_t* drop;
    int32_t *surv_idx, *surv_ptr;
    uint32_t* status;
    void* workspace;
    // after an estimate call that counted and staged the survivors along the way (all three null otherwise):
    const uint32_t* kept;              // [K] survivors per snapshot
    const int32_t* staged;             // [n] a snapshot's survivors in queue order, from its first request's place on
    const int32_t* loc_ptr;            // [K*S] survivors of the snapshot before each of its queues
};
// True when pard_compact gives every snapshot to one workgroup for this promised bound (the form the
// estimate kernels can prepare).
bool compact_per_snapshot(int64_t max_snapshot);
int64_t compact_workspace_bytes(int64_t n, int64_t num_snapshots);
hipError_t launch_compact(const CompactArgs& a, hipStream_t stream);

// ---- State Planner side (pard_planner.hip) ------------------------------------------
constexpr int kMaxWaitSamples = 16384;             // samples of the arrival process one workgroup holds in LDS
constexpr int32_t kMaxWaitLatency = 1 << 25;       // durations above this are not sampled (sums of 64 must fit 32 bits)

hipError_t launch_queue_lengths(const PlanDev& plan, int64_t n, const int32_t* stage, const int32_t* snap_ptr,
                                int32_t* qlen, hipStream_t stream);
struct SubArgs {
    PlanDev plan;
    const int32_t* qlen;               // [K*S]
    const int32_t* qdelay;             // [K*S] monitored queueing delays, or null: derived from qlen
    int32_t variant;                   // PARD_SUB_*
    int64_t rank;                      // 1-based order statistic of the sampled totals (full variant)
    int32_t num_samples;
    const int32_t* samples;            // [num_samples]
    const uint32_t* picks;             // [num_samples * S]
    uint32_t* drawn;                   // [S][num_samples] scratch: the arrival each (sample, stage) pair draws
    unsigned long long* sub;           // [K*S] out
};
hipError_t launch_sub_latency(const SubArgs& a, hipStream_t stream);
hipError_t launch_priority_modes(const PlanDev& plan, int32_t series_len, int32_t window, const int32_t* rate,
                                 const int32_t* prev_mode, int32_t* mode_out, hipStream_t stream);
hipError_t launch_queue_delay(int32_t K, int32_t S, int32_t len, uint32_t window, const int32_t* time, const int32_t* delay,
                              const int32_t* now, int32_t* q, hipStream_t stream);
hipError_t launch_set_modes(StageRec* recs, const int32_t* modes, int64_t count, hipStream_t stream);

// ---- reactive policies (pard_reactive.hip) --------------------------------------------
hipError_t launch_window_scan(const PlanDev& plan, int64_t n, const int32_t* deadline, const int32_t* order, const int32_t* seg_ptr,
                              const int32_t* now, uint8_t* drop, int32_t* first, hipStream_t stream);
hipError_t launch_slo_split(const PlanDev& plan, int64_t n, const int32_t* arrival, const int32_t* deadline, const int32_t* stage,
                            const int32_t* snap_ptr, const int32_t* now, uint8_t* drop, hipStream_t stream);

}  // namespace pard
