// Small snapshots: one wave evaluates one whole snapshot of at most 128 queued requests.
//
// The same result as the on-chip path for larger snapshots (paper Section 3.2 Eq.(1),(2),(4),
// DAG maximum; Section 3.3 ordering), by other means: a workgroup sized for hundreds of
// requests spends nearly all of its time on fixed costs (clearing and scanning bucket
// counters, barriers) when a snapshot holds a few dozen.  Here a request is a 64-bit word
// stage | order key | local index held in a register; a bitonic network over the wave's
// lanes sorts the words, after which lane p holds the request of queue slot p:
//   1. load deadline/stage (arrival for FCFS stages), form the word; deadlines go to LDS by
//      local index
//   2. sort (register exchanges across lanes; no LDS, no counters)
//   3. queue starts from the places where the stage changes along the sorted order
//   4. per stage: cost at full queue length; per path entry: downstream suffix sum, maximum
//      per stage
//   5. per queue slot: own-stage cost at its position + downstream maximum, drop decision;
//      the queue order leaves coalesced, estimate and decision return to request order
//      through LDS and leave coalesced as well.
//      Sequentially consistent variant (the position counts only the kept requests ahead,
//      Section 4.1): every queue is a chain of decisions.  Guess that everybody is kept, evaluate
//      every slot at the position the guess implies, take the decisions as the next guess: after
//      t rounds the first t slots of every queue are final, and a guess that reproduces itself
//      is the in-order result.  The guess is a lane mask, a position a population count.
// The workgroup is a single wave, so its barriers cost next to nothing and up to 32 snapshots
// are in flight per compute unit.  (Measured on 131,072 snapshots of 64 requests: 0.13 ms against
// 0.33 ms for the workgroup path; letting each wave loop over snapshots, with the next snapshot's
// loads issued ahead and the DAG's tables parked in LDS, needed 105 registers, halved the waves
// per SIMD and came out at 0.16 ms - the kernel issues about 560 instructions per snapshot, 320 of
// them vector ALU, and is bound by that once enough waves hide the load latency.)
#include "pard_device.hpp"

namespace pard {

namespace {

// Ascending bitonic sort of 64 * R distinct words, element e = r * 64 + lane.
template <int R>
__device__ __forceinline__ void sort_words(unsigned long long (&c)[R], const int lane) {
    constexpr int N = kWave * R;
#pragma unroll
    for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (j >= kWave) {                              // partner in the same lane
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const int r2 = r ^ (j / kWave);
                    if (r2 > r) {
                        const bool ascending = ((r * kWave) & k) == 0;
                        const unsigned long long a = c[r], b = c[r2];
                        const bool swap = ascending ? a > b : a < b;
                        c[r] = swap ? b : a;
                        c[r2] = swap ? a : b;
                    }
                }
            } else {                                       // partner in lane ^ j
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const unsigned long long other = __shfl_xor(c[r], j);
                    const bool lower = (lane & j) == 0;
                    const bool ascending = ((r * kWave + lane) & k) == 0;
                    const bool keep_min = lower == ascending;
                    c[r] = (keep_min == (other < c[r])) ? other : c[r];
                }
            }
        }
    }
}

constexpr unsigned long long kNoRequest = ~0ull;          // sorts behind every request
constexpr int kStageShift = 40, kKeyShift = 8;            // word = stage << 40 | key << 8 | local index

// LDS words (4 bytes) a snapshot of up to 64 * R requests and S stages needs.
__host__ __device__ constexpr int wave_lds_words(int R, int S) { return kWave * R + 17 * S + 2 + kWave; }

// Lanes l of slot row r (slots r * 64 + l) with first <= r * 64 + l < end.
__device__ __forceinline__ unsigned long long row_mask(int r, int first, int end) {
    int a = first - r * kWave, b = end - r * kWave;
    a = a < 0 ? 0 : a;
    b = b > kWave ? kWave : b;
    if (b <= a) return 0ull;
    const unsigned long long below_b = b == kWave ? ~0ull : (1ull << b) - 1ull;
    return below_b & ~((1ull << a) - 1ull);
}

template <int R, bool CONSISTENT>
__global__ __launch_bounds__(kWave, 8) void wave_snapshot_kernel(FusedArgs A) {
    constexpr int N = kWave * R;
    extern __shared__ __align__(16) uint32_t lds[];
    const PlanDev& P = A.plan;
    const int S = P.S;
    uint32_t* by_id = lds;                                                             // [N] deadline, later est | drop << 31
    unsigned long long* cfull = reinterpret_cast<unsigned long long*>(lds + N);        // [S]
    unsigned long long* down = cfull + S;                                              // [S]
    StageRec* recs = reinterpret_cast<StageRec*>(lds + N + 4 * S);                     // [S]
    int32_t* seg_start = reinterpret_cast<int32_t*>(lds + N + 16 * S);                 // [S + 1]
    uint32_t* ent = lds + N + 17 * S + 2;                                              // [64] the DAG's path entries (up to 64)
    static_assert(sizeof(StageRec) == 48, "LDS layout");

    const int u = blockIdx.x;
    const int lane = threadIdx.x;
    const int dag = P.shared ? 0 : u;
    const int32_t* lat_dag = P.lat + (int64_t)dag * S * PARD_LAT_ENTRIES;
    const int e_lo = P.dag_entry_ptr[dag], n_entries = P.dag_entry_ptr[dag + 1] - e_lo;
    const int32_t now = A.now[u];
    // snapshot bounds, made safe whatever snap_ptr holds
    const int64_t n = A.n;
    int64_t lo = A.snap_ptr[u], hi = A.snap_ptr[u + 1];
    if (lo < 0) lo = 0;
    if (lo > n) lo = n;
    if (hi > n) hi = n;
    int64_t m64 = hi - lo;
    if (m64 < 0) m64 = 0;
    const int limit = A.cap < N ? A.cap : N;
    if (m64 > limit) {
        m64 = limit;
        if (lane == 0) atomicOr(A.status, kStatusSnapshotTooLarge);
    }
    const int m = (int)m64;

    // ---- 1. loads, words ----------------------------------------------------------------
    int32_t dl[R], st[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = r * kWave + lane;
        // read once / written once and not read again by this call: streaming accesses (131,072 snapshots of 64: 134 -> 118 us)
        dl[r] = e < m ? __builtin_nontemporal_load(A.deadline + lo + e) : 0;
        st[r] = e < m ? __builtin_nontemporal_load(A.stage + lo + e) : 0;
    }
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(P.recs + (int64_t)dag * S);
        uint32_t* dst = reinterpret_cast<uint32_t*>(recs);
        for (int i = lane; i < S * (int)(sizeof(StageRec) / 4); i += kWave) dst[i] = src[i];
        for (int i = lane; i < S; i += kWave) down[i] = 0;
    }
    // The path entries (stage | end of the entry's path << 8) are fetched now, behind the request loads: walked in
    // memory after the sort they are a chain of dependent loads, one per stage of a path.
    const bool entries_cached = n_entries <= kWave;
    if (entries_cached && lane < n_entries)
        ent[lane] = (uint32_t)P.entry_stage[e_lo + lane] | ((uint32_t)(P.entry_end[e_lo + lane] - e_lo) << 8);
    __syncthreads();
    unsigned long long c[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = r * kWave + lane;
        const int s = clamp_stage(st[r], S);
        const int mode = P.uniform_mode >= 0 ? P.uniform_mode : (recs[s].mode & 0xFF);
        int32_t arr = 0;
        if (mode == PARD_ORDER_FCFS && e < m) arr = A.arrival[lo + e];
        const uint32_t k = order_key(mode, dl[r], arr);
        c[r] = e < m ? ((unsigned long long)s << kStageShift) | ((unsigned long long)k << kKeyShift) | (unsigned)e : kNoRequest;
        by_id[e] = (uint32_t)dl[r];
    }

    // ---- 2. queue order -----------------------------------------------------------------
    sort_words<R>(c, lane);

    // ---- 3. queue starts: slot p opens every queue after its predecessor's up to its own -----
    int sp[R];                               // stage of slot p = r * 64 + lane; S behind the last request
#pragma unroll
    for (int r = 0; r < R; ++r) sp[r] = r * kWave + lane < m ? (int)(c[r] >> kStageShift) : S;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int prev = __shfl_up(sp[r], 1);
        const int carry = r > 0 ? __shfl(sp[r > 0 ? r - 1 : 0], kWave - 1) : -1;
        if (lane == 0) prev = carry;
        for (int s = prev + 1; s <= sp[r]; ++s) seg_start[s] = r * kWave + lane;
        if (r == R - 1 && lane == kWave - 1)
            for (int s = sp[r] + 1; s <= S; ++s) seg_start[s] = N;      // all N slots taken: m = N
    }
    __syncthreads();

    // ---- 4. full-queue costs, downstream maximum per stage ------------------------------------
    for (int i = lane; i < S; i += kWave)
        cfull[i] = stage_cost(recs[i], (uint32_t)(seg_start[i + 1] - seg_start[i]), lat_dag + i * PARD_LAT_ENTRIES);
    __syncthreads();
    if (A.sub) {
        for (int i = lane; i < S; i += kWave) {
            const int64_t v = A.sub[(int64_t)u * S + i];
            down[i] = v < 0 ? 0ull : ((uint64_t)v < kCostCap ? (unsigned long long)v : (unsigned long long)kCostCap);
        }
    } else if (entries_cached) {
        if (lane < n_entries) {
            const uint32_t me = ent[lane];
            const int end = (int)(me >> 8);
            unsigned long long sum = 0;
            for (int t = lane + 1; t < end; ++t) sum += cfull[ent[t] & 0xFFu];
            atomicMax(&down[me & 0xFFu], sum);
        }
    } else {
        for (int e = e_lo + lane; e < e_lo + n_entries; e += kWave) {
            const int end = P.entry_end[e];
            unsigned long long sum = 0;
            for (int t = e + 1; t < end; ++t) sum += cfull[P.entry_stage[t]];
            atomicMax(&down[P.entry_stage[e]], sum);
        }
    }
    int32_t dq[R];                           // deadline of the request in slot p
#pragma unroll
    for (int r = 0; r < R; ++r) dq[r] = (int32_t)by_id[(uint32_t)c[r] & (N - 1)];   // a slot without request reads a deadline it never uses
    __syncthreads();

    // ---- 5. estimate and decision per queue slot; back to request order through LDS ----------
    int32_t est[R];
    uint8_t drp[R];
    if (CONSISTENT) {
        unsigned long long keep[R];
        int q0[R];
        unsigned long long dn[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const bool ok = r * kWave + lane < m;
            keep[r] = __ballot(ok);
            q0[r] = ok ? seg_start[sp[r]] : 0;
            dn[r] = ok ? down[sp[r]] : 0ull;
            est[r] = 0;
            drp[r] = 0;
        }
        for (int round = 0; round <= N; ++round) {
            unsigned long long next[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int p = r * kWave + lane;
                const bool ok = p < m;
                if (ok) {
                    uint32_t ahead = 0;
#pragma unroll
                    for (int r2 = 0; r2 <= r; ++r2) ahead += (uint32_t)__popcll(keep[r2] & row_mask(r2, q0[r], p));
                    finish_request(stage_cost_short(recs[sp[r]], ahead, lat_dag + sp[r] * PARD_LAT_ENTRIES) + dn[r], now, dq[r],
                                   est[r], drp[r]);
                }
                next[r] = __ballot(ok && drp[r] == 0);
            }
            bool same = true;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                same = same && next[r] == keep[r];
                keep[r] = next[r];
            }
            if (same) break;
        }
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int p = r * kWave + lane;
            est[r] = 0;
            drp[r] = 0;
            if (p < m) {
                const int k = sp[r];
                const uint32_t pos = (uint32_t)(p - seg_start[k]);
                finish_request(stage_cost_short(recs[k], pos, lat_dag + k * PARD_LAT_ENTRIES) + down[k], now, dq[r], est[r], drp[r]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = r * kWave + lane;
        if (p < m) {
            const uint32_t id = (uint32_t)c[r] & (N - 1);
            by_id[id] = (uint32_t)est[r] | ((uint32_t)drp[r] << 31);
            A.order[lo + p] = (int32_t)(lo + id);
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = r * kWave + lane;
        if (e < m) {
            const uint32_t v = by_id[e];
            __builtin_nontemporal_store((int32_t)(v & 0x7FFFFFFFu), A.est + lo + e);
            __builtin_nontemporal_store((uint8_t)(v >> 31), A.drop + lo + e);
        }
    }
    for (int i = lane; i < S; i += kWave) A.seg_ptr[(int64_t)u * S + i] = (int32_t)lo + seg_start[i];
    if (u == P.K - 1 && lane == 0) A.seg_ptr[(int64_t)P.K * S] = (int32_t)(lo + m);
}

}  // namespace

bool wave_path_covers(const FusedArgs& a) { return a.cap <= 2 * kWave; }

template <int R>
static void launch_rows(const FusedArgs& a, size_t bytes, hipStream_t stream) {
    if (a.consistent) wave_snapshot_kernel<R, true><<<dim3((unsigned)a.plan.K), dim3(kWave), bytes, stream>>>(a);
    else wave_snapshot_kernel<R, false><<<dim3((unsigned)a.plan.K), dim3(kWave), bytes, stream>>>(a);
}

hipError_t launch_wave(const FusedArgs& a, hipStream_t stream) {
    const int R = a.cap <= kWave ? 1 : 2;
    const size_t bytes = (size_t)wave_lds_words(R, a.plan.S) * 4;
    if (R == 1) launch_rows<1>(a, bytes, stream);
    else launch_rows<2>(a, bytes, stream);
    return hipGetLastError();
}

}  // namespace pard
