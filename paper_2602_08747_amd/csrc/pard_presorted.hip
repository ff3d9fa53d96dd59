// On-chip path for snapshots whose requests already come in queue order.
//
// A queue snapshot is normally taken in arrival order, and with one SLO per pipeline the
// deadlines (the low-budget-first keys, Section 3.3) then rise along the request array.  For such
// a snapshot the segmented stable sort of the path degenerates to a stable split by stage: the
// queue position of a request is the number of earlier requests of its stage.  This kernel
// checks that property while it loads a snapshot and, when it holds, produces exactly what the
// general on-chip kernel produces (paper Section 3.2 Eq.(1),(2),(4), DAG maximum) without
// bucket counters, scatter or rank loop; a snapshot that is not in key order is only marked, and
// the general kernel, launched right behind this one, takes the marked snapshots (and returns at
// once for all others).
//
// One workgroup of T threads per snapshot of up to 16 T requests.  Wave w owns the local
// indices [1024 w, 1024 (w + 1)) as four sub-blocks of 256; in sub-block j lane l holds the four
// requests 1024 w + 256 j + 4 l + c.  Steps:
//   1. load deadline/stage with 16-byte accesses; per lane and sub-block count the requests of
//      every stage in 3-bit fields of one word, which also gives a request's rank among the
//      lane's own requests of its stage; check that the deadlines never fall
//   2. per sub-block an inclusive scan of the counts across the wave's lanes (six DPP adds on two
//      words of three 10-bit fields); sub-block totals to LDS
//   3. one wave turns the 4 T / 64 sub-block totals into each sub-block's first queue slot per
//      stage, the queue starts and lengths, the stage costs at full queue length and the
//      downstream maxima over the path CSR
//   4. per request: queue slot = sub-block's first slot of its stage + requests of that stage in
//      earlier lanes + rank inside the lane; own-stage cost in the exact short-queue form,
//      estimate, drop decision; outputs leave in request order, the queue order via LDS.
#include "pard_device.hpp"

namespace pard {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
// The request arrays are read exactly once, and the estimates and decisions are written once and not looked at
// again by this call: streaming loads and stores (they leave the caches early).  The queue order is stored
// normally: the compaction that follows reads it again, slot by slot.  Measured on 4096 snapshots of 8192:
// streaming stores for estimates and decisions 122.8 -> 117.0 us per call and the compaction 47.7 -> 46.4;
// for the queue order as well 119.3 and 52.0.
template <typename V> __device__ __forceinline__ void out_store(V* p, V v) { *p = v; }
__device__ __forceinline__ int4 in_load(const int4* p) {
    const v4i x = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p));
    return make_int4(x.x, x.y, x.z, x.w);
}

constexpr int kPsStages = kPresortedMaxStages;     // 3-bit count fields of stages 0..5 plus one for slots that are not live
constexpr uint32_t kDeadStage = 7;
constexpr int kPsEntries = 128;                    // path entries of a DAG kept in LDS (longer lists are read in place)

template <int T>
struct PresortedLds {
    static constexpr int CAP = 16 * T;
    static constexpr int SUB = T / kWave * 4;                 // sub-blocks of 256 requests
    __align__(16) uint16_t ord[CAP + 8];                      // queue slot -> local index
    __align__(16) uint32_t lat[8 * PARD_LAT_ENTRIES];         // the DAG's latency tables (rows beyond the stages are never written)
    __align__(16) uint32_t quick[8][8];                       // B-1, 1/B, 1/W, aW | bW, queue start, downstream (lo, hi); rows
                                                              // beyond the stages are zero (B-1 = 0 keeps every table index in range)
    uint32_t tot[SUB][2];                                     // per sub-block: requests per stage, 10-bit fields
    __align__(16) uint16_t first_slot[SUB][8];                // per sub-block and stage: queue slot of its first request there
    int32_t edge_lo[SUB], edge_hi[SUB];                       // first and last deadline of a sub-block
    StageRec recs[kPsStages];
    unsigned long long cfull[kPsStages];
    unsigned long long down[kPsStages];
    int32_t seg_start[kPsStages + 1];
    uint32_t disorder[T / kWave];                             // per wave: it saw a deadline fall
    uint32_t ktot[SUB];                                       // kept slots per sub-block
    uint32_t ent[kPsEntries];                                 // the DAG's path entries: stage | (end of the entry's path) << 8
    uint32_t verdict;                                         // 0: in order and finished here, 1: left to the general kernel
};

// Value of the previous lane (lane 0 keeps `own`).
__device__ __forceinline__ int32_t from_previous_lane(int32_t v, int32_t own) {
    return __builtin_amdgcn_update_dpp(own, v, 0x138, 0xF, 0xF, false);               // wave_shr:1
}

// FULL: the snapshot holds exactly 16 T requests and every array is 16-byte aligned at its start.
template <int T, bool FULL>
__device__ __forceinline__ void presorted_body(const FusedArgs& A, PresortedLds<T>& L, const int u, const int64_t lo,
                                               const int m, const bool aligned, const int off) {
    constexpr int SUB = PresortedLds<T>::SUB;
    const PlanDev& P = A.plan;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int S = P.S;
    const int dag = P.shared ? 0 : u;
    const int32_t* lat_dag = P.lat + (int64_t)dag * S * PARD_LAT_ENTRIES;
    // Local index i stands for request lo_s + i; with 16-byte accesses lo_s is lo rounded down to a
    // multiple of four, and the `off` slots in front of the snapshot are not live.
    const int64_t lo_s = lo - off;
    const int m_s = m + off;
    auto live = [&](int idx) { return FULL || (idx >= off && idx < m_s); };
    auto whole = [&](int base) { return FULL || (aligned && base >= off && base + 3 < m_s); };
    const int32_t now = A.now[u];
    const int wbase = wave * 1024 + lane * 4;

    // ---- 1. loads, LDS set-up meanwhile ---------------------------------------------------
    int32_t dl[4][4];
    int32_t st[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int base = wbase + j * 256;
        if (FULL || (aligned && base < m_s && lo_s + base + 3 < A.n)) {
            const int4 d4 = in_load(reinterpret_cast<const int4*>(A.deadline + lo_s + base));
            const int4 s4 = in_load(reinterpret_cast<const int4*>(A.stage + lo_s + base));
            dl[j][0] = d4.x; dl[j][1] = d4.y; dl[j][2] = d4.z; dl[j][3] = d4.w;
            st[j][0] = s4.x; st[j][1] = s4.y; st[j][2] = s4.z; st[j][3] = s4.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const bool ok = live(base + c);
                dl[j][c] = ok ? A.deadline[lo_s + base + c] : 0;
                st[j][c] = ok ? A.stage[lo_s + base + c] : 0;
            }
        }
    }
    for (int i = tid; i < S * PARD_LAT_ENTRIES; i += T) L.lat[i] = (uint32_t)lat_dag[i];
    // The path entries are walked by one wave while the others wait (step 3): from LDS that walk is a few reads, from
    // memory a chain of dependent loads, one per stage of a path.  They are fetched here, behind the request loads.
    const int e_lo = P.dag_entry_ptr[dag], n_entries = P.dag_entry_ptr[dag + 1] - e_lo;
    const bool entries_cached = n_entries <= kPsEntries;
    if (entries_cached)
        for (int e = tid; e < n_entries; e += T)
            L.ent[e] = (uint32_t)P.entry_stage[e_lo + e] | ((uint32_t)(P.entry_end[e_lo + e] - e_lo) << 8);
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(P.recs + (int64_t)dag * S);
        uint32_t* dst = reinterpret_cast<uint32_t*>(L.recs);
        for (int i = tid; i < S * (int)(sizeof(StageRec) / 4); i += T) dst[i] = src[i];
        if (tid < kPsStages) L.down[tid] = 0;
        if (tid < SUB) L.ktot[tid] = 0;
        if (tid >= S && tid < 8) *reinterpret_cast<uint4*>(&L.quick[tid][0]) = *reinterpret_cast<uint4*>(&L.quick[tid][4]) = make_uint4(0, 0, 0, 0);
    }

    // ---- counts per lane and sub-block, order check -----------------------------------------
    uint32_t sr[4];                         // per request one byte: stage | rank among the lane's own requests of that stage << 3
    uint32_t ex0[4], ex1[4];                // requests per stage in earlier lanes of the sub-block (10-bit fields)
    bool falls = false;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int base = wbase + j * 256;
        uint32_t c24 = 0;                   // eight 3-bit counters
        sr[j] = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t k;
            if (!FULL && !live(base + c)) {
                // slots that are not live: no stage, and a deadline that keeps the sequence rising
                k = kDeadStage;
                dl[j][c] = base + c < off ? (int32_t)0x80000000 : kInt32Max;
            } else {
                k = (uint32_t)clamp_stage((int32_t)st[j][c], S);
            }
            const uint32_t f = k * 3u;
            sr[j] |= (k | (((c24 >> f) & 7u) << 3)) << (8 * c);
            c24 += 1u << f;
        }
        falls |= (dl[j][1] < dl[j][0]) | (dl[j][2] < dl[j][1]) | (dl[j][3] < dl[j][2]);
        const int32_t before = from_previous_lane(dl[j][3], dl[j][0]);
        falls |= dl[j][0] < before;
        if (lane == 0) L.edge_lo[wave * 4 + j] = dl[j][0];
        if (lane == kWave - 1) L.edge_hi[wave * 4 + j] = dl[j][3];
        // stages 0..2 and 3..5 as three 10-bit fields each (a sub-block holds 256 requests)
        const uint32_t a = c24 & 0x1FFu, b = (c24 >> 9) & 0x1FFu;
        const uint32_t own0 = (a | (a << 7) | (a << 14)) & 0x00701C07u;
        const uint32_t own1 = (b | (b << 7) | (b << 14)) & 0x00701C07u;
        const uint32_t inc0 = wave_inclusive_sum(own0);
        const uint32_t inc1 = wave_inclusive_sum(own1);
        if (lane == kWave - 1) { L.tot[wave * 4 + j][0] = inc0; L.tot[wave * 4 + j][1] = inc1; }
        ex0[j] = inc0 - own0;
        ex1[j] = inc1 - own1;
        // the three words are final here: keep the compiler from carrying the sixteen stages along instead
        asm volatile("" : "+v"(sr[j]), "+v"(ex0[j]), "+v"(ex1[j]));
    }
    const bool wave_saw_fall = __ballot(falls) != 0ull;          // all lanes take part
    if (lane == 0) L.disorder[wave] = wave_saw_fall ? 1u : 0u;
    __syncthreads();

    // ---- 3. one wave: first slots per sub-block, queue starts, stage costs, downstream maxima ----
    if (wave == 0) {
        // lane i < SUB takes sub-block i; exclusive prefix over the sub-blocks per stage
        uint32_t t0 = 0, t1 = 0;
        bool broken = false;
        if (lane < SUB) {
            t0 = L.tot[lane][0];
            t1 = L.tot[lane][1];
            if (lane > 0) broken = L.edge_lo[lane] < L.edge_hi[lane - 1];
        }
        if (lane < T / kWave) broken |= L.disorder[lane] != 0u;
        const bool disorder = __ballot(broken) != 0ull;
        uint32_t cnt[kPsStages], pre[kPsStages];
        cnt[0] = t0 & 1023u; cnt[1] = (t0 >> 10) & 1023u; cnt[2] = (t0 >> 20) & 1023u;
        cnt[3] = t1 & 1023u; cnt[4] = (t1 >> 10) & 1023u; cnt[5] = (t1 >> 20) & 1023u;
        uint32_t start = 0;                  // queue start of stage k (same in every lane)
#pragma unroll
        for (int k = 0; k < kPsStages; ++k) {
            const uint32_t inc = wave_inclusive_sum(cnt[k]);
            const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)inc, kWave - 1);
            pre[k] = start + inc - cnt[k];
            if (lane == 0) L.seg_start[k] = (int32_t)start;
            if (lane == k && k < S) {
                const StageRec& r = L.recs[k];
                L.cfull[k] = stage_cost(r, total, reinterpret_cast<const int32_t*>(L.lat) + k * PARD_LAT_ENTRIES);
                L.quick[k][0] = (uint32_t)r.B - 1u;
                L.quick[k][1] = __float_as_uint(r.rcpB);
                L.quick[k][2] = __float_as_uint(r.rcpW);
                L.quick[k][3] = r.aW;
                L.quick[k][4] = r.bW;
                L.quick[k][5] = start;
            }
            start += total;
        }
        if (lane == 0) L.seg_start[kPsStages] = (int32_t)start;
        if (lane < SUB) {
            uint4 v;
            v.x = pre[0] | (pre[1] << 16); v.y = pre[2] | (pre[3] << 16); v.z = pre[4] | (pre[5] << 16); v.w = 0u;
            *reinterpret_cast<uint4*>(&L.first_slot[lane][0]) = v;
        }
        if (lane == 0) L.verdict = disorder ? 1u : 0u;
        if (!disorder) {
            // downstream maximum per stage over the path CSR (or as given); only this wave is involved
            __builtin_amdgcn_s_waitcnt(0);
            __builtin_amdgcn_wave_barrier();
            if (A.sub) {
                if (lane < S) {
                    const int64_t v = A.sub[(int64_t)u * S + lane];
                    L.down[lane] = v < 0 ? 0ull : ((uint64_t)v < kCostCap ? (unsigned long long)v : (unsigned long long)kCostCap);
                }
            } else if (entries_cached) {
                for (int e = lane; e < n_entries; e += kWave) {
                    const uint32_t me = L.ent[e];
                    const int end = (int)(me >> 8);
                    unsigned long long sum = 0;
                    for (int t = e + 1; t < end; ++t) sum += L.cfull[L.ent[t] & 0xFFu];
                    atomicMax(&L.down[me & 0xFFu], sum);
                }
            } else {
                for (int e = e_lo + lane; e < e_lo + n_entries; e += kWave) {
                    const int end = P.entry_end[e];
                    unsigned long long sum = 0;
                    for (int t = e + 1; t < end; ++t) sum += L.cfull[P.entry_stage[t]];
                    atomicMax(&L.down[P.entry_stage[e]], sum);
                }
            }
            __builtin_amdgcn_s_waitcnt(0);
            __builtin_amdgcn_wave_barrier();
            if (lane < S) {
                const unsigned long long d = L.down[lane];
                L.quick[lane][6] = (uint32_t)d;
                L.quick[lane][7] = (uint32_t)(d >> 32);
            }
        }
    }
    __syncthreads();
    if (L.verdict != 0u) {                   // not in key order: the general kernel takes this snapshot
        if (tid == 0) A.todo[u] = 1u;
        return;
    }
    if (tid == 0) A.todo[u] = 0u;

    // ---- 4. queue slot, estimate, drop decision -------------------------------------------------
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int base = wbase + j * 256;
        // requests of every stage in earlier lanes of this sub-block: six 10-bit fields of a 64-bit word
        const unsigned long long before = (unsigned long long)ex0[j] | ((unsigned long long)ex1[j] << 30);
        const uint16_t* fs = &L.first_slot[wave * 4 + j][0];
        int32_t est[4];
        uint8_t drp[4];
        asm volatile("" ::: "memory");       // one sub-block at a time (register pressure)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t k = (sr[j] >> (8 * c)) & 7u;     // slots that are not live compute on the zeroed rows of stage 7 and are discarded
            const uint32_t slot = (uint32_t)fs[k] + ((uint32_t)(before >> (k * 10u)) & 1023u) + ((sr[j] >> (8 * c + 3)) & 7u);
            const uint4 qa = *reinterpret_cast<const uint4*>(&L.quick[k][0]);     // B-1, 1/B, 1/W, aW
            const uint4 qb = *reinterpret_cast<const uint4*>(&L.quick[k][4]);     // bW, queue start, downstream
            const uint32_t pos = slot - qb.y;
            const uint32_t q = (uint32_t)(((float)(pos + qa.x) + 0.5f) * __uint_as_float(qa.y));
            const uint32_t p = __umul24(q, qb.x);
            const uint32_t wait = __umul24(q, qa.w) + (uint32_t)(((float)p + 0.5f) * __uint_as_float(qa.z));
            const uint32_t seen = pos < qa.x ? pos : qa.x;
            const uint64_t dn = (uint64_t)qb.z | ((uint64_t)qb.w << 32);
            const uint64_t e64 = (uint64_t)wait + L.lat[k * PARD_LAT_ENTRIES + seen] + dn;
            finish_request(e64, now, dl[j][c], est[c], drp[c]);
            if (live(base + c)) {
                L.ord[slot] = (uint16_t)((uint32_t)(base + c) | ((uint32_t)drp[c] << 15));   // local index < 2^13
                if (A.kept && !drp[c]) atomicAdd(&L.ktot[(slot + (uint32_t)off) >> 8], 1u);     // kept slots per sub-block of the slot layout
            }
        }
        if (whole(base)) {
            stream_store(reinterpret_cast<int4*>(A.est + lo_s + base), make_int4(est[0], est[1], est[2], est[3]));
            stream_store(reinterpret_cast<uint32_t*>(A.drop + lo_s + base),
                      (uint32_t)drp[0] | ((uint32_t)drp[1] << 8) | ((uint32_t)drp[2] << 16) | ((uint32_t)drp[3] << 24));
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (live(base + c)) { A.est[lo_s + base + c] = est[c]; A.drop[lo_s + base + c] = drp[c]; }
        }
    }
    __syncthreads();

    // ---- queue order and queue offsets out --------------------------------------------------------
    // (an entry of ord[] is local index | drop << 15)
    const int32_t b32 = (int32_t)lo_s;
    uint32_t entry[4][4];                    // this thread's sixteen queue slots (slot = local index - off)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int base = wbase + j * 256;
        // queue slot q sits at order[lo + q] = order[lo_s + (q + off)]
        if (whole(base)) {
            if (off == 0) {
                const uint2 o = *reinterpret_cast<const uint2*>(L.ord + base);
                entry[j][0] = o.x & 0xFFFFu; entry[j][1] = o.x >> 16;
                entry[j][2] = o.y & 0xFFFFu; entry[j][3] = o.y >> 16;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c) entry[j][c] = L.ord[base - off + c];
            }
            out_store(reinterpret_cast<int4*>(A.order + lo_s + base),
                      make_int4(b32 + (int32_t)(entry[j][0] & 0x7FFFu), b32 + (int32_t)(entry[j][1] & 0x7FFFu),
                                b32 + (int32_t)(entry[j][2] & 0x7FFFu), b32 + (int32_t)(entry[j][3] & 0x7FFFu)));
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                entry[j][c] = 0x8000u;       // not a slot: counts as dropped below
                if (live(base + c)) {
                    entry[j][c] = L.ord[base - off + c];
                    A.order[lo_s + base + c] = b32 + (int32_t)(entry[j][c] & 0x7FFFu);
                }
            }
        }
    }
    if (tid < S) A.seg_ptr[(int64_t)u * S + tid] = (int32_t)lo + L.seg_start[tid];
    if (u == P.K - 1 && tid == 0) A.seg_ptr[(int64_t)P.K * S] = (int32_t)(lo + m);
    if (!A.kept) return;

    // ---- survivors of this snapshot in queue order, staged at the snapshot's own place ----------------
    // (the compaction's last kernel moves them to their final place once the counts of all snapshots are known)
    uint32_t keep[4];
    uint32_t c0 = 0, c1 = 0;                 // kept slots per sub-block: three 10-bit fields, and the fourth
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        keep[j] = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) keep[j] |= ((entry[j][c] >> 15) ^ 1u) << c;
        const uint32_t cnt = (uint32_t)__popc(keep[j]);
        if (j < 3) c0 |= cnt << (10 * j); else c1 = cnt;
    }
    const uint32_t i0 = wave_inclusive_sum(c0), i1 = wave_inclusive_sum(c1);
    // kept slots in earlier sub-blocks: every wave scans the sub-block totals itself
    const uint32_t tk = lane < SUB ? L.ktot[lane] : 0u;
    const uint32_t ik = wave_inclusive_sum(tk);
    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)ik, kWave - 1);
    const uint32_t xk = ik - tk;
    const uint32_t e0 = i0 - c0, e1 = i1 - c1;
    int32_t* stage_at = A.staged + lo + staging_shift(u, (uint32_t)m, total);
    // a queue's first slot, in this layout, for the threads that happen to hold it
    int qs[kPsStages];
#pragma unroll
    for (int k = 0; k < kPsStages; ++k) qs[k] = L.seg_start[k] + off;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int base = wbase + j * 256;
        const uint32_t sub_before = (uint32_t)__builtin_amdgcn_readlane((int)xk, wave * 4 + j);
        uint32_t o = sub_before + (j < 3 ? (e0 >> (10 * j)) & 1023u : e1);
        // survivors of the snapshot before each queue: written by whoever holds the queue's first slot
#pragma unroll
        for (int k = 0; k < kPsStages; ++k)
            if (k < S && (qs[k] >> 2) == (base >> 2) && qs[k] < m_s)
                A.loc_ptr[(int64_t)u * S + k] = (int32_t)(o + (uint32_t)__popc(keep[j] & ((1u << (qs[k] & 3)) - 1u)));
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (keep[j] & (1u << c)) { stage_at[o] = b32 + (int32_t)(entry[j][c] & 0x7FFFu); ++o; }
    }
    if (tid < S && L.seg_start[tid] + off >= m_s) A.loc_ptr[(int64_t)u * S + tid] = (int32_t)total;   // queues that start at the end
    if (tid == 0) A.kept[u] = total;
}

// Six waves per SIMD (three workgroups of 512 per compute unit): measured faster than four (128 registers) and
// as fast as eight, which no longer fits the registers without spilling.
#ifndef PARD_PS_WAVES
#define PARD_PS_WAVES 6
#endif
template <int T>
__global__ __launch_bounds__(T, PARD_PS_WAVES) void presorted_snapshot_kernel(FusedArgs A) {
    constexpr int kCap = 16 * T;
    __shared__ PresortedLds<T> L;
    const int u = blockIdx.x;
    const int64_t n = A.n;
    // snapshot bounds, made safe whatever snap_ptr holds
    int64_t lo = A.snap_ptr[u], hi = A.snap_ptr[u + 1];
    if (lo < 0) lo = 0;
    if (lo > n) lo = n;
    if (hi > n) hi = n;
    int64_t m64 = hi - lo;
    if (m64 < 0) m64 = 0;
    const int limit = A.cap < kCap ? A.cap : kCap;
    if (m64 > limit) {
        // larger than promised: the general kernel truncates it and raises the status bit
        if (threadIdx.x == 0) A.todo[u] = 1u;
        return;
    }
    const int m = (int)m64;
    if (m >= 256) {
        // A first look at 64 deadlines spread evenly over the snapshot, before anything else is loaded: a snapshot
        // in random order fails it at once and costs a few cache lines here instead of a whole pass.  Every wave
        // looks at the same 64 values, so the decision needs no barrier.  (A snapshot in queue order passes: a
        // subsequence of a rising sequence rises.)
        const int lane = threadIdx.x & (kWave - 1);
        const int32_t d = A.deadline[lo + ((lane * m) >> 6)];
        if (__ballot(d < from_previous_lane(d, d)) != 0ull) {
            if (threadIdx.x == 0) A.todo[u] = 1u;
            return;
        }
    }
    const uintptr_t bits = reinterpret_cast<uintptr_t>(A.deadline) | reinterpret_cast<uintptr_t>(A.stage) |
                           reinterpret_cast<uintptr_t>(A.est) | reinterpret_cast<uintptr_t>(A.order) |
                           (reinterpret_cast<uintptr_t>(A.drop) << 2);
    const int shift = (int)(lo & 3);
    const bool aligned = (bits & 15) == 0 && m + shift <= kCap;
    const int off = aligned ? shift : 0;
    if (m == kCap && aligned && off == 0) presorted_body<T, true>(A, L, u, lo, m, true, 0);
    else presorted_body<T, false>(A, L, u, lo, m, aligned, off);
}

}  // namespace

// Promised bounds of at most 512 requests stay with the general kernel: the smallest workgroup here is laid out for 1024
// requests, and below about half of that the general kernel's smaller capacities are as fast or faster (65,536
// snapshots of 256 in queue order: 0.210 ms per call through this kernel, 0.148 through the general one; of 512:
// 0.234 either way; 43,690 of 768: 0.181 against 0.270).
bool presorted_path_covers(const FusedArgs& a) {
    return a.todo != nullptr && a.plan.presorted_ok && !a.consistent && a.plan.uniform_mode == PARD_ORDER_LBF &&
           a.plan.S <= kPresortedMaxStages && a.cap > 512 && a.cap <= PARD_FUSED_SNAPSHOT_CAPACITY;
}

hipError_t launch_presorted(const FusedArgs& a, hipStream_t stream) {
    const dim3 grid((unsigned)a.plan.K);
    if (a.cap <= 1024) presorted_snapshot_kernel<64><<<grid, dim3(64), 0, stream>>>(a);
    else if (a.cap <= 2048) presorted_snapshot_kernel<128><<<grid, dim3(128), 0, stream>>>(a);
    else if (a.cap <= 4096) presorted_snapshot_kernel<256><<<grid, dim3(256), 0, stream>>>(a);
    else presorted_snapshot_kernel<512><<<grid, dim3(512), 0, stream>>>(a);
    return hipGetLastError();
}

}  // namespace pard
